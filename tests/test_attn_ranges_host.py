"""Host check of the slot bookkeeping of the attention kernels (csrc/attn_ranges.h: which partial slots the
wavefronts write, which the merge reads), compiled for the CPU and replayed with plain loops.  No GPU."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("ranges") / "attn_ranges_check")
    subprocess.check_call(["g++", "-O1", "-std=c++17", os.path.join(HERE, "host", "attn_ranges_check.cpp"), "-o", exe])

    def run(H, W, clamp, lens):
        out = subprocess.check_output([exe, str(H), str(W), str(int(clamp))] + [str(n) for n in lens], text=True)
        unwritten, double, pairs, waves = (int(v) for v in out.split())
        return unwritten, double, pairs, waves
    return run


def test_every_slot_the_merge_reads_is_written(checker):
    """Launches sized for the tokens that are there (W <= total) and launches sized for an upper bound far above
    (W > total: a graph captured for 4096 tokens serving 2 .. 40): with the kernels' clamp of the working
    wavefronts no merge reads a slot that was not written, and no slot is written twice."""
    cases = [(72, 3072, [16]), (72, 2304, [2]), (72, 2304, [33]), (12, 3072, [1, 0, 5, 0, 0, 17]), (4, 24, [0, 5, 0, 17, 3]),
             (32, 3072, [1024, 700, 1, 0, 333]), (8, 7, [300]), (8, 3072, [1]), (1, 64, [1]), (5, 3072, [0, 0, 0])]
    for H, W, lens in cases:
        unwritten, double, pairs, waves = checker(H, W, True, lens)
        assert unwritten == 0 and double == 0, (H, W, lens, unwritten, double)
        assert pairs == H * sum(1 for n in lens if n > 0)
        assert waves == min(W, H * sum(lens))


def test_the_clamp_is_what_makes_it_so(checker):
    """The same replay without the clamp: 72 heads, 16 cached tokens and a launch of 3072 wavefronts leave
    unwritten slots between the working wavefronts (the failure the clamp removes)."""
    unwritten, double, _, _ = checker(72, 3072, False, [16])
    assert unwritten > 0 and double == 0
