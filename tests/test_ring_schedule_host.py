"""The LDS ring of the persistent projection kernel (csrc/kv_gemm_fold.hip), replayed on the host.

The kernel streams the k blocks of all of a workgroup's tiles through a ring of 5 slots, two units (weights,
activations) per k block, with a load cursor that runs two k blocks ahead of the matrix cores and crosses from one
tile to the next before the current tile's last two k blocks are consumed.  This model restates that schedule
(slot rotation, which unit is issued early and which late, where the cursor switches tiles, where the row table
lives at a tile's end) and checks what the kernel relies on:
  * every k block is consumed from slots that hold exactly that block's two units, issued at least one barrier earlier;
  * no slot is overwritten between the issue of a unit and the last read of it;
  * the row table's slot is free from the last barrier of a tile until the next tile's first early loads;
  * after the workgroup's last tile the cursor stays on that tile's last k block (loads go on, nobody reads them).
It runs for every combination of 1..4 tiles per workgroup and 2..9 k blocks per tile (2 and 3 are the special cases of
the loop structure: a tile's first k block is its last but one; the main loop is empty).
"""
import itertools

import pytest

SLOTS = 5


def next2(s):
    return (s + 2) % SLOTS


def replay(my_tiles, nks, switch_late=False, late_into_second=False):
    """Returns the list of consumed (tile, kb); raises AssertionError where the schedule breaks.  The two flags plant
    mistakes (the cursor leaves a tile one k block late; the late loads go into the second unit's slot)."""
    content = [None] * SLOTS          # what a slot holds: (unit, tile, kb), unit 0 = first (weights), 1 = second (activations)
    issued_at = [None] * SLOTS        # barrier count at which the slot's current content was issued
    barriers = 0
    ld = {"tile": 0, "kb": 0, "step": 1}

    def issue(slot, unit):
        content[slot] = (unit, ld["tile"], ld["kb"])
        issued_at[slot] = barriers

    def next_load_tile(c_j):
        if c_j + 1 < my_tiles:
            ld["tile"], ld["kb"] = c_j + 1, 0
        else:
            ld["kb"], ld["step"] = nks - 1, 0

    # prologue: k blocks 0 and 1 of tile 0 into slots 0..3, then a barrier
    for s in range(2):
        issue(2 * s, 0)
        issue(2 * s + 1, 1)
        ld["kb"] += 1
    barriers += 1
    s1, s2 = 0, 1
    consumed = []

    def stage(tile, kb):
        nonlocal s1, s2, barriers
        n1, n2 = next2(s1), next2(s2)
        early, late = next2(n1), (s2 if late_into_second else s1)
        # the block being consumed sits in (s1, s2) and was issued before the last barrier
        for slot, unit in ((s1, 0), (s2, 1)):
            assert content[slot] == (unit, tile, kb), ("consumed slot holds", content[slot], "wanted", (unit, tile, kb))
            assert issued_at[slot] < barriers, "unit consumed without a barrier after its issue"
        # sub-step 0: early loads (first unit of the block two ahead) into the spare slot
        assert early not in (s1, s2, n1, n2), "early loads overwrite a slot still in use"
        issue(early, 0)
        # barrier early in sub-step 1: block g+1 must be complete and a barrier old
        barriers += 1
        for slot in (n1, n2):
            assert issued_at[slot] < barriers
        # behind the barrier: all reads of block g are done, its first slot takes the late loads
        assert late not in (n1, n2, early)
        issue(late, 1)
        ld["kb"] += ld["step"]
        consumed.append((tile, kb))
        s1, s2 = n1, n2

    for c_j in range(my_tiles):
        if nks == 2:
            next_load_tile(c_j)
        stage(c_j, 0)
        for kb in range(1, nks - 2):
            stage(c_j, kb)
        if nks > 2:
            if not switch_late:
                next_load_tile(c_j)
            stage(c_j, nks - 2)
            if switch_late:
                next_load_tile(c_j)
        stage(c_j, nks - 1)
        # tile end: the row table takes the slot of the second unit of the block just consumed
        s_tab = (s2 - 2) % SLOTS
        in_flight_or_landed = {s1, s2, next2(s1), (s1 - 2) % SLOTS}     # block g+1 (2 slots), early and late loads of g+2
        assert s_tab not in in_flight_or_landed, "the row table's slot is in use"
        assert next2(next2(s1)) == s_tab, "the next stage's early loads are what reclaims the table's slot"
    return consumed, ld


@pytest.mark.parametrize("my_tiles,nks", list(itertools.product(range(1, 5), range(2, 10))))
def test_ring_schedule_consumes_every_block_from_the_right_slots(my_tiles, nks):
    consumed, ld = replay(my_tiles, nks)
    assert consumed == [(t, k) for t in range(my_tiles) for k in range(nks)]
    # after the last tile the cursor rests on that tile's last k block
    assert ld["tile"] == my_tiles - 1 and ld["kb"] == nks - 1 and ld["step"] == 0


@pytest.mark.parametrize("mistake", ["switch_late", "late_into_second"])
def test_ring_model_catches_planted_mistakes(mistake):
    """The model is not vacuous: a cursor that leaves a tile one k block late, or late loads that go into the slot of
    the block's second unit, break an assertion."""
    with pytest.raises(AssertionError):
        replay(3, 6, **{mistake: True})
