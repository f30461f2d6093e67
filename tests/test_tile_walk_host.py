"""The row placement used by the full-size GPU parity tests (host arithmetic only, no GPU)."""
from paper_2501_01792_amd import synth
from tile_walk import tile_walk_rows as _tile_walk_rows


def test_tile_walk_strata_cover_what_they_claim():
    """The row placement itself (host arithmetic, no GPU work): on the OPT-66B-shaped layer it names rows in the
    first and last tile of several workgroups, both edges of a tile, band edges, XCD seams, the last row, and rows
    beyond 2^31 and 2^32 bytes into the checkpoint tensor."""
    strata = _tile_walk_rows(synth.CONFIGS["opt66b"])
    labels = " | ".join(l for l, _ in strata)
    for word in ("workgroup 0 first", "workgroup 255 last", "row 255 of", "band edge", "XCD range seam", "last row",
                 "past 2^31", "past 2^32"):
        assert word in labels, word
    rows = [m for _, m in strata]
    assert 30 <= len(rows) <= 80 and len(set(rows)) == len(rows) and max(rows) == synth.CONFIGS["opt66b"].M - 1
    assert any(m * 9216 * 2 >= 1 << 32 for m in rows)
    # a ragged problem: the last row tile is partial and is sampled
    cfg = synth.LayerConfig("ragged", 1024, 8, 3, 300, 0.0, 1)         # M = 900 = 3 tiles + 132 rows
    rows = [m for _, m in _tile_walk_rows(cfg)]
    assert 768 in rows and 899 in rows and max(rows) == 899
