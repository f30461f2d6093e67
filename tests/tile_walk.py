"""Where to sample a full-size regeneration: rows placed by the projection kernel's tile walk (test helper)."""


def tile_walk_rows(cfg, grid=256, tile=256, group_m=4, xcds=8):
    """Checkpoint rows of a full-size configuration chosen by where the large-problem projection kernel meets
    them, as (stratum, global row) pairs.  The kernel is persistent: workgroup p of `grid` takes tiles p, p + grid,
    p + 2 grid, ... of the walk; tile numbers are regrouped so that each of the 8 XCDs owns a contiguous range, and
    that range is walked in bands of 4 row tiles, column-major inside a band.  A sampled row is compared over all
    2d output features, i.e. over every column tile of its row tile (each held by another workgroup).  This
    mirrors the walk only to decide WHERE to look; the expected values come from the oracle."""
    M, d = cfg.M, cfg.d
    tiles_m, tiles_n = (M + tile - 1) // tile, (2 * d + tile - 1) // tile
    n_tiles = tiles_m * tiles_n
    grid = min(grid, n_tiles)

    def coords(pid):                                       # position in the walk -> (row tile, column tile)
        per, rem = divmod(n_tiles, xcds)
        xcd, local = pid % xcds, pid // xcds
        t = xcd * per + min(xcd, rem) + local
        band = group_m * tiles_n
        g = t // band
        first_m = g * group_m
        rows = min(tiles_m - first_m, group_m)
        inb = t - g * band
        return first_m + inb % rows, inb // rows

    picks = []

    def add(label, tm, r):
        m = tm * tile + r
        if 0 <= m < M:
            picks.append((label, m))

    # a handful of workgroups: the first and the last tile each of them walks (cold pipeline / drained ring)
    for p in (0, 1, grid // 2, grid - 1):
        my = (n_tiles - p + grid - 1) // grid
        for which, jj in (("first", 0), ("last", my - 1)):
            tm, tn = coords(p + jj * grid)
            add("workgroup %d %s tile (row tile %d, column tile %d)" % (p, which, tm, tn), tm, 0)
            add("workgroup %d %s tile, last row" % (p, which), tm, tile - 1)
    # rows inside a tile: its edges, the seam between the two wavefront rows, MFMA block seams
    mid = tiles_m // 2
    for r in (0, 15, 16, 127, 128, 255):
        add("row %d of row tile %d" % (r, mid), mid, r)
    # band edges of the walk (bands of 4 row tiles) and the seams between the XCDs' ranges of tiles
    for tm in (3, 4, tiles_m - 5, tiles_m - 4):
        add("band edge, row tile %d" % tm, tm, 1)
    per = n_tiles // xcds
    for x in (1, 4, 7):
        for t in (x * per - 1, x * per):                   # last tile of one XCD's range, first of the next
            pid = (t - (t // per) * per) * xcds + t // per if n_tiles % xcds == 0 else None
            if pid is not None and pid < n_tiles:
                tm, tn = coords(pid)
                add("XCD range seam at tile %d (row tile %d)" % (t, tm), tm, 2)
    # the last row tile (partial when M is not a multiple of 256) and the last row of all
    add("first row of the last row tile", tiles_m - 1, 0)
    picks.append(("last row", M - 1))
    # rows whose byte offset into the checkpoint tensor needs more than 31 bits
    far = (1 << 31) // (2 * d) + 1
    if far < M:
        picks.append(("first row past 2^31 bytes", far))
        picks.append(("row past 2^31 bytes, mid tile", (far // tile + 1) * tile + 77))
    if 2 * far < M:
        picks.append(("first row past 2^32 bytes", 2 * far))
    seen, out = set(), []
    for label, m in picks:
        if m not in seen and 0 <= m < M:
            seen.add(m)
            out.append((label, m))
    return out
