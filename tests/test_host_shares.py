"""Invariants of the kernels' work-share arithmetic (which workgroup streams which units,
which workgroups share an item), evaluated on the host through the library.

The kernels rely on: every unit is streamed exactly once; a workgroup's range is contiguous
and the ranges of an XCD's workgroups are balanced within one unit; an item (a row slice of a
linear layer) is always finished inside one XCD; only the first and the last item of a
workgroup's range can be shared with other workgroups (two partial-sum slots per workgroup);
and a workgroup is the first part of at most one shared item (one counter line per
workgroup)."""
import ctypes as C

import pytest

from paper_2505_23219_amd import binding as B


def share(lib, items, per_item, j, G, item=0):
    out = (C.c_int * 5)()
    lib.ghd_debug_share(items, per_item, j, G, item, out)
    return list(out)


CASES = [
    # items, units per item, workgroups
    (48, 32, 256), (16, 32, 256), (86, 32, 256), (16, 86, 256), (125, 32, 256),   # the 7B layers (256-row groups)
    (96, 16, 256), (172, 16, 256), (500, 8, 256),                                  # row-split variants
    (3, 2, 256), (1, 1, 256), (7, 5, 256), (300, 1, 256), (9, 1000, 256),
    (5, 3, 16), (40, 7, 24), (13, 9, 8), (11, 4, 7), (2, 50, 5),                   # small grids, also not a multiple of 8
    # row blocks x k-steps of the packed 7B / 13B matrices (wide ones tile by tile, narrow ones in
    # blocks of four tiles), one and two shares per workgroup
    (768, 128, 256), (64, 128, 256), (1376, 128, 256), (64, 344, 256), (2000, 128, 512),
    (960, 160, 256), (80, 160, 256), (1728, 160, 256), (80, 432, 256), (2000, 160, 512),
]


@pytest.mark.parametrize("items,per_item,G", CASES)
def test_share_invariants(items, per_item, G):
    lib = B.lib()
    nx = 8 if G % 8 == 0 else 1
    Gx = G // nx
    total = items * per_item
    ranges = [share(lib, items, per_item, j, G)[:2] for j in range(G)]
    # every unit exactly once, ranges contiguous in workgroup order inside an XCD
    covered = 0
    for x in range(nx):
        i0, i1 = items * x // nx, items * (x + 1) // nx
        pos = i0 * per_item
        sizes = []
        for j in range(x * Gx, (x + 1) * Gx):
            c0, c1 = ranges[j]
            if c0 == c1:
                continue
            assert c0 == pos and c1 > c0
            sizes.append(c1 - c0)
            pos = c1
        assert pos == i1 * per_item                       # the XCD's items, all of them
        covered += pos - i0 * per_item
        if sizes:
            assert max(sizes) - min(sizes) <= 1
            assert len(sizes) == min(Gx, (i1 - i0) * per_item)
    assert covered == total
    # per item: its parts are exactly the workgroups whose range meets it
    first_count = {}
    for item in range(items):
        lo, hi = item * per_item, (item + 1) * per_item
        parts = [j for j in range(G) if ranges[j][0] < hi and ranges[j][1] > lo]
        assert parts == list(range(parts[0], parts[-1] + 1))
        assert parts[0] // Gx == parts[-1] // Gx          # inside one XCD
        for j in parts:
            _, _, first, last, begins = share(lib, items, per_item, j, G, item)
            assert (first, last) == (parts[0], parts[-1])
            assert begins == (1 if ranges[j][0] >= lo else 0)
        if len(parts) > 1:
            first_count[parts[0]] = first_count.get(parts[0], 0) + 1
    assert all(v == 1 for v in first_count.values())      # one counter line per workgroup is enough
    # only the first and the last item of a range can be shared
    for j in range(G):
        c0, c1 = ranges[j]
        if c0 == c1:
            continue
        for item in range(c0 // per_item + 1, (c1 - 1) // per_item):
            assert item * per_item >= c0 and (item + 1) * per_item <= c1


@pytest.mark.parametrize("M,N,K", [(64, 12288, 4096), (64, 4096, 4096), (64, 22016, 4096), (64, 4096, 11008),
                                   (64, 32000, 4096), (1, 32000, 4096), (128, 22016, 4096), (128, 32000, 4096),
                                   (64, 15360, 5120), (64, 27648, 5120), (16, 160000, 4096), (128, 16384 * 16, 64),
                                   (1, 4096, 4096), (16, 4096, 11008), (17, 4096, 11008), (8, 5120, 13824), (3, 130, 688)])
def test_linear_plan(M, N, K):
    """The cut of a linear layer.  A wide matrix (640 tiles of 16 rows or more) is dealt out in
    whole tiles, so that no share has more tiles than the kernel keeps accumulators for (8 up to
    64 rows of x, 4 above), with as few shares per workgroup as that takes.  So is a narrow one at
    up to 16 rows of x if its tiles spread evenly enough over the workgroups; otherwise a narrow
    one streams a k range of one block of four tiles at a time, one share per workgroup."""
    lib = B.lib()
    G = 256
    out = (C.c_int * 3)()
    rc = lib.ghd_debug_plan(M, N, K, G, out)
    ntiles = (N + 15) // 16
    cap = 8 if M <= 64 else 4

    def most(P):
        worst = 0
        for j in range(G * P):
            c0, c1 = share(lib, ntiles, 1, j, G * P)[:2]
            worst = max(worst, c1 - c0)
        return worst

    feasible = [P for P in range(1, 9) if most(P) <= cap]
    whole = bool(feasible)
    if ntiles < 640:
        if M > 16:
            whole = False
        elif whole:
            P = feasible[0]
            excess = most(P) * P * G / ntiles - 1.0
            whole = excess * (2.0 * N * K / 6.4e6) < 3.0
        if not whole:
            assert rc == 0 and list(out) == [4, 1, 0]
            return
    if not feasible:
        assert rc == -1
        return
    assert rc == 0 and out[2] == 1 and out[1] == feasible[0] and out[0] == most(feasible[0]) and 1 <= out[0] <= cap


def test_linear_plan_known_shapes():
    """7B-shaped output and down projections (256 tiles on 256 workgroups) go whole-tile at one
    row of x; the 13B-shaped ones (320 tiles: shares of one and two) do not."""
    lib = B.lib()
    out = (C.c_int * 3)()
    for (M, N, K), want in [((1, 4096, 4096), [1, 1, 1]), ((16, 4096, 11008), [1, 1, 1]), ((17, 4096, 4096), [4, 1, 0]),
                            ((1, 5120, 5120), [4, 1, 0]), ((1, 5120, 13824), [4, 1, 0]), ((64, 22016, 4096), [6, 1, 1]),
                            ((64, 12288, 4096), [3, 1, 1]), ((128, 22016, 4096), [3, 2, 1])]:
        assert lib.ghd_debug_plan(M, N, K, 256, out) == 0 and list(out) == want, (M, N, K, list(out))


def attn_share(lib, nh, ntile, j, G, head):
    out = (C.c_int * 6)()
    lib.ghd_debug_attn_share(nh, ntile, j, G, head, out)
    return list(out)


@pytest.mark.parametrize("nh,ntile,G", [
    (32, 33, 256), (40, 129, 256), (32, 1, 256), (4, 3, 256), (2, 5, 256), (256, 2, 256), (100, 17, 256),
    (1, 40, 256), (7, 9, 256), (3, 2, 8), (5, 4, 16), (9, 3, 24), (4, 6, 7), (300, 2, 256),
])
def test_attention_share_invariants(nh, ntile, G):
    """Every (head, key tile) pair belongs to exactly one workgroup; the parts of a head are
    consecutive workgroups of one XCD, at most 64 of them (the merge keeps one part per
    lane), each with a contiguous, non-empty tile range, in order."""
    lib = B.lib()
    nx = 8 if G % 8 == 0 else 1
    Gx = G // nx
    for head in range(nh):
        parts = {}
        for j in range(G):
            first, np_, me, t0, t1, mine = attn_share(lib, nh, ntile, j, G, head)
            if not mine or me >= np_:
                continue
            parts[me] = (j, first, np_, t0, t1)
        assert parts, head
        np_ = next(iter(parts.values()))[2]
        first = next(iter(parts.values()))[1]
        assert sorted(parts) == list(range(np_)) and 1 <= np_ <= 64
        pos = 0
        for me in range(np_):
            j, f, n, t0, t1 = parts[me]
            assert (f, n) == (first, np_) and j == first + me
            assert j // Gx == first // Gx                 # one XCD
            assert t0 == pos and t1 > t0
            pos = t1
        assert pos == ntile
        sizes = [parts[me][4] - parts[me][3] for me in range(np_)]
        assert max(sizes) - min(sizes) <= 1 and sizes[-1] == min(sizes)   # the last part gets a short range
