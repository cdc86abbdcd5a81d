"""How the forward, dX and dW GEMMs divide their work among workgroups, checked on the host for many shapes.

The kernels compute an output tile either whole, in one workgroup, or in pieces along K: as the head and tail of
"runs" (two contributors at most), or split among a group of workgroups.  The function that tells a workgroup its
items is compiled for host and device alike; `eqat_plan_item` calls the host side of it with the launch geometry the
library would use.  Here every workgroup's items are listed and it is checked that every K-tile pair of every tile is
computed exactly once, that what a piece says about its tile (contributors, first contributor, counter) is what the
pieces of that tile really are, and that no two tiles cut in one launch share a counter.  No GPU is needed (without one
the library plans for the 256 compute units of an MI355X).
"""
import ctypes

import numpy as np
import pytest

import paper_2407_11062_amd as eq


def items_of_launch(T, I, O, gemm):
    L = eq.lib()
    d = eq.make_desc(T, I, O, 2, 32, eq.BF16, eq.BF16)
    item = (ctypes.c_int32 * 12)()
    exists = ctypes.c_int32(0)

    def ask(block, j):
        rc = L.eqat_plan_item(ctypes.byref(d), gemm, block, j, item, ctypes.byref(exists))
        assert rc == 0, eq.lib().eqat_status_string(rc)
        return bool(exists.value), list(item)

    _, first = ask(0, 0)
    grid, pairs, tiles_m, tiles_n = first[8], first[9], first[10], first[11]
    out = []
    for block in range(grid):
        j = 0
        while True:
            ok, it = ask(block, j)
            if not ok:
                break
            out.append((block, j, it))
            j += 1
            assert j <= 64, "a workgroup with more than 64 items"
    # past the launch: an error, not an item
    assert L.eqat_plan_item(ctypes.byref(d), gemm, grid, 0, item, ctypes.byref(exists)) != 0
    return out, grid, pairs, tiles_m, tiles_n


def check_launch(T, I, O, gemm):
    items, grid, pairs, tiles_m, tiles_n = items_of_launch(T, I, O, gemm)
    M, N, K = (T, O, I) if gemm == 0 else (T, I, O) if gemm == 1 else (I, O, T)
    assert pairs == ((K + 63) // 64 + 1) // 2
    assert grid % 8 == 0 or grid == tiles_m * tiles_n
    cover = np.zeros((tiles_m, tiles_n, pairs), dtype=np.int32)
    pieces = {}                                   # tile -> list of (contributor index in its XCD, xcd, kb, ke, item)
    for block, j, (tm, tn, kb, ke, parts, first, fixed, ctr, *_rest) in items:
        assert 0 <= tm < tiles_m and 0 <= tn < tiles_n, (block, j, tm, tn)
        assert 0 <= kb < ke <= pairs, (block, j, kb, ke)
        cover[tm, tn, kb:ke] += 1
        pieces.setdefault((tm, tn), []).append((block >> 3, block & 7, kb, ke, parts, first, fixed, ctr))
    assert (cover == 1).all(), f"{int((cover != 1).sum())} K-tile pairs computed {sorted(set(cover.ravel()))} times"
    counters = {}
    for tile, ps in pieces.items():
        ps.sort(key=lambda p: p[2])
        xcds = {p[1] for p in ps}
        assert len(xcds) == 1, f"tile {tile} has pieces on XCDs {xcds}"
        parts, first, fixed, ctr = ps[0][4:]
        assert all(p[4:] == (parts, first, fixed, ctr) for p in ps), f"the pieces of tile {tile} disagree about it"
        assert parts == len(ps)
        if parts == 1:
            assert ps[0][2] == 0 and ps[0][3] == pairs
            continue
        # contributors first .. first + parts - 1 of the XCD, in the order of their K ranges, which join up
        assert [p[0] for p in ps] == list(range(first, first + parts)), (tile, [p[0] for p in ps], first, parts)
        assert ps[0][2] == 0 and ps[-1][3] == pairs and all(a[3] == b[2] for a, b in zip(ps, ps[1:]))
        assert fixed in (0, 1) and (fixed == 1 or parts == 2), "runs have two contributors"
        assert 0 <= ctr < 2 * grid
        assert ctr not in counters, f"tiles {tile} and {counters.get(ctr)} share counter {ctr}"
        counters[ctr] = tile
    return len(counters), grid, tiles_m * tiles_n


BENCH_SHAPES = [      # (tokens, in, out) of the benchmark's linears
    (8192, 4096, 4096), (8192, 4096, 11008), (8192, 11008, 4096),
    (4096, 4096, 4096), (4096, 4096, 11008), (4096, 11008, 4096),
    (4096, 5120, 5120), (4096, 5120, 13824), (4096, 13824, 5120),
    (4096, 8192, 8192), (4096, 8192, 1024), (4096, 8192, 28672), (4096, 28672, 8192), (4096, 8192, 10240), (4096, 8192, 57344),
]


@pytest.mark.parametrize("T,I,O", BENCH_SHAPES)
@pytest.mark.parametrize("gemm", [0, 1, 2], ids=["fwd", "dx", "dw"])
def test_every_k_tile_pair_of_every_tile_is_computed_once_at_the_benchmark_shapes(T, I, O, gemm):
    check_launch(T, I, O, gemm)


def test_the_three_ways_of_dividing_the_work_all_occur():
    # 13B q projection: 320 tiles = 1.25 rounds: a whole tile each, the other 64 tiles split four ways
    cut, grid, ntiles = check_launch(4096, 5120, 5120, 0)
    assert (cut, grid, ntiles) == (64, 256, 320)
    # 1.625 rounds: more than half a round beyond the first: runs
    cut, grid, ntiles = check_launch(4096, 5120, 6656, 0)
    assert grid == 256 and ntiles == 416 and cut > 64
    # 7B gate projection: 5.375 rounds: five whole tiles each, then 96 tiles split two ways
    cut, grid, ntiles = check_launch(8192, 4096, 11008, 0)
    assert (cut, grid, ntiles) == (96, 256, 1376)
    # whole rounds, or too many of them: nothing is cut
    assert check_launch(8192, 4096, 4096, 0)[0] == 0
    assert check_launch(8192, 4096, 16640, 0)[0] == 0            # 8.125 rounds
    # few big tiles: 128 x 128 tiles, two workgroups per compute unit, one workgroup per tile
    cut, grid, ntiles = check_launch(2048, 4096, 4096, 0)
    assert cut == 0 and grid == ntiles == 512


def test_many_ragged_shapes():
    rng = np.random.default_rng(20240711)
    for _ in range(120):
        T = int(rng.integers(1, 40)) * int(rng.choice([64, 100, 256, 300]))
        I = 32 * int(rng.integers(1, 300))
        O = 8 * int(rng.integers(1, 1200))
        for gemm in (0, 1, 2):
            check_launch(T, I, O, gemm)


def test_bad_arguments():
    L = eq.lib()
    item = (ctypes.c_int32 * 12)()
    ex = ctypes.c_int32(0)
    d = eq.make_desc(512, 512, 512, 2, 32, eq.BF16, eq.BF16)
    r = ctypes.byref(d)
    assert L.eqat_plan_item(r, 3, 0, 0, item, ctypes.byref(ex)) != 0
    assert L.eqat_plan_item(r, 0, -1, 0, item, ctypes.byref(ex)) != 0
    assert L.eqat_plan_item(r, 0, 0, -1, item, ctypes.byref(ex)) != 0
    assert L.eqat_plan_item(r, 0, 0, 0, None, ctypes.byref(ex)) != 0
    assert L.eqat_plan_item(r, 0, 0, 0, item, None) != 0
    f32 = eq.make_desc(512, 512, 512, 2, 32, eq.F32, eq.F32)
    assert L.eqat_plan_item(ctypes.byref(f32), 0, 0, 0, item, ctypes.byref(ex)) != 0
    assert L.eqat_plan_item(r, 0, 0, 0, item, ctypes.byref(ex)) == 0 and ex.value == 1
