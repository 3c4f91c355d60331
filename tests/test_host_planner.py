"""CPU tests of the library's host side: the C ABI loads and exports every
declared symbol, the planner's geometry agrees with the oracle's independent
planner and with the paper's worked examples, error codes, and the box-task
tables of the one-pass halo kernels -- interpreted here on numpy arrays --
reproduce the oracle's nested halo exchange and its adjoint."""
import os
import random
import re

import numpy as np
import pytest

import paper_2006_03108_amd as dd
from oracle import geometry as geo
from oracle import primitives as prim

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "distdl.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(distdl_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(dd.lib, name), name
    for name in ("distdl_halo_fwd", "distdl_halo_adj", "distdl_bcast_fwd", "distdl_bcast_adj",
                 "distdl_sumreduce_fwd", "distdl_sumreduce_adj", "distdl_conv_fwd", "distdl_conv_bwd",
                 "distdl_affine_fwd", "distdl_affine_bwd"):
        assert name in declared


def _random_setups(count, seed):
    rnd = random.Random(seed)
    out = []
    while len(out) < count:
        D = rnd.randint(1, 3)
        P = [rnd.randint(1, 4) for _ in range(D)]
        k = [rnd.randint(1, 5) for _ in range(D)]
        s = [rnd.randint(1, 3) for _ in range(D)]
        dil = [rnd.randint(1, 2) for _ in range(D)]
        p = [rnd.randint(0, 3) for _ in range(D)]
        n = [rnd.randint(P[d] * 2, P[d] * 7) for d in range(D)]
        out.append((n, P, k, s, p, dil))
    return out


@pytest.mark.parametrize("n,P,k,s,p,dil", _random_setups(60, 1))
def test_planner_agrees_with_oracle_geometry(n, P, k, s, p, dil):
    D = len(n)
    try:
        part = geo.Partition.for_kernel(n, P, k, s, p, dil)
    except geo.EmptyPartition:
        with pytest.raises(dd.DistdlError) as e:
            dd.distdl_plan_create(D, 1, 1, 1, n, P, k, s, p, dil)
        assert e.value.code == dd.ERR_EMPTY_PARTITION
        return
    except geo.HaloTooWide:
        with pytest.raises(dd.DistdlError) as e:
            dd.distdl_plan_create(D, 1, 1, 1, n, P, k, s, p, dil)
        assert e.value.code == dd.ERR_HALO_TOO_WIDE
        return
    plan = dd.distdl_plan_create(D, 2, 3, 4, n, P, k, s, p, dil)
    assert plan.n_workers == part.n_workers
    for w in range(part.n_workers):
        q = plan.query(w)
        for d in range(D):
            g = part.g(w, d)
            assert q["in_start"][d] == g["in_start"] and q["in_size"][d] == g["in_size"]
            assert q["out_start"][d] == g["out_start"] and q["out_size"][d] == g["out_size"]
            assert q["halo"][d] == g["halo"] and q["pad"][d] == g["pad"] and q["extra"][d] == g["extra"]
            assert q["buf_shape"][d] == g["buf"] and q["bulk_off"][d] == g["bulk_off"]
            assert q["conv_origin"][d] == g["origin"]


def test_planner_on_the_papers_pooling_example():
    # App. B.1 fourth example: n = 20, k = 2, s = 2, P = 6
    plan = dd.distdl_plan_create(1, 1, 1, 1, [20], [6], [2], [2], [0], [1])
    got = [(plan.query(w)["halo"][0], plan.query(w)["extra"][0]) for w in range(6)]
    assert got == [((0, 0), (0, 0)), ((0, 0), (0, 0)), ((0, 1), (0, 0)),
                   ((0, 2), (1, 0)), ((0, 1), (2, 0)), ((0, 0), (1, 0))]


def test_error_codes():
    def code(fn):
        with pytest.raises(dd.DistdlError) as e:
            fn()
        return e.value.code
    assert code(lambda: dd.distdl_plan_create(4, 1, 1, 1, [4] * 4, [1] * 4, [1] * 4, [1] * 4, [0] * 4, [1] * 4)) == dd.ERR_INVALID_ARG
    assert code(lambda: dd.distdl_plan_create(1, 0, 1, 1, [4], [1], [1], [1], [0], [1])) == dd.ERR_INVALID_ARG
    assert code(lambda: dd.distdl_plan_create(1, 1, 1, 1, [4], [1], [1], [0], [0], [1])) == dd.ERR_INVALID_ARG
    assert code(lambda: dd.distdl_plan_create(1, 1, 1, 1, [3], [4], [1], [1], [0], [1])) == dd.ERR_EMPTY_PARTITION
    assert code(lambda: dd.distdl_plan_create(1, 1, 1, 1, [8], [4], [7], [1], [3], [1])) == dd.ERR_HALO_TOO_WIDE
    assert code(lambda: dd.distdl_plan_create_explicit(1, 1, 1, [2], [[2, 5]], [[(0, 0), (3, 0)]])) == dd.ERR_HALO_TOO_WIDE
    assert code(lambda: dd.distdl_plan_create_explicit(1, 1, 1, [2], [[0, 5]], [[(0, 0), (0, 0)]])) == dd.ERR_EMPTY_PARTITION
    assert code(lambda: dd.distdl_affine_plan_create(4, 3, 8, 2, 4)) == dd.ERR_EMPTY_PARTITION
    assert code(lambda: dd.distdl_affine_plan_create(0, 3, 8, 1, 1)) == dd.ERR_INVALID_ARG
    assert "worker" in dd.distdl_last_error() or "sizes" in dd.distdl_last_error()
    plan = dd.distdl_plan_create(1, 1, 1, 1, [8], [2], [3], [1], [1], [1])
    with pytest.raises(dd.DistdlError):
        plan.query(2)


def _as3(arr, D):
    """[n_b, n_c, spatial...] -> view with 3 feature dims."""
    return arr.reshape(arr.shape[:2] + (1,) * (3 - D) + arr.shape[2:])


def _box(org, ext):
    return (slice(None), slice(None)) + tuple(slice(o, o + e) for o, e in zip(org, ext))


def _interpret(tasks, bufs, D, adjoint):
    views = [_as3(b, D) for b in bufs]
    for t in tasks:
        dst = views[t["dst"]]
        if not t["srcs"]:
            dst[_box(t["org"], t["ext"])] = 0
        elif not adjoint:
            (sw, sorg), = t["srcs"]
            dst[_box(t["org"], t["ext"])] = views[sw][_box(sorg, t["ext"])]
        else:
            assert [s[0] for s in t["srcs"]] == sorted(s[0] for s in t["srcs"])
            for sw, sorg in t["srcs"]:
                dst[_box(t["org"], t["ext"])] += views[sw][_box(sorg, t["ext"])]
                views[sw][_box(sorg, t["ext"])] = 0


TABLE_SETUPS = [s for s in _random_setups(120, 2)]


@pytest.mark.parametrize("n,P,k,s,p,dil", TABLE_SETUPS[:50] + [
    ([64], [4], [3], [1], [1], [1]), ([12, 12], [2, 2], [3, 3], [1, 1], [1, 1], [1, 1]),
    ([4], [2], [7], [1], [3], [1]),                      # pad and halo on the same side
    ([9, 9], [3, 3], [5, 5], [1, 1], [2, 2], [1, 1]),    # bulk 3 covered from both sides
    ([21, 22, 23], [2, 2, 2], [5, 5, 5], [2, 2, 2], [2, 2, 2], [1, 1, 1])])
def test_task_tables_reproduce_the_oracle_halo_exchange(n, P, k, s, p, dil):
    D = len(n)
    try:
        part = geo.Partition.for_kernel(n, P, k, s, p, dil)
    except ValueError:
        pytest.skip("geometry rejected")
    plan = dd.distdl_plan_create(D, 2, 2, 2, n, P, k, s, p, dil)
    rng = np.random.default_rng(0)
    xg = rng.standard_normal((2, 2) + tuple(n))
    want = prim.halo_exchange(prim.scatter_bulk(xg, part, fill=np.nan), part)
    got = prim.scatter_bulk(xg, part, fill=np.nan)
    _interpret(dd.distdl_debug_tasks(plan, False), got, D, False)
    for a, b in zip(got, want):
        assert np.array_equal(a, b)

    y = [rng.standard_normal(b.shape) for b in want]
    want = prim.halo_exchange_adjoint([t.copy() for t in y], part)
    got = [t.copy() for t in y]
    _interpret(dd.distdl_debug_tasks(plan, True), got, D, True)
    for a, b in zip(got, want):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def test_task_tables_cover_every_non_bulk_cell_once():
    part = geo.Partition.for_kernel([10, 11, 9], [2, 3, 2], [5, 3, 4], [1, 1, 2], [2, 1, 1], [1, 1, 1])
    plan = dd.distdl_plan_create(3, 1, 1, 1, [10, 11, 9], [2, 3, 2], [5, 3, 4], [1, 1, 2], [2, 1, 1], [1, 1, 1])
    hits = [np.zeros(part.buf_shape(w), dtype=int) for w in range(part.n_workers)]
    for t in dd.distdl_debug_tasks(plan, False):
        hits[t["dst"]][_box(t["org"], t["ext"])[2:]] += 1
    for w in range(part.n_workers):
        expect = np.ones(part.buf_shape(w), dtype=int)
        expect[part.bulk_slices(w)] = 0
        assert np.array_equal(hits[w], expect)
    # adjoint: every halo cell is read-and-cleared exactly once, every pad cell zeroed once
    hits = [np.zeros(part.buf_shape(w), dtype=int) for w in range(part.n_workers)]
    for t in dd.distdl_debug_tasks(plan, True):
        if not t["srcs"]:
            hits[t["dst"]][_box(t["org"], t["ext"])[2:]] += 1
        for sw, sorg in t["srcs"]:
            hits[sw][_box(sorg, t["ext"])[2:]] += 1
    for w in range(part.n_workers):
        expect = np.ones(part.buf_shape(w), dtype=int)
        expect[part.bulk_slices(w)] = 0
        assert np.array_equal(hits[w], expect)


def test_explicit_plan_matches_app_b2_example():
    plan = dd.distdl_plan_create_explicit(2, 1, 1, [2, 2], [[5, 7], [6, 4]], [[(0, 2), (4, 0)], [(0, 0), (3, 0)]])
    part = geo.Partition.explicit([[5, 7], [6, 4]], [[(0, 2), (4, 0)], [(0, 0), (3, 0)]])
    assert [plan.query(w)["buf_shape"] for w in range(4)] == [list(part.buf_shape(w)) for w in range(4)]
    xg = np.arange(120.0).reshape(1, 1, 12, 10)
    want = prim.halo_exchange(prim.scatter_bulk(xg, part, fill=-1.0), part)
    got = prim.scatter_bulk(xg, part, fill=-1.0)
    _interpret(dd.distdl_debug_tasks(plan, False), got, 2, False)
    for a, b in zip(got, want):
        assert np.array_equal(a, b)


def test_index_decode_division_is_exact():
    rnd = random.Random(3)
    edge = [1, 2, 3, 5, 7, 16, 255, 256, 257, 65535, 65536, 2**31 - 1, 2**31, 2**32 - 1]
    for d in edge + [rnd.randint(1, 2**32 - 1) for _ in range(200)] + [rnd.randint(1, 5000) for _ in range(300)]:
        for n in edge + [0, d - 1, d, d + 1, 2 * d - 1, 2 * d] + [rnd.randint(0, 2**32 - 1) for _ in range(40)]:
            n &= 0xFFFFFFFF
            assert dd.lib.distdl_debug_fastdiv(n, d) == n // d, (n, d)


def test_repartition_plan_blocks_follow_the_balanced_rule_and_errors():
    """The generalized all-to-all's planner (no GPU): its blocks are the oracle's balanced blocks, row-major."""
    from oracle import primitives as prim
    for shape, Ps, Pd in [((3, 10, 9, 8), (1, 2, 3, 2), (3, 1, 2, 4)), ((11,), (4,), (3,)), ((6, 7), (2, 3), (3, 1))]:
        plan = dd.distdl_repart_plan_create(shape, Ps, Pd)
        for side, P in ((0, Ps), (1, Pd)):
            want = [(tuple(s.start for s in sl), tuple(s.stop - s.start for s in sl))
                    for sl in prim.partition_blocks(shape, P)]
            assert plan.blocks(side) == want
    with pytest.raises(dd.DistdlError) as e:
        dd.distdl_repart_plan_create((3, 4), (4, 1), (1, 1))
    assert e.value.code == dd.binding.ERR_EMPTY_PARTITION
    with pytest.raises(dd.DistdlError):
        dd.distdl_repart_plan_create((3, 4, 5, 6, 7), (1,) * 5, (1,) * 5)
    with pytest.raises(dd.DistdlError):
        dd.distdl_repart_plan_create((0, 4), (1, 1), (1, 1))


def test_conv_kernel_family_falls_back_when_no_window_fits():
    """Layers whose staged patch fits no window of the matrix-core correlation (wide dilated kernels with many
    channels) must be routed to the direct kernels by the planner, not fail when the launch is prepared."""
    path = lambda *a, **k: dd.distdl_debug_conv_path(dd.distdl_plan_create(*a, **k))
    # the volumetric configuration and the 2-D one: 32-wide and 16-wide matrix-core tiles
    assert path(3, 1, 32, 32, [64, 64, 64], [2, 2, 2], [5] * 3, [2] * 3, [2] * 3, [1] * 3) == (1, 1, 1)
    assert path(2, 8, 16, 16, [256, 256], [2, 2], [3, 3], [1, 1], [1, 1], [1, 1]) == (2, 2, 2)
    # channel counts that are no multiples of 4: direct kernels throughout (3 -> 5 channels still fit 16-wide tiles)
    assert path(2, 2, 33, 35, [40, 40], [2, 2], [3, 3], [1, 1], [1, 1], [1, 1])[:2] == (0, 0)
    # k = 3 with dilation 16, k = 7 with dilation 6, 32 channels: the patch of even the narrowest window exceeds
    # the pieces a thread can stage; k = 3 with dilation 3 still fits
    assert path(2, 1, 32, 32, [80, 80], [2, 2], [3, 3], [1, 1], [16, 16], [16, 16])[:2] == (0, 0)
    assert path(2, 1, 32, 32, [90, 90], [2, 2], [7, 7], [1, 1], [18, 18], [6, 6])[:2] == (0, 0)
    assert path(2, 1, 32, 32, [60, 64], [2, 2], [3, 3], [1, 1], [12, 12], [12, 12])[:2] == (1, 1)   # the narrowest window
    assert path(2, 1, 32, 32, [80, 80], [2, 2], [3, 3], [1, 1], [3, 3], [3, 3])[:2] == (1, 1)


def test_table_cache_policy_never_rewrites_a_block_another_reader_may_hold():
    """The device-table cache (pointer arrays, GEMM descriptors), run without a device: eight blocks per stream with
    least-recently-used replacement, no replacement across streams, blocks selected during capture pinned for good,
    unknown tables refused during capture, and an error instead of an eviction when nothing may be reused."""
    pol = dd.distdl_debug_slot_policy
    # steady state: a repeated table reuses its block
    assert pol([0, 0, 0, 0], [7, 8, 7, 8], [0] * 4) == [0, 1, 0, 1]
    # the ninth distinct table on a stream replaces that stream's least recently used block
    seq = list(range(1, 10))
    assert pol([0] * 9, seq, [0] * 9) == [0, 1, 2, 3, 4, 5, 6, 7, 0]
    assert pol([0] * 10, [1, 2, 3, 4, 5, 6, 7, 8, 1, 9], [0] * 10)[-1] == 1      # table 1 was touched again: 2 goes
    # another stream never takes over a block: the same table on stream 1 gets a block of its own, and stream 1's
    # ninth table replaces one of ITS blocks
    got = pol([0, 1] + [1] * 8, [5, 5] + list(range(10, 18)), [0] * 10)
    assert got[0] == 0 and got[1] == 1 and got[-1] == 1 and 0 not in got[1:]
    # a table first seen during capture is refused (its copy would read host memory at replay)
    assert pol([0, 0], [1, 2], [0, 1]) == [0, dd.ERR_INVALID_ARG]
    # a block selected during capture is pinned: eight more tables on the stream leave it alone ...
    got = pol([0] * 11, [1, 1] + list(range(2, 11)), [0, 1] + [0] * 9)
    assert got[1] == 0 and 0 not in got[2:]
    # ... and the recorded table is still found afterwards
    assert pol([0] * 12, [1, 1] + list(range(2, 11)) + [1], [0, 1] + [0] * 10)[-1] == 0
    # 64 blocks, all pinned by captures: the next new table fails with NOMEM instead of evicting one
    streams, tables, cap = [], [], []
    for t in range(64):
        streams += [0, 0]
        tables += [100 + t, 100 + t]
        cap += [0, 1]
    got = pol(streams + [0], tables + [999], cap + [0])
    assert sorted(set(got[:-1])) == list(range(64)) and got[-1] == dd.ERR_NOMEM
