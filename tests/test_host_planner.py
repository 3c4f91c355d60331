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
