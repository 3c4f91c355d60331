"""Pins for oracle/primitives.py: closed forms, operator identities of Sec. 3,
the adjoint test, nested == direct halo exchange, integer multiplicities of
H*, and the App. B.2 2x2 example."""
import os

import numpy as np
import pytest

from oracle import geometry as geo
from oracle import primitives as prim

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(7)


# ------------------------------------------------------------ broadcast / reduce
def test_broadcast_closed_form():
    x = np.arange(5.0)
    out = prim.broadcast(x, 3)
    assert len(out) == 3 and all(np.array_equal(o, x) for o in out)
    out[0][0] = 99                      # out-of-place: independent realizations
    assert x[0] == 0 and out[1][0] == 0


def test_sum_reduce_closed_form_integers():
    xs = [np.full(4, float(i + 1)) for i in range(5)]
    assert np.array_equal(prim.sum_reduce(xs), np.full(4, 15.0))
    ys = [np.arange(3.0), 10 * np.arange(3.0)]
    assert np.array_equal(prim.broadcast_adjoint(ys, clear_inputs=True), 11 * np.arange(3.0))
    assert all(not y.any() for y in ys)          # K_i applied


def _matrix_of(op, n_in):
    cols = []
    for e in range(n_in):
        v = np.zeros(n_in)
        v[e] = 1.0
        cols.append(np.concatenate([np.ravel(o) for o in op(v)]))
    return np.stack(cols, axis=1)


def test_reduce_is_broadcast_transposed():
    # Sec. 3: R = B*, R* = B, all-reduce B R is self-adjoint
    c, k = 3, 4
    B = _matrix_of(lambda v: prim.broadcast(v, k), c)
    R = _matrix_of(lambda v: [prim.sum_reduce(list(v.reshape(k, c)))], k * c)
    assert np.array_equal(R, B.T)
    A = _matrix_of(lambda v: prim.all_reduce(list(v.reshape(k, c))), k * c)
    assert np.array_equal(A, B @ R) and np.array_equal(A, A.T)


def test_broadcast_adjoint_test():
    x = RNG.standard_normal(16)
    y = [RNG.standard_normal(16) for _ in range(4)]
    Fx = prim.broadcast(x, 4)
    Fsy = prim.broadcast_adjoint(y)
    assert prim.adjoint_test_ratio(Fx, y, x, Fsy) < 1e-12
    # a planted mistake (dropping one replica) must fail the same test
    bad = prim.broadcast_adjoint(y[:3])
    assert prim.adjoint_test_ratio(Fx, y, x, bad) > 1e-3


# ------------------------------------------------------------ halo exchange
def _random_partitions(count, seed):
    import random
    rnd = random.Random(seed)
    out = []
    while len(out) < count:
        D = rnd.randint(1, 3)
        P = [rnd.randint(1, 3) for _ in range(D)]
        k = [rnd.randint(1, 5) for _ in range(D)]
        s = [rnd.randint(1, 3) for _ in range(D)]
        dil = [rnd.randint(1, 2) for _ in range(D)]
        p = [rnd.randint(0, 3) for _ in range(D)]
        n = [rnd.randint(P[d] * 3, P[d] * 7) for d in range(D)]
        try:
            out.append(geo.Partition.for_kernel(n, P, k, s, p, dil))
        except ValueError:
            continue
    return out


PARTS = _random_partitions(25, 3)


def _random_bufs(part, n_b=2, n_c=2):
    return [RNG.standard_normal((n_b, n_c) + part.buf_shape(w)) for w in range(part.n_workers)]


@pytest.mark.parametrize("part", PARTS)
def test_halo_nested_equals_direct_and_definition(part):
    xg = RNG.standard_normal((2, 2) + part.global_in_shape())
    a = prim.scatter_bulk(xg, part, fill=np.nan)        # stale contents must not matter
    b = prim.scatter_bulk(xg, part, fill=123.0)
    prim.halo_exchange(a, part)
    prim.halo_exchange_direct(b, part)
    for w in range(part.n_workers):
        assert np.array_equal(a[w], b[w])
        assert np.array_equal(a[w], prim.expected_buffer_after_halo(xg, part, w))
    assert np.array_equal(prim.gather_bulk(a, part), xg)   # bulk untouched


@pytest.mark.parametrize("part", PARTS)
def test_halo_adjoint_nested_equals_direct(part):
    y = _random_bufs(part)
    a = [t.copy() for t in y]
    b = [t.copy() for t in y]
    prim.halo_exchange_adjoint(a, part)
    prim.halo_exchange_adjoint_direct(b, part)
    for w in range(part.n_workers):
        np.testing.assert_allclose(a[w], b[w], rtol=0, atol=1e-12)
        mask = np.ones(part.buf_shape(w), dtype=bool)
        mask[part.bulk_slices(w)] = False
        assert not a[w][:, :, mask].any()               # halo and pad cleared


@pytest.mark.parametrize("part", PARTS)
def test_halo_adjoint_test(part):
    x = _random_bufs(part)
    y = _random_bufs(part)
    Fx = prim.halo_exchange([t.copy() for t in x], part)
    Fsy = prim.halo_exchange_adjoint([t.copy() for t in y], part)
    assert prim.adjoint_test_ratio(Fx, y, x, Fsy) < 1e-6


def test_planted_halo_mistakes_fail_the_adjoint_test():
    part = geo.Partition.for_kernel([12, 12], [2, 2], [5, 5], [1, 1], [2, 2], [1, 1])
    x, y = _random_bufs(part), _random_bufs(part)
    Fx = prim.halo_exchange([t.copy() for t in x], part)
    # (i) an adjoint that adds into the bulk but forgets to clear the halos;
    # (ii) one that clears the halos but never adds them into the bulk
    no_clear = [t.copy() for t in y]
    good = prim.halo_exchange_adjoint([t.copy() for t in y], part)
    for w in range(part.n_workers):                      # keep halo values: not K_b S
        keep = y[w].copy()
        keep[(slice(None), slice(None)) + part.bulk_slices(w)] = \
            good[w][(slice(None), slice(None)) + part.bulk_slices(w)]
        no_clear[w] = keep
    assert prim.adjoint_test_ratio(Fx, y, x, no_clear) > 1e-3
    assign = [t.copy() for t in y]                        # bulk untouched: no add
    for w in range(part.n_workers):
        mask = np.ones(part.buf_shape(w), dtype=bool)
        mask[part.bulk_slices(w)] = False
        assign[w][:, :, mask] = 0
    assert prim.adjoint_test_ratio(Fx, y, x, assign) > 1e-3


def test_halo_adjoint_multiplicities_are_integer_counts():
    """H* of all-ones: every bulk cell ends at 1 + (number of other workers'
    buffers that hold a copy of it) -- brute-force count, exact in fp."""
    part = geo.Partition.for_kernel([9, 10, 11], [2, 3, 2], [5, 3, 5], [2, 1, 1], [2, 1, 2], [1, 1, 1])
    ones = [np.ones((1, 1) + part.buf_shape(w)) for w in range(part.n_workers)]
    prim.halo_exchange_adjoint(ones, part)
    n_glob = part.global_in_shape()
    count = np.zeros(n_glob)
    for w in range(part.n_workers):
        lo = [part.g(w, d)["in_start"] - part.g(w, d)["halo"][0] for d in range(3)]
        hi = [part.g(w, d)["in_start"] + part.g(w, d)["in_size"] + part.g(w, d)["halo"][1] for d in range(3)]
        count[tuple(slice(l, h) for l, h in zip(lo, hi))] += 1
    got = prim.gather_bulk(ones, part)[0, 0]
    assert np.array_equal(got, count)
    assert got.max() >= 4                                # an edge band is hit


def test_rank2_example_of_app_b2():
    rows = {}
    for line in open(os.path.join(GOLDEN, "halo_2x2_example.txt")):
        line = line.split("#")[0].strip()
        if line:
            tok = line.split()
            rows[tok[0]] = [tuple(int(v) for v in t.split(",")) for t in tok[2:]]
    bulk = [[5, 7], [6, 4]]                              # unequal domains
    part = geo.Partition.explicit(bulk, [rows["dim0"], rows["dim1"]])
    xg = np.arange(12 * 10, dtype=np.float64).reshape(1, 1, 12, 10)
    bufs = prim.scatter_bulk(xg, part, fill=-1.0)
    assert bufs[0].shape[2:] == (7, 6) and bufs[3].shape[2:] == (11, 7)
    prim.halo_exchange(bufs, part)
    # worker 3's corner halo (4 rows x 3 cols) holds worker 0's bottom-right block,
    # which reached it through worker 1 (dim 0 first) and worker 2
    assert np.array_equal(bufs[3][0, 0, :4, :3], xg[0, 0, 1:5, 3:6])
    # worker 1: left halo of width 3 over its bulk rows and its bottom halo rows
    assert np.array_equal(bufs[1][0, 0, :, :3], xg[0, 0, 0:7, 3:6])
    # workers 0 and 2 take nothing horizontally
    assert bufs[0].shape[3] == 6 and bufs[2].shape[3] == 6
    # adjoint: ones -> multiplicities; cell (4, 5) is held by workers 0, 1, 2, 3
    ones = [np.ones_like(b) for b in bufs]
    prim.halo_exchange_adjoint(ones, part)
    got = prim.gather_bulk(ones, part)[0, 0]
    assert got[4, 5] == 4 and got[0, 0] == 1 and got[4, 0] == 2 and got[0, 5] == 2
    assert got[5, 5] == 4 and got[6, 5] == 4 and got[7, 5] == 2 and got[6, 2] == 2 and got[8, 2] == 1


def test_halo_operator_matrix_is_transposed():
    """H and H* as explicit matrices on a tiny case: H* == H^T exactly."""
    part = geo.Partition.for_kernel([5, 4], [2, 2], [3, 3], [1, 1], [1, 1], [1, 1])
    sizes = [int(np.prod(part.buf_shape(w))) for w in range(part.n_workers)]
    total = sum(sizes)

    def split(v):
        out, o = [], 0
        for w, s in enumerate(sizes):
            out.append(v[o:o + s].reshape((1, 1) + part.buf_shape(w)).copy())
            o += s
        return out

    def apply(op, v):
        return np.concatenate([np.ravel(t) for t in op(split(v), part)])

    H = np.stack([apply(prim.halo_exchange, e) for e in np.eye(total)], axis=1)
    Hs = np.stack([apply(prim.halo_exchange_adjoint, e) for e in np.eye(total)], axis=1)
    assert np.array_equal(Hs, H.T)
    assert set(np.unique(H)) == {0.0, 1.0}


@pytest.mark.parametrize("n,P,k,s,p", [((11,), (3,), (5,), (1,), (2,)), ((10, 20), (3, 6), (2, 2), (2, 2), (0, 0)),
                                       ((9, 9), (3, 3), (5, 5), (1, 1), (2, 2)),
                                       ((20, 18, 22), (2, 3, 2), (5, 3, 5), (2, 1, 2), (2, 1, 2))])
def test_adjoint_multiplicity_closed_form_matches_nested_adjoint(n, P, k, s, p):
    """H* of all-ones counts the copies of every cell (an exact integer pin that a wrong slab, a dropped
    corner or a missed clear would break); the closed form used at full size on the GPU agrees with it."""
    part = geo.Partition.for_kernel(n, P, k, s, p, (1,) * len(n))
    ones = [np.ones((1, 2) + part.buf_shape(w)) for w in range(part.n_workers)]
    got = prim.halo_exchange_adjoint(ones, part)
    for w in range(part.n_workers):
        want = np.zeros(part.buf_shape(w))
        want[part.bulk_slices(w)] = prim.adjoint_multiplicity(part, w)
        assert np.array_equal(got[w][0, 0], want) and np.array_equal(got[w][0, 1], want)


@pytest.mark.parametrize("bulk,halo", [([[5, 7], [6, 4]], [[(0, 2), (4, 0)], [(0, 0), (3, 0)]]),
                                       ([[4, 4], [5, 3], [6, 6]], [[(0, 1), (1, 0)], [(0, 3), (0, 0)], [(0, 6), (6, 0)]])])
def test_adjoint_multiplicity_on_explicit_widths(bulk, halo):
    """Same pin on partitions with hand-given widths (App. B.2), against the cell-by-cell statement of H*."""
    part = geo.Partition.explicit(bulk, halo)
    ones = [np.ones((1, 1) + part.buf_shape(w)) for w in range(part.n_workers)]
    got = prim.halo_exchange_adjoint_direct(ones, part)
    for w in range(part.n_workers):
        assert np.array_equal(got[w][0, 0][part.bulk_slices(w)], prim.adjoint_multiplicity(part, w))


@pytest.mark.parametrize("shape,Ps,Pd", [((6, 7), (2, 3), (3, 1)), ((4, 16, 5, 5), (1, 1, 2, 2), (1, 2, 1, 1)),
                                         ((3, 10, 9, 8), (1, 2, 3, 2), (3, 1, 2, 4)), ((11,), (4,), (3,))])
def test_repartition_is_a_permutation_with_inverse_adjoint(shape, Ps, Pd):
    """The generalized all-to-all only re-cuts the tensor: the blocks of the result are the destination
    partition's slices of the global tensor (checked with an index pattern, independent of the routine),
    going back restores the source blocks, and <T x, y> == <x, T^-1 y>."""
    full = np.arange(int(np.prod(shape)), dtype=np.float64).reshape(shape)
    src = [full[sl].copy() for sl in prim.partition_blocks(shape, Ps)]
    dst = prim.repartition(src, shape, Ps, Pd)
    assert len(dst) == int(np.prod(Pd))
    seen = np.concatenate([b.ravel() for b in dst])
    assert np.array_equal(np.sort(seen), full.ravel())                  # every element exactly once
    w = 0
    import itertools
    for coords in itertools.product(*[range(p) for p in Pd]):
        lo = [geo.balanced_split(shape[d], Pd[d])[coords[d]][0] for d in range(len(shape))]
        assert dst[w].flat[0] == full[tuple(lo)]                          # block w starts where the balanced rule says
        assert dst[w].shape == tuple(geo.balanced_split(shape[d], Pd[d])[coords[d]][1] for d in range(len(shape)))
        w += 1
    back = prim.repartition(dst, shape, Pd, Ps)
    for a, b in zip(back, src):
        assert np.array_equal(a, b)
    y = [RNG.standard_normal(b.shape) for b in dst]
    x = [RNG.standard_normal(b.shape) for b in src]
    lhs = prim.inner(prim.repartition(x, shape, Ps, Pd), y)
    rhs = prim.inner(x, prim.repartition(y, shape, Pd, Ps))
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1.0)
