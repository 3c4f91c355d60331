"""Pins for oracle/layers.py: brute-force loops on tiny inputs, independent
library routines (PyTorch CPU fp64 conv / linear / max_pool with autograd),
special cases, bilinear dot-product identities, and partitioned ==
unpartitioned for the distributed algorithms of Sec. 4."""
import itertools
import random

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import geometry as geo
from oracle import layers
from oracle import primitives as prim

RNG = np.random.default_rng(11)
T = lambda a: torch.from_numpy(np.ascontiguousarray(a))


def _brute_conv(x, w, b, s, p, dil):
    n_b, n_ci = x.shape[:2]
    n_co, k = w.shape[0], w.shape[2:]
    D = len(k)
    out = [geo.output_length(x.shape[2 + d], k[d], s[d], p[d], dil[d]) for d in range(D)]
    y = np.zeros((n_b, n_co) + tuple(out))
    for n in range(n_b):
        for co in range(n_co):
            for o in itertools.product(*[range(t) for t in out]):
                acc = b[co] if b is not None else 0.0
                for ci in range(n_ci):
                    for kap in itertools.product(*[range(t) for t in k]):
                        i = [o[d] * s[d] - p[d] + kap[d] * dil[d] for d in range(D)]
                        if all(0 <= i[d] < x.shape[2 + d] for d in range(D)):
                            acc += w[(co, ci) + kap] * x[(n, ci) + tuple(i)]
                y[(n, co) + o] = acc
    return y


CONV_CASES = [
    # x spatial, k, s, p, dil
    ((9,), (3,), (1,), (1,), (1,)),
    ((11,), (5,), (2,), (2,), (1,)),
    ((10,), (2,), (2,), (0,), (1,)),
    ((7, 8), (3, 3), (1, 1), (1, 1), (1, 1)),
    ((9, 7), (3, 2), (2, 1), (0, 1), (2, 1)),
    ((6, 7, 5), (3, 3, 3), (2, 2, 1), (1, 1, 0), (1, 1, 1)),
    ((9, 9, 9), (5, 5, 5), (2, 2, 2), (2, 2, 2), (1, 1, 1)),
]


@pytest.mark.parametrize("shape,k,s,p,dil", CONV_CASES)
def test_conv_forward_vs_brute_force_and_torch(shape, k, s, p, dil):
    x = RNG.standard_normal((2, 3) + shape)
    w = RNG.standard_normal((4, 3) + k)
    b = RNG.standard_normal(4)
    y = layers.conv_forward(x, w, b, s, p, dil)
    if np.prod(shape) <= 400:
        np.testing.assert_allclose(y, _brute_conv(x, w, b, s, p, dil), rtol=1e-12, atol=1e-12)
    conv = {1: F.conv1d, 2: F.conv2d, 3: F.conv3d}[len(shape)]
    ref = conv(T(x), T(w), T(b), stride=s, padding=p, dilation=dil).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape,k,s,p,dil", CONV_CASES)
def test_conv_backward_vs_torch_autograd(shape, k, s, p, dil):
    x = RNG.standard_normal((2, 3) + shape)
    w = RNG.standard_normal((4, 3) + k)
    b = RNG.standard_normal(4)
    conv = {1: F.conv1d, 2: F.conv2d, 3: F.conv3d}[len(shape)]
    tx, tw, tb = (T(a).requires_grad_(True) for a in (x, w, b))
    ty = conv(tx, tw, tb, stride=s, padding=p, dilation=dil)
    dy = RNG.standard_normal(tuple(ty.shape))
    ty.backward(T(dy))
    dx, dw, db = layers.conv_backward(x, w, dy, s, p, dil)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-11)
    # conv is linear in x and in w: <Conv x, dy> = <x, dx> = <w, dw> (bias off)
    y0 = layers.conv_forward(x, w, None, s, p, dil)
    lhs = np.sum(y0 * dy)
    assert abs(lhs - np.sum(x * dx)) < 1e-9 * abs(lhs) + 1e-9
    assert abs(lhs - np.sum(w * dw)) < 1e-9 * abs(lhs) + 1e-9


def test_conv_k1_is_a_per_pixel_gemm():
    x = RNG.standard_normal((2, 5, 6, 7))
    w = RNG.standard_normal((3, 5, 1, 1))
    y = layers.conv_forward(x, w, None, (1, 1), (0, 0), (1, 1))
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


def test_affine_vs_library_and_autograd():
    x = RNG.standard_normal((5, 7))
    W = RNG.standard_normal((4, 7))
    b = RNG.standard_normal(4)
    dy = RNG.standard_normal((5, 4))
    y = layers.affine_forward(x, W, b)
    tx, tW, tb = (T(a).requires_grad_(True) for a in (x, W, b))
    ty = F.linear(tx, tW, tb)
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-13, atol=1e-13)
    ty.backward(T(dy))
    dx, dW, db = layers.affine_backward(x, W, dy)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dW, tW.grad.numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-13, atol=1e-13)
    # element-wise definition on one entry
    assert abs(y[2, 1] - (sum(W[1, f] * x[2, f] for f in range(7)) + b[1])) < 1e-13


# ------------------------------------------------------------ distributed conv
def _random_conv_setups(count, seed):
    rnd = random.Random(seed)
    out = []
    while len(out) < count:
        D = rnd.randint(1, 3)
        P = [rnd.randint(1, 3) for _ in range(D)]
        k = [rnd.randint(1, 5) for _ in range(D)]
        s = [rnd.randint(1, 3) for _ in range(D)]
        dil = [rnd.randint(1, 2) for _ in range(D)]
        p = [rnd.randint(0, 3) for _ in range(D)]
        n = [rnd.randint(P[d] * 3, P[d] * 6) for d in range(D)]
        try:
            geo.Partition.for_kernel(n, P, k, s, p, dil)
        except ValueError:
            continue
        out.append((n, P, k, s, p, dil))
    return out


SETUPS = _random_conv_setups(20, 5) + [
    ([64], [4], [3], [1], [1], [1]),                                  # cfg1
    ([16, 16], [2, 2], [3, 3], [1, 1], [1, 1], [1, 1]),               # cfg2, scaled
    ([21, 22, 23], [2, 2, 2], [5, 5, 5], [2, 2, 2], [2, 2, 2], [1, 1, 1]),   # cfg5u-like, uneven
    ([28, 28], [2, 2], [5, 5], [1, 1], [2, 2], [1, 1]),               # cfg4 conv1
    ([14, 14], [2, 2], [5, 5], [1, 1], [0, 0], [1, 1]),               # cfg4 conv2
]


@pytest.mark.parametrize("n,P,k,s,p,dil", SETUPS)
def test_distributed_conv_equals_sequential(n, P, k, s, p, dil):
    part = geo.Partition.for_kernel(n, P, k, s, p, dil)
    x = RNG.standard_normal((2, 3) + tuple(n))
    w = RNG.standard_normal((2, 3) + tuple(k))
    b = RNG.standard_normal(2)
    y_seq = layers.conv_forward(x, w, b, s, p, dil)
    bufs = prim.scatter_bulk(x, part, fill=np.nan)
    y_parts = layers.dist_conv_forward(bufs, w, b, part, s, dil)
    np.testing.assert_allclose(prim.gather_out(y_parts, part), y_seq, rtol=1e-12, atol=1e-12)

    dy = RNG.standard_normal(y_seq.shape)
    dx_seq, dw_seq, db_seq = layers.conv_backward(x, w, dy, s, p, dil)
    dx_bufs, dw, db = layers.dist_conv_adjoint(bufs, w, prim.scatter_out(dy, part), part, s, dil)
    np.testing.assert_allclose(prim.gather_bulk(dx_bufs, part), dx_seq, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dw, dw_seq, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, db_seq, rtol=1e-11, atol=1e-11)
    for wk in range(part.n_workers):                     # halos / pads end cleared
        mask = np.ones(part.buf_shape(wk), dtype=bool)
        mask[part.bulk_slices(wk)] = False
        assert not dx_bufs[wk][:, :, mask].any()


# ------------------------------------------------------------ distributed affine
@pytest.mark.parametrize("n_b,n_fi,n_fo,P_fo,P_fi", [(4, 10, 6, 2, 2), (3, 7, 5, 3, 2), (5, 9, 4, 1, 1),
                                                     (2, 400, 120, 2, 2), (6, 8, 8, 1, 4)])
def test_distributed_affine_equals_sequential(n_b, n_fi, n_fo, P_fo, P_fi):
    x = RNG.standard_normal((n_b, n_fi))
    W = RNG.standard_normal((n_fo, n_fi))
    b = RNG.standard_normal(n_fo)
    dy = RNG.standard_normal((n_b, n_fo))
    rows, cols = layers.feature_blocks(n_fo, P_fo), layers.feature_blocks(n_fi, P_fi)
    x_parts = [x[:, c] for c in cols]
    W_parts = [[W[r][:, c] for c in cols] for r in rows]
    b_parts = [b[r] for r in rows]
    y = layers.dist_affine_forward(x_parts, W_parts, b_parts, P_fo, P_fi)
    np.testing.assert_allclose(np.concatenate(y, axis=1), layers.affine_forward(x, W, b), rtol=1e-12, atol=1e-12)
    dx, dW, db = layers.dist_affine_adjoint(x_parts, W_parts, [dy[:, r] for r in rows], P_fo, P_fi)
    dx_s, dW_s, db_s = layers.affine_backward(x, W, dy)
    np.testing.assert_allclose(np.concatenate(dx, axis=1), dx_s, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(np.block(dW), dW_s, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(np.concatenate(db), db_s, rtol=1e-12, atol=1e-12)
    # bilinear identities: <y - b, dy> = <x, dx> = <W, dW>
    lhs = np.sum(layers.affine_forward(x, W, None) * dy)
    assert abs(lhs - np.sum(x * dx_s)) < 1e-10 * max(1, abs(lhs))
    assert abs(lhs - np.sum(W * dW_s)) < 1e-10 * max(1, abs(lhs))


@pytest.mark.parametrize("n,P,k,s,p,ci,co,Pco,Pci", [((9, 8), (2, 2), (3, 3), (1, 1), (1, 1), 5, 4, 2, 2),
                                                     ((11,), (3,), (5,), (2,), (2,), 6, 7, 3, 2),
                                                     ((8, 6, 7), (2, 1, 2), (3, 3, 3), (2, 1, 1), (1, 1, 1), 4, 3, 1, 3)])
def test_channel_partitioned_conv_equals_unpartitioned(n, P, k, s, p, ci, co, Pco, Pci):
    """The full Sec. 4 algorithm (broadcast of x over P_co, sum-reduce of y over P_ci, bias on one sub-partition)
    against the plain definition of the layer and of its adjoint."""
    D = len(n)
    dil = (1,) * D
    part = geo.Partition.for_kernel(n, P, k, s, p, dil)
    x = RNG.standard_normal((2, ci) + n)
    w = RNG.standard_normal((co, ci) + k)
    b = RNG.standard_normal(co)
    y_ref = layers.conv_forward(x, w, b, s, p, dil)
    dy = RNG.standard_normal(y_ref.shape)
    dx_ref, dw_ref, db_ref = layers.conv_backward(x, w, dy, s, p, dil)
    rows, cols = layers.feature_blocks(co, Pco), layers.feature_blocks(ci, Pci)
    x_bufs = [prim.scatter_bulk(x[:, c], part, fill=np.nan) for c in cols]
    w_blocks = [[w[r][:, c] for c in cols] for r in rows]
    y = layers.dist_conv_cp_forward(x_bufs, w_blocks, [b[r] for r in rows], part, Pco, Pci, s, dil)
    got = np.concatenate([prim.gather_out(y[i], part) for i in range(Pco)], axis=1)
    np.testing.assert_allclose(got, y_ref, rtol=1e-12, atol=1e-12)
    dy_parts = [prim.scatter_out(dy[:, r], part) for r in rows]
    dx, dw, db = layers.dist_conv_cp_adjoint(x_bufs, w_blocks, dy_parts, part, Pco, Pci, s, dil)
    np.testing.assert_allclose(np.concatenate([prim.gather_bulk(dx[j], part) for j in range(Pci)], axis=1), dx_ref,
                               rtol=1e-12, atol=1e-12)
    dw_full = np.zeros_like(dw_ref)
    for i, r in enumerate(rows):
        for j, c in enumerate(cols):
            dw_full[r, c] = dw[i][j]
    np.testing.assert_allclose(dw_full, dw_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(np.concatenate(db), db_ref, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------ pooling and glue
@pytest.mark.parametrize("n,P", [((28, 28), (2, 2)), ((10, 10), (2, 2)), ((10, 20), (3, 6)), ((11, 9), (2, 2))])
def test_distributed_maxpool_equals_torch(n, P):
    k, s = (2, 2), (2, 2)
    part = geo.Partition.for_kernel(n, P, k, s, (0, 0), (1, 1))
    x = RNG.standard_normal((2, 3) + n)
    tx = T(x).requires_grad_(True)
    ty = F.max_pool2d(tx, 2, 2)
    dy = RNG.standard_normal(tuple(ty.shape))
    ty.backward(T(dy))
    bufs = prim.scatter_bulk(x, part, fill=np.nan)
    ys, args = layers.dist_maxpool_forward(bufs, part, k, s)
    np.testing.assert_array_equal(prim.gather_out(ys, part), ty.detach().numpy())
    dx = layers.dist_maxpool_adjoint(prim.scatter_out(dy, part), args, part,
                                     [b.shape for b in bufs], k, s)
    np.testing.assert_allclose(prim.gather_bulk(dx, part), tx.grad.numpy(), rtol=0, atol=1e-14)


@pytest.mark.parametrize("n,P,k,s,p", [((13, 11), (2, 2), (3, 3), (2, 2), (1, 1)), ((9, 12), (3, 2), (2, 2), (2, 2), (1, 1)),
                                       ((64, 48), (4, 3), (2, 2), (2, 2), (1, 1)), ((12, 7), (3, 1), (4, 3), (2, 1), (2, 1))])
def test_distributed_maxpool_with_padding_ignores_the_padding(n, P, k, s, p):
    """Padding cells never win the max and never receive gradient.  Pinned on all-negative inputs (where a zero
    in the padding would win every border window) against torch's max_pool2d with padding and its autograd, and
    against a window loop written out here that visits only in-domain cells."""
    part = geo.Partition.for_kernel(n, P, k, s, p, (1, 1))
    x = -np.abs(RNG.standard_normal((2, 3) + n)) - 0.5
    tx = T(x).requires_grad_(True)
    ty = F.max_pool2d(tx, k, s, p)
    dy = RNG.standard_normal(tuple(ty.shape))
    ty.backward(T(dy))
    bufs = prim.scatter_bulk(x, part, fill=np.nan)
    ys, args = layers.dist_maxpool_forward(bufs, part, k, s)
    y = prim.gather_out(ys, part)
    np.testing.assert_array_equal(y, ty.detach().numpy())
    assert (y < 0).all(), "a zero from the padding won a window"
    dx_bufs = layers.dist_maxpool_adjoint(prim.scatter_out(dy, part), args, part, [b.shape for b in bufs], k, s)
    np.testing.assert_allclose(prim.gather_bulk(dx_bufs, part), tx.grad.numpy(), rtol=0, atol=1e-14)
    # the definition, cell by cell: first maximum in row-major tap order over the taps inside the domain
    want = np.empty_like(y)
    dx_want = np.zeros_like(x)
    for b, c, o0, o1 in np.ndindex(*y.shape):
        best, where = None, None
        for t0 in range(k[0]):
            for t1 in range(k[1]):
                i0, i1 = o0 * s[0] - p[0] + t0, o1 * s[1] - p[1] + t1
                if 0 <= i0 < n[0] and 0 <= i1 < n[1] and (best is None or x[b, c, i0, i1] > best):
                    best, where = x[b, c, i0, i1], (i0, i1)
        want[b, c, o0, o1] = best
        dx_want[(b, c) + where] += dy[b, c, o0, o1]
    np.testing.assert_array_equal(y, want)
    np.testing.assert_allclose(prim.gather_bulk(dx_bufs, part), dx_want, rtol=0, atol=1e-14)
    # with zeros competing the border windows would differ: the reading matters on these inputs
    zero_pad = F.max_pool2d(F.pad(T(x), (p[1], p[1], p[0], p[0])), k, s).numpy()
    assert not np.array_equal(zero_pad, y)


def test_maxpool_tie_goes_to_first_tap():
    xp = np.zeros((1, 1, 2, 2))
    y, arg = layers.maxpool_valid(xp, (2, 2), (2, 2), (1, 1), (0, 0))
    assert y[0, 0, 0, 0] == 0 and arg[0, 0, 0, 0] == 0
    dxp = layers.maxpool_valid_adjoint(np.ones((1, 1, 1, 1)), arg, xp.shape, (2, 2), (2, 2), (0, 0))
    assert np.array_equal(dxp[0, 0], [[1, 0], [0, 0]])


@pytest.mark.parametrize("n,P,k,s,p", [((28, 28), (2, 2), (2, 2), (2, 2), (0, 0)), ((10, 20), (3, 6), (2, 2), (2, 2), (0, 0)),
                                       ((13, 11), (2, 2), (3, 3), (2, 2), (1, 1)), ((12,), (3,), (4,), (2,), (1,))])
def test_distributed_avgpool_equals_library_pool_and_is_adjoint(n, P, k, s, p):
    """Pinned against torch's avg_pool (zero padding counted in the divisor) and its autograd, against the
    reshape-mean closed form when windows tile the input, and by the dot-product test of the whole operator."""
    D = len(n)
    part = geo.Partition.for_kernel(n, P, k, s, p, (1,) * D)
    x = RNG.standard_normal((2, 3) + n)
    tx = T(x).requires_grad_(True)
    pool = F.avg_pool2d if D == 2 else F.avg_pool1d
    ty = pool(tx, k, s, p, count_include_pad=True)
    dy = RNG.standard_normal(tuple(ty.shape))
    ty.backward(T(dy))
    bufs = prim.scatter_bulk(x, part, fill=np.nan)
    ys = layers.dist_avgpool_forward(bufs, part, k, s)
    np.testing.assert_allclose(prim.gather_out(ys, part), ty.detach().numpy(), rtol=0, atol=1e-14)
    dx = layers.dist_avgpool_adjoint(prim.scatter_out(dy, part), part, [b.shape for b in bufs], k, s)
    np.testing.assert_allclose(prim.gather_bulk(dx, part), tx.grad.numpy(), rtol=0, atol=1e-14)
    if k == s and all(pp == 0 for pp in p) and all(nn % kk == 0 for nn, kk in zip(n, k)):
        blocks = x.reshape(2, 3, n[0] // k[0], k[0], n[1] // k[1], k[1]).mean(axis=(3, 5))
        np.testing.assert_allclose(prim.gather_out(ys, part), blocks, rtol=0, atol=1e-14)
    # <Pool x, dy> == <x, Pool* dy> on the partitioned spaces (halo and pad cells of x do not matter: H overwrites them)
    lhs = sum(np.sum(a * b) for a, b in zip(ys, prim.scatter_out(dy, part)))
    rhs = np.sum(prim.gather_bulk(dx, part) * x)
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1.0)


def test_relu_and_mse():
    x = np.array([-1.0, 0.0, 2.0])
    assert np.array_equal(layers.relu(x), [0, 0, 2])
    assert np.array_equal(layers.relu_backward(x, np.ones(3)), [0, 0, 1])
    y = RNG.standard_normal((4, 10))
    t = RNG.standard_normal((4, 10))
    loss, g = layers.mse_loss(y, t)
    ty = T(y).requires_grad_(True)
    tl = F.mse_loss(ty, T(t))
    tl.backward()
    assert abs(loss - tl.item()) < 1e-14
    np.testing.assert_allclose(g, ty.grad.numpy(), rtol=1e-14, atol=1e-16)


def test_repartition_is_a_permutation_with_inverse_adjoint():
    part = geo.Partition.for_kernel((10, 10), (2, 2), (2, 2), (2, 2), (0, 0), (1, 1))
    y = RNG.standard_normal((3, 4, 5, 5))
    parts = prim.scatter_out(y, part)
    f = layers.repartition_spatial_to_features(parts, part, 2)
    assert [t.shape for t in f] == [(3, 50), (3, 50)]
    np.testing.assert_array_equal(np.concatenate(f, axis=1), y.reshape(3, -1))
    back = layers.repartition_features_to_spatial(f, part, 4)
    for a, b in zip(back, parts):
        np.testing.assert_array_equal(a, b)
