"""GPU parity of the calls that widen the path beyond the ten named ones: average / max pooling through the
halo plan for any kernel size, stride and padding (Sec. 4 pooling algorithms, App. B.1 unbalanced cases) and the
all-reduce A = B R (Sec. 3), against the oracle."""
import numpy as np
import pytest
import torch

import paper_2006_03108_amd as dd
import synthetic_inputs as syn
from oracle import geometry as geo
from oracle import layers
from oracle import primitives as prim
from tests.gpu_util import assert_close, from_cl, require_gpu, to_cl

pytestmark = pytest.mark.gpu
TOL32 = 1e-5

POOL_CASES = [
    # D, n_b, c, n, P, k, s, p
    (2, 2, 8, (10, 20), (3, 6), (2, 2), (2, 2), (0, 0)),       # App. B.1 unbalanced examples, two dimensions
    (2, 3, 6, (28, 28), (2, 2), (2, 2), (2, 2), (0, 0)),
    (2, 2, 5, (13, 11), (2, 2), (3, 3), (2, 2), (1, 1)),       # overlapping windows with zero padding
    (1, 2, 4, (12,), (3,), (4,), (2,), (1,)),
    (3, 1, 16, (12, 10, 14), (2, 2, 2), (2, 3, 2), (2, 1, 2), (0, 1, 0)),
    (2, 2, 8, (13, 17), (2, 2), (2, 2), (3, 3), (0, 0)),       # stride > kernel: cells that no window covers
    (3, 2, 16, (12, 10, 14), (2, 2, 2), (2, 2, 2), (2, 2, 2), (0, 0, 0)),
    (2, 1, 32, (64, 48), (4, 3), (2, 2), (2, 2), (1, 1)),      # zero padding inside tiled windows
]


def _pool_setup(case):
    D, n_b, c, n, P, k, s, p = case
    one = (1,) * D
    part = geo.Partition.for_kernel(n, P, k, s, p, one)
    plan = dd.distdl_plan_create(D, n_b, c, c, n, P, k, s, p, one)
    r = syn.streams(31, 2)
    x = syn.normal(r[0], (n_b, c) + tuple(n))
    dy = syn.normal(r[1], (n_b, c) + part.global_out_shape())
    return part, plan, x, dy


@pytest.mark.parametrize("case", POOL_CASES, ids=[str(c[3]) + "k" + str(c[5]) for c in POOL_CASES])
def test_avgpool_fwd_bwd_and_adjoint_test(case):
    require_gpu()
    D, n_b, c, n, P, k, s, p = case
    part, plan, x, dy = _pool_setup(case)
    bufs_o = prim.scatter_bulk(x.astype(np.float64), part, fill=np.nan)
    y_want = layers.dist_avgpool_forward(bufs_o, part, k, s)
    dx_want = layers.dist_avgpool_adjoint(prim.scatter_out(dy.astype(np.float64), part), part,
                                          [b.shape for b in bufs_o], k, s)
    g_x = [to_cl(b) for b in prim.scatter_bulk(x, part, fill=np.float32(9.0))]
    g_y = [torch.empty((n_b,) + part.out_shape(w) + (c,), device="cuda") for w in range(part.n_workers)]
    dd.distdl_avgpool_fwd(plan, g_x, g_y)
    g_dy = [to_cl(t) for t in prim.scatter_out(dy, part)]
    g_dx = [torch.full_like(t, -5.0) for t in g_x]
    dd.distdl_avgpool_bwd(plan, g_dy, g_dx)
    # dot-product test on the device results: <Pool x, dy> == <x, Pool* dy> (x restricted to the bulk)
    res = torch.zeros(2, dtype=torch.float64, device="cuda")
    g_xb = [to_cl(b) for b in prim.scatter_bulk(x, part, fill=np.float32(0.0))]
    dd.distdl_dot(g_y, g_dy, res[0:1])
    dd.distdl_dot(g_xb, g_dx, res[1:2])
    torch.cuda.synchronize()
    for w in range(part.n_workers):
        assert_close(from_cl(g_y[w]), y_want[w], TOL32, f"avgpool y worker {w}")
        assert_close(from_cl(g_dx[w]), dx_want[w], TOL32, f"avgpool dx worker {w}")
    lhs, rhs = res.cpu().tolist()
    assert abs(lhs - rhs) <= TOL32 * max(abs(lhs), abs(rhs), 1e-30)


@pytest.mark.parametrize("case", POOL_CASES, ids=[str(c[3]) + "k" + str(c[5]) for c in POOL_CASES])
def test_maxpool_general_kernels(case):
    require_gpu()
    D, n_b, c, n, P, k, s, p = case
    part, plan, x, dy = _pool_setup(case)
    bufs_o = prim.scatter_bulk(x.astype(np.float64), part, fill=np.nan)
    y_want, args = layers.dist_maxpool_forward(bufs_o, part, k, s)
    dx_want = layers.dist_maxpool_adjoint(prim.scatter_out(dy.astype(np.float64), part), args, part,
                                          [b.shape for b in bufs_o], k, s)
    g_x = [to_cl(b) for b in prim.scatter_bulk(x, part, fill=np.float32(9.0))]
    g_y = [torch.empty((n_b,) + part.out_shape(w) + (c,), device="cuda") for w in range(part.n_workers)]
    dd.distdl_maxpool_fwd(plan, g_x, g_y)
    g_dy = [to_cl(t) for t in prim.scatter_out(dy, part)]
    g_dx = [torch.full_like(t, -5.0) for t in g_x]
    dd.distdl_maxpool_bwd(plan, g_x, g_dy, g_dx)
    torch.cuda.synchronize()
    for w in range(part.n_workers):
        assert np.array_equal(from_cl(g_y[w]), y_want[w].astype(np.float32)), f"maxpool y worker {w}"
        assert_close(from_cl(g_dx[w]), dx_want[w], TOL32, f"maxpool dx worker {w}")


@pytest.mark.parametrize("case", [POOL_CASES[2], POOL_CASES[3], POOL_CASES[4], POOL_CASES[7]],
                         ids=lambda c: str(c[3]) + "k" + str(c[5]))
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_maxpool_padding_never_wins(case, dtype):
    """Padded plans on all-negative inputs: a zero from the padding would win every border window and swallow its
    gradient; the maximum runs over in-domain cells only (all four kernel forms: element-wise and 16-byte forward,
    gather and window backward)."""
    require_gpu()
    D, n_b, c, n, P, k, s, p = case
    one = (1,) * D
    part = geo.Partition.for_kernel(n, P, k, s, p, one)
    plan = dd.distdl_plan_create(D, n_b, c, c, n, P, k, s, p, one, dtype)
    r = syn.streams(35, 2)
    x = syn.to_bf16_values(-np.abs(syn.normal(r[0], (n_b, c) + tuple(n))) - 0.5)
    dy = syn.to_bf16_values(syn.normal(r[1], (n_b, c) + part.global_out_shape()))
    bufs_o = prim.scatter_bulk(x.astype(np.float64), part, fill=np.nan)
    y_want, args = layers.dist_maxpool_forward(bufs_o, part, k, s)
    dx_want = layers.dist_maxpool_adjoint(prim.scatter_out(dy.astype(np.float64), part), args, part,
                                          [b.shape for b in bufs_o], k, s)
    g_x = [to_cl(b, dtype) for b in prim.scatter_bulk(x, part, fill=np.float32(9.0))]
    g_y = [torch.empty((n_b,) + part.out_shape(w) + (c,), device="cuda", dtype=dtype) for w in range(part.n_workers)]
    dd.distdl_maxpool_fwd(plan, g_x, g_y)
    g_dy = [to_cl(t, dtype) for t in prim.scatter_out(dy, part)]
    g_dx = [torch.full_like(t, -5.0) for t in g_x]
    dd.distdl_maxpool_bwd(plan, g_x, g_dy, g_dx)
    torch.cuda.synchronize()
    for w in range(part.n_workers):
        got = from_cl(g_y[w])
        assert (got < 0).all(), f"a padding zero won a window of worker {w}"
        assert np.array_equal(got, y_want[w].astype(np.float32)), f"maxpool y worker {w}"
        assert_close(from_cl(g_dx[w]), dx_want[w], TOL32 if dtype == torch.float32 else 2e-2, f"maxpool dx worker {w}")


def test_maxpool_rejects_windows_that_lie_in_the_padding():
    require_gpu()
    plan = dd.distdl_plan_create(1, 1, 4, 4, [12], [2], [2], [2], [3], [1])   # padding 3 with a 2-wide window
    part = geo.Partition.for_kernel((12,), (2,), (2,), (2,), (3,), (1,))
    g_x = [torch.zeros((1,) + part.buf_shape(w) + (4,), device="cuda") for w in range(2)]
    g_y = [torch.zeros((1,) + part.out_shape(w) + (4,), device="cuda") for w in range(2)]
    with pytest.raises(dd.DistdlError) as e:
        dd.distdl_maxpool_fwd(plan, g_x, g_y)
    assert e.value.code == dd.ERR_UNSUPPORTED


@pytest.mark.parametrize("case", [POOL_CASES[0], POOL_CASES[2], POOL_CASES[4], POOL_CASES[5]],
                         ids=lambda c: str(c[3]) + "k" + str(c[5]))
def test_pooling_bf16(case):
    """bf16 tensors through max and average pooling: the max is exact (a selection), sums round to bf16 (2e-2)."""
    require_gpu()
    D, n_b, c, n, P, k, s, p = case
    one, bf = (1,) * D, torch.bfloat16
    part = geo.Partition.for_kernel(n, P, k, s, p, one)
    plan = dd.distdl_plan_create(D, n_b, c, c, n, P, k, s, p, one, bf)
    r = syn.streams(33, 2)
    x = syn.to_bf16_values(syn.normal(r[0], (n_b, c) + tuple(n)))
    dy = syn.to_bf16_values(syn.normal(r[1], (n_b, c) + part.global_out_shape()))
    bufs_o = prim.scatter_bulk(x.astype(np.float64), part, fill=np.nan)
    dyo = prim.scatter_out(dy.astype(np.float64), part)
    shapes = [b.shape for b in bufs_o]
    ymax, args = layers.dist_maxpool_forward(bufs_o, part, k, s)
    dxmax = layers.dist_maxpool_adjoint(dyo, args, part, shapes, k, s)
    yavg = layers.dist_avgpool_forward(bufs_o, part, k, s)
    dxavg = layers.dist_avgpool_adjoint(dyo, part, shapes, k, s)
    g_x = [to_cl(b, bf) for b in prim.scatter_bulk(x, part, fill=np.float32(9.0))]
    new_y = lambda: [torch.empty((n_b,) + part.out_shape(w) + (c,), device="cuda", dtype=bf) for w in range(part.n_workers)]
    g_dy = [to_cl(t, bf) for t in prim.scatter_out(dy, part)]
    y1, y2 = new_y(), new_y()
    dx1, dx2 = [torch.full_like(t, -5.0) for t in g_x], [torch.full_like(t, -5.0) for t in g_x]
    dd.distdl_maxpool_fwd(plan, g_x, y1)
    dd.distdl_maxpool_bwd(plan, g_x, g_dy, dx1)
    dd.distdl_avgpool_fwd(plan, g_x, y2)
    dd.distdl_avgpool_bwd(plan, g_dy, dx2)
    torch.cuda.synchronize()
    for w in range(part.n_workers):
        assert np.array_equal(from_cl(y1[w]), ymax[w].astype(np.float32)), f"maxpool y worker {w}"
        assert_close(from_cl(dx1[w]), dxmax[w], 2e-2, f"maxpool dx worker {w}")
        assert_close(from_cl(y2[w]), yavg[w], 2e-2, f"avgpool y worker {w}")
        assert_close(from_cl(dx2[w]), dxavg[w], 2e-2, f"avgpool dx worker {w}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("count,k,G", [(16, 4, 1), (4099, 3, 2), (1 << 20, 2, 2), (1000, 70, 1), (0, 2, 1)])
def test_allreduce_matches_oracle_and_is_self_adjoint(count, k, G, dtype):
    require_gpu()
    r = syn.streams(41, 2)
    conv = syn.to_bf16_values if dtype == torch.bfloat16 else (lambda a: a)
    xs = [conv(syn.normal(r[0], (count,))) for _ in range(G * k)]
    ys = [conv(syn.normal(r[1], (count,))) for _ in range(G * k)]
    dev = lambda arrs: [torch.from_numpy(a).cuda().to(dtype) for a in arrs]
    gx, gy = dev(xs), dev(ys)
    gx0, gy0 = [t.clone() for t in gx], [t.clone() for t in gy]
    dd.distdl_allreduce(gx, k)
    dd.distdl_allreduce(gy, k)
    torch.cuda.synchronize()
    tol = TOL32 if dtype == torch.float32 else 2e-2
    for g in range(G):
        want = prim.all_reduce([xs[g * k + i].astype(np.float64) for i in range(k)])
        for i in range(k):
            if count:
                assert_close(gx[g * k + i].float().cpu().numpy(), want[i], tol, f"group {g} replica {i}")
            assert torch.equal(gx[g * k + i], gx[g * k])          # all replicas bit-identical
    if count and dtype == torch.float32:
        # A = A*: <A x, y> == <x, A y>
        res = torch.zeros(2, dtype=torch.float64, device="cuda")
        dd.distdl_dot(gx, gy0, res[0:1])
        dd.distdl_dot(gx0, gy, res[1:2])
        torch.cuda.synchronize()
        lhs, rhs = res.cpu().tolist()
        assert abs(lhs - rhs) <= TOL32 * max(abs(lhs), abs(rhs))


def test_allreduce_rejects_bad_arguments():
    require_gpu()
    import ctypes as C
    a = torch.zeros(8, device="cuda")
    ptrs = (C.c_void_p * 2)(a.data_ptr(), a.data_ptr())
    counts = (C.c_int64 * 1)(8)
    assert dd.lib.distdl_allreduce(None, counts, 1, 2, 0, None) == dd.binding.ERR_NULL
    assert dd.lib.distdl_allreduce(ptrs, counts, 1, 0, 0, None) == dd.binding.ERR_INVALID_ARG
    assert dd.lib.distdl_allreduce(ptrs, counts, 0, 2, 0, None) == dd.binding.ERR_INVALID_ARG
    assert dd.lib.distdl_allreduce(ptrs, counts, 1, 2, 7, None) == dd.binding.ERR_UNSUPPORTED
