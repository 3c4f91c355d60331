"""GPU parity of the channel-partitioned convolution layer (Sec. 4, P_co x P_ci x feature-space partition)
against the oracle's step-by-step algorithm."""
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

CASES = [
    # D, n_b, ci, co, n, P, Pco, Pci, k, s, p
    (2, 2, 5, 4, (9, 8), (2, 2), 2, 2, (3, 3), (1, 1), (1, 1)),              # direct kernels (odd channel blocks)
    (1, 2, 6, 7, (11,), (3,), 3, 2, (5,), (2,), (2,)),
    (3, 1, 64, 64, (16, 14, 18), (2, 1, 2), 2, 2, (3, 3, 3), (2, 1, 1), (1, 1, 1)),   # MFMA kernels, 32-channel blocks
    (2, 2, 16, 24, (20, 20), (2, 2), 1, 2, (3, 3), (1, 1), (1, 1)),          # only the sum-reduce over P_ci
    (2, 2, 16, 24, (20, 20), (2, 2), 3, 1, (3, 3), (1, 1), (1, 1)),          # only the broadcast over P_co
]


@pytest.mark.parametrize("case", CASES, ids=[f"{c[4]}co{c[6]}ci{c[7]}" for c in CASES])
@pytest.mark.parametrize("with_bias", [True, False], ids=["bias", "nobias"])
def test_convcp_fwd_bwd_against_oracle(case, with_bias):
    require_gpu()
    D, n_b, ci, co, n, P, Pco, Pci, k, s, p = case
    dil = (1,) * D
    part = geo.Partition.for_kernel(n, P, k, s, p, dil)
    S = part.n_workers
    r = syn.streams(61, 4)
    x = syn.normal(r[0], (n_b, ci) + tuple(n))
    w = syn.normal(r[1], (co, ci) + tuple(k), std=syn.he_normal_std((co, ci) + tuple(k)))
    b = syn.normal(r[2], (co,)) if with_bias else None
    dy = syn.normal(r[3], (n_b, co) + part.global_out_shape())
    rows, cols = layers.feature_blocks(co, Pco), layers.feature_blocks(ci, Pci)
    # oracle
    xo = [prim.scatter_bulk(x[:, c].astype(np.float64), part, fill=np.nan) for c in cols]
    wo = [[w[rr][:, c].astype(np.float64) for c in cols] for rr in rows]
    bo = [b[rr].astype(np.float64) for rr in rows] if with_bias else None
    y_want = layers.dist_conv_cp_forward(xo, wo, bo, part, Pco, Pci, s, dil)
    dyo = [prim.scatter_out(dy[:, rr].astype(np.float64), part) for rr in rows]
    dx_want, dw_want, db_want = layers.dist_conv_cp_adjoint(xo, wo, dyo, part, Pco, Pci, s, dil, want_bias=with_bias)
    # library
    plan = dd.distdl_convcp_plan_create(D, n_b, ci, co, n, P, Pco, Pci, k, s, p, dil)
    assert plan.S == S
    for j, c in enumerate(cols):
        assert plan.channels(0, j) == (c.start, c.stop - c.start)
    g_x = [to_cl(bb) for c in cols for bb in prim.scatter_bulk(x[:, c], part, fill=np.float32(5.0))]
    g_w = [torch.from_numpy(np.ascontiguousarray(w[rr][:, c])).cuda() for rr in rows for c in cols]
    g_b = [torch.from_numpy(np.ascontiguousarray(b[rr])).cuda() for rr in rows] if with_bias else None
    g_y = [torch.full((n_b,) + part.out_shape(sw) + (rr.stop - rr.start,), -1.0, device="cuda") for rr in rows for sw in range(S)]
    dd.distdl_convcp_fwd(plan, g_x, g_w, g_b, g_y)
    g_dy = [to_cl(t) for rr in rows for t in prim.scatter_out(dy[:, rr], part)]
    g_dx = [torch.full_like(t, 9.0) for t in g_x]
    g_dw = [torch.full_like(t, 9.0) for t in g_w]
    g_db = [torch.full_like(t, 9.0) for t in g_b] if with_bias else None
    dd.distdl_convcp_bwd(plan, g_x, g_w, g_dy, g_dx, g_dw, g_db)
    torch.cuda.synchronize()
    for i in range(Pco):
        for sw in range(S):
            assert_close(from_cl(g_y[i * S + sw]), y_want[i][sw], TOL32, f"y block {i} worker {sw}")
        for j in range(Pci):
            assert_close(g_dw[i * Pci + j].cpu().numpy(), dw_want[i][j], TOL32, f"dw block ({i},{j})")
        if with_bias:
            assert_close(g_db[i].cpu().numpy(), db_want[i], TOL32, f"db block {i}")
    for j in range(Pci):
        for sw in range(S):
            assert_close(from_cl(g_dx[j * S + sw]), dx_want[j][sw], TOL32, f"dx block {j} worker {sw}")


def test_convcp_bf16():
    """bf16 tensors through the channel-partitioned layer (partial outputs are rounded to bf16 before the sum-reduce
    over the input-channel blocks); bar 2e-2."""
    require_gpu()
    D, n_b, ci, co, n, P, Pco, Pci, k, s, p = 3, 1, 64, 64, (16, 14, 18), (2, 1, 2), 2, 2, (3, 3, 3), (2, 1, 1), (1, 1, 1)
    dil, bf = (1,) * D, torch.bfloat16
    part = geo.Partition.for_kernel(n, P, k, s, p, dil)
    S = part.n_workers
    r = syn.streams(62, 4)
    x = syn.to_bf16_values(syn.normal(r[0], (n_b, ci) + tuple(n)))
    w = syn.to_bf16_values(syn.normal(r[1], (co, ci) + tuple(k), std=syn.he_normal_std((co, ci) + tuple(k))))
    b = syn.to_bf16_values(syn.normal(r[2], (co,)))
    dy = syn.to_bf16_values(syn.normal(r[3], (n_b, co) + part.global_out_shape()))
    rows, cols = layers.feature_blocks(co, Pco), layers.feature_blocks(ci, Pci)
    xo = [prim.scatter_bulk(x[:, c].astype(np.float64), part, fill=np.nan) for c in cols]
    wo = [[w[rr][:, c].astype(np.float64) for c in cols] for rr in rows]
    y_want = layers.dist_conv_cp_forward(xo, wo, [b[rr].astype(np.float64) for rr in rows], part, Pco, Pci, s, dil)
    dyo = [prim.scatter_out(dy[:, rr].astype(np.float64), part) for rr in rows]
    dx_want, dw_want, db_want = layers.dist_conv_cp_adjoint(xo, wo, dyo, part, Pco, Pci, s, dil, want_bias=True)
    plan = dd.distdl_convcp_plan_create(D, n_b, ci, co, n, P, Pco, Pci, k, s, p, dil, bf)
    g_x = [to_cl(bb, bf) for c in cols for bb in prim.scatter_bulk(x[:, c], part, fill=np.float32(5.0))]
    g_w = [torch.from_numpy(np.ascontiguousarray(w[rr][:, c])).to(bf).cuda() for rr in rows for c in cols]
    g_b = [torch.from_numpy(np.ascontiguousarray(b[rr])).to(bf).cuda() for rr in rows]
    g_y = [torch.full((n_b,) + part.out_shape(sw) + (rr.stop - rr.start,), -1.0, device="cuda", dtype=bf)
           for rr in rows for sw in range(S)]
    dd.distdl_convcp_fwd(plan, g_x, g_w, g_b, g_y)
    g_dy = [to_cl(t, bf) for rr in rows for t in prim.scatter_out(dy[:, rr], part)]
    g_dx = [torch.full_like(t, 9.0) for t in g_x]
    g_dw = [torch.full_like(t, 9.0) for t in g_w]
    g_db = [torch.full_like(t, 9.0) for t in g_b]
    dd.distdl_convcp_bwd(plan, g_x, g_w, g_dy, g_dx, g_dw, g_db)
    torch.cuda.synchronize()
    tol = 2e-2
    for i in range(Pco):
        for sw in range(S):
            assert_close(from_cl(g_y[i * S + sw]), y_want[i][sw], tol, f"y block {i} worker {sw}")
        for j in range(Pci):
            assert_close(g_dw[i * Pci + j].float().cpu().numpy(), dw_want[i][j], tol, f"dw block ({i},{j})")
        assert_close(g_db[i].float().cpu().numpy(), db_want[i], tol, f"db block {i}")
    for j in range(Pci):
        for sw in range(S):
            assert_close(from_cl(g_dx[j * S + sw]), dx_want[j][sw], tol, f"dx block {j} worker {sw}")


def test_convcp_rejects_bad_arguments():
    require_gpu()
    with pytest.raises(dd.DistdlError) as e:
        dd.distdl_convcp_plan_create(2, 1, 2, 4, (8, 8), (2, 2), 2, 3, (3, 3), (1, 1), (1, 1), (1, 1))
    assert e.value.code == dd.binding.ERR_EMPTY_PARTITION
    with pytest.raises(dd.DistdlError):
        dd.distdl_convcp_plan_create(2, 1, 4, 4, (8, 8), (2, 2), 0, 1, (3, 3), (1, 1), (1, 1), (1, 1))
