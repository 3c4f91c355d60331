"""Pins for oracle/network.py: the distributed network equals the sequential
one (the claim of Sec. 5), the sequential one equals an independent PyTorch
CPU fp64 network with autograd, and the loss gradient passes a
finite-difference check."""
import numpy as np
import torch
import torch.nn.functional as F

import synthetic_inputs as syn
from oracle import network

CASE = syn.cnn_case(dict(syn.CONFIGS["cfg4"], n_b=6))
IMG = CASE["images"].astype(np.float64)
TGT = CASE["target"].astype(np.float64)
PAR = {k: v.astype(np.float64) for k, v in CASE["params"].items()}
_rng = np.random.default_rng(1)
for _k in PAR:                                           # non-zero biases exercise db
    if _k.endswith("_b"):
        PAR[_k] = 0.1 * _rng.standard_normal(PAR[_k].shape)


def _torch_step():
    t = {k: torch.from_numpy(v.copy()).requires_grad_(True) for k, v in PAR.items()}
    x = torch.from_numpy(IMG.copy()).requires_grad_(True)
    h = F.max_pool2d(F.relu(F.conv2d(x, t["c1_w"], t["c1_b"], padding=2)), 2)
    h = F.max_pool2d(F.relu(F.conv2d(h, t["c3_w"], t["c3_b"])), 2)
    h = h.reshape(h.shape[0], -1)
    h = F.relu(F.linear(h, t["c5_w"], t["c5_b"]))
    h = F.relu(F.linear(h, t["f6_w"], t["f6_b"]))
    out = F.linear(h, t["out_w"], t["out_b"])
    loss = F.mse_loss(out, torch.from_numpy(TGT))
    loss.backward()
    g = {k: v.grad.numpy() for k, v in t.items()}
    g["images"] = x.grad.numpy()
    return loss.item(), out.detach().numpy(), g


def test_sequential_matches_torch_autograd():
    loss, out, g = network.sequential_step(IMG, TGT, PAR)
    tl, tout, tg = _torch_step()
    assert abs(loss - tl) < 1e-13
    np.testing.assert_allclose(out, tout, rtol=1e-12, atol=1e-13)
    for k in tg:
        np.testing.assert_allclose(g[k], tg[k], rtol=1e-10, atol=1e-13, err_msg=k)


def test_distributed_equals_sequential():
    loss_s, out_s, g_s = network.sequential_step(IMG, TGT, PAR)
    loss_d, out_d, g_d = network.distributed_step(IMG, TGT, PAR)
    assert abs(loss_s - loss_d) < 1e-13
    np.testing.assert_allclose(out_d, out_s, rtol=1e-12, atol=1e-13)
    for k in g_s:
        np.testing.assert_allclose(g_d[k], g_s[k], rtol=1e-10, atol=1e-13, err_msg=k)


def test_finite_difference_of_loss_gradient():
    _, _, g = network.distributed_step(IMG, TGT, PAR)
    rng = np.random.default_rng(0)
    for name in ("c1_w", "c3_w", "c3_b", "c5_w", "out_w", "f6_b"):
        idx = tuple(rng.integers(0, s) for s in PAR[name].shape)
        h = 1e-6
        p_hi = {k: v.copy() for k, v in PAR.items()}
        p_lo = {k: v.copy() for k, v in PAR.items()}
        p_hi[name][idx] += h
        p_lo[name][idx] -= h
        fd = (network.distributed_step(IMG, TGT, p_hi)[0] - network.distributed_step(IMG, TGT, p_lo)[0]) / (2 * h)
        assert abs(fd - g[name][idx]) < 1e-7 + 1e-5 * abs(fd), (name, idx, fd, g[name][idx])
