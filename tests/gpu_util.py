"""Helpers for the GPU parity tests: layout marshalling between the oracle's
logical [n_b, n_c, spatial...] numpy arrays and the library's channels-last
device buffers, and the parity norms."""
import numpy as np
import torch

from oracle import geometry as geo


def require_gpu():
    assert torch.cuda.is_available(), "GPU tests need a HIP device (run them with -m gpu on the GPU box)"
    return torch.device("cuda:0")


def to_cl(arr, dtype=torch.float32):
    """numpy [n, c, s...] -> contiguous device tensor [n, s..., c]."""
    t = torch.from_numpy(np.ascontiguousarray(np.moveaxis(arr, 1, -1)))
    return t.to(dtype).cuda().contiguous()


def from_cl(t):
    """device tensor [n, s..., c] -> numpy [n, c, s...] (float64 for parity math)."""
    return np.moveaxis(t.detach().to(torch.float32).cpu().numpy(), -1, 1)


def w_to_dev(w):
    return torch.from_numpy(np.ascontiguousarray(w)).float().cuda()


def oracle_partition(cfg):
    return geo.Partition.for_kernel(cfg["in_shape"], cfg["P"], cfg["ksize"], cfg["stride"], cfg["padding"],
                                    cfg["dilation"])


def rel_errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    l2 = np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-300)
    mx = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
    return l2, mx


def assert_close(got, want, tol, what=""):
    l2, mx = rel_errors(got, want)
    assert l2 <= tol and mx <= tol, f"{what}: rel l2 {l2:.3e}, rel max {mx:.3e} > {tol:.1e}"
