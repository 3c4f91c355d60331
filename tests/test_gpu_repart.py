"""GPU parity of the generalized all-to-all (Sec. 3): blocks of one balanced partition re-cut into another;
bit-exact against the oracle, the adjoint is the inverse."""
import numpy as np
import pytest
import torch

import paper_2006_03108_amd as dd
import synthetic_inputs as syn
from oracle import primitives as prim
from tests.gpu_util import require_gpu

pytestmark = pytest.mark.gpu

CASES = [
    ((11,), (4,), (3,)),
    ((6, 7), (2, 3), (3, 1)),
    ((4, 16, 5, 5), (1, 1, 2, 2), (1, 2, 1, 1)),            # spatial 2 x 2 -> channel blocks
    ((3, 10, 9, 8), (1, 2, 3, 2), (3, 1, 2, 4)),            # 16-byte rows on both sides
    ((5, 12, 7, 32), (1, 3, 2, 1), (5, 1, 1, 4)),           # wide rows, vector path
    ((2, 9, 31, 33), (2, 1, 4, 3), (1, 3, 2, 5)),           # odd extents: element path
    ((256, 16, 10, 10), (1, 1, 2, 2), (2, 2, 1, 1)),        # the example network's activations, batch split
    ((3, 8, 20, 12), (1, 1, 1, 1), (1, 2, 3, 2)),           # scatter of a global tensor (Sec. 3) ...
    ((3, 8, 20, 12), (1, 2, 3, 2), (1, 1, 1, 1)),           # ... and gather
]


def _blocks(shape, P, full):
    return [np.ascontiguousarray(full[sl]) for sl in prim.partition_blocks(shape, P)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("shape,Ps,Pd", CASES, ids=[str(c[0]) for c in CASES])
def test_repart_fwd_adj_bit_exact(shape, Ps, Pd, dtype):
    require_gpu()
    r = syn.streams(51, 2)
    full = syn.normal(r[0], shape)
    if dtype == torch.bfloat16:
        full = syn.to_bf16_values(full)
    src = _blocks(shape, Ps, full)
    want = prim.repartition(src, shape, Ps, Pd)
    plan = dd.distdl_repart_plan_create(shape, Ps, Pd, dtype)
    g_src = [torch.from_numpy(b).cuda().to(dtype) for b in src]
    g_dst = [torch.full(b.shape, -7.0, device="cuda", dtype=dtype) for b in want]
    dd.distdl_repart_fwd(plan, g_src, g_dst)
    g_back = [torch.full_like(t, 3.0) for t in g_src]
    dd.distdl_repart_adj(plan, g_dst, g_back)
    torch.cuda.synchronize()
    for w, (g, b) in enumerate(zip(g_dst, want)):
        assert np.array_equal(g.float().cpu().numpy(), b), f"destination block {w}"
    for w, (g, b) in enumerate(zip(g_back, g_src)):
        assert torch.equal(g, b), f"source block {w} after the inverse"
    if dtype == torch.float32:
        # <T x, y> == <x, T* y> with the device inner product
        y = [torch.from_numpy(syn.normal(r[1], b.shape)).cuda() for b in want]
        ty = [torch.empty_like(t) for t in g_src]
        dd.distdl_repart_adj(plan, y, ty)
        res = torch.zeros(2, dtype=torch.float64, device="cuda")
        dd.distdl_dot(g_dst, y, res[0:1])
        dd.distdl_dot(g_src, ty, res[1:2])
        torch.cuda.synchronize()
        lhs, rhs = res.cpu().tolist()
        assert abs(lhs - rhs) <= 1e-6 * max(abs(lhs), abs(rhs), 1e-30)


def test_repart_unaligned_pointers_take_the_element_path():
    require_gpu()
    shape, Ps, Pd = (3, 10, 9, 8), (1, 2, 3, 2), (3, 1, 2, 4)
    full = syn.normal(syn.streams(52, 1)[0], shape)
    src = _blocks(shape, Ps, full)
    want = prim.repartition(src, shape, Ps, Pd)
    plan = dd.distdl_repart_plan_create(shape, Ps, Pd)
    g_src = []
    for b in src:
        flat = torch.zeros(b.size + 1, device="cuda")
        v = flat[1:].view(b.shape)
        v.copy_(torch.from_numpy(b))
        assert v.data_ptr() % 16 == 4
        g_src.append(v)
    g_dst = [torch.empty(b.shape, device="cuda") for b in want]
    dd.distdl_repart_fwd(plan, g_src, g_dst)
    torch.cuda.synchronize()
    for g, b in zip(g_dst, want):
        assert np.array_equal(g.cpu().numpy(), b)


def test_repart_large_sampled():
    """A tensor far beyond the cache (1 GiB), spatial 4 x 4 -> (batch, channel) blocks: sampled against the
    definition through an index pattern."""
    require_gpu()
    shape, Ps, Pd = (32, 32, 512, 512), (1, 1, 4, 4), (4, 4, 1, 1)
    plan = dd.distdl_repart_plan_create(shape, Ps, Pd)
    pat = lambda i0, i1, i2, i3: ((i0 * 32 + i1) * 512 + i2) * 512 + i3     # < 2^28: not exact in fp32, so use % 2^24
    g_src = []
    for (st, sz) in plan.blocks(0):
        ax = [torch.arange(st[d], st[d] + sz[d], device="cuda", dtype=torch.int64) for d in range(4)]
        v = pat(ax[0][:, None, None, None], ax[1][None, :, None, None], ax[2][None, None, :, None], ax[3][None, None, None, :])
        g_src.append((v % 16777216).to(torch.float32))
    g_dst = [torch.empty(sz, device="cuda") for (_, sz) in plan.blocks(1)]
    dd.distdl_repart_fwd(plan, g_src, g_dst)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    for w, (st, sz) in enumerate(plan.blocks(1)):
        idx = [rng.integers(0, sz[d], size=2000) for d in range(4)]
        got = g_dst[w][tuple(torch.from_numpy(a).cuda() for a in idx)].cpu().numpy()
        want = (pat(*(idx[d] + st[d] for d in range(4))) % 16777216).astype(np.float32)
        assert np.array_equal(got, want), f"block {w}"
