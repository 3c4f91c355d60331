"""The inner product for callers that cannot allocate (distdl_dot_static: partial sums in a static device array)
against distdl_dot, through the C ABI.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import paper_2006_03108_amd as dd
from oracle import primitives as prim
from tests.gpu_util import require_gpu

pytestmark = pytest.mark.gpu


def _pair(rng, counts, dtype):
    a = [rng.standard_normal(c).astype(np.float32) for c in counts]
    b = [rng.standard_normal(c).astype(np.float32) for c in counts]
    to = lambda t: torch.from_numpy(t).to(dtype).cuda()
    return [to(t) for t in a], [to(t) for t in b]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_dot_static_matches_dot_on_two_calls_in_a_row(dtype):
    """Two calls back to back, the second on a smaller input: the shared scratch array keeps the first call's
    partial sums, none of which may leak into the second result.  Same kernels and summation order as distdl_dot,
    so the results agree bit for bit; both are also held against the oracle's inner product."""
    require_gpu()
    rng = np.random.default_rng(11)
    big = _pair(rng, [300_000, 77, 0, 1 << 20] + [4099] * 40, dtype)          # 44 arrays: two launches of partials
    small = _pair(rng, [513, 3], dtype)
    res = torch.full((4,), 123.0, dtype=torch.float64, device="cuda")
    dd.distdl_dot_static(big[0], big[1], res[0:1])
    dd.distdl_dot_static(small[0], small[1], res[1:2])
    dd.distdl_dot(big[0], big[1], res[2:3])
    dd.distdl_dot(small[0], small[1], res[3:4])
    torch.cuda.synchronize()
    got = res.cpu().numpy()
    assert got[0] == got[2] and got[1] == got[3]
    for value, (a, b) in ((got[0], big), (got[1], small)):
        want = prim.inner([t.float().cpu().numpy().astype(np.float64) for t in a],
                          [t.float().cpu().numpy().astype(np.float64) for t in b])
        assert abs(value - want) <= 1e-9 * max(abs(want), 1.0)


def test_dot_static_rejects_what_exceeds_its_limit():
    require_gpu()
    t = torch.ones(8, device="cuda")
    res = torch.zeros(1, dtype=torch.float64, device="cuda")
    with pytest.raises(dd.DistdlError) as e:
        dd.distdl_dot_static([t] * 97, [t] * 97, res)
    assert e.value.code == dd.ERR_INVALID_ARG and "96" in str(e.value)
    dd.distdl_dot_static([t] * 96, [t] * 96, res)
    torch.cuda.synchronize()
    assert res.item() == 96 * 8
