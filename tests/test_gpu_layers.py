"""GPU parity of the partitioned convolution and affine layers against the
CPU oracle, through the C ABI (rel 1e-5 fp32, 2e-2 bf16)."""
import numpy as np
import pytest
import torch

import paper_2006_03108_amd as dd
import synthetic_inputs as syn
from oracle import geometry as geo
from oracle import layers
from oracle import primitives as prim
from tests.gpu_util import assert_close, from_cl, oracle_partition, require_gpu, to_cl, w_to_dev

pytestmark = pytest.mark.gpu
TOL32, TOL16 = 1e-5, 2e-2


def _conv_case(name, **override):
    cfg = dict(syn.CONFIGS[name])
    cfg.update(override)
    part = oracle_partition(cfg)
    case = syn.conv_case(cfg, part.global_out_shape())
    return cfg, part, case


def _off_by_one_element(shape, value, dtype):
    """A tensor of that shape whose storage starts one element into an allocation: aligned to its element only."""
    n = int(np.prod(shape))
    flat = torch.full((n + 1,), value, device="cuda", dtype=dtype)
    return flat[1:].view(shape)


def _run_conv(cfg, part, case, use_bias, dtype=torch.float32, misaligned_outputs=False):
    plan = dd.distdl_plan_create(cfg["D"], cfg["n_b"], cfg["c_in"], cfg["c_out"], cfg["in_shape"], cfg["P"],
                                 cfg["ksize"], cfg["stride"], cfg["padding"], cfg["dilation"], dtype)
    x_bufs = [to_cl(b, dtype) for b in prim.scatter_bulk(case["x"], part, fill=np.float32(3.0))]
    w = w_to_dev(case["w"]).to(dtype)
    bias = w_to_dev(case["bias"]).to(dtype) if use_bias else None
    y_shapes = [(cfg["n_b"],) + part.out_shape(wk) + (cfg["c_out"],) for wk in range(part.n_workers)]
    if misaligned_outputs:
        y = [_off_by_one_element(sh, 7.0, dtype) for sh in y_shapes]
    else:
        y = [torch.full(sh, 7.0, device="cuda", dtype=dtype) for sh in y_shapes]
    dd.distdl_conv_fwd(plan, x_bufs, w, bias, y)
    dy = [to_cl(t, dtype) for t in prim.scatter_out(case["dy"], part)]
    if misaligned_outputs:
        dx_bufs = [_off_by_one_element(tuple(b.shape), 5.0, dtype) for b in x_bufs]
    else:
        dx_bufs = [torch.full_like(b, 5.0) for b in x_bufs]
    dw = torch.full_like(w, 9.0)
    db = torch.full((cfg["c_out"],), 9.0, device="cuda", dtype=dtype) if use_bias else None
    ws = torch.empty(max(dd.distdl_conv_bwd_workspace(plan), 16), dtype=torch.uint8, device="cuda")
    dd.distdl_conv_bwd(plan, x_bufs, w, dy, dx_bufs, dw, db, ws)
    torch.cuda.synchronize()
    return x_bufs, y, dx_bufs, dw, db


CONV_FULL = [
    ("cfg1", {}, True),
    ("cfg1", {}, False),
    ("cfg2", dict(in_shape=(64, 64), n_b=2), True),
    ("cfg2", {}, True),            # the 2-D configuration at its full size, every element (the oracle takes seconds)
    ("cfg5", dict(in_shape=(24, 24, 24), P=(2, 2, 2), c_in=8, c_out=8), True),
    ("cfg5u", dict(in_shape=(21, 23, 22), P=(2, 2, 2), c_in=32, c_out=32), False),
    ("cfg2", dict(in_shape=(19, 23), n_b=3, c_in=3, c_out=5, P=(2, 3), ksize=(3, 4), stride=(2, 1),
                  padding=(1, 2), dilation=(1, 2)), True),
    # matrix-core path: channel counts that are multiples of 4, several output-channel tiles, odd geometry
    ("cfg2", dict(in_shape=(23, 41), n_b=2, c_in=4, c_out=40, P=(2, 3), ksize=(3, 4), stride=(2, 1),
                  padding=(1, 2), dilation=(1, 2)), True),
    ("cfg1", dict(in_shape=(200,), n_b=3, c_in=8, c_out=8, P=(3,), ksize=(7,), stride=(3,), padding=(2,)), True),
    ("cfg5", dict(in_shape=(13, 17, 40), P=(2, 2, 2), c_in=12, c_out=20, ksize=(2, 3, 4), stride=(1, 2, 3),
                  padding=(1, 0, 2)), False),
    ("cfg5", dict(in_shape=(18, 18, 70), P=(1, 2, 1), c_in=32, c_out=32, ksize=(5, 5, 5), stride=(2, 2, 2),
                  padding=(2, 2, 2)), True),
    # dilated kernels at matrix-core shapes (32 and 64 channels), 3-D and 2-D, with stride
    ("cfg5", dict(in_shape=(26, 22, 70), P=(2, 2, 1), c_in=32, c_out=32, ksize=(3, 3, 3), stride=(1, 1, 1),
                  padding=(2, 2, 2), dilation=(2, 2, 2)), True),
    ("cfg5", dict(in_shape=(30, 30, 76), P=(2, 1, 2), c_in=32, c_out=64, ksize=(3, 2, 3), stride=(2, 1, 2),
                  padding=(3, 1, 2), dilation=(3, 2, 2)), False),
    ("cfg2", dict(in_shape=(70, 90), n_b=2, c_in=16, c_out=16, ksize=(3, 3), stride=(1, 1), padding=(2, 2),
                  dilation=(2, 2)), True),
    # few channels (16 x 16 matrix-core tiles): planes stacked per unit, ragged batches and partitions, 3-D, dilation
    ("cfg2", dict(in_shape=(28, 28), n_b=37, c_in=1, c_out=6, ksize=(5, 5), padding=(2, 2)), True),
    ("cfg2", dict(in_shape=(14, 14), n_b=37, c_in=6, c_out=16, ksize=(5, 5), padding=(0, 0)), True),
    ("cfg2", dict(in_shape=(45, 150), n_b=3, c_in=16, c_out=16, P=(3, 1)), True),
    ("cfg2", dict(in_shape=(33, 29), n_b=5, c_in=16, c_out=12, ksize=(5, 5), padding=(2, 2), P=(2, 3)), False),
    ("cfg2", dict(in_shape=(31, 37), n_b=2, c_in=3, c_out=8, ksize=(3, 3), padding=(2, 2), dilation=(2, 2), P=(2, 2)), True),
    ("cfg5", dict(in_shape=(11, 14, 19), P=(2, 1, 2), c_in=4, c_out=8, ksize=(3, 3, 3), stride=(2, 1, 1),
                  padding=(1, 1, 1)), True),
    ("cfg1", dict(in_shape=(300,), n_b=4, c_in=5, c_out=7, P=(3,), ksize=(5,), padding=(2,)), True),
    ("cfg1", dict(in_shape=(130,), n_b=9, c_in=8, c_out=8, P=(2,), ksize=(7,), padding=(3,)), False),
    ("cfg2", dict(in_shape=(20, 24), n_b=6, c_in=12, c_out=4, ksize=(1, 1), padding=(0, 0)), True),
    ("cfg2", dict(in_shape=(28, 28), n_b=4, c_in=1, c_out=6, ksize=(5, 5), padding=(2, 2)), True),   # cfg4 conv1
    ("cfg2", dict(in_shape=(14, 14), n_b=4, c_in=6, c_out=16, ksize=(5, 5), padding=(0, 0)), True),  # cfg4 conv2
    # a single worker per dimension: no neighbour to exchange with, only the padding to clear
    ("cfg2", dict(in_shape=(40, 44), n_b=1, c_in=16, c_out=16, P=(1, 1)), True),
    ("cfg5", dict(in_shape=(12, 14, 36), P=(1, 1, 1), c_in=32, c_out=32), True),
    # several channel tiles (the second output tile half full): the weight gradient's shared tap and its db sums
    ("cfg2", dict(in_shape=(40, 70), n_b=2, c_in=64, c_out=48, ksize=(3, 3), padding=(1, 1), P=(2, 2)), True),
    ("cfg2", dict(in_shape=(36, 40), n_b=3, c_in=32, c_out=64, ksize=(5, 5), stride=(2, 2), padding=(2, 2), P=(2, 1)), True),
    # three and four workers per dimension in 3-D: interior workers (halo on both sides of every dimension, no
    # padding), every element compared; uneven bulks in the second
    ("cfg5", dict(in_shape=(40, 38, 44), P=(3, 3, 3)), True),
    ("cfg5u", dict(in_shape=(50, 46, 54), P=(4, 4, 4), c_in=8, c_out=16), False),
    # wide dilated kernels with 32 channels: dilation 12 still finds a (32-wide) window of the matrix-core
    # correlation, dilation 16 does not and must run on the direct kernels
    ("cfg2", dict(in_shape=(60, 64), n_b=1, c_in=32, c_out=32, ksize=(3, 3), padding=(12, 12), dilation=(12, 12)), True),
    ("cfg2", dict(in_shape=(80, 72), n_b=1, c_in=32, c_out=32, ksize=(3, 3), padding=(16, 16), dilation=(16, 16)), True),
]


@pytest.mark.parametrize("name,override,use_bias", CONV_FULL,
                         ids=[f"{n}-{i}" for i, (n, _, _) in enumerate(CONV_FULL)])
def test_conv_fwd_bwd_against_partitioned_oracle(name, override, use_bias):
    require_gpu()
    cfg, part, case = _conv_case(name, **override)
    x_bufs, y, dx_bufs, dw, db = _run_conv(cfg, part, case, use_bias)
    o_bufs = prim.scatter_bulk(case["x"].astype(np.float64), part, fill=np.nan)
    bias = case["bias"] if use_bias else None
    y_want = layers.dist_conv_forward(o_bufs, case["w"], bias, part, cfg["stride"], cfg["dilation"])
    dx_want, dw_want, db_want = layers.dist_conv_adjoint(o_bufs, case["w"], prim.scatter_out(case["dy"], part), part,
                                                         cfg["stride"], cfg["dilation"], use_bias)
    for wk in range(part.n_workers):
        assert np.array_equal(from_cl(x_bufs[wk]), o_bufs[wk].astype(np.float32)), "x <- H x must be exact"
        assert_close(from_cl(y[wk]), y_want[wk], TOL32, f"y worker {wk}")
        assert_close(from_cl(dx_bufs[wk]), dx_want[wk], TOL32, f"dx worker {wk}")
        mask = np.ones(part.buf_shape(wk), dtype=bool)
        mask[part.bulk_slices(wk)] = False
        assert not from_cl(dx_bufs[wk])[:, :, mask].any()
    assert_close(dw.cpu().numpy(), dw_want, TOL32, "dw")
    if use_bias:
        assert_close(db.cpu().numpy(), db_want, TOL32, "db")


@pytest.mark.gpu
def test_small_channel_conv_repeated_launches_give_identical_bits():
    """The 16-channel kernels are deterministic (fixed summation order, one writer per cell): any difference between
    repeated launches of the 2-D configuration at full size (ragged windows in the data gradient) is a hazard."""
    require_gpu()
    cfg, part, case = _conv_case("cfg2")
    plan = dd.distdl_plan_create(cfg["D"], cfg["n_b"], cfg["c_in"], cfg["c_out"], cfg["in_shape"], cfg["P"],
                                 cfg["ksize"], cfg["stride"], cfg["padding"], cfg["dilation"], torch.float32)
    x_bufs = [to_cl(b, torch.float32) for b in prim.scatter_bulk(case["x"], part, fill=np.float32(3.0))]
    w = w_to_dev(case["w"])
    dy = [to_cl(t, torch.float32) for t in prim.scatter_out(case["dy"], part)]
    ws = torch.empty(max(dd.distdl_conv_bwd_workspace(plan), 16), dtype=torch.uint8, device="cuda")

    def run():
        y = [torch.full_like(t, float("nan")) for t in dy]
        dx = [torch.full_like(b, float("nan")) for b in x_bufs]
        dw = torch.full_like(w, float("nan"))
        dd.distdl_conv_fwd(plan, x_bufs, w, None, y)
        dd.distdl_conv_bwd(plan, x_bufs, w, dy, dx, dw, None, ws)
        torch.cuda.synchronize()
        return y + dx + [dw]

    first = run()
    assert not any(bool(torch.isnan(t).any()) for t in first)
    for _ in range(20):
        assert all(torch.equal(a, b) for a, b in zip(run(), first))


@pytest.mark.gpu
@pytest.mark.parametrize("idx", [2, 10])  # a 16-channel 2-D layer and a 32-channel strided 3-D layer
def test_conv_outputs_aligned_to_their_element_only(idx):
    """y and dx^ that start 4 bytes into an allocation: the kernels that store 16 bytes at a time must not be chosen."""
    require_gpu()
    name, override, use_bias = CONV_FULL[idx]
    cfg, part, case = _conv_case(name, **override)
    x_bufs, y, dx_bufs, dw, db = _run_conv(cfg, part, case, use_bias, misaligned_outputs=True)
    o_bufs = prim.scatter_bulk(case["x"].astype(np.float64), part, fill=np.nan)
    bias = case["bias"] if use_bias else None
    y_want = layers.dist_conv_forward(o_bufs, case["w"], bias, part, cfg["stride"], cfg["dilation"])
    dx_want, dw_want, _ = layers.dist_conv_adjoint(o_bufs, case["w"], prim.scatter_out(case["dy"], part), part,
                                                   cfg["stride"], cfg["dilation"], use_bias)
    for wk in range(part.n_workers):
        assert y[wk].data_ptr() % 16 != 0 and dx_bufs[wk].data_ptr() % 16 != 0
        assert_close(from_cl(y[wk]), y_want[wk], TOL32, f"y worker {wk}")
        assert_close(from_cl(dx_bufs[wk]), dx_want[wk], TOL32, f"dx worker {wk}")
    assert_close(dw.cpu().numpy(), dw_want, TOL32, "dw")


def _random_small_cases(count):
    """Seeded random layers with at most 16 channels: D, kernel, dilation, leading-dimension stride, ragged shapes
    and partitions (the geometry the 16 x 16-tile kernels choose their windows and units from)."""
    rng = np.random.default_rng(77)
    cases = []
    while len(cases) < count:
        D = int(rng.integers(1, 4))
        k = tuple(int(rng.choice([1, 3, 5])) if d >= D - 2 else int(rng.choice([1, 2, 3])) for d in range(D))
        dil = tuple(int(rng.choice([1, 1, 2])) for _ in range(D))
        stride = tuple(int(rng.choice([1, 2])) if d < D - 2 else 1 for d in range(D))
        P = tuple(int(rng.integers(1, 4)) for _ in range(D))
        pad = tuple(int(rng.integers(0, (k[d] - 1) * dil[d] // 2 + 1)) for d in range(D))
        lo = [max((k[d] - 1) * dil[d] + 1, 2 * P[d] * stride[d] + (k[d] - 1) * dil[d]) for d in range(D)]
        shape = tuple(int(rng.integers(lo[d], lo[d] + (40 if d == D - 1 else 14))) for d in range(D))
        cfg = dict(D=D, n_b=int(rng.integers(1, 12)), c_in=int(rng.integers(1, 17)), c_out=int(rng.integers(1, 17)),
                   in_shape=shape, P=P, ksize=k, stride=stride, padding=pad, dilation=dil, seed=len(cases))
        try:
            oracle_partition(cfg)
        except Exception:
            continue
        cases.append(cfg)
    return cases


@pytest.mark.parametrize("cfg", _random_small_cases(24), ids=lambda c: f"D{c['D']}c{c['c_in']}-{c['c_out']}k{'x'.join(map(str, c['ksize']))}")
def test_conv_small_channel_random_layers(cfg):
    require_gpu()
    part = oracle_partition(cfg)
    case = syn.conv_case(cfg, part.global_out_shape())
    x_bufs, y, dx_bufs, dw, db = _run_conv(cfg, part, case, True)
    o_bufs = prim.scatter_bulk(case["x"].astype(np.float64), part, fill=np.nan)
    y_want = layers.dist_conv_forward(o_bufs, case["w"], case["bias"], part, cfg["stride"], cfg["dilation"])
    dx_want, dw_want, db_want = layers.dist_conv_adjoint(o_bufs, case["w"], prim.scatter_out(case["dy"], part), part,
                                                         cfg["stride"], cfg["dilation"], True)
    for wk in range(part.n_workers):
        assert_close(from_cl(y[wk]), y_want[wk], TOL32, f"y worker {wk}")
        assert_close(from_cl(dx_bufs[wk]), dx_want[wk], TOL32, f"dx worker {wk}")
    assert_close(dw.cpu().numpy(), dw_want, TOL32, "dw")
    assert_close(db.cpu().numpy(), db_want, TOL32, "db")


CONV_BF16 = [
    # matrix-core path (channel counts that are multiples of 4), 3-D strided, 2-D, dilated; then the direct kernels
    ("cfg5", dict(in_shape=(24, 22, 40), P=(2, 2, 1), c_in=32, c_out=32), True),
    ("cfg5u", dict(in_shape=(21, 23, 22), P=(2, 2, 2), c_in=32, c_out=32), False),
    ("cfg2", dict(in_shape=(64, 64), n_b=2), True),
    ("cfg2", dict(in_shape=(23, 41), n_b=2, c_in=4, c_out=40, P=(2, 3), ksize=(3, 4), stride=(2, 1), padding=(1, 2),
                  dilation=(1, 2)), True),
    ("cfg2", dict(in_shape=(19, 23), n_b=3, c_in=3, c_out=5, P=(2, 3), ksize=(3, 4), stride=(2, 1), padding=(1, 2),
                  dilation=(1, 2)), True),
    ("cfg1", dict(), True),
    # 24 input channels: the last 16-channel chunk of the bf16 matrix-core kernel is half empty
    ("cfg5", dict(in_shape=(14, 18, 36), P=(2, 1, 2), c_in=24, c_out=8, ksize=(3, 3, 3), stride=(1, 2, 1),
                  padding=(1, 1, 1)), True),
    # several channel tiles, the second output tile half full: db sums of the weight-gradient kernel per tile
    ("cfg2", dict(in_shape=(40, 70), n_b=2, c_in=64, c_out=48, ksize=(3, 3), padding=(1, 1), P=(2, 2)), True),
    # 20 output channels: not a multiple of 8, so the forward kernel stores 8-byte channel quads instead of 16-byte
    # pieces, and the data gradient (20 contraction channels) widens bf16 to fp32 while staging
    ("cfg2", dict(in_shape=(37, 45), n_b=2, c_in=40, c_out=20, ksize=(3, 3), padding=(1, 1), stride=(2, 1), P=(2, 2)), True),
]


@pytest.mark.parametrize("name,override,use_bias", CONV_BF16, ids=[f"{n}-{i}" for i, (n, _, _) in enumerate(CONV_BF16)])
def test_conv_bf16_fwd_bwd_against_partitioned_oracle(name, override, use_bias):
    """bf16 tensors (inputs, weights, bias, outputs, gradients), fp32 accumulation: the oracle runs in fp64 on the
    same bf16-representable inputs; bar 2e-2."""
    require_gpu()
    cfg, part, case = _conv_case(name, **override)
    bf = torch.bfloat16
    x, w, dyv = syn.to_bf16_values(case["x"]), syn.to_bf16_values(case["w"]), syn.to_bf16_values(case["dy"])
    bias = syn.to_bf16_values(case["bias"] + 0.25) if use_bias else None
    plan = dd.distdl_plan_create(cfg["D"], cfg["n_b"], cfg["c_in"], cfg["c_out"], cfg["in_shape"], cfg["P"],
                                 cfg["ksize"], cfg["stride"], cfg["padding"], cfg["dilation"], bf)
    x_bufs = [to_cl(b, bf) for b in prim.scatter_bulk(x, part, fill=np.float32(3.0))]
    gw = torch.from_numpy(np.ascontiguousarray(w)).to(bf).cuda()
    gb = torch.from_numpy(np.ascontiguousarray(bias)).to(bf).cuda() if use_bias else None
    y = [torch.full((cfg["n_b"],) + part.out_shape(wk) + (cfg["c_out"],), 7.0, device="cuda", dtype=bf)
         for wk in range(part.n_workers)]
    dd.distdl_conv_fwd(plan, x_bufs, gw, gb, y)
    dy = [to_cl(t, bf) for t in prim.scatter_out(dyv, part)]
    dx_bufs = [torch.full_like(b, 5.0) for b in x_bufs]
    dw = torch.full_like(gw, 9.0)
    db = torch.full((cfg["c_out"],), 9.0, device="cuda", dtype=bf) if use_bias else None
    ws = torch.empty(max(dd.distdl_conv_bwd_workspace(plan), 16), dtype=torch.uint8, device="cuda")
    dd.distdl_conv_bwd(plan, x_bufs, gw, dy, dx_bufs, dw, db, ws)
    torch.cuda.synchronize()
    o_bufs = prim.scatter_bulk(x.astype(np.float64), part, fill=np.nan)
    y_want = layers.dist_conv_forward(o_bufs, w.astype(np.float64), bias, part, cfg["stride"], cfg["dilation"])
    dx_want, dw_want, db_want = layers.dist_conv_adjoint(o_bufs, w.astype(np.float64), prim.scatter_out(dyv, part), part,
                                                         cfg["stride"], cfg["dilation"], use_bias)
    for wk in range(part.n_workers):
        assert np.array_equal(from_cl(x_bufs[wk]), o_bufs[wk].astype(np.float32)), "x <- H x must be exact"
        assert_close(from_cl(y[wk]), y_want[wk], TOL16, f"y worker {wk}")
        assert_close(from_cl(dx_bufs[wk]), dx_want[wk], TOL16, f"dx worker {wk}")
    assert_close(dw.float().cpu().numpy(), dw_want, TOL16, "dw")
    if use_bias:
        assert_close(db.float().cpu().numpy(), db_want, TOL16, "db")


@pytest.mark.parametrize("name,override,dtype", [
    ("cfg2", dict(in_shape=(64, 64), n_b=4), torch.float32),                                   # 16 x 16-tile kernels
    ("cfg5", dict(in_shape=(24, 22, 40), P=(2, 2, 1)), torch.float32),                          # 32-wide kernels
    ("cfg5", dict(in_shape=(24, 22, 40), P=(2, 2, 1)), torch.bfloat16),                         # bf16 matrix cores
    ("cfg2", dict(in_shape=(19, 23), n_b=3, c_in=3, c_out=5, P=(2, 3), stride=(2, 1)), torch.float32),   # direct kernels
], ids=["small16", "wide", "bf16", "direct"])
def test_conv_is_run_to_run_identical(name, override, dtype):
    """No float atomics anywhere: partial sums are combined in a fixed order (Sec. 2 footnote on floating-point
    addition in parallel), so two runs on the same inputs agree bit for bit."""
    require_gpu()
    cfg, part, case = _conv_case(name, **override)
    if dtype == torch.bfloat16:
        case = {k: (syn.to_bf16_values(v) if isinstance(v, np.ndarray) else v) for k, v in case.items()}
    first = _run_conv(cfg, part, case, True, dtype)
    second = _run_conv(cfg, part, case, True, dtype)
    for a, b in zip(first[1] + first[2] + [first[3], first[4]], second[1] + second[2] + [second[3], second[4]]):
        assert torch.equal(a, b)


def test_conv_cfg2_full_size():
    """cfg2 at its full size against the sequential definition (Sec. 5 claim:
    distributed == sequential)."""
    require_gpu()
    cfg, part, case = _conv_case("cfg2")
    x_bufs, y, dx_bufs, dw, db = _run_conv(cfg, part, case, True)
    y_want = layers.conv_forward(case["x"], case["w"], case["bias"], cfg["stride"], cfg["padding"], cfg["dilation"])
    dx_want, dw_want, db_want = layers.conv_backward(case["x"], case["w"], case["dy"], cfg["stride"], cfg["padding"],
                                                     cfg["dilation"])
    assert_close(prim.gather_out([from_cl(t) for t in y], part), y_want, TOL32, "y")
    assert_close(prim.gather_bulk([from_cl(t) for t in dx_bufs], part), dx_want, TOL32, "dx")
    assert_close(dw.cpu().numpy(), dw_want, TOL32, "dw")
    assert_close(db.cpu().numpy(), db_want, TOL32, "db")


def test_conv_rejects_bad_arguments():
    require_gpu()
    plan = dd.distdl_plan_create_explicit(1, 1, 1, [2], [[4, 4]], [[(0, 1), (1, 0)]])
    t = torch.zeros(8, device="cuda")
    with pytest.raises(dd.DistdlError) as e:
        dd.distdl_conv_fwd(plan, [t, t], t, None, [t, t])
    assert e.value.code == dd.ERR_UNSUPPORTED
    plan = dd.distdl_plan_create(1, 1, 1, 1, [8], [2], [3], [1], [1], [1])
    with pytest.raises(dd.DistdlError) as e:
        dd.distdl_conv_bwd(plan, [t, t], t, [t, t], [t, t], t, None, torch.zeros(4, dtype=torch.uint8, device="cuda")[:0])
    assert e.value.code in (dd.ERR_INVALID_ARG, dd.ERR_NULL)


# ---------------------------------------------------------------- affine
AFFINE_CASES = [
    # n_b, n_fi, n_fo, P_fo, P_fi
    (256, 4096, 4096, 2, 2),       # cfg3
    (256, 400, 120, 2, 2), (256, 120, 84, 2, 2), (256, 84, 10, 2, 2),   # cfg4 / App. C table
    (7, 13, 9, 3, 2), (5, 33, 17, 1, 1), (64, 256, 192, 1, 4), (33, 130, 70, 4, 1),
    (128, 3000, 1024, 1, 3),       # K splits that straddle the column workers' segments, ragged last K stage
    (200, 2064, 3096, 1, 2),       # small batch, wide layer: ragged tiles in M, N and K
    (100, 1048, 528, 2, 1),        # small batch: ragged M, N and K tails in the forward and the data-gradient product, two row workers
    (37, 264, 72, 1, 1),           # one tile, output rows of 72 (no whole 16-column groups at the edge), K tail of 8
    (48, 192, 264, 3, 1),          # data gradient summed over three row workers whose K (88) ends inside a 64-k step
]


@pytest.mark.parametrize("n_b,n_fi,n_fo,P_fo,P_fi", AFFINE_CASES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("use_bias", [True, False], ids=["bias", "nobias"])
def test_affine_fwd_bwd(n_b, n_fi, n_fo, P_fo, P_fi, dtype, use_bias):
    require_gpu()
    if n_fi == 4096 and not use_bias:
        pytest.skip("full size covered with bias")
    case = syn.affine_case(syn.CONFIGS["cfg3"], n_b, n_fi, n_fo)
    conv = syn.to_bf16_values if dtype == torch.bfloat16 else (lambda a: a)
    x, W, b, dy = (conv(case[k]) for k in ("x", "W", "b", "dy"))
    tol = TOL32 if dtype == torch.float32 else TOL16
    rows, cols = layers.feature_blocks(n_fo, P_fo), layers.feature_blocks(n_fi, P_fi)
    x_parts = [x[:, c] for c in cols]
    W_parts = [[W[r][:, c] for c in cols] for r in rows]
    b_parts = [b[r] for r in rows] if use_bias else None
    dy_parts = [dy[:, r] for r in rows]
    y_want = layers.dist_affine_forward(x_parts, W_parts, b_parts, P_fo, P_fi)
    dx_want, dW_want, db_want = layers.dist_affine_adjoint(x_parts, W_parts, dy_parts, P_fo, P_fi)

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()
    g_x = [dev(t) for t in x_parts]
    g_W = [dev(W_parts[i][j]) for i in range(P_fo) for j in range(P_fi)]
    g_b = [dev(t) for t in b_parts] if use_bias else None
    g_dy = [dev(t) for t in dy_parts]
    g_y = [torch.full(t.shape, 3.0, dtype=dtype, device="cuda") for t in y_want]
    g_dx = [torch.full(t.shape, 3.0, dtype=dtype, device="cuda") for t in dx_want]
    g_dW = [torch.full(dW_want[i][j].shape, 3.0, dtype=dtype, device="cuda") for i in range(P_fo) for j in range(P_fi)]
    g_db = [torch.full(t.shape, 3.0, dtype=dtype, device="cuda") for t in db_want] if use_bias else None
    plan = dd.distdl_affine_plan_create(n_b, n_fi, n_fo, P_fo, P_fi, dtype)
    dd.distdl_affine_fwd(plan, g_x, g_W, g_b, g_y)
    dd.distdl_affine_bwd(plan, g_x, g_W, g_dy, g_dx, g_dW, g_db)
    torch.cuda.synchronize()
    host = lambda t: t.float().cpu().numpy()
    for i in range(P_fo):
        assert_close(host(g_y[i]), y_want[i], tol, f"y_{i}")
        if use_bias:
            assert_close(host(g_db[i]), db_want[i], tol, f"db_{i}")
        for j in range(P_fi):
            assert_close(host(g_dW[i * P_fi + j]), dW_want[i][j], tol, f"dW_{i}{j}")
    for j in range(P_fi):
        assert_close(host(g_dx[j]), dx_want[j], tol, f"dx_{j}")
    # whole-layer check against the sequential definition
    assert_close(np.concatenate([host(t) for t in g_y], axis=1), layers.affine_forward(x, W, b if use_bias else None),
                 tol, "y vs sequential")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n_b,n_fi,n_fo,P_fo,P_fi", [(256, 1024, 768, 2, 2), (100, 1048, 528, 2, 1)])
def test_affine_step_replayed_from_a_graph_matches_eager(n_b, n_fi, n_fo, P_fo, P_fi, dtype):
    """A warmed-up affine forward + adjoint (in bf16: the streaming kernels fed by global -> LDS loads, the bias
    gradient inside the weight-gradient launch) recorded into a HIP graph and replayed on
    new data, with eager work and synchronisations between the replays, must reproduce the eager step bit for bit;
    the eager step itself is checked against the oracle."""
    require_gpu()
    rows, cols = layers.feature_blocks(n_fo, P_fo), layers.feature_blocks(n_fi, P_fi)
    rng = np.random.default_rng(11)
    conv = syn.to_bf16_values if dtype == torch.bfloat16 else (lambda a: a)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()
    W = conv((rng.standard_normal((n_fo, n_fi)) / np.sqrt(n_fi)).astype(np.float32))
    b = conv(rng.standard_normal(n_fo).astype(np.float32))
    g_W = [dev(W[r][:, c]) for r in rows for c in cols]
    g_b = [dev(b[r]) for r in rows]
    new_batch = lambda: (conv(rng.standard_normal((n_b, n_fi)).astype(np.float32)),
                         conv(rng.standard_normal((n_b, n_fo)).astype(np.float32)))
    g_x = [torch.zeros((n_b, c.stop - c.start), dtype=dtype, device="cuda") for c in cols]
    g_dy = [torch.zeros((n_b, r.stop - r.start), dtype=dtype, device="cuda") for r in rows]
    g_y = [torch.zeros_like(t) for t in g_dy]
    g_dx = [torch.zeros_like(t) for t in g_x]
    g_dW = [torch.zeros_like(t) for t in g_W]
    g_db = [torch.zeros_like(t) for t in g_b]
    plan = dd.distdl_affine_plan_create(n_b, n_fi, n_fo, P_fo, P_fi, dtype)

    def step():
        dd.distdl_affine_fwd(plan, g_x, g_W, g_b, g_y)
        dd.distdl_affine_bwd(plan, g_x, g_W, g_dy, g_dx, g_dW, g_db)

    def load(x, dy):
        for dst, c in zip(g_x, cols):
            dst.copy_(dev(x[:, c]))
        for dst, r in zip(g_dy, rows):
            dst.copy_(dev(dy[:, r]))

    snapshot = lambda: [t.clone() for t in g_y + g_dx + g_dW + g_db]
    batches = [new_batch() for _ in range(3)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    eager = []
    with torch.cuda.stream(side):
        for x, dy in batches:
            load(x, dy)
            step()
            eager.append(snapshot())
    side.synchronize()
    # the last eager step against the oracle
    x, dy = batches[-1]
    tol = TOL32 if dtype == torch.float32 else TOL16
    host = lambda t: t.float().cpu().numpy()
    y_want = layers.affine_forward(x, W, b)
    assert_close(np.concatenate([host(t) for t in g_y], axis=1), y_want, tol, "y")
    dx_want, dW_want, db_want = layers.affine_backward(x, W, dy)
    assert_close(np.concatenate([host(t) for t in g_dx], axis=1), dx_want, tol, "dx")
    for i, r in enumerate(rows):
        assert_close(host(g_db[i]), db_want[r], tol, f"db_{i}")
        for j, c in enumerate(cols):
            assert_close(host(g_dW[i * P_fi + j]), dW_want[r][:, c], tol, f"dW_{i}{j}")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for (x, dy), want in zip(batches, eager):
        load(x, dy)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(snapshot(), want):
            assert torch.equal(got, ref)


def _round_bf16(x):
    """fp64 -> the nearest bf16-representable value, ties to even (8 significant bits), and the spacing there."""
    m, e = np.frexp(np.asarray(x, dtype=np.float64))
    return np.ldexp(np.round(m * 256.0) / 256.0, e), np.ldexp(1.0, e - 8)


def _assert_rounded_sum(got, want64, what):
    """A bf16 result is the fp32-accumulated sum rounded once to nearest-even: it equals the oracle's fp64 value
    rounded the same way, except where the fp32 accumulation error (about 1e-6 of the output scale) carries the sum
    across a rounding boundary, and then it is the neighbouring bf16 value.  Truncation, or rounding the partial
    sums, would move a large share of the elements by one step (the planted-mistake check below shows it)."""
    ref, step = _round_bf16(want64)
    diff = np.abs(got.astype(np.float64) - ref)
    scale = float(np.sqrt(np.mean(np.asarray(want64, dtype=np.float64) ** 2)))
    assert np.all(diff <= step * 1.0001 + 2e-6 * scale), f"{what}: {np.sum(diff > step * 1.0001 + 2e-6 * scale)} elements off by more than one bf16 step"
    exact = float(np.mean(diff == 0))
    assert exact >= 0.99, f"{what}: only {exact:.4f} of the elements are the correctly rounded value"


def test_bf16_rounding_pin_detects_truncation():
    """The pin itself: truncating instead of rounding to nearest fails it."""
    rng = np.random.default_rng(5)
    v = rng.standard_normal(20000)
    ok = syn.to_bf16_values(v.astype(np.float32))
    _assert_rounded_sum(ok, v.astype(np.float32).astype(np.float64), "rounded")
    trunc = (v.astype(np.float32).view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)
    with pytest.raises(AssertionError):
        _assert_rounded_sum(trunc, v.astype(np.float32).astype(np.float64), "truncated")


def test_bf16_outputs_are_the_rounded_fp32_sums():
    """bf16 layers (bf16 MFMAs, fp32 accumulation): every output tensor of the affine layer (streaming kernels) and
    of a strided 32-channel convolution (forward, data gradient through H*, weight and bias gradient) against the
    oracle's fp64 result rounded to bf16 with ties to even."""
    require_gpu()
    dtype = torch.bfloat16
    host = lambda t: t.float().cpu().numpy()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()
    # affine
    n_b, n_fi, n_fo = 64, 256, 192
    rng = np.random.default_rng(21)
    x = syn.to_bf16_values(rng.standard_normal((n_b, n_fi)).astype(np.float32))
    W = syn.to_bf16_values((rng.standard_normal((n_fo, n_fi)) / np.sqrt(n_fi)).astype(np.float32))
    b = syn.to_bf16_values(rng.standard_normal(n_fo).astype(np.float32))
    dy = syn.to_bf16_values(rng.standard_normal((n_b, n_fo)).astype(np.float32))
    g_y, g_dx, g_dW, g_db = (torch.zeros(sh, dtype=dtype, device="cuda") for sh in ((n_b, n_fo), (n_b, n_fi), (n_fo, n_fi), (n_fo,)))
    plan = dd.distdl_affine_plan_create(n_b, n_fi, n_fo, 1, 1, dtype)
    dd.distdl_affine_fwd(plan, [dev(x)], [dev(W)], [dev(b)], [g_y])
    dd.distdl_affine_bwd(plan, [dev(x)], [dev(W)], [dev(dy)], [g_dx], [g_dW], [g_db])
    torch.cuda.synchronize()
    dx_w, dW_w, db_w = layers.affine_backward(x, W, dy)
    for got, want, what in ((g_y, layers.affine_forward(x, W, b), "affine y"), (g_dx, dx_w, "affine dx"),
                            (g_dW, dW_w, "affine dW"), (g_db, db_w, "affine db")):
        _assert_rounded_sum(host(got), want, what)
    # convolution: one worker, so that no halo sum adds a second rounding to dx
    cfg, part, case = _conv_case("cfg5u", in_shape=(21, 23, 22), P=(1, 1, 1), c_in=32, c_out=32)
    xc, wc, bc, dyc = (syn.to_bf16_values(case[k]) for k in ("x", "w", "bias", "dy"))
    plan = dd.distdl_plan_create(cfg["D"], cfg["n_b"], cfg["c_in"], cfg["c_out"], cfg["in_shape"], cfg["P"],
                                 cfg["ksize"], cfg["stride"], cfg["padding"], cfg["dilation"], dtype)
    x_bufs = [to_cl(t, dtype) for t in prim.scatter_bulk(xc, part, fill=np.float32(3.0))]
    g_w, g_bias = w_to_dev(wc).to(dtype), w_to_dev(bc).to(dtype)
    y = [torch.zeros((cfg["n_b"],) + part.out_shape(0) + (cfg["c_out"],), device="cuda", dtype=dtype)]
    dd.distdl_conv_fwd(plan, x_bufs, g_w, g_bias, y)
    g_dy = [to_cl(t, dtype) for t in prim.scatter_out(dyc, part)]
    dx = [torch.zeros_like(t) for t in x_bufs]
    dw, db = torch.zeros_like(g_w), torch.zeros_like(g_bias)
    ws = torch.empty(max(dd.distdl_conv_bwd_workspace(plan), 16), dtype=torch.uint8, device="cuda")
    dd.distdl_conv_bwd(plan, x_bufs, g_w, g_dy, dx, dw, db, ws)
    torch.cuda.synchronize()
    bufs = prim.scatter_bulk(xc.astype(np.float64), part)
    y_want = layers.dist_conv_forward(bufs, wc, bc, part, cfg["stride"], cfg["dilation"])  # leaves H x in bufs
    dx_want, dw_want, db_want = layers.dist_conv_adjoint(bufs, wc, prim.scatter_out(dyc.astype(np.float64), part), part,
                                                         cfg["stride"], cfg["dilation"], True)
    _assert_rounded_sum(from_cl(y[0]), y_want[0], "conv y")
    _assert_rounded_sum(from_cl(dx[0]), dx_want[0], "conv dx")
    _assert_rounded_sum(host(dw), dw_want, "conv dw")
    _assert_rounded_sum(host(db), db_want, "conv db")


# ---------------------------------------------------------------- full-size volumetric configuration
def _sample_indices(rng, shape, count):
    return [tuple(int(rng.integers(0, s)) for s in shape) for _ in range(count)]


@pytest.mark.parametrize("name,dtype", [("cfg5", torch.float32), ("cfg5u", torch.float32), ("cfg5", torch.bfloat16)],
                         ids=["cfg5", "cfg5u", "cfg5-bf16"])
def test_conv_full_size_sampled(name, dtype):
    """The volumetric configuration at its full size, in the launch configuration the benchmark
    times: sampled outputs against the plain definition of Sec. 4 (cross-correlation and its
    adjoint), computed one by one in fp64; halo cells against the global tensor (exact).  bf16: the same on
    bf16-representable inputs at the bf16 bar."""
    require_gpu()
    cfg = dict(syn.CONFIGS[name])
    part = oracle_partition(cfg)
    case = syn.conv_case(cfg, part.global_out_shape())
    tol = TOL32 if dtype == torch.float32 else TOL16
    if dtype == torch.bfloat16:
        case = {k: (syn.to_bf16_values(v) if isinstance(v, np.ndarray) else v) for k, v in case.items()}
    x, w, dy, bias = case["x"], case["w"].astype(np.float64), case["dy"], case["bias"]
    x_bufs, y, dx_bufs, dw, db = _run_conv(cfg, part, case, True, dtype)
    s, p, k = cfg["stride"], cfg["padding"], cfg["ksize"]
    n_in, n_out = cfg["in_shape"], part.global_out_shape()
    rng = np.random.default_rng(0)

    # H: sampled workers' buffers equal the zero-extended global tensor, bit for bit
    for wk in (0, 21, 42, 63):
        assert np.array_equal(from_cl(x_bufs[wk]), prim.expected_buffer_after_halo(x, part, wk)), f"H worker {wk}"

    def window(o):
        """Input window of output index o with zero padding, [ci, k0, k1, k2] in fp64."""
        win = np.zeros((cfg["c_in"],) + tuple(k))
        lo = [o[d] * s[d] - p[d] for d in range(3)]
        src = tuple(slice(max(lo[d], 0), min(lo[d] + k[d], n_in[d])) for d in range(3))
        dst = tuple(slice(max(lo[d], 0) - lo[d], min(lo[d] + k[d], n_in[d]) - lo[d]) for d in range(3))
        win[(slice(None),) + dst] = x[(0, slice(None)) + src]
        return win

    y_glob_scale = 0.0
    errs = []
    owner = {}
    for wk in range(part.n_workers):
        owner[tuple(part.g(wk, d)["out_start"] for d in range(3))] = wk
    y_host = {}
    for o in _sample_indices(rng, n_out, 200):
        wk = next(wkk for wkk in range(part.n_workers)
                  if all(part.g(wkk, d)["out_start"] <= o[d] < part.g(wkk, d)["out_start"] + part.g(wkk, d)["out_size"]
                         for d in range(3)))
        if wk not in y_host:
            y_host[wk] = from_cl(y[wk])
        lo = tuple(o[d] - part.g(wk, d)["out_start"] for d in range(3))
        want = np.einsum("ocijk,cijk->o", w, window(o)) + bias
        got = y_host[wk][(0, slice(None)) + lo]
        errs.append(np.abs(got - want).max())
        y_glob_scale = max(y_glob_scale, np.abs(want).max())
    assert max(errs) <= tol * y_glob_scale, (max(errs), y_glob_scale)

    # dw: sampled entries; dw[co,ci,kappa] = sum_o dy[co,o] x[ci, o*s - p + kappa]
    dw_host = dw.float().cpu().numpy()
    dy64 = dy[0].astype(np.float64)
    worst, scale = 0.0, np.abs(dw_host).max()
    for (co, ci, k0, k1, k2) in _sample_indices(rng, (cfg["c_out"], cfg["c_in"]) + tuple(k), 24):
        kap = (k0, k1, k2)
        # output range whose tap kappa lies inside the input
        o_lo = [max(0, -((kap[d] - p[d]) // s[d])) for d in range(3)]
        o_hi = [min(n_out[d] - 1, (n_in[d] - 1 + p[d] - kap[d]) // s[d]) for d in range(3)]
        osl = tuple(slice(o_lo[d], o_hi[d] + 1) for d in range(3))
        isl = tuple(slice(o_lo[d] * s[d] - p[d] + kap[d], o_hi[d] * s[d] - p[d] + kap[d] + 1, s[d]) for d in range(3))
        want = float(np.sum(dy64[(co,) + osl] * x[(0, ci) + isl].astype(np.float64)))
        worst = max(worst, abs(dw_host[co, ci, k0, k1, k2] - want))
    assert worst <= tol * scale, (worst, scale)
    db_want = dy64.sum(axis=(1, 2, 3))
    assert_close(db.float().cpu().numpy(), db_want, tol, "db")

    # dx: sampled input cells; dx[ci,i] = sum_{co,kappa: (i + p - kappa) % s == 0} w[co,ci,kappa] dy[co,(i+p-kappa)/s]
    dx_host = {}
    worst, scale = 0.0, 0.0
    for i in _sample_indices(rng, n_in, 120):
        wk = next(wkk for wkk in range(part.n_workers)
                  if all(part.g(wkk, d)["in_start"] <= i[d] < part.g(wkk, d)["in_start"] + part.g(wkk, d)["in_size"]
                         for d in range(3)))
        if wk not in dx_host:
            dx_host[wk] = from_cl(dx_bufs[wk])
        loc = tuple(i[d] - part.g(wk, d)["in_start"] + part.g(wk, d)["bulk_off"] for d in range(3))
        want = np.zeros(cfg["c_in"])
        for kap in np.ndindex(*k):
            q = [i[d] + p[d] - kap[d] for d in range(3)]
            if all(q[d] % s[d] == 0 and 0 <= q[d] // s[d] < n_out[d] for d in range(3)):
                o = tuple(q[d] // s[d] for d in range(3))
                want += w[(slice(None), slice(None)) + kap].T @ dy64[(slice(None),) + o]
        got = dx_host[wk][(0, slice(None)) + loc]
        worst = max(worst, np.abs(got - want).max())
        scale = max(scale, np.abs(want).max())
    assert worst <= tol * scale, (worst, scale)
    # halo and pad cells of dx end cleared (H* ran)
    for wk in list(dx_host)[:4]:
        mask = np.ones(part.buf_shape(wk), dtype=bool)
        mask[part.bulk_slices(wk)] = False
        assert not dx_host[wk][:, :, mask].any()


@pytest.mark.parametrize("name", ["cfg5", "cfg5u"])
def test_conv_full_size_whole_workers(name):
    """The volumetric configuration at its full size, in the launch configuration the benchmark times: every
    element of a corner, an edge, a face, an interior and the far-corner worker against the oracle -- y from the
    oracle's local correlation on that worker's buffer after H; the local gradient dx^ over the whole padded
    buffer (halo and padding cells included) before H*; and dx after H*, whose bulk (band cells that H* adds
    into included) must equal the sequential layer's gradient on that region, with halo and padding cleared."""
    require_gpu()
    cfg = dict(syn.CONFIGS[name])
    part = oracle_partition(cfg)
    case = syn.conv_case(cfg, part.global_out_shape())
    s, p, k, dil = cfg["stride"], cfg["padding"], cfg["ksize"], cfg["dilation"]
    plan = dd.distdl_plan_create(cfg["D"], cfg["n_b"], cfg["c_in"], cfg["c_out"], cfg["in_shape"], cfg["P"], k, s, p, dil)
    x_bufs = [to_cl(b) for b in prim.scatter_bulk(case["x"], part, fill=np.float32(3.0))]
    w, bias = w_to_dev(case["w"]), w_to_dev(case["bias"])
    y = [torch.full((cfg["n_b"],) + part.out_shape(wk) + (cfg["c_out"],), 7.0, device="cuda")
         for wk in range(part.n_workers)]
    dd.distdl_conv_fwd(plan, x_bufs, w, bias, y)
    dy_parts = prim.scatter_out(case["dy"], part)
    dy = [to_cl(t) for t in dy_parts]
    dx_local = [torch.full_like(b, 5.0) for b in x_bufs]
    dw, db = torch.full_like(w, 9.0), torch.full_like(bias, 9.0)
    ws = torch.empty(max(dd.distdl_conv_bwd_workspace(plan), 16), dtype=torch.uint8, device="cuda")
    dd.distdl_conv_local_bwd(plan, x_bufs, w, dy, dx_local, dw, db, ws)      # [dConv]* and R dw, R db; no H*
    dx = [torch.full_like(b, 5.0) for b in x_bufs]
    dw2, db2 = torch.full_like(w, 9.0), torch.full_like(bias, 9.0)
    dd.distdl_conv_bwd(plan, x_bufs, w, dy, dx, dw2, db2, ws)                # the whole adjoint algorithm
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2) and torch.equal(db, db2)
    if name == "cfg5":
        pick = {"corner": (0, 0, 0), "edge": (0, 0, 1), "face": (0, 1, 2), "interior": (1, 2, 1)}
    else:   # uneven bulks: an interior worker with a 63 / 62 / 63 bulk and the far corner (right-hand padding)
        pick = {"interior": (1, 2, 1), "far corner": (3, 3, 3)}
    n_in, n_out = cfg["in_shape"], part.global_out_shape()

    def oracle_side(wk):
        """The three oracle results for worker wk (plain calls of oracle.layers; run side by side in threads only
        to keep the test short, numpy releases the interpreter lock inside them)."""
        xb = prim.expected_buffer_after_halo(case["x"], part, wk)             # H x, cell by cell from the global tensor
        origin = [part.g(wk, d)["origin"] for d in range(3)]
        y_want = layers.conv_valid(xb, case["w"], case["bias"], part.out_shape(wk), s, dil, origin)
        dxp_want, _, _ = layers.conv_valid_adjoint(xb, case["w"], dy_parts[wk], s, dil, origin)
        return xb, y_want, dxp_want

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(len(pick)) as pool:
        oracle = dict(zip(pick, pool.map(oracle_side, [part.worker_id(c) for c in pick.values()])))
    for label, coords in pick.items():
        wk = part.worker_id(coords)
        xb, y_want, dxp_want = oracle[label]
        assert np.array_equal(from_cl(x_bufs[wk]), xb), f"H x, {label} worker"
        assert_close(from_cl(y[wk]), y_want, TOL32, f"y, {label} worker")
        assert_close(from_cl(dx_local[wk]), dxp_want, TOL32, f"dx^ before H*, {label} worker")
        # after H*: the sequential gradient on the worker's bulk.  Outputs that touch the bulk [a0, a1] of a
        # dimension are o_lo .. o_hi; the sequential adjoint on that slab of dy, cropped to the bulk
        geom = [part.g(wk, d) for d in range(3)]
        a0 = [g["in_start"] for g in geom]
        a1 = [g["in_start"] + g["in_size"] - 1 for g in geom]
        span = [dil[d] * (k[d] - 1) for d in range(3)]
        o_lo = [max(0, -((-(a0[d] + p[d] - span[d])) // s[d])) for d in range(3)]
        o_hi = [min(n_out[d] - 1, (a1[d] + p[d]) // s[d]) for d in range(3)]
        v0 = [o_lo[d] * s[d] - p[d] for d in range(3)]                          # global index of the slab's first cell
        vshape = tuple((o_hi[d] - o_lo[d]) * s[d] + span[d] + 1 for d in range(3))
        dy_slab = case["dy"][(slice(None), slice(None)) + tuple(slice(o_lo[d], o_hi[d] + 1) for d in range(3))]
        slab, _, _ = layers.conv_valid_adjoint(np.zeros((cfg["n_b"], cfg["c_in"]) + vshape), case["w"], dy_slab, s, dil,
                                               [0, 0, 0], want_bias=False)
        crop = tuple(slice(a0[d] - v0[d], a1[d] - v0[d] + 1) for d in range(3))
        got = from_cl(dx[wk])
        bulk = (slice(None), slice(None)) + part.bulk_slices(wk)
        assert_close(got[bulk], slab[(slice(None), slice(None)) + crop], TOL32, f"dx after H*, bulk of the {label} worker")
        mask = np.ones(part.buf_shape(wk), dtype=bool)
        mask[part.bulk_slices(wk)] = False
        assert not got[:, :, mask].any(), f"halo / padding of dx not cleared, {label} worker"
        # and H* changed exactly the band cells: away from them dx^ is untouched
        inner = tuple(slice(g["bulk_off"] + 4, g["bulk_off"] + g["in_size"] - 4) for g in geom)
        assert np.array_equal(got[(slice(None), slice(None)) + inner],
                              from_cl(dx_local[wk])[(slice(None), slice(None)) + inner])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_conv_step_replayed_from_a_graph_matches_eager(dtype):
    """The 32-channel strided layer (matrix-core kernels, eight parity-class launches, fused db sums): a warmed-up
    forward + backward recorded into a HIP graph and replayed on new data must reproduce the eager step bit for bit."""
    require_gpu()
    cfg, part, case = _conv_case("cfg5u", in_shape=(21, 23, 22), P=(2, 2, 2), c_in=32, c_out=32)
    plan = dd.distdl_plan_create(cfg["D"], cfg["n_b"], cfg["c_in"], cfg["c_out"], cfg["in_shape"], cfg["P"],
                                 cfg["ksize"], cfg["stride"], cfg["padding"], cfg["dilation"], dtype)
    rng = np.random.default_rng(3)
    new_x = lambda: [to_cl(b, dtype) for b in prim.scatter_bulk(rng.standard_normal(case["x"].shape).astype(np.float32),
                                                                  part, fill=np.float32(3.0))]
    new_dy = lambda: [to_cl(t, dtype) for t in prim.scatter_out(rng.standard_normal(case["dy"].shape).astype(np.float32),
                                                                 part)]
    x_bufs, dy = new_x(), new_dy()
    w, bias = w_to_dev(case["w"]).to(dtype), w_to_dev(case["bias"]).to(dtype)
    y = [torch.zeros((cfg["n_b"],) + part.out_shape(wk) + (cfg["c_out"],), device="cuda", dtype=dtype)
         for wk in range(part.n_workers)]
    dx = [torch.zeros_like(b) for b in x_bufs]
    dw, db = torch.zeros_like(w), torch.zeros_like(bias)
    ws = torch.empty(max(dd.distdl_conv_bwd_workspace(plan), 16), dtype=torch.uint8, device="cuda")

    def step():
        dd.distdl_conv_fwd(plan, x_bufs, w, bias, y)
        dd.distdl_conv_bwd(plan, x_bufs, w, dy, dx, dw, db, ws)

    def load(xs, dys):                      # into the recorded buffers, by eager copies
        for dst, src in zip(x_bufs, xs):
            dst.copy_(src)
        for dst, src in zip(dy, dys):
            dst.copy_(src)

    snapshot = lambda: [t.clone() for t in (y[0], y[-1], dx[0], dx[-1], dw, db, x_bufs[3])]
    batches = [(new_x(), new_dy()) for _ in range(3)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    eager = []
    with torch.cuda.stream(side):
        for xs, dys in batches:
            load(xs, dys)
            step()
            eager.append(snapshot())
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for (xs, dys), want in zip(batches, eager):
        load(xs, dys)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(snapshot(), want):
            assert torch.equal(got, ref)
