"""Seeded synthetic inputs shared by the tests, the smoke check and the
benchmark.  This module draws numbers and nothing else: it contains none of
the method's arithmetic and imports neither the oracle nor the HIP library.

Every tensor comes from numpy's Generator(PCG64(seed)), one child stream per
tensor in the order listed, in the paper's logical shapes
([n_b, n_c, m_0..] activations, [n_co, n_ci, k_0..] conv weights,
[n_fo, n_fi] affine weights).
"""
import numpy as np

CONFIGS = {
    # name: description of the workload (shapes are the benchmark's own)
    "cfg1": dict(D=1, n_b=1, c_in=1, c_out=1, in_shape=(64,), P=(4,), ksize=(3,),
                 stride=(1,), padding=(1,), dilation=(1,), seed=0, vec=16, k_workers=4),
    "cfg2": dict(D=2, n_b=8, c_in=16, c_out=16, in_shape=(256, 256), P=(2, 2), ksize=(3, 3),
                 stride=(1, 1), padding=(1, 1), dilation=(1, 1), seed=1),
    "cfg3": dict(n_b=256, n_fi=4096, n_fo=4096, P_fo=2, P_fi=2, seed=2),
    "cfg4": dict(n_b=256, image=(1, 28, 28), classes=10, P=(2, 2), seed=3),
    "cfg5": dict(D=3, n_b=1, c_in=32, c_out=32, in_shape=(256, 256, 256), P=(4, 4, 4),
                 ksize=(5, 5, 5), stride=(2, 2, 2), padding=(2, 2, 2), dilation=(1, 1, 1), seed=4),
    # parity-only variant of cfg5 with uneven partition sizes in every dimension
    "cfg5u": dict(D=3, n_b=1, c_in=32, c_out=32, in_shape=(250, 250, 250), P=(4, 4, 4),
                  ksize=(5, 5, 5), stride=(2, 2, 2), padding=(2, 2, 2), dilation=(1, 1, 1), seed=5),
}


def streams(seed, n):
    """n independent child generators of one seed."""
    return [np.random.Generator(np.random.PCG64(s))
            for s in np.random.SeedSequence(seed).spawn(n)]


def normal(rng, shape, std=1.0, dtype=np.float32):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x.astype(dtype, copy=False)


def uniform(rng, shape, lo, hi, dtype=np.float32):
    return (rng.random(size=shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)).astype(dtype)


def he_normal_std(w_shape):
    fan_in = int(np.prod(w_shape[1:]))
    return float(np.sqrt(2.0 / fan_in))


def xavier_uniform_bound(n_fo, n_fi):
    return float(np.sqrt(6.0 / (n_fo + n_fi)))


def conv_case(cfg, out_shape, **override):
    """x, w, dy (and a small bias) for a sliding-kernel config.  out_shape is
    the global output extent, supplied by the caller (from the oracle's or the
    library's own geometry) and used only to size the cotangent dy.
    Keyword overrides replace config entries (same structure, other extents)."""
    c = dict(cfg)
    c.update(override)
    r = streams(c["seed"], 4)
    out_shape = tuple(out_shape)
    w_shape = (c["c_out"], c["c_in"]) + tuple(c["ksize"])
    return dict(
        cfg=c,
        x=normal(r[0], (c["n_b"], c["c_in"]) + tuple(c["in_shape"])),
        w=normal(r[1], w_shape, std=he_normal_std(w_shape)),
        dy=normal(r[2], (c["n_b"], c["c_out"]) + out_shape),
        bias=normal(r[3], (c["c_out"],), std=0.1),
        out_shape=out_shape)


def vector_case(seed, count, k, G=1):
    """Inputs for broadcast / sum-reduce: G source vectors and G*k replica
    cotangents, all N(0,1)."""
    r = streams(seed, 2)
    return dict(src=[normal(r[0], (count,)) for _ in range(G)],
                reps=[normal(r[1], (count,)) for _ in range(G * k)])


def affine_case(cfg, n_b=None, n_fi=None, n_fo=None):
    c = dict(cfg)
    for key, v in (("n_b", n_b), ("n_fi", n_fi), ("n_fo", n_fo)):
        if v is not None:
            c[key] = v
    r = streams(c["seed"], 4)
    bound = xavier_uniform_bound(c["n_fo"], c["n_fi"])
    return dict(
        cfg=c,
        x=normal(r[0], (c["n_b"], c["n_fi"])),
        W=uniform(r[1], (c["n_fo"], c["n_fi"]), -bound, bound),
        dy=normal(r[2], (c["n_b"], c["n_fo"])),
        b=normal(r[3], (c["n_fo"],), std=0.1))


def to_bf16_values(x):
    """The same draws rounded to the nearest bf16-representable value
    (round-to-nearest-even), returned as fp32."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).to(torch.float32).numpy()


def cnn_case(cfg):
    """Images U(0,1), labels uniform in 0..classes-1 as one-hot targets, and
    the parameters of conv5x5(6)-pool-conv5x5(16)-pool-affine 400-120-84-10:
    conv weights He-normal, affine weights Xavier-uniform, biases zero."""
    c = dict(cfg)
    r = streams(c["seed"], 8)
    n_b = c["n_b"]
    images = uniform(r[0], (n_b,) + tuple(c["image"]), 0.0, 1.0)
    labels = r[1].integers(0, c["classes"], size=n_b)
    target = np.zeros((n_b, c["classes"]), dtype=np.float32)
    target[np.arange(n_b), labels] = 1.0
    shapes = dict(c1=(6, 1, 5, 5), c3=(16, 6, 5, 5))
    params = {}
    for i, (name, shp) in enumerate(shapes.items()):
        params[name + "_w"] = normal(r[2 + i], shp, std=he_normal_std(shp))
        params[name + "_b"] = np.zeros((shp[0],), dtype=np.float32)
    for i, (name, (fo, fi)) in enumerate((("c5", (120, 400)), ("f6", (84, 120)), ("out", (10, 84)))):
        bnd = xavier_uniform_bound(fo, fi)
        params[name + "_w"] = uniform(r[4 + i], (fo, fi), -bnd, bnd)
        params[name + "_b"] = np.zeros((fo,), dtype=np.float32)
    return dict(cfg=c, images=images, labels=labels, target=target, params=params)
