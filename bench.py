#!/usr/bin/env python3
"""Benchmark of the partitioned-convolution hot path on one MI355X.

One step = distdl_conv_fwd (halo exchange H + local convolution) followed by
distdl_conv_bwd (local [dConv]* for dx and dw, sum-reduce of dw over the
workers, adjoint halo exchange H*) on the volumetric configuration:
fp32 [1, 32, 256^3] input, [32, 32, 5, 5, 5] weights, stride 2, padding 2,
4 x 4 x 4 = 64 virtual workers.  Inputs are seeded synthetic N(0,1) tensors
already resident in HBM when the timed region starts.

Prints ONE JSON line (see the keys below).  `--workload cfg2|cfg3` times the
other single-GPU configurations with the same harness.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def _dev_randn(shape, seed, std=1.0, dtype=None):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    t = torch.randn(shape, generator=g, device="cuda", dtype=torch.float32)
    if std != 1.0:
        t *= std
    return t if dtype is None else t.to(dtype)


def _prod(v):
    out = 1
    for t in v:
        out *= int(t)
    return out


class ConvWorkload:
    """cfg5 / cfg2: partitioned convolution forward + backward."""

    def __init__(self, name, dtype="f32"):
        import torch
        import paper_2006_03108_amd as dd
        import synthetic_inputs as syn
        self.dd, self.torch, self.name = dd, torch, name
        self.tag = name if dtype == "f32" else name + "-bf16"
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        c = self.cfg = dict(syn.CONFIGS[name])
        self.plan = dd.distdl_plan_create(c["D"], c["n_b"], c["c_in"], c["c_out"], c["in_shape"], c["P"], c["ksize"],
                                          c["stride"], c["padding"], c["dilation"], tdt)
        P = self.plan.n_workers
        geoms = [self.plan.query(w) for w in range(P)]
        self.out_global = [max(g["out_start"][d] + g["out_size"][d] for g in geoms) for d in range(c["D"])]
        taps = _prod(c["ksize"])
        w_std = syn.he_normal_std((c["c_out"], c["c_in"]) + tuple(c["ksize"]))
        # channels-last device buffers; bulk = N(0,1), halo / pad cells start as noise and are overwritten by H
        self.x = [_dev_randn([c["n_b"]] + g["buf_shape"] + [c["c_in"]], 1000 + w).to(tdt) for w, g in enumerate(geoms)]
        self.dy = [_dev_randn([c["n_b"]] + g["out_size"] + [c["c_out"]], 2000 + w).to(tdt) for w, g in enumerate(geoms)]
        self.y = [torch.empty_like(t) for t in self.dy]
        self.dx = [torch.empty_like(t) for t in self.x]
        self.w = _dev_randn((c["c_out"], c["c_in"]) + tuple(c["ksize"]), 7, std=w_std).to(tdt)
        self.dw = torch.empty_like(self.w)
        self.ws = torch.empty(max(dd.distdl_conv_bwd_workspace(self.plan), 16), dtype=torch.uint8, device="cuda")
        stats = dd.distdl_plan_stats(self.plan)
        esz = 4 if dtype == "f32" else 2
        per_cell = c["n_b"] * c["c_in"] * esz
        self.flops_fwd = 2.0 * c["n_b"] * c["c_out"] * c["c_in"] * taps * _prod(self.out_global)
        self.flops_step = 3.0 * self.flops_fwd
        nw = taps * c["c_in"] * c["c_out"]
        self.alg = {   # algorithmic bytes or flops per launch, by kernel-name prefix
            "halo_fwd": ("hbm", (2 * stats["halo_cells"] + stats["pad_cells"]) * per_cell),
            "halo_adj": ("hbm", (2 * stats["halo_cells"] + 2 * stats["band_cells"] + stats["pad_cells"]) * per_cell),
            "conv_fwd": ("mfma", self.flops_fwd),
            # launched once per stride-parity class; the classes share the layer's flops
            "conv_bwd_data_mfma": ("mfma", self.flops_fwd / _prod(c["stride"])),
            "conv_bwd_data": ("mfma", self.flops_fwd),
            "conv_bwd_weight": ("mfma", self.flops_fwd),
            "conv_reduce_dw": ("hbm", None),     # filled from the workspace geometry below
            "conv_relayout_w": ("hbm", 2 * nw * esz),
        }
        self.nw = nw
        # least bytes each contraction must move (operands once, results once): for the second roofline
        # min(MFMA peak, arithmetic intensity x HBM peak)
        xb = sum(t.numel() for t in self.x) * esz
        yb = sum(t.numel() for t in self.dy) * esz
        self.min_bytes = {"conv_fwd": xb + yb + nw * esz,
                          # a parity class reads all of dy and writes its share of dx^
                          "conv_bwd_data_mfma": yb + (xb + nw * esz) / _prod(c["stride"]),
                          "conv_bwd_data": xb + yb + nw * esz,
                          "conv_bwd_weight": xb + yb + nw * 4}
        self.metric = ("partitioned conv fwd+bwd TFLOP/s (halo exchange H, H* and dw sum-reduce included); "
                       "halo+bcast+sumreduce fwd/adj GB/s and fraction of HBM peak under movement_* and <kernel>_GBs")
        self.unit = "TFLOP/s"
        # arithmetic types: fp32 throughout for fp32 tensors; bf16 tensors are multiplied in bf16 with fp32
        # accumulation when the channel counts are multiples of 8, else widened to fp32
        self.dtype = "f32" if dtype == "f32" else "bf16"
        self.storage = dtype
        self.kernel_dtype = {}
        if dtype == "bf16":
            self.kernel_dtype = {"conv_fwd": "bf16" if c["c_in"] % 8 == 0 else "f32",
                                 "conv_bwd_data_mfma": "bf16" if c["c_out"] % 8 == 0 else "f32",
                                 "conv_bwd_data": "f32",
                                 "conv_bwd_weight": "bf16" if c["c_in"] % 8 == 0 and c["c_out"] % 8 == 0 else "f32"}
        self.describe = {"workload": f"{self.tag}: conv{c['D']}d fwd+bwd {'fp32' if dtype == 'f32' else 'bf16 (fp32 accumulation)'} x[{c['n_b']},{c['c_in']}," +
                         ",".join(str(v) for v in c["in_shape"]) + f"] w[{c['c_out']},{c['c_in']}," +
                         ",".join(str(v) for v in c["ksize"]) + f"] stride {c['stride'][0]} pad {c['padding'][0]}, " +
                         "P=" + "x".join(str(v) for v in c["P"]) + f" ({P} virtual workers); tensors resident in HBM "
                         "in the library's channels-last layout (a caller holding the paper's planes-first order "
                         "converts with distdl_layout_convert, rate under layout_*_GBs; not part of the timed step)",
                         "halo_cells": stats["halo_cells"], "pad_cells": stats["pad_cells"],
                         "band_cells": stats["band_cells"]}

    def step(self):
        dd = self.dd
        dd.distdl_conv_fwd(self.plan, self.x, self.w, None, self.y)
        dd.distdl_conv_bwd(self.plan, self.x, self.w, self.dy, self.dx, self.dw, None, self.ws)

    def value(self, seconds_per_step):
        return self.flops_step / seconds_per_step / 1e12

    def cpu_baseline(self):
        """The oracle's distributed conv forward + adjoint on a bounded sample of the same workload: the same
        channels, kernel and stride on a 96^3 (cfg5) or 256^2, batch 4 (cfg2) input over 2 workers per dimension.
        The steps are the oracle's own functions in the order of its dist_conv_forward / dist_conv_adjoint (H, B w,
        Conv per worker, [dConv]* per worker, R dw, R db, H*); the per-worker steps, which are independent, run on a
        pool of host threads (numpy releases the interpreter lock inside them), one per virtual worker."""
        import os
        from concurrent.futures import ThreadPoolExecutor
        import synthetic_inputs as syn
        from oracle import geometry as geo, layers, primitives as prim
        c = dict(self.cfg)
        if c["D"] == 3:
            c.update(in_shape=(96, 96, 96), P=(2, 2, 2))
        else:
            c.update(in_shape=(256, 256), n_b=4)
        part = geo.Partition.for_kernel(c["in_shape"], c["P"], c["ksize"], c["stride"], c["padding"], c["dilation"])
        case = syn.conv_case(c, part.global_out_shape())
        P = part.n_workers
        threads = max(1, min(P, os.cpu_count() or 1, 16))
        origin = [[part.g(wk, d)["origin"] for d in range(part.D)] for wk in range(P)]
        t0 = time.perf_counter()
        bufs = prim.scatter_bulk(case["x"].astype(np.float64), part)
        dy = prim.scatter_out(case["dy"], part)
        prim.halo_exchange(bufs, part)
        w_hat = prim.broadcast(np.asarray(case["w"], dtype=np.float64), P)
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(lambda wk: layers.conv_valid(bufs[wk], w_hat[wk], None, part.out_shape(wk), c["stride"],
                                                       c["dilation"], origin[wk]), range(P)))
            back = list(pool.map(lambda wk: layers.conv_valid_adjoint(bufs[wk], w_hat[wk], dy[wk], c["stride"],
                                                                      c["dilation"], origin[wk], True), range(P)))
        prim.sum_reduce([b[1] for b in back])
        prim.sum_reduce([b[2] for b in back])
        prim.halo_exchange_adjoint([b[0] for b in back], part)
        dt = time.perf_counter() - t0
        flops = 3 * 2.0 * c["n_b"] * c["c_out"] * c["c_in"] * _prod(c["ksize"]) * _prod(part.global_out_shape())
        return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
                "sample": f"oracle H, Conv, [dConv]*, R dw, R db, H* (numpy fp64, {threads} threads: one per virtual "
                          f"worker) on x[{c['n_b']},{c['c_in']}," + ",".join(str(v) for v in c["in_shape"]) + "], P=" +
                          "x".join(str(v) for v in c["P"]) + f", {flops / 1e9:.2f} GFLOP in {dt:.1f} s"}


class AffineWorkload:
    """cfg3: distributed affine forward + backward (fp32 or bf16)."""

    def __init__(self, name, dtype):
        import torch
        import paper_2006_03108_amd as dd
        import synthetic_inputs as syn
        self.dd, self.torch = dd, torch
        self.tag = "cfg3" if dtype == "f32" else "cfg3-bf16"
        c = self.cfg = dict(syn.CONFIGS["cfg3"])
        td = torch.float32 if dtype == "f32" else torch.bfloat16
        self.plan = dd.distdl_affine_plan_create(c["n_b"], c["n_fi"], c["n_fo"], c["P_fo"], c["P_fi"], td)
        fo, fi = c["n_fo"] // c["P_fo"], c["n_fi"] // c["P_fi"]
        bound = syn.xavier_uniform_bound(c["n_fo"], c["n_fi"])
        self.x = [_dev_randn((c["n_b"], fi), 10 + j, dtype=td) for j in range(c["P_fi"])]
        self.W = [((torch.rand((fo, fi), device="cuda", generator=torch.Generator(device="cuda").manual_seed(20 + k))
                    * 2 - 1) * bound).to(td) for k in range(c["P_fo"] * c["P_fi"])]
        self.b = [torch.zeros(fo, device="cuda", dtype=td) for _ in range(c["P_fo"])]
        self.dy = [_dev_randn((c["n_b"], fo), 30 + i, dtype=td) for i in range(c["P_fo"])]
        self.y = [torch.empty_like(t) for t in self.dy]
        self.dx = [torch.empty_like(t) for t in self.x]
        self.dW = [torch.empty_like(t) for t in self.W]
        self.db = [torch.empty_like(t) for t in self.b]
        self.flops_fwd = 2.0 * c["n_b"] * c["n_fi"] * c["n_fo"]
        self.flops_step = 3.0 * self.flops_fwd
        esz = 4 if dtype == "f32" else 2
        self.alg = {"affine_fwd": ("mfma", self.flops_fwd), "affine_bwd_x": ("mfma", self.flops_fwd),
                    "affine_bwd_w": ("mfma", self.flops_fwd), "affine_bwd_direct": ("mfma", 2 * self.flops_fwd),
                    "affine_bias_grad": ("hbm", (c["n_b"] + 1) * c["n_fo"] * esz)}
        # bytes every kernel must at least move (operands once, result once): the HBM side of the roofline
        self.min_bytes = {"affine_fwd": (c["n_fi"] * c["n_fo"] + c["n_b"] * (c["n_fi"] + c["n_fo"])) * esz,
                          "affine_bwd_x": (c["n_fi"] * c["n_fo"] + c["n_b"] * (c["n_fi"] + c["n_fo"])) * esz,
                          "affine_bwd_w": (c["n_fi"] * c["n_fo"] + c["n_b"] * (c["n_fi"] + c["n_fo"])) * esz}
        self.metric = "distributed affine fwd+bwd TFLOP/s (broadcast of x, sum-reduce over P_fi included)"
        self.unit = "TFLOP/s"
        self.dtype = dtype
        self.describe = {"workload": f"cfg3: affine fwd+bwd {dtype} x[{c['n_b']},{c['n_fi']}] W[{c['n_fo']},{c['n_fi']}]"
                                     f" on a {c['P_fo']}x{c['P_fi']} weight partition"}

    def step(self):
        self.dd.distdl_affine_fwd(self.plan, self.x, self.W, self.b, self.y)
        self.dd.distdl_affine_bwd(self.plan, self.x, self.W, self.dy, self.dx, self.dW, self.db)

    def value(self, seconds_per_step):
        return self.flops_step / seconds_per_step / 1e12

    def cpu_baseline(self):
        import synthetic_inputs as syn
        from oracle import layers
        c = self.cfg
        case = syn.affine_case(c)
        rows, cols = layers.feature_blocks(c["n_fo"], c["P_fo"]), layers.feature_blocks(c["n_fi"], c["P_fi"])
        x_parts = [case["x"][:, s] for s in cols]
        W_parts = [[case["W"][r][:, s] for s in cols] for r in rows]
        t0 = time.perf_counter()
        layers.dist_affine_forward(x_parts, W_parts, [case["b"][r] for r in rows], c["P_fo"], c["P_fi"])
        layers.dist_affine_adjoint(x_parts, W_parts, [case["dy"][:, r] for r in rows], c["P_fo"], c["P_fi"])
        dt = time.perf_counter() - t0
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
        return {"value": self.flops_step / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                "sample": f"oracle dist_affine_forward+dist_affine_adjoint (numpy fp64 matmul) on the full cfg3 "
                          f"shapes, {self.flops_step / 1e9:.1f} GFLOP in {dt:.1f} s"}


class MovementWorkload:
    """The data-movement primitives alone: H and H* on the cfg5 geometry (fp32, 32 channels, 4 x 4 x 4 workers,
    buffers of 4.9 GB, far beyond the 256 MB cache) and B, B*, R, R* over k = 4 replicas of 256 MiB with two
    rotating sets of arrays.  value = algorithmic bytes of the six calls / time."""

    K, COUNT, SETS = 4, 1 << 26, 2

    def __init__(self, sweep):
        import torch
        import paper_2006_03108_amd as dd
        import synthetic_inputs as syn
        self.dd, self.torch, self.tag, self.sweep_on = dd, torch, "movement", sweep
        c = self.cfg = dict(syn.CONFIGS["cfg5"])
        self.plan = dd.distdl_plan_create(c["D"], c["n_b"], c["c_in"], c["c_out"], c["in_shape"], c["P"], c["ksize"],
                                          c["stride"], c["padding"], c["dilation"])
        geoms = [self.plan.query(w) for w in range(self.plan.n_workers)]
        self.x = [_dev_randn([c["n_b"]] + g["buf_shape"] + [c["c_in"]], 1000 + w) for w, g in enumerate(geoms)]
        self.g = [_dev_randn([c["n_b"]] + g["buf_shape"] + [c["c_in"]], 3000 + w) for w, g in enumerate(geoms)]
        k, n = self.K, self.COUNT
        self.one = [_dev_randn((n,), 50 + s) for s in range(self.SETS)]
        self.many = [[_dev_randn((n,), 60 + 10 * s + i) for i in range(k)] for s in range(self.SETS)]
        self.turn = 0
        stats = dd.distdl_plan_stats(self.plan)
        per_cell = c["n_b"] * c["c_in"] * 4
        coll = (k + 1) * n * 4
        self.alg = {
            "halo_fwd": ("hbm", (2 * stats["halo_cells"] + stats["pad_cells"]) * per_cell),
            "halo_adj": ("hbm", (2 * stats["halo_cells"] + 2 * stats["band_cells"] + stats["pad_cells"]) * per_cell),
            "bcast": ("hbm", coll), "sumreduce": ("hbm", coll),
        }
        # planes-first <-> channels-last conversion of the same buffers (for callers that hold the paper's logical
        # order): reads and writes every buffer once; timed on its own, not part of the step
        buf_bytes = sum(t.numel() for t in self.x) * 4
        self.alg["layout_to_cl"] = self.alg["layout_from_cl"] = ("hbm", 2 * buf_bytes)
        self.bytes_step = self.alg["halo_fwd"][1] + self.alg["halo_adj"][1] + 4 * coll
        self.metric = "halo + broadcast + sum-reduce forward and adjoint GB/s (algorithmic bytes)"
        self.unit = "GB/s"
        self.dtype = "f32"
        self.describe = {"workload": "movement: H, H* on the cfg5 geometry (fp32 [1,32,256^3], P=4x4x4, halo 2/1, "
                                     f"pad 2/1) + B, B*, R, R* over k={k} replicas of {n * 4 >> 20} MiB, channels-last",
                         "halo_cells": stats["halo_cells"], "pad_cells": stats["pad_cells"],
                         "band_cells": stats["band_cells"]}

    def step(self):
        dd, s = self.dd, self.turn % self.SETS
        self.turn += 1
        dd.distdl_bcast_fwd([self.one[s]], self.many[s], self.K)
        dd.distdl_bcast_adj([self.one[s]], self.many[s], self.K, False)
        dd.distdl_halo_fwd(self.plan, self.x)
        dd.distdl_sumreduce_adj([self.one[s]], self.many[s], self.K)
        dd.distdl_sumreduce_fwd(self.many[s], [self.one[s]], self.K, False)
        dd.distdl_halo_adj(self.plan, self.g)

    def value(self, seconds_per_step):
        return self.bytes_step / seconds_per_step / 1e9

    def layout_rates(self):
        """distdl_layout_convert on the 64 padded buffers of this geometry, both directions (4.9 GB in, 4.9 GB
        out per call), kernel time from the library's HIP events."""
        dd, torch = self.dd, self.torch
        other = [torch.empty_like(t) for t in self.x]
        out = {}
        dd.distdl_profile_enable(True)
        for name, to_cl, src, dst in (("layout_to_cl", True, other, self.x), ("layout_from_cl", False, self.x, other)):
            for _ in range(2):
                dd.distdl_layout_convert(self.plan, 0, to_cl, src, dst)
            torch.cuda.synchronize()
            dd.distdl_profile_report()
            for _ in range(5):
                dd.distdl_layout_convert(self.plan, 0, to_cl, src, dst)
            rep = dd.distdl_profile_report()
            ms = sum(v[1] for v in rep.values()) / 5
            nbytes = self.alg[name][1]
            out[name] = {"avg_ms": ms, "algorithmic_bytes": nbytes, "achieved": nbytes / (ms * 1e-3) / 1e9,
                         "unit": "GB/s", "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        dd.distdl_profile_enable(False)
        return out

    def achievable_copy(self):
        """What a plain device-to-device copy reaches on this chip (the practical ceiling of any streaming kernel):
        2 GiB read + 2 GiB written, by the library's plain copy kernel (distdl_copy_ref) and by torch's copy_, median
        of 9 timed with events on the launch stream."""
        torch, dd = self.torch, self.dd
        n = 1 << 29                                    # fp32 elements: 2 GiB
        src = torch.empty(n, device="cuda").normal_()
        dst = torch.empty_like(src)
        out = {"bytes_moved": 2 * n * 4}
        for name, call in (("library_copy", lambda: dd.distdl_copy_ref(src, dst)),
                           ("torch_copy", lambda: dst.copy_(src))):
            times = []
            for _ in range(11):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                call()
                e1.record()
                e1.synchronize()
                times.append(e0.elapsed_time(e1))
            ms = sorted(times[2:])[len(times[2:]) // 2]
            out[name + "_GBs"] = 2 * n * 4 / (ms * 1e-3) / 1e9
        out["best_GBs"] = max(out["library_copy_GBs"], out["torch_copy_GBs"])
        out["frac_hbm_peak"] = out["best_GBs"] / HBM_PEAK_GBS
        return out

    def sweep(self):
        """B and R over k in {2, 4, 64} replicas of 1 MiB .. 1 GiB (fp32), array sets rotated through a pool of
        20 GiB so that no call finds its operands in the cache; kernel time from the library's HIP events."""
        dd, torch = self.dd, self.torch
        pool = torch.empty(5 << 30, dtype=torch.float32, device="cuda")
        pool.normal_()
        dd.distdl_profile_enable(True)
        rows = []
        for k in (2, 4, 64):
            for mib in (1, 4, 16, 64, 256, 1024):
                n = mib << 18
                per_set = (k + 1) * n
                if per_set > pool.numel():
                    continue
                nsets = min(pool.numel() // per_set, max(2, (1 << 30) // (per_set * 4) + 1), 16)
                sets = [[pool[(s * (k + 1) + i) * n:(s * (k + 1) + i + 1) * n] for i in range(k + 1)]
                        for s in range(nsets)]
                reps = max(nsets, 8)
                for direction in ("bcast", "sumreduce"):
                    torch.cuda.synchronize()
                    dd.distdl_profile_report()
                    for r in range(reps):
                        a = sets[r % nsets]
                        if direction == "bcast":
                            dd.distdl_bcast_fwd([a[0]], a[1:], k)
                        else:
                            dd.distdl_sumreduce_fwd(a[1:], [a[0]], k, False)
                    rep = dd.distdl_profile_report()
                    ms = sum(v[1] for v in rep.values()) / reps
                    gbs = per_set * 4 / (ms * 1e-3) / 1e9
                    rows.append({"op": direction, "k": k, "MiB_per_replica": mib, "ms": round(ms, 5),
                                 "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 3),
                                 "cache_resident": per_set * 4 * nsets <= (256 << 20)})
        del pool, sets
        torch.cuda.empty_cache()

        def timed(name, call, nbytes, reps=6, extra=None):
            for _ in range(2):
                call()
            torch.cuda.synchronize()
            dd.distdl_profile_report()
            for _ in range(reps):
                call()
            rep = dd.distdl_profile_report()
            ms = sum(v[1] for v in rep.values()) / reps
            row = {"op": name, "ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                   "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 3), "algorithmic_bytes": nbytes,
                   "kernels": {k: round(v[1] / reps, 5) for k, v in rep.items()}}
            row.update(extra or {})
            rows.append(row)

        # the halo kernels on the same volume cut along two dimensions only (4 x 4 x 1 workers): every face is made
        # of whole 32 KB rows, none of 128-256 byte pieces -- what the kernels reach when the access pattern is benign
        c = self.cfg
        hp = dd.distdl_plan_create(3, 1, c["c_in"], c["c_in"], c["in_shape"], (4, 4, 1), c["ksize"], c["stride"],
                                   c["padding"], c["dilation"])
        hg = [hp.query(w) for w in range(hp.n_workers)]
        hb = [_dev_randn([1] + g["buf_shape"] + [c["c_in"]], 300 + w) for w, g in enumerate(hg)]
        hst = dd.distdl_plan_stats(hp)
        cell = c["c_in"] * 4
        timed("halo_fwd_rows_only", lambda: dd.distdl_halo_fwd(hp, hb), (2 * hst["halo_cells"] + hst["pad_cells"]) * cell,
              extra={"P": [4, 4, 1]})
        timed("halo_adj_rows_only", lambda: dd.distdl_halo_adj(hp, hb),
              (2 * hst["halo_cells"] + 2 * hst["band_cells"] + hst["pad_cells"]) * cell, extra={"P": [4, 4, 1]})
        del hb, hp
        # all-reduce A = B R in place over k = 4 replicas of 256 MiB: k reads + k writes
        reps4 = [_dev_randn((1 << 26,), 70 + i) for i in range(4)]
        timed("allreduce", lambda: dd.distdl_allreduce(reps4, 4), 2 * 4 * (1 << 28), extra={"k": 4, "MiB_per_replica": 256})
        del reps4
        # generalized all-to-all of a 1 GiB tensor: spatial 4 x 4 blocks -> (batch, channel) 4 x 4 blocks
        shape = (32, 32, 512, 512)
        rp = dd.distdl_repart_plan_create(shape, (1, 1, 4, 4), (4, 4, 1, 1))
        src = [_dev_randn(sz, 80 + w) for w, (_, sz) in enumerate(rp.blocks(0))]
        dst = [torch.empty(sz, device="cuda") for (_, sz) in rp.blocks(1)]
        timed("repart_fwd", lambda: dd.distdl_repart_fwd(rp, src, dst), 2 * 4 * _prod(shape), extra={"shape": list(shape)})
        timed("repart_adj", lambda: dd.distdl_repart_adj(rp, dst, src), 2 * 4 * _prod(shape), extra={"shape": list(shape)})
        del src, dst
        # pooling 2^3 / stride 2 on the volumetric input, 4 x 4 x 4 workers (no halos: reads the input, writes 1/8)
        c = self.cfg
        pp = dd.distdl_plan_create(3, 1, c["c_in"], c["c_in"], c["in_shape"], c["P"], (2, 2, 2), (2, 2, 2), (0, 0, 0), (1, 1, 1))
        geoms = [pp.query(w) for w in range(pp.n_workers)]
        px = [_dev_randn([1] + g["buf_shape"] + [c["c_in"]], 90 + w) for w, g in enumerate(geoms)]
        py = [torch.empty([1] + g["out_size"] + [c["c_in"]], device="cuda") for g in geoms]
        pdx = [torch.empty_like(t) for t in px]
        n_in = sum(t.numel() for t in px) * 4
        n_out = sum(t.numel() for t in py) * 4
        timed("maxpool_fwd", lambda: dd.distdl_maxpool_fwd(pp, px, py), n_in + n_out)
        timed("avgpool_fwd", lambda: dd.distdl_avgpool_fwd(pp, px, py), n_in + n_out)
        timed("maxpool_bwd", lambda: dd.distdl_maxpool_bwd(pp, px, py, pdx), 2 * n_in + n_out)
        timed("avgpool_bwd", lambda: dd.distdl_avgpool_bwd(pp, py, pdx), n_in + n_out)
        del px, py, pdx
        # channel-partitioned convolution: 64 -> 64 channels as 2 x 2 blocks of 32, 5^3 / stride 2 on 128^3 over
        # 2 x 2 x 2 spatial workers (every block is the cfg5 per-worker contraction); reported in TFLOP/s
        cp_shape, cp_P, cc = (128, 128, 128), (2, 2, 2), 64
        cp = dd.distdl_convcp_plan_create(3, 1, cc, cc, cp_shape, cp_P, 2, 2, c["ksize"], c["stride"], c["padding"],
                                          c["dilation"])
        S = cp.S
        g0 = [cp.block_plan(0, 0).query(w) for w in range(S)]
        cx = [_dev_randn([1] + g["buf_shape"] + [32], 200 + i) for i in range(2) for g in g0]
        cw = [_dev_randn((32, 32) + tuple(c["ksize"]), 210 + i) * 0.02 for i in range(4)]
        cb = [_dev_randn((32,), 220 + i) for i in range(2)]
        cy = [torch.empty([1] + g["out_size"] + [32], device="cuda") for i in range(2) for g in g0]
        cdy = [_dev_randn(list(t.shape), 230 + i) for i, t in enumerate(cy)]
        cdx = [torch.empty_like(t) for t in cx]
        cdw = [torch.empty_like(t) for t in cw]
        cdb = [torch.empty_like(t) for t in cb]
        out_cells = sum(_prod(g["out_size"]) for g in g0)
        fl = 2 * out_cells * cc * cc * _prod(c["ksize"])
        for name, call, nfl in (("convcp_fwd", lambda: dd.distdl_convcp_fwd(cp, cx, cw, cb, cy), fl),
                                ("convcp_bwd", lambda: dd.distdl_convcp_bwd(cp, cx, cw, cdy, cdx, cdw, cdb), 2 * fl)):
            timed(name, call, 0, reps=3)
            row = rows[-1]
            row.update({"TFLOP/s": round(nfl / (row["ms"] * 1e-3) / 1e12, 1), "algorithmic_flops": nfl,
                        "frac_mfma_peak": round(nfl / (row["ms"] * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS["f32"], 3),
                        "config": "64->64 channels, P_co x P_ci = 2 x 2, 128^3 over 2x2x2 workers, 5^3 stride 2"})
            for key in ("GB/s", "frac_hbm_peak", "algorithmic_bytes"):
                row.pop(key)
        dd.distdl_profile_enable(False)
        return rows

    def cpu_baseline(self):
        """The oracle's nested halo exchange and adjoint plus broadcast / sum-reduce and adjoints on a bounded
        sample: 32 channels on a 192^3 volume over 2 x 2 x 2 workers, k = 4 replicas of 32 Mi elements."""
        import synthetic_inputs as syn
        from oracle import geometry as geo, primitives as prim
        c = dict(self.cfg)
        c.update(in_shape=(192, 192, 192), P=(2, 2, 2))
        part = geo.Partition.for_kernel(c["in_shape"], c["P"], c["ksize"], c["stride"], c["padding"], c["dilation"])
        r = syn.streams(11, 3)
        x = syn.normal(r[0], (c["n_b"], c["c_in"]) + tuple(c["in_shape"])).astype(np.float64)
        bufs = prim.scatter_bulk(x, part)
        gb = [syn.normal(r[1], b.shape).astype(np.float64) for b in bufs]
        v = syn.normal(r[2], (1 << 25,)).astype(np.float64)
        halo = pad = 0
        for w in range(part.n_workers):
            g = [part.g(w, d) for d in range(part.D)]
            inner = _prod(d["halo"][0] + d["in_size"] + d["halo"][1] for d in g)
            halo += inner - _prod(d["in_size"] for d in g)
            pad += _prod(part.buf_shape(w)) - inner
        t0 = time.perf_counter()
        prim.halo_exchange(bufs, part)
        prim.halo_exchange_adjoint(gb, part)
        reps = prim.broadcast(v, self.K)
        prim.broadcast_adjoint(reps)
        prim.sum_reduce(reps)
        prim.sum_reduce_adjoint(v, self.K)
        dt = time.perf_counter() - t0
        per_cell = c["n_b"] * c["c_in"] * 8
        moved = (4 * halo + 2 * pad) * per_cell + 4 * (self.K + 1) * v.size * 8
        return {"value": moved / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                "sample": f"oracle halo_exchange + halo_exchange_adjoint (nested form, numpy fp64) on x[1,32,192,192,192], "
                          f"P=2x2x2, and broadcast / sum_reduce and adjoints over k={self.K} replicas of 32 Mi fp64 "
                          f"elements; {moved / 1e6:.0f} MB (fp64; the band term of H* counted as halo) in {dt:.2f} s"}


class SmallCnn:
    """cfg4: conv5x5(6)-ReLU-pool2-conv5x5(16)-ReLU-pool2-affine 400-120-84-10 (ReLU after the first two affine
    layers), MSE loss; conv / pool layers on a 2 x 2 spatial partition, affine layers on 2 x 2 weight partitions.
    Every step is a call of the library; this class only owns the device tensors and the order of the calls.
    `params`: the numpy weights (c1_w, c1_b, c3_w, c3_b, c5_w, c5_b, f6_w, f6_b, out_w, out_b)."""

    P, PF = (2, 2), 2

    def __init__(self, n_b, params):
        import torch
        import paper_2006_03108_amd as dd
        self.dd, self.torch, self.n_b = dd, torch, n_b
        one = (1, 1)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        new = lambda shapes: [torch.empty(s, device="cuda") for s in shapes]
        like = lambda ts: [torch.empty_like(t) for t in ts]

        def sliding(c_in, c_out, in_shape, k, stride, pad):
            plan = dd.distdl_plan_create(2, n_b, c_in, c_out, in_shape, self.P, (k, k), (stride, stride), (pad, pad), one)
            geoms = [plan.query(w) for w in range(plan.n_workers)]
            x = [torch.zeros([n_b] + g["buf_shape"] + [c_in], device="cuda") for g in geoms]
            y = [torch.empty([n_b] + g["out_size"] + [c_out], device="cuda") for g in geoms]
            return plan, x, y, like(x)

        self.c1, self.c1_x, self.c1_y, self.c1_dx = sliding(1, 6, (28, 28), 5, 1, 2)
        self.p2, self.p2_x, self.p2_y, self.p2_dx = sliding(6, 6, (28, 28), 2, 2, 0)
        self.c3, self.c3_x, self.c3_y, self.c3_dx = sliding(6, 16, (14, 14), 5, 1, 0)
        self.p4, self.p4_x, self.p4_y, self.p4_dx = sliding(16, 16, (10, 10), 2, 2, 0)
        self.c1_ws = torch.empty(max(dd.distdl_conv_bwd_workspace(self.c1), 16), dtype=torch.uint8, device="cuda")
        self.c3_ws = torch.empty(max(dd.distdl_conv_bwd_workspace(self.c3), 16), dtype=torch.uint8, device="cuda")
        # conv weights in the library's [c_out][c_in][taps] order == the usual [c_out, c_in, k, k], contiguous
        self.w1, self.b1, self.w3, self.b3 = dev(params["c1_w"]), dev(params["c1_b"]), dev(params["c3_w"]), dev(params["c3_b"])
        self.dw1, self.db1, self.dw3, self.db3 = (torch.empty_like(t) for t in (self.w1, self.b1, self.w3, self.b3))

        def split(n, parts):
            out, at = [], 0
            for r in range(parts):
                z = n // parts + (1 if r < n % parts else 0)
                out.append(slice(at, at + z))
                at += z
            return out

        def affine(W, b):
            n_fo, n_fi = W.shape
            rows, cols = split(n_fo, self.PF), split(n_fi, self.PF)
            plan = dd.distdl_affine_plan_create(n_b, n_fi, n_fo, self.PF, self.PF)
            Wp = [dev(W[r][:, c]) for r in rows for c in cols]
            bp = [dev(b[r]) for r in rows]
            y = new([(n_b, r.stop - r.start) for r in rows])
            return dict(plan=plan, W=Wp, b=bp, y=y, dW=like(Wp), db=like(bp), rows=rows, cols=cols)

        self.a5 = affine(params["c5_w"], params["c5_b"])
        self.a6 = affine(params["f6_w"], params["f6_b"])
        self.ao = affine(params["out_w"], params["out_b"])
        self.r1, self.r3 = like(self.c1_y), like(self.c3_y)
        self.f = new([(n_b, c.stop - c.start) for c in self.a5["cols"]])
        self.r5, self.r6 = like(self.a5["y"]), like(self.a6["y"])
        self.t = like(self.ao["y"])
        self.d_out, self.d_r6, self.d_a6, self.d_r5, self.d_a5 = (like(self.ao["y"]), like(self.r6), like(self.a6["y"]),
                                                                 like(self.r5), like(self.a5["y"]))
        self.d_f, self.d_s4, self.d_r3, self.d_a3 = like(self.f), like(self.p4_y), like(self.r3), like(self.c3_y)
        self.d_s2, self.d_r1, self.d_a1 = like(self.p2_y), like(self.r1), like(self.c1_y)
        self.loss = torch.zeros(1, dtype=torch.float64, device="cuda")

    def load_batch(self, image_bufs, target):
        """image_bufs: per worker the channels-last padded buffer [n_b, buf_0, buf_1, 1] of conv1 with the bulk
        filled; target: [n_b, 10] one-hot."""
        for dst, src in zip(self.c1_x, image_bufs):
            dst.copy_(src)
        for dst, rows in zip(self.t, self.ao["rows"]):
            dst.copy_(self.torch.from_numpy(np.ascontiguousarray(target[:, rows], dtype=np.float32)))

    def step(self):
        dd = self.dd
        a5, a6, ao = self.a5, self.a6, self.ao
        # forward
        dd.distdl_conv_fwd(self.c1, self.c1_x, self.w1, self.b1, self.c1_y)
        dd.distdl_relu_fwd(self.c1_y, self.r1)
        dd.distdl_bulk_copy(self.p2, self.r1, self.p2_x, True)
        dd.distdl_maxpool_fwd(self.p2, self.p2_x, self.p2_y)
        dd.distdl_bulk_copy(self.c3, self.p2_y, self.c3_x, True)
        dd.distdl_conv_fwd(self.c3, self.c3_x, self.w3, self.b3, self.c3_y)
        dd.distdl_relu_fwd(self.c3_y, self.r3)
        dd.distdl_bulk_copy(self.p4, self.r3, self.p4_x, True)
        dd.distdl_maxpool_fwd(self.p4, self.p4_x, self.p4_y)
        dd.distdl_repartition_fwd(self.p4, self.p4_y, self.f)
        dd.distdl_affine_fwd(a5["plan"], self.f, a5["W"], a5["b"], a5["y"])
        dd.distdl_relu_fwd(a5["y"], self.r5)
        dd.distdl_affine_fwd(a6["plan"], self.r5, a6["W"], a6["b"], a6["y"])
        dd.distdl_relu_fwd(a6["y"], self.r6)
        dd.distdl_affine_fwd(ao["plan"], self.r6, ao["W"], ao["b"], ao["y"])
        dd.distdl_mse_fwd_bwd(ao["y"], self.t, self.d_out, self.loss)
        # backward
        dd.distdl_affine_bwd(ao["plan"], self.r6, ao["W"], self.d_out, self.d_r6, ao["dW"], ao["db"])
        dd.distdl_relu_bwd(a6["y"], self.d_r6, self.d_a6)
        dd.distdl_affine_bwd(a6["plan"], self.r5, a6["W"], self.d_a6, self.d_r5, a6["dW"], a6["db"])
        dd.distdl_relu_bwd(a5["y"], self.d_r5, self.d_a5)
        dd.distdl_affine_bwd(a5["plan"], self.f, a5["W"], self.d_a5, self.d_f, a5["dW"], a5["db"])
        dd.distdl_repartition_adj(self.p4, self.d_f, self.d_s4)
        dd.distdl_maxpool_bwd(self.p4, self.p4_x, self.d_s4, self.p4_dx)
        dd.distdl_bulk_copy(self.p4, self.d_r3, self.p4_dx, False)
        dd.distdl_relu_bwd(self.c3_y, self.d_r3, self.d_a3)
        dd.distdl_conv_bwd(self.c3, self.c3_x, self.w3, self.d_a3, self.c3_dx, self.dw3, self.db3, self.c3_ws)
        dd.distdl_bulk_copy(self.c3, self.d_s2, self.c3_dx, False)
        dd.distdl_maxpool_bwd(self.p2, self.p2_x, self.d_s2, self.p2_dx)
        dd.distdl_bulk_copy(self.p2, self.d_r1, self.p2_dx, False)
        dd.distdl_relu_bwd(self.c1_y, self.d_r1, self.d_a1)
        dd.distdl_conv_bwd(self.c1, self.c1_x, self.w1, self.d_a1, self.c1_dx, self.dw1, self.db1, self.c1_ws)


class SmallCnnWorkload:
    """cfg4 end to end: one forward + backward step of the small CNN on batch 256; launch-latency bound, so the
    figure is the step time and the number of kernel launches, not a roofline fraction."""

    def __init__(self):
        import torch
        import paper_2006_03108_amd as dd
        import synthetic_inputs as syn
        self.dd, self.torch, self.tag = dd, torch, "cfg4"
        self.case = syn.cnn_case(syn.CONFIGS["cfg4"])
        n_b = self.case["images"].shape[0]
        self.net = SmallCnn(n_b, self.case["params"])
        geoms = [self.net.c1.query(w) for w in range(4)]
        bufs = []
        img = torch.from_numpy(self.case["images"]).cuda()           # [n_b, 1, 28, 28]
        for g in geoms:
            b = torch.zeros([n_b] + g["buf_shape"] + [1], device="cuda")
            sl = [slice(g["in_start"][d], g["in_start"][d] + g["in_size"][d]) for d in range(2)]
            o = g["bulk_off"]
            b[:, o[0]:o[0] + g["in_size"][0], o[1]:o[1] + g["in_size"][1], 0] = img[:, 0, sl[0], sl[1]]
            bufs.append(b)
        self.net.load_batch(bufs, self.case["target"])
        self.alg = {}
        self.flops_step = 3 * 2.0 * n_b * (6 * 25 * 28 * 28 + 16 * 6 * 25 * 10 * 10 + 400 * 120 + 120 * 84 + 84 * 10)
        self.metric = "small CNN forward + backward step time (launch-latency bound)"
        self.unit = "us/step"
        self.dtype = "f32"
        self.higher_is_better = False
        self.describe = {"workload": f"cfg4: conv5x5(6)-pool2-conv5x5(16)-pool2-affine 400-120-84-10 with ReLU, MSE, "
                                     f"batch {n_b} of 28x28 images, conv / pool P=2x2, affine 2x2 weight partitions, fp32",
                         "flops_per_step": self.flops_step}

    def step(self):
        self.net.step()

    def value(self, seconds_per_step):
        return seconds_per_step * 1e6

    def cpu_baseline(self):
        from oracle import network
        c = self.case
        par = {k: v.astype(np.float64) for k, v in c["params"].items()}
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            network.distributed_step(c["images"].astype(np.float64), c["target"].astype(np.float64), par)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        return {"value": dt * 1e6, "unit": "us/step", "cores": 1, "kind": "oracle",
                "sample": f"oracle network.distributed_step (numpy fp64) on the full cfg4 batch, mean of {reps} steps"}


def kernel_rooflines(workload, report, traffic):
    """Per-kernel roofline entries from the library's HIP-event timings."""
    out = {}
    for name, (count, total_ms) in report.items():
        key = next((k for k in sorted(workload.alg, key=len, reverse=True) if name.startswith(k)), None)
        avg_ms = total_ms / count
        entry = {"launches": count, "avg_ms": avg_ms, "total_ms": total_ms}
        if key is not None:
            bound, work = workload.alg[key]
            if work is None and key == "conv_reduce_dw":
                nparts = workload.dd.distdl_conv_bwd_workspace(workload.plan) // (4 * (workload.nw + workload.cfg["c_out"]))
                work = (nparts + 1) * workload.nw * 4
            if bound == "hbm":
                ach = work / (avg_ms * 1e-3) / 1e9
                entry.update(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                             algorithmic_bytes=work)
            else:
                ach = work / (avg_ms * 1e-3) / 1e12
                kdt = getattr(workload, "kernel_dtype", {}).get(key, workload.dtype)   # the MFMA type of this kernel
                peak = MFMA_PEAK_TFLOPS[kdt]
                entry.update(bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak,
                             algorithmic_flops=work, mfma_dtype=kdt)
                mb = getattr(workload, "min_bytes", {}).get(key)
                if mb:   # also against min(MFMA peak, arithmetic intensity x HBM peak)
                    roof = min(peak, work / mb * HBM_PEAK_GBS / 1e3)
                    entry.update(min_bytes=mb, roofline_tflops=roof, frac_of_roofline=ach / roof)
            tr = traffic.get(f"{workload.tag}/{name}")
            entry["traffic"] = None if tr is None else tr["fetch_bytes"] + tr["write_bytes"]
            if tr is not None:
                entry["traffic_fetch"], entry["traffic_write"] = tr["fetch_bytes"], tr["write_bytes"]
        out[name] = entry
    return out


def load_traffic():
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the
    readings of a plain 1 GiB copy (summaries and commands under profiles/); keyed
    "<workload>/<profiling scope of the library>"."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(path):
        with open(path) as f:
            return json.load(f)
    return {}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", choices=["cfg5", "cfg5-bf16", "cfg2", "cfg3", "cfg3-bf16", "cfg4", "movement"])
    ap.add_argument("--no-movement", action="store_true",
                    help="with the default workload: skip the movement kernels' own figures and the other configurations")
    ap.add_argument("--sweep", action="store_true",
                    help="with --workload movement: also the size sweep of broadcast / sum-reduce")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", default=None, metavar="PATH",
                    help="also write the full report (per-kernel tables of every workload, sweep rows) to this file")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB copy (copy_ref_kernel) before the timed region, as the "
                         "known-size reference for rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all P virtual workers share its HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    import paper_2006_03108_amd as dd
    torch.cuda.set_device(0)
    if args.workload == "movement":
        wl = MovementWorkload(args.sweep)
    elif args.workload == "cfg4":
        wl = SmallCnnWorkload()
    elif args.workload in ("cfg5", "cfg2"):
        wl = ConvWorkload(args.workload)
    elif args.workload == "cfg5-bf16":
        wl = ConvWorkload("cfg5", "bf16")
    else:
        wl = AffineWorkload("cfg3", "bf16" if args.workload.endswith("bf16") else "f32")
    if args.calibrate_copy:
        src = torch.ones(1 << 28, device="cuda")
        dst = torch.empty_like(src)
        dd.distdl_copy_ref(src, dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    dd.distdl_profile_enable(True)      # HIP events around every kernel, on the launch stream
    dd.distdl_profile_report()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    report = dd.distdl_profile_report()
    dd.distdl_profile_enable(False)
    sec = elapsed / args.steps
    kernels = kernel_rooflines(wl, report, load_traffic())
    launches_per_step = sum(k["launches"] for k in kernels.values()) / args.steps
    dominant = max(kernels, key=lambda k: kernels[k]["total_ms"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": dk.get("bound"), "achieved": dk.get("achieved"), "peak": dk.get("peak"),
                "unit": dk.get("unit"), "frac": dk.get("frac"), "traffic": dk.get("traffic"),
                "avg_ms": dk["avg_ms"], "launches": dk["launches"]}
    line = {
        "metric": wl.metric, "value": wl.value(sec), "unit": wl.unit, "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": getattr(wl, "higher_is_better", True),
        "scaling": "weak", "kernel_launches_per_step": launches_per_step,
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic", "config": wl.describe,
        "roofline": roofline, "kernels": kernels,
    }
    def side_run(make, steps):
        """One more workload timed with the same harness (profiling scopes on); its own small report."""
        w = make()
        for _ in range(3):
            w.step()
        torch.cuda.synchronize()
        dd.distdl_profile_enable(True)
        dd.distdl_profile_report()
        t0 = time.perf_counter()
        for _ in range(steps):
            w.step()
        torch.cuda.synchronize()
        s_sec = (time.perf_counter() - t0) / steps
        kern = kernel_rooflines(w, dd.distdl_profile_report(), load_traffic())
        dd.distdl_profile_enable(False)
        return w, {"metric": w.metric, "value": w.value(s_sec), "unit": w.unit, "steps": steps,
                   "ms_per_step": s_sec * 1e3, "dtype": w.dtype, "config": w.describe, "kernels": kern}

    def graph_step_ms(w, steps):
        """Launch-bound workloads: the same step recorded once into a HIP graph and replayed (a warmed-up step
        allocates nothing and copies no tables).  None if the runtime refuses the capture."""
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(3):
                    w.step()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                w.step()
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e3
        except RuntimeError as e:
            print(f"bench.py: graph capture failed: {e}", file=sys.stderr)
            return None

    if args.workload in ("cfg2", "cfg3", "cfg3-bf16", "cfg4"):
        line["ms_per_step_graph"] = graph_step_ms(wl, args.steps)
    detail = dict(line)                     # everything, for --detail; the printed line stays short
    if args.workload == "cfg5" and not args.no_movement:
        # the other half of the metric: the movement primitives on their own (H, H* on this geometry, B, R and
        # adjoints on large arrays), timed after the convolution step
        del wl.y, wl.dx, wl.ws, wl.x, wl.dy
        torch.cuda.empty_cache()
        mv, rep = side_run(lambda: MovementWorkload(False), 10)
        rep["frac_hbm_peak"] = rep["value"] / HBM_PEAK_GBS
        rep["layout"] = mv.layout_rates()
        del mv.x, mv.g
        torch.cuda.empty_cache()
        rep["achievable_copy"] = mv.achievable_copy()
        for kern in rep["kernels"].values():
            if kern.get("bound") == "hbm":
                kern["frac_of_achievable_copy"] = kern["achieved"] / rep["achievable_copy"]["best_GBs"]
        detail["movement"] = rep
        del mv
        torch.cuda.empty_cache()
        # the remaining single-GPU configurations, for reference (same harness, no CPU leg)
        detail["other_configs"] = {}
        for tag, make, steps in (("cfg2", lambda: ConvWorkload("cfg2"), 50),
                                 ("cfg5-bf16", lambda: ConvWorkload("cfg5", "bf16"), 20),
                                 ("cfg3", lambda: AffineWorkload("cfg3", "f32"), 50),
                                 ("cfg3-bf16", lambda: AffineWorkload("cfg3", "bf16"), 50),
                                 ("cfg4", lambda: SmallCnnWorkload(), 50)):
            w, rep = side_run(make, steps)
            rep["kernel_launches_per_step"] = sum(k["launches"] for k in rep["kernels"].values()) / steps
            if tag in ("cfg2", "cfg3", "cfg3-bf16", "cfg4"):
                rep["ms_per_step_graph"] = graph_step_ms(w, steps)
            detail["other_configs"][tag] = rep
            del w
    if getattr(wl, "sweep_on", False):
        detail["sweep"] = wl.sweep()
    if args.workload == "movement":
        detail["layout"] = wl.layout_rates()
        detail["achievable_copy"] = wl.achievable_copy()
        for kern in detail["kernels"].values():
            if kern.get("bound") == "hbm":
                kern["frac_of_achievable_copy"] = kern["achieved"] / detail["achievable_copy"]["best_GBs"]
    if not args.no_cpu_baseline:
        detail["cpu_baseline"] = wl.cpu_baseline()
    print(json.dumps(compact_line(detail, args.workload)))
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump(detail, f, indent=1)


def compact_line(detail, workload):
    """The one printed line: the contract's keys, `roofline`, `cpu_baseline`, and every figure of the metric as a
    top-level scalar (movement kernels in GB/s and as a fraction of the 8 TB/s HBM peak, contraction kernels as a
    fraction of the MFMA peak of their type, the other configurations' step rates), short enough to survive a
    log tail.  The per-kernel tables go to the --detail file."""
    r3 = lambda v: None if v is None else float(f"{v:.4g}")
    line = {k: v for k, v in detail.items() if k not in ("kernels", "movement", "other_configs", "sweep", "layout",
                                                         "achievable_copy")}

    def kernel_scalars(kernels, prefix=""):
        for name, k in kernels.items():
            if k.get("bound") == "hbm":
                line[f"{prefix}{name}_GBs"] = r3(k["achieved"])
                line[f"{prefix}{name}_frac_hbm"] = r3(k["frac"])
            elif k.get("bound") == "mfma":
                line[f"{prefix}{name}_TFLOPs"] = r3(k["achieved"])
                line[f"{prefix}{name}_frac_mfma"] = r3(k["frac"])
            line[f"{prefix}{name}_ms"] = r3(k["avg_ms"])

    if workload == "movement":
        kernel_scalars(detail["kernels"])
        mv = detail
        line["movement_GBs"], line["movement_frac_hbm"] = r3(detail["value"]), r3(detail["value"] / HBM_PEAK_GBS)
    else:
        kernel_scalars({k: v for k, v in detail["kernels"].items() if v.get("bound")})
        mv = detail.get("movement")
        if mv:
            line["movement_GBs"], line["movement_frac_hbm"] = r3(mv["value"]), r3(mv["frac_hbm_peak"])
            line["movement_ms_per_step"] = r3(mv["ms_per_step"])
            kernel_scalars(mv["kernels"])
    if "TFLOP" in detail["unit"]:
        line["step_frac_mfma"] = r3(detail["value"] / MFMA_PEAK_TFLOPS[detail["dtype"]])
    if mv:
        for name, k in mv.get("layout", {}).items():
            line[f"{name}_GBs"], line[f"{name}_frac_hbm"] = r3(k["achieved"]), r3(k["frac"])
        if "achievable_copy" in mv:
            line["copy_ref_GBs"] = r3(mv["achievable_copy"]["library_copy_GBs"])
            line["copy_ref_frac_hbm"] = r3(mv["achievable_copy"]["library_copy_GBs"] / HBM_PEAK_GBS)
    for tag, rep in detail.get("other_configs", {}).items():
        key = tag.replace("-", "_")
        line[f"{key}_value"], line[f"{key}_unit"] = r3(rep["value"]), rep["unit"]
        line[f"{key}_ms_per_step"] = r3(rep["ms_per_step"])
        if rep.get("ms_per_step_graph"):
            line[f"{key}_ms_per_step_graph"] = r3(rep["ms_per_step_graph"])
        if "TFLOP" in rep["unit"]:
            line[f"{key}_frac_mfma"] = r3(rep["value"] / MFMA_PEAK_TFLOPS[rep["dtype"]])
            if rep.get("ms_per_step_graph"):
                line[f"{key}_frac_mfma_graph"] = r3(rep["value"] * rep["ms_per_step"] / rep["ms_per_step_graph"] /
                                                    MFMA_PEAK_TFLOPS[rep["dtype"]])
        for name, k in rep["kernels"].items():
            if k.get("bound") == "mfma":
                line[f"{key}_{name}_frac_mfma"] = r3(k["frac"])
                line[f"{key}_{name}_ms"] = r3(k["avg_ms"])
    return line


if __name__ == "__main__":
    main()
