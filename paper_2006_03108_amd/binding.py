"""ctypes binding of include/distdl.h: same names, argument marshalling only.

Tensors are torch tensors on the GPU (used for device memory and the current
stream); every computation happens inside libdistdl.so.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdistdl.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2006_03108_amd/build.py`")
lib = C.CDLL(_LIB_PATH)

DISTDL_F32, DISTDL_BF16 = 0, 1
MAX_DIMS = 3
ERR_INVALID_ARG, ERR_NULL, ERR_UNSUPPORTED, ERR_EMPTY_PARTITION, ERR_HALO_TOO_WIDE, ERR_HIP, ERR_NOMEM = \
    -1, -2, -3, -4, -5, -6, -7


class DistdlError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"distdl error {code}: {msg}")
        self.code = code


class WorkerGeom(C.Structure):
    _fields_ = [("in_start", C.c_int64 * 3), ("in_size", C.c_int64 * 3),
                ("out_start", C.c_int64 * 3), ("out_size", C.c_int64 * 3),
                ("halo", (C.c_int32 * 2) * 3), ("pad", (C.c_int32 * 2) * 3), ("extra", (C.c_int32 * 2) * 3),
                ("buf_shape", C.c_int64 * 3), ("bulk_off", C.c_int64 * 3), ("conv_origin", C.c_int64 * 3)]


_vp, _i, _i64 = C.c_void_p, C.c_int, C.c_int64
_pp = C.POINTER(C.c_void_p)
_p64, _p32 = C.POINTER(C.c_int64), C.POINTER(C.c_int32)
_SIGS = {
    "distdl_plan_create": [C.POINTER(_vp), _i, _i64, _i64, _i64, _p64, _p32, _p32, _p32, _p32, _p32, _i],
    "distdl_plan_create_explicit": [C.POINTER(_vp), _i, _i64, _i64, _p32, _p64, _p32, _i],
    "distdl_plan_num_workers": [_vp],
    "distdl_plan_query": [_vp, _i, C.POINTER(WorkerGeom)],
    "distdl_plan_destroy": [_vp],
    "distdl_halo_fwd": [_vp, _pp, _vp],
    "distdl_halo_adj": [_vp, _pp, _vp],
    "distdl_bcast_fwd": [_pp, _pp, _p64, _i, _i, _i, _vp],
    "distdl_bcast_adj": [_pp, _pp, _p64, _i, _i, _i, _i, _vp],
    "distdl_sumreduce_fwd": [_pp, _pp, _p64, _i, _i, _i, _i, _vp],
    "distdl_sumreduce_adj": [_pp, _pp, _p64, _i, _i, _i, _vp],
    "distdl_allreduce": [_pp, _p64, _i, _i, _i, _vp],
    "distdl_convcp_plan_create": [C.POINTER(_vp), _i, _i64, _i64, _i64, _p64, _p32, _i, _i, _p32, _p32, _p32, _p32, _i],
    "distdl_convcp_plan_destroy": [_vp],
    "distdl_convcp_block_plan": [_vp, _i, _i],
    "distdl_convcp_channels": [_vp, _i, _i, _p64, _p64],
    "distdl_convcp_fwd": [_vp, _pp, _pp, _pp, _pp, _vp],
    "distdl_convcp_bwd": [_vp, _pp, _pp, _pp, _pp, _pp, _pp, _vp],
    "distdl_repart_plan_create": [C.POINTER(_vp), _i, _p64, C.POINTER(C.c_int32), C.POINTER(C.c_int32), _i],
    "distdl_repart_plan_destroy": [_vp],
    "distdl_repart_plan_num_blocks": [_vp, _i, ],
    "distdl_repart_plan_block": [_vp, _i, _i, _p64, _p64],
    "distdl_repart_fwd": [_vp, _pp, _pp, _vp],
    "distdl_repart_adj": [_vp, _pp, _pp, _vp],
    "distdl_conv_fwd": [_vp, _pp, _vp, _vp, _pp, _vp],
    "distdl_conv_bwd": [_vp, _pp, _vp, _pp, _pp, _vp, _vp, _vp, C.c_size_t, _vp],
    "distdl_conv_local_fwd": [_vp, _pp, _vp, _vp, _pp, _vp],
    "distdl_conv_local_bwd": [_vp, _pp, _vp, _pp, _pp, _vp, _vp, _vp, C.c_size_t, _vp],
    "distdl_layout_convert": [_vp, _i, _i, _pp, _pp, _vp],
    "distdl_copy_ref": [_vp, _vp, C.c_size_t, _vp],
    "distdl_debug_slot_policy": [_p32, _p32, _p32, _i, _p32],
    "distdl_debug_conv_path": [_vp, _p32],
    "distdl_affine_plan_create": [C.POINTER(_vp), _i64, _i64, _i64, _i, _i, _i],
    "distdl_affine_plan_destroy": [_vp],
    "distdl_affine_fwd": [_vp, _pp, _pp, _pp, _pp, _vp],
    "distdl_affine_bwd": [_vp, _pp, _pp, _pp, _pp, _pp, _pp, _vp],
    "distdl_dot": [_pp, _pp, _p64, _i, _i, _vp, _vp],
    "distdl_dot_static": [_pp, _pp, _p64, _i, _i, _vp, _vp],
    "distdl_relu_fwd": [_pp, _pp, _p64, _i, _vp],
    "distdl_relu_bwd": [_pp, _pp, _pp, _p64, _i, _vp],
    "distdl_maxpool_fwd": [_vp, _pp, _pp, _vp],
    "distdl_maxpool_bwd": [_vp, _pp, _pp, _pp, _vp],
    "distdl_avgpool_fwd": [_vp, _pp, _pp, _vp],
    "distdl_avgpool_bwd": [_vp, _pp, _pp, _vp],
    "distdl_bulk_copy": [_vp, _pp, _pp, _i, _vp],
    "distdl_repartition_fwd": [_vp, _pp, _i, _pp, _vp],
    "distdl_repartition_adj": [_vp, _pp, _i, _pp, _vp],
    "distdl_mse_fwd_bwd": [_pp, _pp, _pp, _p64, _i, _vp, _vp],
    "distdl_plan_stats": [_vp, _p64],
    "distdl_profile_enable": [_i],
    "distdl_profile_report": [C.c_char_p, C.c_size_t],
    "distdl_debug_task_count": [_vp, _i],
    "distdl_debug_get_task": [_vp, _i, _i, _p32, _i],
}
EXPORTS = sorted(list(_SIGS) + ["distdl_conv_bwd_workspace", "distdl_last_error", "distdl_debug_fastdiv"])
for _name, _args in _SIGS.items():
    getattr(lib, _name).argtypes = _args
    getattr(lib, _name).restype = C.c_int
lib.distdl_conv_bwd_workspace.argtypes = [_vp]
lib.distdl_conv_bwd_workspace.restype = C.c_size_t
lib.distdl_debug_fastdiv.argtypes = [C.c_uint32, C.c_uint32]
lib.distdl_debug_fastdiv.restype = C.c_uint32
lib.distdl_convcp_block_plan.restype = C.c_void_p
lib.distdl_last_error.argtypes = []
lib.distdl_last_error.restype = C.c_char_p


def _check(rc):
    if rc < 0:
        raise DistdlError(rc, lib.distdl_last_error().decode())
    return rc


def _ptrs(tensors):
    """Host array of device pointers from a list of tensors (None -> NULL)."""
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def _arr(ctype, values):
    return (ctype * len(values))(*[int(v) for v in values])


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(dtype):
    if dtype in (torch.float32, DISTDL_F32, "f32"):
        return DISTDL_F32
    if dtype in (torch.bfloat16, DISTDL_BF16, "bf16"):
        return DISTDL_BF16
    raise DistdlError(ERR_UNSUPPORTED, f"dtype {dtype}")


class Plan:
    """Owner of a distdl_plan handle."""

    def __init__(self, handle, D):
        self.handle, self.D = handle, D
        self.n_workers = _check(lib.distdl_plan_num_workers(handle))

    def query(self, worker):
        g = WorkerGeom()
        _check(lib.distdl_plan_query(self.handle, worker, C.byref(g)))
        D = self.D
        return dict(
            in_start=list(g.in_start)[:D], in_size=list(g.in_size)[:D],
            out_start=list(g.out_start)[:D], out_size=list(g.out_size)[:D],
            halo=[tuple(g.halo[d]) for d in range(D)], pad=[tuple(g.pad[d]) for d in range(D)],
            extra=[tuple(g.extra[d]) for d in range(D)], buf_shape=list(g.buf_shape)[:D],
            bulk_off=list(g.bulk_off)[:D], conv_origin=list(g.conv_origin)[:D])

    def destroy(self):
        if self.handle:
            lib.distdl_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def distdl_plan_create(D, n_b, n_c_in, n_c_out, in_shape, P, ksize, stride, padding, dilation, dtype=torch.float32):
    h = C.c_void_p()
    _check(lib.distdl_plan_create(C.byref(h), D, n_b, n_c_in, n_c_out, _arr(C.c_int64, in_shape),
                                  _arr(C.c_int32, P), _arr(C.c_int32, ksize), _arr(C.c_int32, stride),
                                  _arr(C.c_int32, padding), _arr(C.c_int32, dilation), _dtype_code(dtype)))
    return Plan(h, D)


def distdl_plan_create_explicit(D, n_b, n_c, P, bulk_sizes, halo_lr, dtype=torch.float32):
    """bulk_sizes: per dimension a list of P[d] sizes; halo_lr: per dimension a
    list of (left, right) pairs."""
    flat_b = [s for d in bulk_sizes for s in d]
    flat_h = [v for d in halo_lr for pair in d for v in pair]
    h = C.c_void_p()
    _check(lib.distdl_plan_create_explicit(C.byref(h), D, n_b, n_c, _arr(C.c_int32, P), _arr(C.c_int64, flat_b),
                                           _arr(C.c_int32, flat_h), _dtype_code(dtype)))
    return Plan(h, D)


def distdl_halo_fwd(plan, bufs):
    _check(lib.distdl_halo_fwd(plan.handle, _ptrs(bufs), _stream()))


def distdl_halo_adj(plan, gbufs):
    _check(lib.distdl_halo_adj(plan.handle, _ptrs(gbufs), _stream()))


def _counts(one):
    return _arr(C.c_int64, [t.numel() for t in one])


def distdl_bcast_fwd(src, dst, k):
    _check(lib.distdl_bcast_fwd(_ptrs(src), _ptrs(dst), _counts(src), len(src), k, _dtype_code(src[0].dtype), _stream()))


def distdl_bcast_adj(gsrc, gdst, k, clear_inputs=False):
    _check(lib.distdl_bcast_adj(_ptrs(gsrc), _ptrs(gdst), _counts(gsrc), len(gsrc), k, _dtype_code(gsrc[0].dtype),
                                int(clear_inputs), _stream()))


def distdl_sumreduce_fwd(src, dst, k, clear_inputs=False):
    _check(lib.distdl_sumreduce_fwd(_ptrs(src), _ptrs(dst), _counts(dst), len(dst), k, _dtype_code(dst[0].dtype),
                                    int(clear_inputs), _stream()))


def distdl_sumreduce_adj(gdst, gsrc, k):
    _check(lib.distdl_sumreduce_adj(_ptrs(gdst), _ptrs(gsrc), _counts(gdst), len(gdst), k,
                                    _dtype_code(gdst[0].dtype), _stream()))


def distdl_allreduce(bufs, k):
    """bufs: G*k tensors, group after group; all replicas of a group end as the group's sum."""
    G = len(bufs) // k
    counts = _arr(C.c_int64, [bufs[g * k].numel() for g in range(G)])
    _check(lib.distdl_allreduce(_ptrs(bufs), counts, G, k, _dtype_code(bufs[0].dtype), _stream()))


class _BorrowedPlan(Plan):
    """A sliding-kernel plan owned by another object (queries only)."""

    def destroy(self):
        self.handle = None


class ConvCpPlan:
    """Owner of a distdl_convcp_plan handle (channel-partitioned convolution layer)."""

    def __init__(self, handle, D, P_co, P_ci):
        self.handle, self.D, self.P_co, self.P_ci = handle, D, P_co, P_ci
        self.spatial = self.block_plan(0, 0)
        self.S = self.spatial.n_workers

    def block_plan(self, i, j):
        h = lib.distdl_convcp_block_plan(self.handle, i, j)
        if not h:
            raise DistdlError(ERR_INVALID_ARG, lib.distdl_last_error().decode())
        return _BorrowedPlan(C.c_void_p(h), self.D)

    def channels(self, output_side, block):
        st, sz = C.c_int64(), C.c_int64()
        _check(lib.distdl_convcp_channels(self.handle, int(output_side), block, C.byref(st), C.byref(sz)))
        return st.value, sz.value

    def __del__(self):
        if getattr(self, "handle", None):
            lib.distdl_convcp_plan_destroy(self.handle)
            self.handle = None


def distdl_convcp_plan_create(D, n_b, n_c_in, n_c_out, in_shape, P, P_co, P_ci, ksize, stride, padding, dilation,
                              dtype=torch.float32):
    h = C.c_void_p()
    _check(lib.distdl_convcp_plan_create(C.byref(h), D, n_b, n_c_in, n_c_out, _arr(C.c_int64, in_shape),
                                         _arr(C.c_int32, P), P_co, P_ci, _arr(C.c_int32, ksize), _arr(C.c_int32, stride),
                                         _arr(C.c_int32, padding), _arr(C.c_int32, dilation), _dtype_code(dtype)))
    return ConvCpPlan(h, D, P_co, P_ci)


def distdl_convcp_fwd(plan, x_bufs, w, bias, y):
    """x_bufs: P_ci * S buffers (block-major), w: P_co * P_ci blocks, bias: P_co arrays or None, y: P_co * S."""
    _check(lib.distdl_convcp_fwd(plan.handle, _ptrs(x_bufs), _ptrs(w), _ptrs(bias) if bias is not None else None,
                                 _ptrs(y), _stream()))


def distdl_convcp_bwd(plan, x_bufs, w, dy, dx_bufs, dw, dbias):
    _check(lib.distdl_convcp_bwd(plan.handle, _ptrs(x_bufs), _ptrs(w), _ptrs(dy), _ptrs(dx_bufs), _ptrs(dw),
                                 _ptrs(dbias) if dbias is not None else None, _stream()))


class RepartPlan:
    """Owner of a distdl_repart_plan handle."""

    def __init__(self, handle, R):
        self.handle, self.R = handle, R

    def blocks(self, side):
        """[(start tuple, size tuple)] of every block of side 0 (source) or 1 (destination)."""
        out = []
        for w in range(_check(lib.distdl_repart_plan_num_blocks(self.handle, side))):
            st, sz = (C.c_int64 * self.R)(), (C.c_int64 * self.R)()
            _check(lib.distdl_repart_plan_block(self.handle, side, w, st, sz))
            out.append((tuple(st), tuple(sz)))
        return out

    def __del__(self):
        if getattr(self, "handle", None):
            lib.distdl_repart_plan_destroy(self.handle)
            self.handle = None


def distdl_repart_plan_create(shape, P_src, P_dst, dtype=torch.float32):
    h = C.c_void_p()
    _check(lib.distdl_repart_plan_create(C.byref(h), len(shape), _arr(C.c_int64, shape), _arr(C.c_int32, P_src),
                                         _arr(C.c_int32, P_dst), _dtype_code(dtype)))
    return RepartPlan(h, len(shape))


def distdl_repart_fwd(plan, src, dst):
    _check(lib.distdl_repart_fwd(plan.handle, _ptrs(src), _ptrs(dst), _stream()))


def distdl_repart_adj(plan, gdst, gsrc):
    _check(lib.distdl_repart_adj(plan.handle, _ptrs(gdst), _ptrs(gsrc), _stream()))


def distdl_conv_bwd_workspace(plan):
    return int(lib.distdl_conv_bwd_workspace(plan.handle))


def distdl_conv_fwd(plan, x_bufs, w, bias, y):
    _check(lib.distdl_conv_fwd(plan.handle, _ptrs(x_bufs), w.data_ptr(), None if bias is None else bias.data_ptr(),
                               _ptrs(y), _stream()))


def distdl_conv_bwd(plan, x_bufs, w, dy, dx_bufs, dw, dbias, workspace):
    _check(lib.distdl_conv_bwd(plan.handle, _ptrs(x_bufs), w.data_ptr(), _ptrs(dy), _ptrs(dx_bufs), dw.data_ptr(),
                               None if dbias is None else dbias.data_ptr(), workspace.data_ptr(),
                               workspace.numel() * workspace.element_size(), _stream()))


def distdl_conv_local_fwd(plan, x_bufs, w, bias, y):
    _check(lib.distdl_conv_local_fwd(plan.handle, _ptrs(x_bufs), w.data_ptr(), None if bias is None else bias.data_ptr(),
                                     _ptrs(y), _stream()))


def distdl_conv_local_bwd(plan, x_bufs, w, dy, dx_bufs, dw, dbias, workspace):
    _check(lib.distdl_conv_local_bwd(plan.handle, _ptrs(x_bufs), w.data_ptr(), _ptrs(dy), _ptrs(dx_bufs), dw.data_ptr(),
                                     None if dbias is None else dbias.data_ptr(), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream()))


def distdl_layout_convert(plan, what, to_channels_last, src, dst):
    """what: 0 padded buffers (input channels), 1 outputs (output channels)."""
    _check(lib.distdl_layout_convert(plan.handle, int(what), int(to_channels_last), _ptrs(src), _ptrs(dst), _stream()))


def distdl_copy_ref(src, dst):
    _check(lib.distdl_copy_ref(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream()))


def distdl_debug_slot_policy(stream_ids, table_ids, capturing):
    """Slot index (or negative error code) each call of the sequence would get from the table cache."""
    n = len(stream_ids)
    out = (C.c_int32 * n)()
    _check(lib.distdl_debug_slot_policy(_arr(C.c_int32, stream_ids), _arr(C.c_int32, table_ids),
                                        _arr(C.c_int32, capturing), n, out))
    return list(out)


def distdl_debug_conv_path(plan):
    """(forward, data gradient, weight gradient) kernel families: 0 direct, 1 32-wide MFMA tiles, 2 16-wide."""
    out = (C.c_int32 * 3)()
    _check(lib.distdl_debug_conv_path(plan.handle, out))
    return tuple(out)


class AffinePlan:
    def __init__(self, handle):
        self.handle = handle

    def destroy(self):
        if self.handle:
            lib.distdl_affine_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def distdl_affine_plan_create(n_b, n_fi, n_fo, P_fo, P_fi, dtype=torch.float32):
    h = C.c_void_p()
    _check(lib.distdl_affine_plan_create(C.byref(h), n_b, n_fi, n_fo, P_fo, P_fi, _dtype_code(dtype)))
    return AffinePlan(h)


def distdl_affine_fwd(plan, x, W, b, y):
    _check(lib.distdl_affine_fwd(plan.handle, _ptrs(x), _ptrs(W), None if b is None else _ptrs(b), _ptrs(y), _stream()))


def distdl_affine_bwd(plan, x, W, dy, dx, dW, db):
    _check(lib.distdl_affine_bwd(plan.handle, _ptrs(x), _ptrs(W), _ptrs(dy), _ptrs(dx), _ptrs(dW),
                                 None if db is None else _ptrs(db), _stream()))


def _numels(ts):
    return _arr(C.c_int64, [t.numel() for t in ts])


def distdl_relu_fwd(x, y):
    _check(lib.distdl_relu_fwd(_ptrs(x), _ptrs(y), _numels(x), len(x), _stream()))


def distdl_relu_bwd(x, dy, dx):
    _check(lib.distdl_relu_bwd(_ptrs(x), _ptrs(dy), _ptrs(dx), _numels(x), len(x), _stream()))


def distdl_maxpool_fwd(plan, x_bufs, y):
    _check(lib.distdl_maxpool_fwd(plan.handle, _ptrs(x_bufs), _ptrs(y), _stream()))


def distdl_maxpool_bwd(plan, x_bufs, dy, dx_bufs):
    _check(lib.distdl_maxpool_bwd(plan.handle, _ptrs(x_bufs), _ptrs(dy), _ptrs(dx_bufs), _stream()))


def distdl_avgpool_fwd(plan, x_bufs, y):
    _check(lib.distdl_avgpool_fwd(plan.handle, _ptrs(x_bufs), _ptrs(y), _stream()))


def distdl_avgpool_bwd(plan, dy, dx_bufs):
    _check(lib.distdl_avgpool_bwd(plan.handle, _ptrs(dy), _ptrs(dx_bufs), _stream()))


def distdl_bulk_copy(plan, dense, bufs, to_bufs):
    _check(lib.distdl_bulk_copy(plan.handle, _ptrs(dense), _ptrs(bufs), int(to_bufs), _stream()))


def distdl_repartition_fwd(plan, src, dst):
    _check(lib.distdl_repartition_fwd(plan.handle, _ptrs(src), len(dst), _ptrs(dst), _stream()))


def distdl_repartition_adj(plan, gdst, gsrc):
    _check(lib.distdl_repartition_adj(plan.handle, _ptrs(gdst), len(gdst), _ptrs(gsrc), _stream()))


def distdl_mse_fwd_bwd(y, t, dy, loss):
    """loss: a 1-element float64 device tensor."""
    _check(lib.distdl_mse_fwd_bwd(_ptrs(y), _ptrs(t), _ptrs(dy), _numels(y), len(y), loss.data_ptr(), _stream()))


def distdl_dot(a, b, result):
    """result: a 1-element float64 device tensor."""
    _check(lib.distdl_dot(_ptrs(a), _ptrs(b), _arr(C.c_int64, [t.numel() for t in a]), len(a),
                          _dtype_code(a[0].dtype), result.data_ptr(), _stream()))


def distdl_dot_static(a, b, result):
    """distdl_dot without any allocation (scratch in a static device array); at most 96 array pairs."""
    _check(lib.distdl_dot_static(_ptrs(a), _ptrs(b), _arr(C.c_int64, [t.numel() for t in a]), len(a),
                                 _dtype_code(a[0].dtype), result.data_ptr(), _stream()))


def distdl_plan_stats(plan):
    out = (C.c_int64 * 4)()
    _check(lib.distdl_plan_stats(plan.handle, out))
    return dict(halo_cells=out[0], pad_cells=out[1], band_cells=out[2], gathered_cells=out[3])


def distdl_profile_enable(on):
    _check(lib.distdl_profile_enable(int(on)))


def distdl_profile_report():
    """{kernel name: (launches, total milliseconds)} since the last report."""
    buf = C.create_string_buffer(1 << 16)
    _check(lib.distdl_profile_report(buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, count, ms = line.split()
        out[name] = (int(count), float(ms))
    return out


def distdl_debug_tasks(plan, adjoint):
    """All box tasks of the forward / adjoint halo table as dicts."""
    out = []
    buf = (C.c_int32 * (8 + 4 * 32))()
    for idx in range(_check(lib.distdl_debug_task_count(plan.handle, int(adjoint)))):
        n = _check(lib.distdl_debug_get_task(plan.handle, int(adjoint), idx, buf, len(buf)))
        v = list(buf)[:n]
        out.append(dict(dst=v[0], org=v[2:5], ext=v[5:8],
                        srcs=[(v[8 + 4 * s], v[9 + 4 * s:12 + 4 * s]) for s in range(v[1])]))
    return out


def distdl_last_error():
    return lib.distdl_last_error().decode()
