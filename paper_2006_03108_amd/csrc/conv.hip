// Partitioned convolution (Sec. 4, Forward / Adjoint Convolution Algorithms
// with P_co = P_ci = 1): x <- H x, the local cross-correlation on every
// worker's padded buffer, and in the adjoint the local [dConv]*, the
// sum-reduce of dw / db over workers and H* on dx.
//
// Layout: channels-last.  x^ is [n_b][B0][B1][B2][Ci], y is [n_b][O0][O1][O2][Co],
// weights arrive as [Co][Ci][T] (T = taps, last fastest) and are re-laid out
// once per call into wt[T][Ci][Co] so that the output-channel axis is the
// contiguous one.
#include <algorithm>

#include "common.h"
#include "conv_core.h"
#include "conv_mfma.h"
#include "profile.h"

namespace distdl {

int plan_prepare_device(distdl_plan* p);
int run_halo(distdl_plan* p, bool adjoint, PtrTable& tab, void* const* bufs_host, hipStream_t st);

struct ConvDev {
  int32_t n_b, ci, co;
  int32_t k[3], s[3], dil[3];
  int32_t taps;
};

static ConvDev conv_params(const distdl_plan* p) {
  ConvDev c;
  c.n_b = (int32_t)p->n_b;
  c.ci = (int32_t)p->n_ci;
  c.co = (int32_t)p->n_co;
  c.taps = 1;
  for (int d = 0; d < 3; ++d) {
    c.k[d] = p->ksize[d];
    c.s[d] = p->stride[d];
    c.dil[d] = p->dilation[d];
    c.taps *= p->ksize[d];
  }
  return c;
}

// wt[(t*Ci + ci)*Co + co] = w[(co*Ci + ci)*T + t]
template <class T>
__global__ void relayout_w_kernel(const T* __restrict__ w, float* __restrict__ wt, int co_n, int ci_n, int taps) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  int total = co_n * ci_n * taps;
  if (idx >= total) return;
  int co = idx % co_n;
  int r = idx / co_n;
  int ci = r % ci_n;
  int t = r / ci_n;
  wt[idx] = ld(w, ((size_t)co * ci_n + ci) * taps + t);
}

// ---- reference-shaped kernels: any D, stride, dilation, channel count -------

template <class T>
__global__ __launch_bounds__(256) void conv_fwd_direct_kernel(const WorkerDev* __restrict__ workers,
                                                              void* const* x_bufs, const float* __restrict__ wt,
                                                              const T* __restrict__ bias, void* const* y_bufs,
                                                              ConvDev c) {
  const WorkerDev wd = workers[blockIdx.y];
  const int64_t total = (int64_t)c.n_b * wd.out[0] * wd.out[1] * wd.out[2] * c.co;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const T* __restrict__ x = (const T*)x_bufs[blockIdx.y];
  T* __restrict__ y = (T*)y_bufs[blockIdx.y];
  int co = (int)(idx % c.co);
  int64_t r = idx / c.co;
  int o2 = (int)(r % wd.out[2]); r /= wd.out[2];
  int o1 = (int)(r % wd.out[1]); r /= wd.out[1];
  int o0 = (int)(r % wd.out[0]);
  int n = (int)(r / wd.out[0]);
  float acc = bias ? ld(bias, co) : 0.f;
  const int64_t s2 = c.ci, s1 = (int64_t)wd.buf[2] * s2, s0 = (int64_t)wd.buf[1] * s1, sn = (int64_t)wd.buf[0] * s0;
  const T* xn = x + n * sn;
  int t = 0;
  for (int t0 = 0; t0 < c.k[0]; ++t0)
    for (int t1 = 0; t1 < c.k[1]; ++t1)
      for (int t2 = 0; t2 < c.k[2]; ++t2, ++t) {
        const T* xc = xn + (wd.origin[0] + o0 * c.s[0] + t0 * c.dil[0]) * s0 +
                          (wd.origin[1] + o1 * c.s[1] + t1 * c.dil[1]) * s1 +
                          (wd.origin[2] + o2 * c.s[2] + t2 * c.dil[2]) * s2;
        const float* wp = wt + (size_t)t * c.ci * c.co + co;
        for (int ci = 0; ci < c.ci; ++ci) acc = fmaf(wp[(size_t)ci * c.co], ld(xc, ci), acc);
      }
  st(y, idx, acc);
}

// dx^[n][cell][ci] over the whole padded buffer (cells no output reads get 0).
template <class T>
__global__ __launch_bounds__(256) void conv_bwd_data_direct_kernel(const WorkerDev* __restrict__ workers,
                                                                   void* const* dy_bufs, const float* __restrict__ wt,
                                                                   void* const* dx_bufs, ConvDev c) {
  const WorkerDev wd = workers[blockIdx.y];
  const int64_t total = (int64_t)c.n_b * wd.buf[0] * wd.buf[1] * wd.buf[2] * c.ci;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const T* __restrict__ dy = (const T*)dy_bufs[blockIdx.y];
  T* __restrict__ dx = (T*)dx_bufs[blockIdx.y];
  int ci = (int)(idx % c.ci);
  int64_t r = idx / c.ci;
  int c2 = (int)(r % wd.buf[2]); r /= wd.buf[2];
  int c1 = (int)(r % wd.buf[1]); r /= wd.buf[1];
  int c0 = (int)(r % wd.buf[0]);
  int n = (int)(r / wd.buf[0]);
  const int64_t so2 = c.co, so1 = (int64_t)wd.out[2] * so2, so0 = (int64_t)wd.out[1] * so1,
                son = (int64_t)wd.out[0] * so0;
  float acc = 0.f;
  int t = 0;
  for (int t0 = 0; t0 < c.k[0]; ++t0) {
    int q0 = c0 - wd.origin[0] - t0 * c.dil[0];
    bool ok0 = q0 >= 0 && q0 % c.s[0] == 0 && q0 / c.s[0] < wd.out[0];
    for (int t1 = 0; t1 < c.k[1]; ++t1) {
      int q1 = c1 - wd.origin[1] - t1 * c.dil[1];
      bool ok1 = q1 >= 0 && q1 % c.s[1] == 0 && q1 / c.s[1] < wd.out[1];
      for (int t2 = 0; t2 < c.k[2]; ++t2, ++t) {
        int q2 = c2 - wd.origin[2] - t2 * c.dil[2];
        bool ok2 = q2 >= 0 && q2 % c.s[2] == 0 && q2 / c.s[2] < wd.out[2];
        if (!(ok0 && ok1 && ok2)) continue;
        const T* dyc = dy + n * son + (q0 / c.s[0]) * so0 + (q1 / c.s[1]) * so1 + (q2 / c.s[2]) * so2;
        const float* wp = wt + ((size_t)t * c.ci + ci) * c.co;
        for (int co = 0; co < c.co; ++co) acc = fmaf(wp[co], ld(dyc, co), acc);
      }
    }
  }
  st(dx, idx, acc);
}

// Partial dw^ / db^ of one worker over one chunk of its (n, o) positions, in
// the wt layout followed by Co bias slots.
template <class T>
__global__ __launch_bounds__(256) void conv_bwd_weight_direct_kernel(const WorkerDev* __restrict__ workers,
                                                                     void* const* x_bufs, void* const* dy_bufs,
                                                                     float* __restrict__ partial, ConvDev c,
                                                                     int nchunks) {
  const int worker = blockIdx.z, chunk = blockIdx.y;
  const WorkerDev wd = workers[worker];
  const int nw = c.taps * c.ci * c.co;
  int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= nw + c.co) return;
  const T* __restrict__ x = (const T*)x_bufs[worker];
  const T* __restrict__ dy = (const T*)dy_bufs[worker];
  const int64_t npos = (int64_t)c.n_b * wd.out[0] * wd.out[1] * wd.out[2];
  const int64_t per = (npos + nchunks - 1) / nchunks;
  const int64_t p0 = chunk * per, p1 = std::min<int64_t>(npos, p0 + per);
  float acc = 0.f;
  if (idx >= nw) {  // bias gradient slot
    int co = idx - nw;
    for (int64_t p = p0; p < p1; ++p) acc += ld(dy, p * c.co + co);
  } else {
    int co = idx % c.co;
    int r = idx / c.co;
    int ci = r % c.ci;
    int t = r / c.ci;
    int t2 = t % c.k[2];
    int t1 = (t / c.k[2]) % c.k[1];
    int t0 = t / (c.k[2] * c.k[1]);
    const int64_t s2 = c.ci, s1 = (int64_t)wd.buf[2] * s2, s0 = (int64_t)wd.buf[1] * s1,
                  sn = (int64_t)wd.buf[0] * s0;
    for (int64_t p = p0; p < p1; ++p) {
      int64_t rr = p;
      int o2 = (int)(rr % wd.out[2]); rr /= wd.out[2];
      int o1 = (int)(rr % wd.out[1]); rr /= wd.out[1];
      int o0 = (int)(rr % wd.out[0]);
      int n = (int)(rr / wd.out[0]);
      const float xv = ld(x, n * sn + (wd.origin[0] + o0 * c.s[0] + t0 * c.dil[0]) * s0 +
                                (wd.origin[1] + o1 * c.s[1] + t1 * c.dil[1]) * s1 +
                                (wd.origin[2] + o2 * c.s[2] + t2 * c.dil[2]) * s2 + ci);
      acc = fmaf(ld(dy, p * c.co + co), xv, acc);
    }
  }
  partial[((size_t)worker * nchunks + chunk) * (nw + c.co) + idx] = acc;
}

// R dw^, R db^ (Sec. 4, adjoint algorithm): sum the partials in worker order
// and write dw in the caller's [Co][Ci][T] shape.
template <int E, class T>
__global__ __launch_bounds__(256) void conv_reduce_dw_kernel(const float* __restrict__ partial, int nparts,
                                                             T* __restrict__ dw, T* __restrict__ db, ConvDev c) {
  // E elements per block, L = 256 / E lanes of partials each (few elements: more lanes, so that the launch still
  // has enough blocks); every lane adds its partials in ascending order (four independent chains for latency),
  // the lanes are then combined in ascending order
  constexpr int L = 256 / E;
  const int nw = c.taps * c.ci * c.co;
  const int e = threadIdx.x % E, lanep = threadIdx.x / E;
  const int idx = blockIdx.x * E + e;
  const size_t slot = (size_t)nw + c.co;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (idx < nw + c.co) {
    int p = lanep;
    for (; p + 3 * L < nparts; p += 4 * L)
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] += partial[(size_t)(p + L * u) * slot + idx];
    for (; p < nparts; p += L) acc[0] += partial[(size_t)p * slot + idx];
  }
  __shared__ float red[L][E];
  red[lanep][e] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  __syncthreads();
  if (lanep != 0 || idx >= nw + c.co) return;
  float sum = red[0][e];
#pragma unroll
  for (int l = 1; l < L; ++l) sum += red[l][e];
  if (idx >= nw) {
    if (db) st(db, idx - nw, sum);
  } else {
    int co = idx % c.co;
    int r = idx / c.co;
    int ci = r % c.ci;
    int t = r / c.ci;
    st(dw, ((size_t)co * c.ci + ci) * c.taps + t, sum);
  }
}

static int direct_chunks(const distdl_plan* p) {
  ConvDev c = conv_params(p);
  int64_t nw = (int64_t)c.taps * c.ci * c.co + c.co;
  int64_t blocks = (nw + 255) / 256 * p->n_workers;
  int64_t want = (2048 + blocks - 1) / blocks;
  int64_t npos = p->n_b * p->max_out_cells;
  return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, 64), npos));
}

static int check_conv_plan(const distdl_plan* p) {
  if (p->explicit_halo) return set_error(DISTDL_ERR_UNSUPPORTED, "conv: plan has no kernel (explicit halo plan)");
  return DISTDL_OK;
}

static int prepare_weights(distdl_plan* p, const void* w, hipStream_t st) {
  ConvDev c = conv_params(p);
  size_t n = (size_t)c.taps * c.ci * c.co;
  if (p->wt_elems < n) {
    if (p->d_wt) (void)hipFree(p->d_wt);  // waits for kernels still reading it
    p->d_wt = nullptr;
    p->wt_elems = 0;
    DISTDL_HIP_TRY(hipMalloc((void**)&p->d_wt, n * sizeof(float)));
    p->wt_elems = n;
  }
  ProfScope prof("conv_relayout_w", st);
  if (p->dtype == DISTDL_BF16)
    hipLaunchKernelGGL(relayout_w_kernel<uint16_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       (const uint16_t*)w, p->d_wt, c.co, c.ci, c.taps);
  else
    hipLaunchKernelGGL(relayout_w_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const float*)w,
                       p->d_wt, c.co, c.ci, c.taps);
  return DISTDL_OK;
}

}  // namespace distdl

using namespace distdl;

extern "C" {

size_t distdl_conv_bwd_workspace(const distdl_plan* plan) {
  if (!plan || plan->explicit_halo) return 0;
  ConvDev c = conv_params(plan);
  size_t nw = (size_t)c.taps * c.ci * c.co + c.co;
  int chunks = direct_chunks(plan);
  if (wgrad_mfma_supported(plan)) chunks = std::max(chunks, wgrad_chunks(plan));
  chunks = std::max(chunks, std::max(wgrad16_chunks(plan, true), wgrad16_chunks(plan, false)));
  return nw * sizeof(float) * plan->n_workers * chunks;
}

int distdl_conv_fwd(distdl_plan* plan, void* const x_bufs_dev[], const void* w_dev, const void* bias_dev,
                    void* const y_dev[], void* stream) {
  return distdl::conv_fwd_core(plan, x_bufs_dev, w_dev, bias_dev, y_dev, (hipStream_t)stream, true);
}

int distdl_conv_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* w_dev, const void* const dy_dev[],
                    void* const dx_bufs_dev[], void* dw_dev, void* dbias_dev, void* workspace_dev,
                    size_t workspace_bytes, void* stream) {
  return distdl::conv_bwd_core(plan, x_bufs_dev, w_dev, dy_dev, dx_bufs_dev, dw_dev, dbias_dev, workspace_dev,
                               workspace_bytes, (hipStream_t)stream, true);
}

int distdl_debug_conv_path(const distdl_plan* plan, int32_t out[3]) {
  if (!plan || !out) return set_error(DISTDL_ERR_NULL, "conv_path: null argument");
  if (plan->explicit_halo) return set_error(DISTDL_ERR_UNSUPPORTED, "conv_path: plan has no kernel");
  // the choices of conv_fwd_core / conv_bwd_core for 16-byte aligned arrays
  const bool vec = plan->n_ci % 4 == 0 && plan->n_co % 4 == 0;
  const bool mfma = corr_mfma_supported(plan);
  out[0] = corr16_fwd_supported(plan, true) ? 2 : mfma ? 1 : 0;
  out[1] = corr16_bwd_supported(plan, true) ? 2 : mfma ? 1 : 0;
  out[2] = wgrad16_supported(plan, vec) ? 2 : (wgrad_mfma_supported(plan) && (plan->dtype != DISTDL_BF16 || vec)) ? 1 : 0;
  return DISTDL_OK;
}

int distdl_conv_local_fwd(distdl_plan* plan, void* const x_bufs_dev[], const void* w_dev, const void* bias_dev,
                          void* const y_dev[], void* stream) {
  return distdl::conv_fwd_core(plan, x_bufs_dev, w_dev, bias_dev, y_dev, (hipStream_t)stream, false);
}

int distdl_conv_local_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* w_dev,
                          const void* const dy_dev[], void* const dx_bufs_dev[], void* dw_dev, void* dbias_dev,
                          void* workspace_dev, size_t workspace_bytes, void* stream) {
  return distdl::conv_bwd_core(plan, x_bufs_dev, w_dev, dy_dev, dx_bufs_dev, dw_dev, dbias_dev, workspace_dev,
                               workspace_bytes, (hipStream_t)stream, false);
}

}  // extern "C"

namespace distdl {

// The two layer calls; `halo` = false leaves out H (forward) / H* (backward) for callers that apply them
// themselves (the channel-partitioned layer exchanges halos once per input block, not once per weight block).
int conv_fwd_core(distdl_plan* plan, void* const x_bufs_dev[], const void* w_dev, const void* bias_dev,
                  void* const y_dev[], hipStream_t st, bool halo) {
  if (!plan || !x_bufs_dev || !w_dev || !y_dev) return set_error(DISTDL_ERR_NULL, "conv_fwd: null argument");
  int rc = check_conv_plan(plan);
  if (rc) return rc;
  const bool bf16 = plan->dtype == DISTDL_BF16;
  const uintptr_t esz = bf16 ? 2 : 4;
  for (int w = 0; w < plan->n_workers; ++w)
    if (!y_dev[w] || (uintptr_t)y_dev[w] % esz) return set_error(DISTDL_ERR_NULL, "conv_fwd: y of worker %d null or misaligned", w);
  if (halo) {
    if ((rc = run_halo(plan, false, plan->tab_x, x_bufs_dev, st))) return rc;  // x <- H x
  } else {
    if ((rc = plan_prepare_device(plan))) return rc;
    for (int w = 0; w < plan->n_workers; ++w)
      if (!x_bufs_dev[w] || (uintptr_t)x_bufs_dev[w] % esz) return set_error(DISTDL_ERR_NULL, "conv_fwd: x of worker %d null or misaligned", w);
  }
  if ((rc = plan->tab_x.upload((const void* const*)x_bufs_dev, plan->n_workers, st))) return rc;
  if ((rc = plan->tab_y.upload((const void* const*)y_dev, plan->n_workers, st))) return rc;
  // 16-byte pieces on both sides: the matrix-core kernels load x in them and store y in them
  bool xvec = true;
  for (int w = 0; w < plan->n_workers; ++w) xvec &= (uintptr_t)x_bufs_dev[w] % 16 == 0 && (uintptr_t)y_dev[w] % 16 == 0;
  const bool aligned = xvec && (uintptr_t)w_dev % 16 == 0;
  if (corr16_fwd_supported(plan, xvec)) {  // few channels: 16 x 16 tiles
    if ((rc = conv_fwd16(plan, (const float*)w_dev, (const float*)bias_dev, xvec, st))) return rc;
    DISTDL_HIP_TRY(hipGetLastError());
    return DISTDL_OK;
  }
  if (aligned && corr_mfma_supported(plan)) {
    if ((rc = conv_fwd_mfma(plan, w_dev, bias_dev, st))) return rc;
    DISTDL_HIP_TRY(hipGetLastError());
    return DISTDL_OK;
  }
  if ((rc = prepare_weights(plan, w_dev, st))) return rc;
  ConvDev c = conv_params(plan);
  int64_t total = plan->n_b * plan->max_out_cells * c.co;
  dim3 grid((unsigned)((total + 255) / 256), plan->n_workers);
  ProfScope prof("conv_fwd_direct", st);
  if (bf16)
    hipLaunchKernelGGL(conv_fwd_direct_kernel<uint16_t>, grid, dim3(256), 0, st, plan->d_workers, plan->tab_x.dev,
                       plan->d_wt, (const uint16_t*)bias_dev, plan->tab_y.dev, c);
  else
    hipLaunchKernelGGL(conv_fwd_direct_kernel<float>, grid, dim3(256), 0, st, plan->d_workers, plan->tab_x.dev,
                       plan->d_wt, (const float*)bias_dev, plan->tab_y.dev, c);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

int conv_bwd_core(distdl_plan* plan, const void* const x_bufs_dev[], const void* w_dev, const void* const dy_dev[],
                  void* const dx_bufs_dev[], void* dw_dev, void* dbias_dev, void* workspace_dev, size_t workspace_bytes,
                  hipStream_t st, bool halo) {
  if (!plan || !x_bufs_dev || !w_dev || !dy_dev || !dx_bufs_dev || !dw_dev || !workspace_dev)
    return set_error(DISTDL_ERR_NULL, "conv_bwd: null argument");
  int rc = check_conv_plan(plan);
  if (rc) return rc;
  const bool bf16 = plan->dtype == DISTDL_BF16;
  const uintptr_t esz = bf16 ? 2 : 4;
  if (workspace_bytes < distdl_conv_bwd_workspace(plan) || (uintptr_t)workspace_dev % 16)
    return set_error(DISTDL_ERR_INVALID_ARG, "conv_bwd: workspace too small or misaligned (%zu < %zu)", workspace_bytes,
                     distdl_conv_bwd_workspace(plan));
  for (int w = 0; w < plan->n_workers; ++w) {
    if (!x_bufs_dev[w] || !dy_dev[w] || !dx_bufs_dev[w]) return set_error(DISTDL_ERR_NULL, "conv_bwd: worker %d has a null array", w);
    if ((uintptr_t)x_bufs_dev[w] % esz || (uintptr_t)dy_dev[w] % esz || (uintptr_t)dx_bufs_dev[w] % esz)
      return set_error(DISTDL_ERR_INVALID_ARG, "conv_bwd: misaligned array");
  }
  if ((rc = plan_prepare_device(plan))) return rc;
  if ((rc = plan->tab_x.upload(x_bufs_dev, plan->n_workers, st))) return rc;
  if ((rc = plan->tab_dy.upload(dy_dev, plan->n_workers, st))) return rc;
  if ((rc = plan->tab_dx.upload((const void* const*)dx_bufs_dev, plan->n_workers, st))) return rc;
  ConvDev c = conv_params(plan);
  bool aligned = true;  // dy is loaded, dx^ stored in 16-byte pieces
  for (int w = 0; w < plan->n_workers; ++w) aligned &= (uintptr_t)dy_dev[w] % 16 == 0 && (uintptr_t)dx_bufs_dev[w] % 16 == 0;
  const bool data_mfma = aligned && corr_mfma_supported(plan);
  bool vec16 = aligned && plan->n_ci % 4 == 0 && plan->n_co % 4 == 0;
  for (int w = 0; w < plan->n_workers; ++w) vec16 &= (uintptr_t)x_bufs_dev[w] % 16 == 0;
  const bool wgrad16 = wgrad16_supported(plan, vec16);
  const bool wgrad_mfma = !wgrad16 && wgrad_mfma_supported(plan) && plan->n_workers * wgrad_chunks(plan) <= 65535 &&
                          (!bf16 || vec16);
  // [dConv]* with respect to x, into the whole padded buffers
  int64_t total = plan->n_b * plan->max_buf_cells * c.ci;
  if (corr16_bwd_supported(plan, aligned)) {
    if ((rc = conv_bwd_data16(plan, (const float*)w_dev, aligned, st))) return rc;
  } else if (data_mfma) {
    if ((rc = conv_bwd_data_mfma(plan, w_dev, st))) return rc;
  } else {
    if ((rc = prepare_weights(plan, w_dev, st))) return rc;
    ProfScope prof("conv_bwd_data_direct", st);
    const dim3 dgrid((unsigned)((total + 255) / 256), plan->n_workers);
    if (bf16)
      hipLaunchKernelGGL(conv_bwd_data_direct_kernel<uint16_t>, dgrid, dim3(256), 0, st, plan->d_workers,
                         plan->tab_dy.dev, plan->d_wt, plan->tab_dx.dev, c);
    else
      hipLaunchKernelGGL(conv_bwd_data_direct_kernel<float>, dgrid, dim3(256), 0, st, plan->d_workers,
                         plan->tab_dy.dev, plan->d_wt, plan->tab_dx.dev, c);
  }
  // [dConv]* with respect to w and b, then R over the workers
  int nchunks = wgrad16 ? wgrad16_chunks(plan, vec16) : wgrad_mfma ? wgrad_chunks(plan) : direct_chunks(plan);
  int nw = c.taps * c.ci * c.co + c.co;
  if (wgrad16) {
    if ((rc = conv_wgrad16(plan, (float*)workspace_dev, vec16, st))) return rc;
  } else if (wgrad_mfma) {
    if ((rc = conv_wgrad_mfma(plan, (float*)workspace_dev, st))) return rc;
  } else {
    ProfScope prof("conv_bwd_weight_direct", st);
    const dim3 wgrid((unsigned)((nw + 255) / 256), nchunks, plan->n_workers);
    if (bf16)
      hipLaunchKernelGGL(conv_bwd_weight_direct_kernel<uint16_t>, wgrid, dim3(256), 0, st, plan->d_workers,
                         plan->tab_x.dev, plan->tab_dy.dev, (float*)workspace_dev, c, nchunks);
    else
      hipLaunchKernelGGL(conv_bwd_weight_direct_kernel<float>, wgrid, dim3(256), 0, st, plan->d_workers,
                         plan->tab_x.dev, plan->tab_dy.dev, (float*)workspace_dev, c, nchunks);
  }
  {
    ProfScope prof("conv_reduce_dw", st);
    const float* part = (const float*)workspace_dev;
    const int nparts = nchunks * plan->n_workers;
    if (nw <= 8192 && bf16)
      hipLaunchKernelGGL((conv_reduce_dw_kernel<16, uint16_t>), dim3((unsigned)((nw + 15) / 16)), dim3(256), 0, st, part,
                         nparts, (uint16_t*)dw_dev, (uint16_t*)dbias_dev, c);
    else if (nw <= 8192)
      hipLaunchKernelGGL((conv_reduce_dw_kernel<16, float>), dim3((unsigned)((nw + 15) / 16)), dim3(256), 0, st, part,
                         nparts, (float*)dw_dev, (float*)dbias_dev, c);
    else if (bf16)
      hipLaunchKernelGGL((conv_reduce_dw_kernel<64, uint16_t>), dim3((unsigned)((nw + 63) / 64)), dim3(256), 0, st, part,
                         nparts, (uint16_t*)dw_dev, (uint16_t*)dbias_dev, c);
    else
      hipLaunchKernelGGL((conv_reduce_dw_kernel<64, float>), dim3((unsigned)((nw + 63) / 64)), dim3(256), 0, st, part,
                         nparts, (float*)dw_dev, (float*)dbias_dev, c);
  }
  DISTDL_HIP_TRY(hipGetLastError());
  // dx <- H* dx
  return halo ? run_halo(plan, true, plan->tab_dx, dx_bufs_dev, st) : DISTDL_OK;
}

}  // namespace distdl
