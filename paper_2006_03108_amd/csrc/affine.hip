// Partitioned affine layer (Sec. 4 "Dense layers", Forward / Adjoint Affine
// Algorithms) on a P_fo x P_fi weight partition held in one HBM.
//
//   forward   y_i  = sum_j x_j W_ij^T + b_i        B x along P_fo is a shared
//                                                  read; R along P_fi is the
//                                                  continuation of the sum
//   adjoint   dW_ij = dy_i^T x_j,  db_i = sum_n dy_i,  dx_j = sum_i dy_i W_ij
#include <algorithm>

#include <cstring>

#include "common.h"
#include "gemm_mfma.h"
#include "profile.h"

struct distdl_affine_plan {
  int64_t n_b = 0, n_fi = 0, n_fo = 0;
  int P_fo = 1, P_fi = 1;
  distdl_dtype dtype = DISTDL_F32;
  std::vector<int64_t> fo_start, fo_size, fi_start, fi_size;
  int64_t max_fo = 0, max_fi = 0;
  distdl::PtrTable tab_x, tab_W, tab_b, tab_y, tab_dy, tab_dx, tab_dW, tab_db;
  int32_t* d_sizes = nullptr;  // [P_fo fo sizes][P_fi fi sizes]
  distdl::DevArray<distdl::GemmBlock> g_fwd, g_dx, g_dw;
  distdl::DevArray<distdl::ColsumBlock> g_db;
  float* d_partial = nullptr;  // fp32 partial tiles of K-split GEMM launches
  size_t partial_floats = 0;
};

namespace distdl {

// ---- reference-shaped kernels (any sizes) -----------------------------------

// grid: (ceil(n_b * max_fo / 256), P_fo)
template <class T>
__global__ __launch_bounds__(256) void affine_fwd_direct_kernel(void* const* x, void* const* W, void* const* b,
                                                                void* const* y, const int32_t* sizes, int n_b,
                                                                int P_fo, int P_fi) {
  const int i = blockIdx.y;
  const int fo = sizes[i];
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)n_b * fo) return;
  int f = (int)(idx % fo);
  int n = (int)(idx / fo);
  float acc = 0.f;
  for (int j = 0; j < P_fi; ++j) {  // R over j, ascending
    const int fi = sizes[P_fo + j];
    const T* xj = (const T*)x[j] + (size_t)n * fi;
    const T* wr = (const T*)W[i * P_fi + j] + (size_t)f * fi;
    float part = 0.f;
    for (int k = 0; k < fi; ++k) part = fmaf(ld(xj, k), ld(wr, k), part);
    if (j == 0 && b && b[i]) part += ld((const T*)b[i], f);  // bias lives on column j = 0
    acc += part;
  }
  st((T*)y[i], idx, acc);
}

// grid: (ceil(n_b * max_fi / 256), P_fi)
template <class T>
__global__ __launch_bounds__(256) void affine_bwd_x_direct_kernel(void* const* dy, void* const* W, void* const* dx,
                                                                  const int32_t* sizes, int n_b, int P_fo, int P_fi) {
  const int j = blockIdx.y;
  const int fi = sizes[P_fo + j];
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)n_b * fi) return;
  int k = (int)(idx % fi);
  int n = (int)(idx / fi);
  float acc = 0.f;
  for (int i = 0; i < P_fo; ++i) {  // R over i, ascending
    const int fo = sizes[i];
    const T* dyi = (const T*)dy[i] + (size_t)n * fo;
    const T* w = (const T*)W[i * P_fi + j] + k;
    float part = 0.f;
    for (int f = 0; f < fo; ++f) part = fmaf(ld(dyi, f), ld(w, (size_t)f * fi), part);
    acc += part;
  }
  st((T*)dx[j], idx, acc);
}

// grid: (ceil(max_fo * max_fi / 16), P_fo * P_fi).  16 outputs x 16 slices of the batch per block: the layers
// that come here are small, so the sum over the batch is split to get enough threads; the slices are added
// in ascending order.
template <class T>
__global__ __launch_bounds__(256) void affine_bwd_w_direct_kernel(void* const* dy, void* const* x, void* const* dW,
                                                                  const int32_t* sizes, int n_b, int P_fo, int P_fi) {
  const int i = blockIdx.y / P_fi, j = blockIdx.y % P_fi;
  const int fo = sizes[i], fi = sizes[P_fo + j];
  const int o = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int64_t idx = (int64_t)blockIdx.x * 16 + o;
  const bool live = idx < (int64_t)fo * fi;
  __shared__ float red[16][16];
  float acc = 0.f;
  if (live) {
    const int k = (int)(idx % fi), f = (int)(idx / fi);
    const T* dyi = (const T*)dy[i];
    const T* xj = (const T*)x[j];
    for (int n = sl; n < n_b; n += 16) acc = fmaf(ld(dyi, (size_t)n * fo + f), ld(xj, (size_t)n * fi + k), acc);
  }
  red[sl][o] = acc;
  __syncthreads();
  if (sl != 0 || !live) return;
  float sum = red[0][o];
#pragma unroll
  for (int t = 1; t < 16; ++t) sum += red[t][o];
  st((T*)dW[blockIdx.y], idx, sum);
}

// grid: (ceil(max_fo / 16), P_fo), same 16 x 16 split
template <class T>
__global__ __launch_bounds__(256) void affine_bwd_b_direct_kernel(void* const* dy, void* const* db,
                                                                  const int32_t* sizes, int n_b) {
  const int i = blockIdx.y;
  const int fo = sizes[i];
  const int o = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int f = blockIdx.x * 16 + o;
  const bool live = f < fo && db[i];
  __shared__ float red[16][16];
  float acc = 0.f;
  if (live) {
    const T* dyi = (const T*)dy[i];
    for (int n = sl; n < n_b; n += 16) acc += ld(dyi, (size_t)n * fo + f);
  }
  red[sl][o] = acc;
  __syncthreads();
  if (sl != 0 || !live) return;
  float sum = red[0][o];
#pragma unroll
  for (int t = 1; t < 16; ++t) sum += red[t][o];
  st((T*)db[i], f, sum);
}

static int check_ptrs(const void* const* p, int n, size_t esz, const char* what, bool nullable = false) {
  for (int i = 0; i < n; ++i) {
    if (!p[i] && !nullable) return set_error(DISTDL_ERR_NULL, "affine: %s[%d] is null", what, i);
    if ((uintptr_t)p[i] % esz) return set_error(DISTDL_ERR_INVALID_ARG, "affine: %s[%d] is misaligned", what, i);
  }
  return DISTDL_OK;
}

static int prepare(distdl_affine_plan* p) {
  if (p->d_sizes) return DISTDL_OK;
  std::vector<int32_t> s;
  for (int64_t v : p->fo_size) s.push_back((int32_t)v);
  for (int64_t v : p->fi_size) s.push_back((int32_t)v);
  DISTDL_HIP_TRY(hipMalloc((void**)&p->d_sizes, s.size() * sizeof(int32_t)));
  DISTDL_HIP_TRY(hipMemcpy(p->d_sizes, s.data(), s.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  return DISTDL_OK;
}

template <class T>
static void fwd_direct(distdl_affine_plan* p, bool has_b, hipStream_t st_) {
  dim3 grid((unsigned)((p->n_b * p->max_fo + 255) / 256), p->P_fo);
  ProfScope prof("affine_fwd_direct", st_);
  hipLaunchKernelGGL(affine_fwd_direct_kernel<T>, grid, dim3(256), 0, st_, p->tab_x.dev, p->tab_W.dev,
                     has_b ? p->tab_b.dev : (void**)nullptr, p->tab_y.dev, p->d_sizes, (int)p->n_b, p->P_fo, p->P_fi);
}

template <class T>
static void bwd_direct(distdl_affine_plan* p, bool has_db, hipStream_t st_) {
  ProfScope prof("affine_bwd_direct", st_);
  hipLaunchKernelGGL(affine_bwd_x_direct_kernel<T>, dim3((unsigned)((p->n_b * p->max_fi + 255) / 256), p->P_fi),
                     dim3(256), 0, st_, p->tab_dy.dev, p->tab_W.dev, p->tab_dx.dev, p->d_sizes, (int)p->n_b, p->P_fo,
                     p->P_fi);
  hipLaunchKernelGGL(affine_bwd_w_direct_kernel<T>,
                     dim3((unsigned)((p->max_fo * p->max_fi + 15) / 16), p->P_fo * p->P_fi), dim3(256), 0, st_,
                     p->tab_dy.dev, p->tab_x.dev, p->tab_dW.dev, p->d_sizes, (int)p->n_b, p->P_fo, p->P_fi);
  if (has_db)
    hipLaunchKernelGGL(affine_bwd_b_direct_kernel<T>, dim3((unsigned)((p->max_fo + 15) / 16), p->P_fo), dim3(256), 0,
                       st_, p->tab_dy.dev, p->tab_db.dev, p->d_sizes, (int)p->n_b);
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_affine_plan_create(distdl_affine_plan** out, int64_t n_b, int64_t n_fi, int64_t n_fo, int P_fo, int P_fi,
                              distdl_dtype dtype) {
  if (!out) return set_error(DISTDL_ERR_NULL, "affine_plan_create: null argument");
  *out = nullptr;
  if (n_b < 1 || n_fi < 1 || n_fo < 1 || P_fo < 1 || P_fi < 1)
    return set_error(DISTDL_ERR_INVALID_ARG, "affine_plan_create: sizes must be >= 1");
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  if (n_fo < P_fo || n_fi < P_fi)
    return set_error(DISTDL_ERR_EMPTY_PARTITION, "affine: %lld x %lld features over %d x %d workers", (long long)n_fo,
                     (long long)n_fi, P_fo, P_fi);
  if (n_b * std::max(n_fi, n_fo) >= (int64_t(1) << 31) || n_fi * n_fo >= (int64_t(1) << 40))
    return set_error(DISTDL_ERR_UNSUPPORTED, "affine: problem too large");
  distdl_affine_plan* p = new (std::nothrow) distdl_affine_plan();
  if (!p) return set_error(DISTDL_ERR_NOMEM, "out of host memory");
  p->n_b = n_b;
  p->n_fi = n_fi;
  p->n_fo = n_fo;
  p->P_fo = P_fo;
  p->P_fi = P_fi;
  p->dtype = dtype;
  auto split = [](int64_t len, int parts, std::vector<int64_t>& start, std::vector<int64_t>& size, int64_t& mx) {
    int64_t at = 0;
    for (int r = 0; r < parts; ++r) {
      int64_t z = len / parts + (r < len % parts ? 1 : 0);
      start.push_back(at);
      size.push_back(z);
      at += z;
      mx = std::max(mx, z);
    }
  };
  split(n_fo, P_fo, p->fo_start, p->fo_size, p->max_fo);
  split(n_fi, P_fi, p->fi_start, p->fi_size, p->max_fi);
  *out = p;
  return DISTDL_OK;
}

int distdl_affine_plan_destroy(distdl_affine_plan* p) {
  if (!p) return DISTDL_OK;
  for (PtrTable* t : {&p->tab_x, &p->tab_W, &p->tab_b, &p->tab_y, &p->tab_dy, &p->tab_dx, &p->tab_dW, &p->tab_db})
    t->release();
  if (p->d_sizes) (void)hipFree(p->d_sizes);
  p->g_fwd.release();
  p->g_dx.release();
  p->g_dw.release();
  p->g_db.release();
  if (p->d_partial) (void)hipFree(p->d_partial);
  delete p;
  return DISTDL_OK;
}

static int ensure_partial(distdl_affine_plan* p, size_t floats) {
  if (floats <= p->partial_floats) return DISTDL_OK;
  if (p->d_partial) (void)hipFree(p->d_partial);
  p->d_partial = nullptr;
  p->partial_floats = 0;
  DISTDL_HIP_TRY(hipMalloc((void**)&p->d_partial, floats * sizeof(float)));
  p->partial_floats = floats;
  return DISTDL_OK;
}

int distdl_affine_fwd(distdl_affine_plan* p, const void* const x_dev[], const void* const W_dev[],
                      const void* const b_dev[], void* const y_dev[], void* stream) {
  if (!p || !x_dev || !W_dev || !y_dev) return set_error(DISTDL_ERR_NULL, "affine_fwd: null argument");
  const size_t esz = dtype_size(p->dtype);
  hipStream_t st_ = (hipStream_t)stream;
  int rc;
  if ((rc = check_ptrs(x_dev, p->P_fi, esz, "x")) || (rc = check_ptrs(W_dev, p->P_fo * p->P_fi, esz, "W")) ||
      (rc = check_ptrs((const void* const*)y_dev, p->P_fo, esz, "y")))
    return rc;
  if (b_dev && (rc = check_ptrs(b_dev, p->P_fo, esz, "b", true))) return rc;
  if ((rc = prepare(p))) return rc;
  const bool bf16 = p->dtype == DISTDL_BF16;
  {  // matrix-core path: y_i = sum_j x_j W_ij^T + b_i, the sum over j inside the K loop
    std::vector<GemmBlock> blocks(p->P_fo);
    for (int i = 0; i < p->P_fo; ++i) {
      GemmBlock& g = blocks[i];
      std::memset(&g, 0, sizeof g);
      g.M = (int32_t)p->n_b;
      g.N = g.ldc = (int32_t)p->fo_size[i];
      g.c = y_dev[i];
      g.bias = b_dev ? b_dev[i] : nullptr;
      g.nseg = std::min(p->P_fi, kGemmMaxSeg + 1);
      for (int j = 0; j < p->P_fi && j < kGemmMaxSeg; ++j)
        g.seg[j] = GemmSeg{x_dev[j], W_dev[i * p->P_fi + j], (int32_t)p->fi_size[j], (int32_t)p->fi_size[j],
                           (int32_t)p->fi_size[j], 0};
    }
    if (gemm_mfma_usable(blocks, bf16, true, true)) {
      const int ns = gemm_mfma_splits(blocks, bf16, true);
      if ((rc = p->g_fwd.upload(blocks, st_)) || (rc = ensure_partial(p, gemm_mfma_partial_floats(blocks, ns)))) return rc;
      if ((rc = launch_gemm_mfma(p->g_fwd.dev, blocks, bf16, true, true, ns, p->d_partial, "affine_fwd_mfma", st_))) return rc;
      DISTDL_HIP_TRY(hipGetLastError());
      return DISTDL_OK;
    }
  }
  if ((rc = p->tab_x.upload(x_dev, p->P_fi, st_)) || (rc = p->tab_W.upload(W_dev, p->P_fo * p->P_fi, st_)) ||
      (rc = p->tab_y.upload((const void* const*)y_dev, p->P_fo, st_)))
    return rc;
  if (b_dev && (rc = p->tab_b.upload(b_dev, p->P_fo, st_))) return rc;
  if (p->dtype == DISTDL_F32) fwd_direct<float>(p, b_dev != nullptr, st_);
  else fwd_direct<uint16_t>(p, b_dev != nullptr, st_);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

int distdl_affine_bwd(distdl_affine_plan* p, const void* const x_dev[], const void* const W_dev[],
                      const void* const dy_dev[], void* const dx_dev[], void* const dW_dev[], void* const db_dev[],
                      void* stream) {
  if (!p || !x_dev || !W_dev || !dy_dev || !dx_dev || !dW_dev) return set_error(DISTDL_ERR_NULL, "affine_bwd: null argument");
  const size_t esz = dtype_size(p->dtype);
  hipStream_t st_ = (hipStream_t)stream;
  int rc;
  if ((rc = check_ptrs(x_dev, p->P_fi, esz, "x")) || (rc = check_ptrs(W_dev, p->P_fo * p->P_fi, esz, "W")) ||
      (rc = check_ptrs(dy_dev, p->P_fo, esz, "dy")) || (rc = check_ptrs((const void* const*)dx_dev, p->P_fi, esz, "dx")) ||
      (rc = check_ptrs((const void* const*)dW_dev, p->P_fo * p->P_fi, esz, "dW")))
    return rc;
  if (db_dev && (rc = check_ptrs((const void* const*)db_dev, p->P_fo, esz, "db", true))) return rc;
  if ((rc = prepare(p))) return rc;
  const bool bf16 = p->dtype == DISTDL_BF16;
  {  // matrix-core path
    std::vector<GemmBlock> bx(p->P_fi), bw((size_t)p->P_fo * p->P_fi);
    std::vector<ColsumBlock> bb(p->P_fo);
    for (int j = 0; j < p->P_fi; ++j) {  // dx_j = sum_i dy_i W_ij
      GemmBlock& g = bx[j];
      std::memset(&g, 0, sizeof g);
      g.M = (int32_t)p->n_b;
      g.N = g.ldc = (int32_t)p->fi_size[j];
      g.c = dx_dev[j];
      g.nseg = std::min(p->P_fo, kGemmMaxSeg + 1);
      for (int i = 0; i < p->P_fo && i < kGemmMaxSeg; ++i)
        g.seg[i] = GemmSeg{dy_dev[i], W_dev[i * p->P_fi + j], (int32_t)p->fo_size[i], (int32_t)p->fo_size[i],
                           (int32_t)p->fi_size[j], 0};
    }
    for (int i = 0; i < p->P_fo; ++i) {
      for (int j = 0; j < p->P_fi; ++j) {  // dW_ij = dy_i^T x_j
        GemmBlock& g = bw[(size_t)i * p->P_fi + j];
        std::memset(&g, 0, sizeof g);
        g.M = (int32_t)p->fo_size[i];
        g.N = g.ldc = (int32_t)p->fi_size[j];
        g.c = dW_dev[i * p->P_fi + j];
        g.nseg = 1;
        g.seg[0] = GemmSeg{dy_dev[i], x_dev[j], (int32_t)p->n_b, (int32_t)p->fo_size[i], (int32_t)p->fi_size[j], 0};
      }
      bb[i] = ColsumBlock{dy_dev[i], db_dev ? db_dev[i] : nullptr, (int32_t)p->n_b, (int32_t)p->fo_size[i]};
    }
    if (gemm_mfma_usable(bx, bf16, true, false) && gemm_mfma_usable(bw, bf16, false, false)) {
      const int nsx = gemm_mfma_splits(bx, bf16, true), nsw = gemm_mfma_splits(bw, bf16, false);
      if ((rc = p->g_dx.upload(bx, st_)) || (rc = p->g_dw.upload(bw, st_)) ||
          (rc = ensure_partial(p, std::max(gemm_mfma_partial_floats(bx, nsx), gemm_mfma_partial_floats(bw, nsw)))))
        return rc;
      // the two launches use the partial buffer one after the other on the stream
      if (db_dev && (rc = p->g_db.upload(bb, st_))) return rc;
      // the bias gradient rides in the weight-gradient launch when its kernel can carry it (it reads the same dy_i)
      GemmColsum cs{p->g_db.dev, p->P_fo, (int)p->max_fo, false};
      bool db_aligned = db_dev != nullptr;  // the fused sums store four features (8 or 16 bytes) at a time
      for (int i = 0; db_dev && i < p->P_fo; ++i) db_aligned &= (uintptr_t)db_dev[i] % (bf16 ? 8 : 16) == 0;
      // dx and dW on one stream, one after the other.  Measured: dW on a side stream between a fork and a join event
      // (its 32 KB workgroups fit next to the 128 KB ones of dx) makes the step slower, eager and from a graph
      // (72 against 61 us at 256 x 4096 x 4096): both launches are bound by what a compute unit can take in.
      rc = launch_gemm_mfma(p->g_dx.dev, bx, bf16, true, false, nsx, p->d_partial, "affine_bwd_x_mfma", st_);
      if (!rc)
        rc = launch_gemm_mfma(p->g_dw.dev, bw, bf16, false, false, nsw, p->d_partial, "affine_bwd_w_mfma", st_,
                              db_aligned ? &cs : nullptr);
      if (!rc && db_dev && !cs.done) launch_colsum(p->g_db.dev, p->P_fo, (int)p->max_fo, bf16, st_);
      if (rc) return rc;
      DISTDL_HIP_TRY(hipGetLastError());
      return DISTDL_OK;
    }
  }
  if ((rc = p->tab_x.upload(x_dev, p->P_fi, st_)) || (rc = p->tab_W.upload(W_dev, p->P_fo * p->P_fi, st_)) ||
      (rc = p->tab_dy.upload(dy_dev, p->P_fo, st_)) ||
      (rc = p->tab_dx.upload((const void* const*)dx_dev, p->P_fi, st_)) ||
      (rc = p->tab_dW.upload((const void* const*)dW_dev, p->P_fo * p->P_fi, st_)))
    return rc;
  if (db_dev && (rc = p->tab_db.upload((const void* const*)db_dev, p->P_fo, st_))) return rc;
  if (p->dtype == DISTDL_F32) bwd_direct<float>(p, db_dev != nullptr, st_);
  else bwd_direct<uint16_t>(p, db_dev != nullptr, st_);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

}  // extern "C"
