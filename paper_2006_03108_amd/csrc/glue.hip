// Point-wise, pooling, repartition and loss glue of the example network (Sec. 4 "point-wise layers" and
// "Sparse layers": Forward / Adjoint Pooling Algorithms; Sec. 3 "Generalized all-to-all"; Sec. 5 / App. C).
// fp32, channels-last.  These calls are small and latency-bound; they exist so that a whole partitioned
// network step can run through the library.
#include <algorithm>
#include <vector>

#include "common.h"
#include "profile.h"

namespace distdl {

int plan_prepare_device(distdl_plan* p);
int run_halo(distdl_plan* p, bool adjoint, PtrTable& tab, void* const* bufs_host, hipStream_t st);

constexpr int kEwArrays = 16;
struct EwArgs {
  const float* a[kEwArrays];
  const float* b[kEwArrays];
  float* out[kEwArrays];
  int64_t count[kEwArrays];
  int32_t n;
  float scale;
};

// mode 0: out = max(a, 0); mode 1: out = a > 0 ? b : 0; mode 2: out = scale * (a - b)
template <int MODE>
__global__ __launch_bounds__(256) void elementwise_kernel(EwArgs e) {
  const int j = blockIdx.y;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < e.count[j]; i += stride) {
    const float a = e.a[j][i];
    if (MODE == 0) e.out[j][i] = a > 0.f ? a : 0.f;
    else if (MODE == 1) e.out[j][i] = a > 0.f ? e.b[j][i] : 0.f;
    else e.out[j][i] = e.scale * (a - e.b[j][i]);
  }
}

template <int MODE>
static int run_elementwise(const void* const a[], const void* const b[], void* const out[], const int64_t count[],
                           int n, float scale, const char* name, hipStream_t st) {
  if (!a || !out || !count || (MODE != 0 && !b)) return set_error(DISTDL_ERR_NULL, "%s: null argument", name);
  if (n < 1) return set_error(DISTDL_ERR_INVALID_ARG, "%s: n = %d", name, n);
  for (int j0 = 0; j0 < n; j0 += kEwArrays) {
    EwArgs e{};
    e.n = std::min(kEwArrays, n - j0);
    e.scale = scale;
    int64_t mx = 0;
    for (int j = 0; j < e.n; ++j) {
      if (count[j0 + j] < 0) return set_error(DISTDL_ERR_INVALID_ARG, "%s: negative count", name);
      if (count[j0 + j] > 0 && (!a[j0 + j] || !out[j0 + j] || (MODE != 0 && !b[j0 + j])))
        return set_error(DISTDL_ERR_NULL, "%s: array %d is null", name, j0 + j);
      e.a[j] = (const float*)a[j0 + j];
      e.b[j] = MODE != 0 ? (const float*)b[j0 + j] : nullptr;
      e.out[j] = (float*)out[j0 + j];
      e.count[j] = count[j0 + j];
      mx = std::max(mx, count[j0 + j]);
    }
    if (mx == 0) continue;
    dim3 grid((unsigned)std::min<int64_t>((mx + 1023) / 1024, 2048), e.n);
    ProfScope prof(name, st);
    hipLaunchKernelGGL(elementwise_kernel<MODE>, grid, dim3(256), 0, st, e);
  }
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

struct PoolDev {
  int32_t n_b, c;
  int32_t k[3], s[3], dil[3];
  FastDiv div_c4, div_s[3];  // by c / 4 and by the strides (vector kernels)
};

static PoolDev pool_params(const distdl_plan* p) {
  PoolDev d;
  d.n_b = (int32_t)p->n_b;
  d.c = (int32_t)p->n_ci;
  for (int i = 0; i < 3; ++i) {
    d.k[i] = p->ksize[i];
    d.s[i] = p->stride[i];
    d.dil[i] = p->dilation[i];
  }
  d.div_c4 = make_fastdiv((uint32_t)std::max<int64_t>(1, p->n_ci / 4));
  for (int i = 0; i < 3; ++i) d.div_s[i] = make_fastdiv((uint32_t)p->stride[i]);
  return d;
}

// Cells outside the global domain are zero padding: the mean counts them as the zeros they hold, the max
// leaves them out (the window maximum is taken over the cells of the tensor itself).
__device__ inline bool in_domain(const WorkerDev& wd, int b0, int b1, int b2) {
  return b0 >= wd.dom_lo[0] && b0 < wd.dom_hi[0] && b1 >= wd.dom_lo[1] && b1 < wd.dom_hi[1] && b2 >= wd.dom_lo[2] &&
         b2 < wd.dom_hi[2];
}

// y[n][o][c] = max over the in-domain cells of the window x^[n][origin + o*s + t*dil][c] (or the window's mean)
template <bool AVG, class T>
__global__ __launch_bounds__(256) void pool_fwd_kernel(const WorkerDev* __restrict__ workers, void* const* x_bufs,
                                                       void* const* y_bufs, PoolDev d) {
  const WorkerDev wd = workers[blockIdx.y];
  const int64_t total = (int64_t)d.n_b * wd.out[0] * wd.out[1] * wd.out[2] * d.c;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const T* __restrict__ x = (const T*)x_bufs[blockIdx.y];
  T* __restrict__ y = (T*)y_bufs[blockIdx.y];
  int c = (int)(idx % d.c);
  int64_t r = idx / d.c;
  int o2 = (int)(r % wd.out[2]); r /= wd.out[2];
  int o1 = (int)(r % wd.out[1]); r /= wd.out[1];
  int o0 = (int)(r % wd.out[0]);
  int n = (int)(r / wd.out[0]);
  const int64_t s2 = d.c, s1 = (int64_t)wd.buf[2] * s2, s0 = (int64_t)wd.buf[1] * s1, sn = (int64_t)wd.buf[0] * s0;
  float best = 0.f, sum = 0.f;
  bool first = true;
  for (int t0 = 0; t0 < d.k[0]; ++t0)
    for (int t1 = 0; t1 < d.k[1]; ++t1)
      for (int t2 = 0; t2 < d.k[2]; ++t2) {
        const int b0 = wd.origin[0] + o0 * d.s[0] + t0 * d.dil[0], b1 = wd.origin[1] + o1 * d.s[1] + t1 * d.dil[1],
                  b2 = wd.origin[2] + o2 * d.s[2] + t2 * d.dil[2];
        const float v = ld(x, n * sn + b0 * s0 + b1 * s1 + b2 * s2 + c);
        sum += v;  // row-major tap order; padding cells hold zeros
        if (!in_domain(wd, b0, b1, b2)) continue;  // padding never wins the max
        if (first || v > best) best = v;
        first = false;
      }
  st(y, idx, AVG ? sum / (float)(d.k[0] * d.k[1] * d.k[2]) : best);
}

// [dPool]* in gather form over the whole padded buffer: a cell receives dy[o] from every window o that
// contains it and whose first maximum (row-major tap order) it is.
// For the mean every window that contains the cell contributes dy[o] / window size.
template <bool AVG, class T>
__global__ __launch_bounds__(256) void pool_bwd_kernel(const WorkerDev* __restrict__ workers, void* const* x_bufs,
                                                       void* const* dy_bufs, void* const* dx_bufs, PoolDev d) {
  const WorkerDev wd = workers[blockIdx.y];
  const int64_t total = (int64_t)d.n_b * wd.buf[0] * wd.buf[1] * wd.buf[2] * d.c;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const T* __restrict__ x = AVG ? nullptr : (const T*)x_bufs[blockIdx.y];
  const T* __restrict__ dy = (const T*)dy_bufs[blockIdx.y];
  T* __restrict__ dx = (T*)dx_bufs[blockIdx.y];
  int c = (int)(idx % d.c);
  int64_t r = idx / d.c;
  int c2 = (int)(r % wd.buf[2]); r /= wd.buf[2];
  int c1 = (int)(r % wd.buf[1]); r /= wd.buf[1];
  int c0 = (int)(r % wd.buf[0]);
  int n = (int)(r / wd.buf[0]);
  const int64_t s2 = d.c, s1 = (int64_t)wd.buf[2] * s2, s0 = (int64_t)wd.buf[1] * s1, sn = (int64_t)wd.buf[0] * s0;
  const int64_t so2 = d.c, so1 = (int64_t)wd.out[2] * so2, so0 = (int64_t)wd.out[1] * so1, son = (int64_t)wd.out[0] * so0;
  float acc = 0.f;
  int tap = 0;
  for (int t0 = 0; t0 < d.k[0]; ++t0)
    for (int t1 = 0; t1 < d.k[1]; ++t1)
      for (int t2 = 0; t2 < d.k[2]; ++t2, ++tap) {
        const int q0 = c0 - wd.origin[0] - t0 * d.dil[0], q1 = c1 - wd.origin[1] - t1 * d.dil[1],
                  q2 = c2 - wd.origin[2] - t2 * d.dil[2];
        if (q0 < 0 || q1 < 0 || q2 < 0 || q0 % d.s[0] || q1 % d.s[1] || q2 % d.s[2]) continue;
        const int o0 = q0 / d.s[0], o1 = q1 / d.s[1], o2 = q2 / d.s[2];
        if (o0 >= wd.out[0] || o1 >= wd.out[1] || o2 >= wd.out[2]) continue;
        if (AVG) {
          acc += ld(dy, n * son + o0 * so0 + o1 * so1 + o2 * so2 + c);
          continue;
        }
        // is this cell (tap index `tap`) the first maximum of window o?
        float best = 0.f;
        int arg = -1, u = 0;
        for (int u0 = 0; u0 < d.k[0]; ++u0)
          for (int u1 = 0; u1 < d.k[1]; ++u1)
            for (int u2 = 0; u2 < d.k[2]; ++u2, ++u) {
              const int b0 = wd.origin[0] + o0 * d.s[0] + u0 * d.dil[0], b1 = wd.origin[1] + o1 * d.s[1] + u1 * d.dil[1],
                        b2 = wd.origin[2] + o2 * d.s[2] + u2 * d.dil[2];
              if (!in_domain(wd, b0, b1, b2)) continue;
              const float v = ld(x, n * sn + b0 * s0 + b1 * s1 + b2 * s2 + c);
              if (arg < 0 || v > best) best = v, arg = u;
            }
        if (arg == tap) acc += ld(dy, n * son + o0 * so0 + o1 * so1 + o2 * so2 + c);
      }
  st(dx, idx, AVG ? acc / (float)(d.k[0] * d.k[1] * d.k[2]) : acc);
}

// Faster forms for channel counts that are multiples of 4 and 16-byte aligned buffers: a thread owns four
// channels of one cell (one 16-byte access per tap).
// streaming accesses for data that is touched once (windows that do not overlap)
__device__ inline void nt_store4(float4* p, float4 v) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, (f32x4*)p);
}
__device__ inline float4 nt_load4(const float4* p) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const f32x4 v = __builtin_nontemporal_load((const f32x4*)p);
  return make_float4(v[0], v[1], v[2], v[3]);
}

template <bool AVG, bool STREAM>
__global__ __launch_bounds__(256) void pool_fwd_vec_kernel(const WorkerDev* __restrict__ workers,
                                                           const FastDiv* __restrict__ divs, void* const* x_bufs,
                                                           void* const* y_bufs, PoolDev d) {
  const WorkerDev wd = workers[blockIdx.y];
  const FastDiv div_o1 = divs[blockIdx.y * 4 + 2], div_o2 = divs[blockIdx.y * 4 + 3];
  const int c4 = d.c >> 2;
  const int64_t total = (int64_t)d.n_b * wd.out[0] * wd.out[1] * wd.out[2] * c4;  // < 2^32 (host check)
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  const float4* __restrict__ x = (const float4*)x_bufs[blockIdx.y];
  float4* __restrict__ y = (float4*)y_bufs[blockIdx.y];
  uint32_t r = fd_div(idx, d.div_c4);
  const int c = (int)(idx - r * c4);
  uint32_t q = fd_div(r, div_o2);
  const int o2 = (int)(r - q * wd.out[2]);
  r = fd_div(q, div_o1);
  const int o1 = (int)(q - r * wd.out[1]);
  const int n = (int)(r / (uint32_t)wd.out[0]), o0 = (int)(r - (uint32_t)n * wd.out[0]);
  const int64_t s2 = c4, s1 = (int64_t)wd.buf[2] * s2, s0 = (int64_t)wd.buf[1] * s1, sn = (int64_t)wd.buf[0] * s0;
  float4 best = make_float4(0.f, 0.f, 0.f, 0.f), sum = best;
  bool first = true;
  for (int t0 = 0; t0 < d.k[0]; ++t0)
    for (int t1 = 0; t1 < d.k[1]; ++t1)
      for (int t2 = 0; t2 < d.k[2]; ++t2) {
        const int b0 = wd.origin[0] + o0 * d.s[0] + t0 * d.dil[0], b1 = wd.origin[1] + o1 * d.s[1] + t1 * d.dil[1],
                  b2 = wd.origin[2] + o2 * d.s[2] + t2 * d.dil[2];
        const float4* xp = x + n * sn + b0 * s0 + b1 * s1 + b2 * s2 + c;
        const float4 v = STREAM ? nt_load4(xp) : *xp;
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;  // row-major tap order; padding cells hold zeros
        if (!AVG && !in_domain(wd, b0, b1, b2)) continue;  // padding never wins the max
        if (first || v.x > best.x) best.x = v.x;
        if (first || v.y > best.y) best.y = v.y;
        if (first || v.z > best.z) best.z = v.z;
        if (first || v.w > best.w) best.w = v.w;
        first = false;
      }
  const float inv = (float)(d.k[0] * d.k[1] * d.k[2]);
  y[idx] = AVG ? make_float4(sum.x / inv, sum.y / inv, sum.z / inv, sum.w / inv) : best;
}

// [dPool]* for windows that do not overlap (stride >= kernel extent, no dilation), in two kernels that
// together write every cell of dx once.  pool_bwd_window_kernel: a thread owns one window (four channels):
// it reads the window once, finds the first maximum per channel (the mean needs no read) and writes every tap
// of the window, dy or zero (dy / window size for the mean).  pool_bwd_uncovered_kernel: the cells that lie
// in no window ("extra" input, the gaps of a stride larger than the kernel, the buffer's tail) are cleared.
template <bool AVG>
__global__ __launch_bounds__(256) void pool_bwd_window_kernel(const WorkerDev* __restrict__ workers,
                                                              const FastDiv* __restrict__ divs, void* const* x_bufs,
                                                              void* const* dy_bufs, void* const* dx_bufs, PoolDev d) {
  const WorkerDev wd = workers[blockIdx.y];
  const FastDiv div_o1 = divs[blockIdx.y * 4 + 2], div_o2 = divs[blockIdx.y * 4 + 3];
  const int c4 = d.c >> 2;
  const int64_t total = (int64_t)d.n_b * wd.out[0] * wd.out[1] * wd.out[2] * c4;  // < 2^32 (host check)
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  const float4* __restrict__ x = AVG ? nullptr : (const float4*)x_bufs[blockIdx.y];
  const float4* __restrict__ dy = (const float4*)dy_bufs[blockIdx.y];
  float4* __restrict__ dx = (float4*)dx_bufs[blockIdx.y];
  uint32_t r = fd_div(idx, d.div_c4);
  const int c = (int)(idx - r * c4);
  uint32_t q = fd_div(r, div_o2);
  const int o2 = (int)(r - q * wd.out[2]);
  r = fd_div(q, div_o1);
  const int o1 = (int)(q - r * wd.out[1]);
  const int n = (int)(r / (uint32_t)wd.out[0]), o0 = (int)(r - (uint32_t)n * wd.out[0]);
  const int64_t s2 = c4, s1 = (int64_t)wd.buf[2] * s2, s0 = (int64_t)wd.buf[1] * s1, sn = (int64_t)wd.buf[0] * s0;
  const int64_t base = n * sn + (wd.origin[0] + o0 * d.s[0]) * s0 + (wd.origin[1] + o1 * d.s[1]) * s1 +
                       (wd.origin[2] + o2 * d.s[2]) * s2 + c;
  const float4 g = nt_load4(dy + idx);
  int ax = 0, ay = 0, az = 0, aw = 0;  // tap of the first maximum, per channel
  if (!AVG) {
    float4 best = make_float4(0.f, 0.f, 0.f, 0.f);
    int u = 0;
    bool first = true;
    const int w0 = wd.origin[0] + o0 * d.s[0], w1 = wd.origin[1] + o1 * d.s[1], w2 = wd.origin[2] + o2 * d.s[2];
    for (int u0 = 0; u0 < d.k[0]; ++u0)
      for (int u1 = 0; u1 < d.k[1]; ++u1)
        for (int u2 = 0; u2 < d.k[2]; ++u2, ++u) {
          const float4 v = nt_load4(x + base + u0 * s0 + u1 * s1 + u2 * s2);
          if (!in_domain(wd, w0 + u0, w1 + u1, w2 + u2)) continue;  // padding never wins the max
          if (first || v.x > best.x) best.x = v.x, ax = u;
          if (first || v.y > best.y) best.y = v.y, ay = u;
          if (first || v.z > best.z) best.z = v.z, az = u;
          if (first || v.w > best.w) best.w = v.w, aw = u;
          first = false;
        }
  }
  const float inv = (float)(d.k[0] * d.k[1] * d.k[2]);
  const float4 share = make_float4(g.x / inv, g.y / inv, g.z / inv, g.w / inv);
  int u = 0;
  for (int u0 = 0; u0 < d.k[0]; ++u0)
    for (int u1 = 0; u1 < d.k[1]; ++u1)
      for (int u2 = 0; u2 < d.k[2]; ++u2, ++u)
        nt_store4(dx + base + u0 * s0 + u1 * s1 + u2 * s2,  // written once, not read again by this kernel
                  AVG ? share : make_float4(u == ax ? g.x : 0.f, u == ay ? g.y : 0.f, u == az ? g.z : 0.f, u == aw ? g.w : 0.f));
}

__global__ __launch_bounds__(256) void pool_bwd_uncovered_kernel(const WorkerDev* __restrict__ workers,
                                                                 const FastDiv* __restrict__ divs, void* const* dx_bufs,
                                                                 PoolDev d) {
  const WorkerDev wd = workers[blockIdx.y];
  const FastDiv div_b1 = divs[blockIdx.y * 4 + 0], div_b2 = divs[blockIdx.y * 4 + 1];
  const int c4 = d.c >> 2;
  const int64_t total = (int64_t)d.n_b * wd.buf[0] * wd.buf[1] * wd.buf[2] * c4;  // < 2^32 (host check)
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  uint32_t r = fd_div(idx, d.div_c4);
  uint32_t q = fd_div(r, div_b2);
  const int c2 = (int)(r - q * wd.buf[2]);
  r = fd_div(q, div_b1);
  const int c1 = (int)(q - r * wd.buf[1]);
  const int c0 = (int)(r % (uint32_t)wd.buf[0]);
  const int q0 = c0 - wd.origin[0], q1 = c1 - wd.origin[1], q2 = c2 - wd.origin[2];
  bool covered = q0 >= 0 && q1 >= 0 && q2 >= 0;
  if (covered) {
    const int o0 = (int)fd_div((uint32_t)q0, d.div_s[0]), o1 = (int)fd_div((uint32_t)q1, d.div_s[1]),
              o2 = (int)fd_div((uint32_t)q2, d.div_s[2]);
    covered = q0 - o0 * d.s[0] < d.k[0] && q1 - o1 * d.s[1] < d.k[1] && q2 - o2 * d.s[2] < d.k[2] && o0 < wd.out[0] &&
              o1 < wd.out[1] && o2 < wd.out[2];
  }
  if (!covered) ((float4*)dx_bufs[blockIdx.y])[idx] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// dense [n][in_size..][c] <-> bulk of the padded buffer
__global__ __launch_bounds__(256) void bulk_copy_kernel(const WorkerDev* __restrict__ workers, void* const* dense,
                                                        void* const* bufs, int n_b, int c_n, int to_bufs) {
  const WorkerDev wd = workers[blockIdx.y];
  const int64_t total = (int64_t)n_b * wd.in_size[0] * wd.in_size[1] * wd.in_size[2] * c_n;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int c = (int)(idx % c_n);
  int64_t r = idx / c_n;
  int i2 = (int)(r % wd.in_size[2]); r /= wd.in_size[2];
  int i1 = (int)(r % wd.in_size[1]); r /= wd.in_size[1];
  int i0 = (int)(r % wd.in_size[0]);
  int n = (int)(r / wd.in_size[0]);
  const int64_t off = ((((int64_t)n * wd.buf[0] + wd.bulk_off[0] + i0) * wd.buf[1] + wd.bulk_off[1] + i1) * wd.buf[2] +
                       wd.bulk_off[2] + i2) * c_n + c;
  float* d = (float*)dense[blockIdx.y];
  float* b = (float*)bufs[blockIdx.y];
  if (to_bufs) b[off] = d[idx];
  else d[idx] = b[off];
}

struct RepartDev {
  int32_t P[3];
  int32_t out_start[3][64], out_size[3][64];  // per dimension, per worker index along it
  int32_t G[3];                                // global output extents
  int32_t n_b, c, P_f;
  int32_t f_start[64], f_size[64];
};

// Features are the row-major flattening of [c][g0][g1][g2] (the framework's flatten of an n_b x n_c x ...
// tensor); feature block j is the balanced split.  to_features = 1: spatial parts -> feature parts;
// 0: the inverse permutation (its adjoint).
__global__ __launch_bounds__(256) void repartition_kernel(void* const* spatial, void* const* feats, RepartDev d,
                                                          int to_features) {
  const int j = blockIdx.y;
  const int64_t total = (int64_t)d.n_b * d.f_size[j];
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int fl = (int)(idx % d.f_size[j]);
  const int n = (int)(idx / d.f_size[j]);
  int f = d.f_start[j] + fl;
  const int g2 = f % d.G[2]; f /= d.G[2];
  const int g1 = f % d.G[1]; f /= d.G[1];
  const int g0 = f % d.G[0];
  const int c = f / d.G[0];
  const int g[3] = {g0, g1, g2};
  int r[3], loc[3], ext[3];
  for (int k = 0; k < 3; ++k) {
    r[k] = 0;
    while (r[k] + 1 < d.P[k] && g[k] >= d.out_start[k][r[k] + 1]) ++r[k];
    loc[k] = g[k] - d.out_start[k][r[k]];
    ext[k] = d.out_size[k][r[k]];
  }
  const int worker = (r[0] * d.P[1] + r[1]) * d.P[2] + r[2];
  const int64_t soff = ((((int64_t)n * ext[0] + loc[0]) * ext[1] + loc[1]) * ext[2] + loc[2]) * d.c + c;
  float* sp = (float*)spatial[worker];
  float* ft = (float*)feats[j];
  if (to_features) ft[idx] = sp[soff];
  else sp[soff] = ft[idx];
}

constexpr int kMseBlocks = 256;
struct MseArgs {
  const float* y[kEwArrays];
  const float* t[kEwArrays];
  int64_t count[kEwArrays];
  int32_t n;
};

__global__ __launch_bounds__(256) void mse_partial_kernel(MseArgs m, double* partial) {
  double acc = 0.0;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int j = 0; j < m.n; ++j)
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < m.count[j]; i += stride) {
      const double dlt = (double)m.y[j][i] - (double)m.t[j][i];
      acc += dlt * dlt;
    }
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
  __shared__ double red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void mse_final_kernel(const double* partial, int n, double inv_count, double* out) {
  double acc = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) acc += partial[i];
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
  __shared__ double red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) *out = ((red[0] + red[1]) + (red[2] + red[3])) * inv_count;
}

static double* g_mse_partial[64] = {};

static int check_pool_plan(const distdl_plan* p, const char* what) {
  if (p->explicit_halo) return set_error(DISTDL_ERR_UNSUPPORTED, "%s: plan has no kernel (explicit halo plan)", what);
  if (p->n_ci != p->n_co) return set_error(DISTDL_ERR_INVALID_ARG, "%s: pooling keeps the channel count", what);
  return DISTDL_OK;
}

// The maximum is taken over the in-domain cells of a window, so every window needs one: per dimension, some tap
// of every output must land inside the domain (padding of at most half the kernel extent guarantees it).
static int check_maxpool_windows(const distdl_plan* p, const char* what) {
  if (p->maxpool_ok > 0) return DISTDL_OK;  // checked before
  for (const WorkerDev& wd : p->workers)
    for (int d = 0; d < 3; ++d)
      for (int o = 0; o < wd.out[d]; ++o) {
        bool any = false;
        for (int t = 0; t < p->ksize[d] && !any; ++t) {
          const int b = wd.origin[d] + o * p->stride[d] + t * p->dilation[d];
          any = b >= wd.dom_lo[d] && b < wd.dom_hi[d];
        }
        if (!any)
          return set_error(DISTDL_ERR_UNSUPPORTED, "%s: a window lies entirely in the zero padding (dimension %d)", what,
                           d - (3 - p->D));
      }
  p->maxpool_ok = 1;
  return DISTDL_OK;
}

// division constants of every worker's buffer and output extents, built on first use
static int ensure_pooldiv(distdl_plan* p) {
  if (p->d_pooldiv) return DISTDL_OK;
  std::vector<FastDiv> h((size_t)p->n_workers * 4);
  for (int w = 0; w < p->n_workers; ++w) {
    const WorkerDev& wd = p->workers[w];
    h[w * 4 + 0] = make_fastdiv((uint32_t)wd.buf[1]);
    h[w * 4 + 1] = make_fastdiv((uint32_t)wd.buf[2]);
    h[w * 4 + 2] = make_fastdiv((uint32_t)wd.out[1]);
    h[w * 4 + 3] = make_fastdiv((uint32_t)wd.out[2]);
  }
  DISTDL_HIP_TRY(hipMalloc((void**)&p->d_pooldiv, h.size() * sizeof(FastDiv)));
  DISTDL_HIP_TRY(hipMemcpy(p->d_pooldiv, h.data(), h.size() * sizeof(FastDiv), hipMemcpyHostToDevice));
  return DISTDL_OK;
}

static bool all_aligned16(const void* const* v, int n) {
  for (int i = 0; i < n; ++i)
    if ((uintptr_t)v[i] % 16) return false;
  return true;
}

static int check_list(const void* const* v, int n, const char* what, int esz = 4) {
  for (int i = 0; i < n; ++i)
    if (!v[i] || (uintptr_t)v[i] % esz) return set_error(DISTDL_ERR_NULL, "%s: array %d null or misaligned", what, i);
  return DISTDL_OK;
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_relu_fwd(const void* const x_dev[], void* const y_dev[], const int64_t count[], int n, void* stream) {
  return run_elementwise<0>(x_dev, nullptr, y_dev, count, n, 0.f, "relu_fwd", (hipStream_t)stream);
}

int distdl_relu_bwd(const void* const x_dev[], const void* const dy_dev[], void* const dx_dev[], const int64_t count[],
                    int n, void* stream) {
  return run_elementwise<1>(x_dev, dy_dev, dx_dev, count, n, 0.f, "relu_bwd", (hipStream_t)stream);
}

static int pool_fwd(distdl_plan* plan, void* const x_bufs_dev[], void* const y_dev[], bool avg, hipStream_t st) {
  const char* what = avg ? "avgpool_fwd" : "maxpool_fwd";
  if (!plan || !x_bufs_dev || !y_dev) return set_error(DISTDL_ERR_NULL, "%s: null argument", what);
  int rc = check_pool_plan(plan, what);
  if (rc) return rc;
  if (!avg && (rc = check_maxpool_windows(plan, what))) return rc;
  const bool bf16 = plan->dtype == DISTDL_BF16;  // bf16 tensors: the element-wise kernels (fp32 arithmetic)
  if ((rc = check_list((const void* const*)y_dev, plan->n_workers, what, bf16 ? 2 : 4))) return rc;
  if ((rc = run_halo(plan, false, plan->tab_x, x_bufs_dev, st))) return rc;  // x <- H x
  if ((rc = plan->tab_x.upload((const void* const*)x_bufs_dev, plan->n_workers, st))) return rc;
  if ((rc = plan->tab_y.upload((const void* const*)y_dev, plan->n_workers, st))) return rc;
  PoolDev d = pool_params(plan);
  int64_t total = plan->n_b * plan->max_out_cells * d.c;
  ProfScope prof(what, st);
  if (!bf16 && d.c % 4 == 0 && all_aligned16((const void* const*)x_bufs_dev, plan->n_workers) &&
      all_aligned16((const void* const*)y_dev, plan->n_workers) && total / 4 < (int64_t(1) << 31) &&
      ensure_pooldiv(plan) == DISTDL_OK) {
    dim3 grid((unsigned)((total / 4 + 255) / 256), plan->n_workers);
    bool stream = true;  // windows that do not overlap: every input is read once
    for (int i = 0; i < 3; ++i) stream = stream && d.s[i] >= (d.k[i] - 1) * d.dil[i] + 1;
#define DISTDL_POOL_FWD(A_, S_)                                                                                     \
  hipLaunchKernelGGL((pool_fwd_vec_kernel<A_, S_>), grid, dim3(256), 0, st, plan->d_workers, plan->d_pooldiv,        \
                     plan->tab_x.dev, plan->tab_y.dev, d)
    if (avg && stream) DISTDL_POOL_FWD(true, true);
    else if (avg) DISTDL_POOL_FWD(true, false);
    else if (stream) DISTDL_POOL_FWD(false, true);
    else DISTDL_POOL_FWD(false, false);
#undef DISTDL_POOL_FWD
    DISTDL_HIP_TRY(hipGetLastError());
    return DISTDL_OK;
  }
  dim3 grid((unsigned)((total + 255) / 256), plan->n_workers);
#define DISTDL_POOL_FWD_G(A_, T_)                                                                                   \
  hipLaunchKernelGGL((pool_fwd_kernel<A_, T_>), grid, dim3(256), 0, st, plan->d_workers, plan->tab_x.dev,            \
                     plan->tab_y.dev, d)
  if (avg && bf16) DISTDL_POOL_FWD_G(true, uint16_t);
  else if (avg) DISTDL_POOL_FWD_G(true, float);
  else if (bf16) DISTDL_POOL_FWD_G(false, uint16_t);
  else DISTDL_POOL_FWD_G(false, float);
#undef DISTDL_POOL_FWD_G
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

static int pool_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* const dy_dev[],
                    void* const dx_bufs_dev[], bool avg, hipStream_t st) {
  const char* what = avg ? "avgpool_bwd" : "maxpool_bwd";
  if (!plan || (!avg && !x_bufs_dev) || !dy_dev || !dx_bufs_dev) return set_error(DISTDL_ERR_NULL, "%s: null argument", what);
  int rc = check_pool_plan(plan, what);
  if (rc) return rc;
  if (!avg && (rc = check_maxpool_windows(plan, what))) return rc;
  const bool bf16 = plan->dtype == DISTDL_BF16;
  const int esz = bf16 ? 2 : 4;
  if ((!avg && (rc = check_list(x_bufs_dev, plan->n_workers, what, esz))) ||
      (rc = check_list(dy_dev, plan->n_workers, what, esz)) ||
      (rc = check_list((const void* const*)dx_bufs_dev, plan->n_workers, what, esz)))
    return rc;
  if ((rc = plan_prepare_device(plan))) return rc;
  if ((!avg && (rc = plan->tab_x.upload(x_bufs_dev, plan->n_workers, st))) ||
      (rc = plan->tab_dy.upload(dy_dev, plan->n_workers, st)) ||
      (rc = plan->tab_dx.upload((const void* const*)dx_bufs_dev, plan->n_workers, st)))
    return rc;
  PoolDev d = pool_params(plan);
  int64_t total = plan->n_b * plan->max_buf_cells * d.c;
  {
    ProfScope prof(what, st);
    bool tiled = !bf16 && d.c % 4 == 0 && all_aligned16(dy_dev, plan->n_workers) &&
                 all_aligned16((const void* const*)dx_bufs_dev, plan->n_workers) &&
                 (avg || all_aligned16(x_bufs_dev, plan->n_workers));
    for (int i = 0; i < 3; ++i) tiled = tiled && d.dil[i] == 1 && d.s[i] >= d.k[i];
    tiled = tiled && total / 4 < (int64_t(1) << 31) && ensure_pooldiv(plan) == DISTDL_OK;
    if (tiled) {
      const int64_t wtotal = plan->n_b * plan->max_out_cells * (d.c / 4);
      dim3 wgrid((unsigned)((wtotal + 255) / 256), plan->n_workers);
      dim3 ugrid((unsigned)((total / 4 + 255) / 256), plan->n_workers);
      if (avg)
        hipLaunchKernelGGL(pool_bwd_window_kernel<true>, wgrid, dim3(256), 0, st, plan->d_workers, plan->d_pooldiv,
                           (void* const*)nullptr, plan->tab_dy.dev, plan->tab_dx.dev, d);
      else
        hipLaunchKernelGGL(pool_bwd_window_kernel<false>, wgrid, dim3(256), 0, st, plan->d_workers, plan->d_pooldiv,
                           plan->tab_x.dev, plan->tab_dy.dev, plan->tab_dx.dev, d);
      // every buffer cell lies in a window (stride == kernel, the windows start at the buffer's first cell and
      // end at its last): nothing to clear
      bool covered = true;
      for (const WorkerDev& wd : plan->workers)
        for (int i = 0; i < 3; ++i)
          covered = covered && d.s[i] == d.k[i] && wd.origin[i] == 0 && wd.out[i] * d.s[i] == wd.buf[i];
      if (!covered)
        hipLaunchKernelGGL(pool_bwd_uncovered_kernel, ugrid, dim3(256), 0, st, plan->d_workers, plan->d_pooldiv,
                           plan->tab_dx.dev, d);
    } else {
    dim3 grid((unsigned)((total + 255) / 256), plan->n_workers);
#define DISTDL_POOL_BWD_G(A_, T_)                                                                                   \
  hipLaunchKernelGGL((pool_bwd_kernel<A_, T_>), grid, dim3(256), 0, st, plan->d_workers,                             \
                     A_ ? (void* const*)nullptr : plan->tab_x.dev, plan->tab_dy.dev, plan->tab_dx.dev, d)
    if (avg && bf16) DISTDL_POOL_BWD_G(true, uint16_t);
    else if (avg) DISTDL_POOL_BWD_G(true, float);
    else if (bf16) DISTDL_POOL_BWD_G(false, uint16_t);
    else DISTDL_POOL_BWD_G(false, float);
#undef DISTDL_POOL_BWD_G
    }
  }
  DISTDL_HIP_TRY(hipGetLastError());
  return run_halo(plan, true, plan->tab_dx, dx_bufs_dev, st);  // dx <- H* dx
}

int distdl_maxpool_fwd(distdl_plan* plan, void* const x_bufs_dev[], void* const y_dev[], void* stream) {
  return pool_fwd(plan, x_bufs_dev, y_dev, false, (hipStream_t)stream);
}

int distdl_maxpool_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* const dy_dev[],
                       void* const dx_bufs_dev[], void* stream) {
  return pool_bwd(plan, x_bufs_dev, dy_dev, dx_bufs_dev, false, (hipStream_t)stream);
}

int distdl_avgpool_fwd(distdl_plan* plan, void* const x_bufs_dev[], void* const y_dev[], void* stream) {
  return pool_fwd(plan, x_bufs_dev, y_dev, true, (hipStream_t)stream);
}

int distdl_avgpool_bwd(distdl_plan* plan, const void* const dy_dev[], void* const dx_bufs_dev[], void* stream) {
  return pool_bwd(plan, nullptr, dy_dev, dx_bufs_dev, true, (hipStream_t)stream);
}

int distdl_bulk_copy(distdl_plan* plan, void* const dense_dev[], void* const bufs_dev[], int to_bufs, void* stream) {
  if (!plan || !dense_dev || !bufs_dev) return set_error(DISTDL_ERR_NULL, "bulk_copy: null argument");
  if (plan->dtype != DISTDL_F32) return set_error(DISTDL_ERR_UNSUPPORTED, "bulk_copy: only fp32 is implemented");
  int rc;
  if ((rc = check_list((const void* const*)dense_dev, plan->n_workers, "bulk_copy dense")) ||
      (rc = check_list((const void* const*)bufs_dev, plan->n_workers, "bulk_copy bufs")))
    return rc;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = plan_prepare_device(plan))) return rc;
  if ((rc = plan->tab_y.upload((const void* const*)dense_dev, plan->n_workers, st)) ||
      (rc = plan->tab_x.upload((const void* const*)bufs_dev, plan->n_workers, st)))
    return rc;
  int64_t total = plan->n_b * plan->max_buf_cells * plan->n_ci;
  ProfScope prof("bulk_copy", st);
  hipLaunchKernelGGL(bulk_copy_kernel, dim3((unsigned)((total + 255) / 256), plan->n_workers), dim3(256), 0, st,
                     plan->d_workers, plan->tab_y.dev, plan->tab_x.dev, (int)plan->n_b, (int)plan->n_ci, to_bufs);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

static int run_repartition(distdl_plan* plan, void* const spatial_dev[], int P_f, void* const feat_dev[],
                           int to_features, hipStream_t st) {
  if (!plan || !spatial_dev || !feat_dev) return set_error(DISTDL_ERR_NULL, "repartition: null argument");
  if (plan->dtype != DISTDL_F32) return set_error(DISTDL_ERR_UNSUPPORTED, "repartition: only fp32 is implemented");
  if (P_f < 1 || P_f > 64) return set_error(DISTDL_ERR_INVALID_ARG, "repartition: P_f = %d not in 1..64", P_f);
  RepartDev d{};
  int64_t feats = plan->n_co;
  for (int k = 0; k < 3; ++k) {
    if (plan->P[k] > 64) return set_error(DISTDL_ERR_UNSUPPORTED, "repartition: more than 64 workers per dimension");
    d.P[k] = plan->P[k];
    d.G[k] = (int32_t)plan->out_shape[k];
    feats *= plan->out_shape[k];
    for (int r = 0; r < plan->P[k]; ++r) {
      d.out_start[k][r] = (int32_t)plan->dims[k][r].out_start;
      d.out_size[k][r] = (int32_t)plan->dims[k][r].out_size;
    }
  }
  if (feats >= (int64_t(1) << 31) || feats < P_f) return set_error(DISTDL_ERR_INVALID_ARG, "repartition: bad feature count");
  d.n_b = (int32_t)plan->n_b;
  d.c = (int32_t)plan->n_co;
  d.P_f = P_f;
  int64_t at = 0, mx = 0;
  for (int j = 0; j < P_f; ++j) {
    int64_t z = feats / P_f + (j < feats % P_f ? 1 : 0);
    d.f_start[j] = (int32_t)at;
    d.f_size[j] = (int32_t)z;
    at += z;
    mx = std::max(mx, z);
  }
  int rc;
  if ((rc = check_list((const void* const*)spatial_dev, plan->n_workers, "repartition spatial")) ||
      (rc = check_list((const void* const*)feat_dev, P_f, "repartition features")))
    return rc;
  if ((rc = plan->tab_y.upload((const void* const*)spatial_dev, plan->n_workers, st)) ||
      (rc = plan->tab_dy.upload((const void* const*)feat_dev, P_f, st)))
    return rc;
  ProfScope prof("repartition", st);
  hipLaunchKernelGGL(repartition_kernel, dim3((unsigned)((plan->n_b * mx + 255) / 256), P_f), dim3(256), 0, st,
                     plan->tab_y.dev, plan->tab_dy.dev, d, to_features);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

int distdl_repartition_fwd(distdl_plan* plan, const void* const src_dev[], int P_f, void* const dst_dev[], void* stream) {
  return run_repartition(plan, (void* const*)src_dev, P_f, dst_dev, 1, (hipStream_t)stream);
}

int distdl_repartition_adj(distdl_plan* plan, const void* const gdst_dev[], int P_f, void* const gsrc_dev[],
                           void* stream) {
  return run_repartition(plan, gsrc_dev, P_f, (void* const*)gdst_dev, 0, (hipStream_t)stream);
}

int distdl_mse_fwd_bwd(const void* const y_dev[], const void* const t_dev[], void* const dy_dev[], const int64_t count[],
                       int n, double* loss_dev, void* stream) {
  if (!y_dev || !t_dev || !dy_dev || !count || !loss_dev) return set_error(DISTDL_ERR_NULL, "mse: null argument");
  if (n < 1 || n > kEwArrays) return set_error(DISTDL_ERR_INVALID_ARG, "mse: n = %d not in 1..%d", n, kEwArrays);
  hipStream_t st = (hipStream_t)stream;
  int64_t total = 0;
  MseArgs m{};
  m.n = n;
  for (int j = 0; j < n; ++j) {
    if (count[j] < 0 || (count[j] > 0 && (!y_dev[j] || !t_dev[j] || !dy_dev[j])))
      return set_error(DISTDL_ERR_NULL, "mse: array %d null or negative count", j);
    m.y[j] = (const float*)y_dev[j];
    m.t[j] = (const float*)t_dev[j];
    m.count[j] = count[j];
    total += count[j];
  }
  if (total == 0) return set_error(DISTDL_ERR_INVALID_ARG, "mse: no elements");
  int dev = 0;
  DISTDL_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(DISTDL_ERR_UNSUPPORTED, "device index %d", dev);
  if (!g_mse_partial[dev]) DISTDL_HIP_TRY(hipMalloc((void**)&g_mse_partial[dev], kMseBlocks * sizeof(double)));
  {
    ProfScope prof("mse", st);
    hipLaunchKernelGGL(mse_partial_kernel, dim3(kMseBlocks), dim3(256), 0, st, m, g_mse_partial[dev]);
    hipLaunchKernelGGL(mse_final_kernel, dim3(1), dim3(256), 0, st, g_mse_partial[dev], kMseBlocks, 1.0 / (double)total,
                       loss_dev);
  }
  // dy = 2 (y - t) / N
  return run_elementwise<2>(y_dev, t_dev, dy_dev, count, n, (float)(2.0 / (double)total), "mse_grad", st);
}

}  // extern "C"
