// Broadcast B, sum-reduce R = B* (Sec. 3 "Broadcast", "Sum-reduce and
// all-reduce") over groups of replicas held in one HBM, and the Euclidean
// inner product over a list of arrays (Sec. 2) for the adjoint test.
//
// Replica pointers travel as kernel arguments when a group has at most
// kMaxPtrs of them; wider groups read them from a device copy of the caller's
// pointer array (cached per device like a plan's tables), so that one thread
// still adds all k replicas of its elements in index order in fp32.
#include <algorithm>
#include <cstdlib>
#include <vector>

#include "common.h"
#include "profile.h"

namespace distdl {

constexpr int kMaxPtrs = 64;
constexpr int kMaxGroups = 16;
constexpr int kCollThreads = 256;

__device__ inline float bf2f(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

struct CollArgs {
  void* one[kMaxGroups];    // per group: the single (source / reduced) array
  void* many[kMaxPtrs];     // replicas, group after group
  int64_t count[kMaxGroups];
  int32_t first[kMaxGroups];  // index of the group's first replica in many[]
  int32_t k[kMaxGroups];      // replicas of the group in this launch
  int32_t wide[kMaxGroups];   // all pointers of the group 16-byte aligned
  void* const* many_dev;      // TAB kernels: all replica pointers in device memory, first[] indexes into it
  int32_t clear_inputs;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Both kernels stream: every element is touched once, so loads carry the
// non-temporal hint, and the grid covers the longest group with one 16-byte
// vector per thread (many short-lived workgroups keep more requests in flight
// than a grid-stride loop over few); the loop only matters beyond 2^31 threads.
template <bool BF16, bool TAB = false>
__global__ __launch_bounds__(kCollThreads) void bcast_kernel(CollArgs a) {
  const int g = blockIdx.y;
  const int64_t count = a.count[g];
  constexpr int V = BF16 ? 8 : 4;
  const int64_t nvec = a.wide[g] ? count / V : 0;
  const int k = a.k[g];
  void* const* rep = (TAB ? a.many_dev : a.many) + a.first[g];
  const int64_t stride = (int64_t)gridDim.x * kCollThreads;
  const int64_t tid = (int64_t)blockIdx.x * kCollThreads + threadIdx.x;
  const u32x4* src = (const u32x4*)a.one[g];
  // The last of three or more replicas is written with the non-temporal hint, the others with plain stores:
  // measured at k = 4, 8 and 64 that mix is 4-7 % faster than either kind alone on replicas of 16-256 MiB and
  // level with plain stores at 1 GiB; with two replicas plain stores are the faster ones.
  const int k_plain = k >= 3 ? k - 1 : k;
  for (int64_t u = tid; u < nvec; u += stride) {
    u32x4 v = __builtin_nontemporal_load(src + u);
    for (int i = 0; i < k_plain; ++i) ((u32x4*)rep[i])[u] = v;
    if (k_plain < k) __builtin_nontemporal_store(v, (u32x4*)rep[k - 1] + u);
  }
  for (int64_t e = nvec * V + tid; e < count; e += stride) {
    if (BF16) {
      uint16_t v = ((const uint16_t*)a.one[g])[e];
      for (int i = 0; i < k; ++i) ((uint16_t*)rep[i])[e] = v;
    } else {
      uint32_t v = ((const uint32_t*)a.one[g])[e];
      for (int i = 0; i < k; ++i) ((uint32_t*)rep[i])[e] = v;
    }
  }
}

template <bool BF16, bool TAB = false>
__global__ __launch_bounds__(kCollThreads) void reduce_kernel(CollArgs a) {
  const int g = blockIdx.y;
  const int64_t count = a.count[g];
  constexpr int V = BF16 ? 8 : 4;
  const int64_t nvec = a.wide[g] ? count / V : 0;
  const int k = a.k[g];
  void* const* rep = (TAB ? a.many_dev : a.many) + a.first[g];
  const int64_t stride = (int64_t)gridDim.x * kCollThreads;
  const int64_t tid = (int64_t)blockIdx.x * kCollThreads + threadIdx.x;
  const bool clear = a.clear_inputs != 0;
  for (int64_t u = tid; u < nvec; u += stride) {
    float acc[V];
    for (int j = 0; j < V; ++j) acc[j] = 0.f;
#pragma unroll 8
    for (int i = 0; i < k; ++i) {  // replica order i = 0 .. k-1; the unrolled loads are issued together
      u32x4 r = __builtin_nontemporal_load((const u32x4*)rep[i] + u);
      for (int j = 0; j < 4; ++j) {
        if (BF16) {
          acc[2 * j] += bf2f(r[j] & 0xffffu);
          acc[2 * j + 1] += bf2f(r[j] >> 16);
        } else {
          acc[j] += __uint_as_float(r[j]);
        }
      }
    }
    if (clear)
      for (int i = 0; i < k; ++i) ((u32x4*)rep[i])[u] = u32x4{0, 0, 0, 0};
    u32x4 o;
    if (BF16) {
      for (int j = 0; j < 4; ++j) o[j] = f2bf(acc[2 * j]) | (f2bf(acc[2 * j + 1]) << 16);
    } else {
      for (int j = 0; j < 4; ++j) o[j] = __float_as_uint(acc[j]);
    }
    __builtin_nontemporal_store(o, (u32x4*)a.one[g] + u);
  }
  for (int64_t e = nvec * V + tid; e < count; e += stride) {
    if (BF16) {
      uint16_t* out = (uint16_t*)a.one[g];
      float acc = 0.f;
      for (int i = 0; i < k; ++i) {
        acc += bf2f(((const uint16_t*)rep[i])[e]);
        if (clear) ((uint16_t*)rep[i])[e] = 0;
      }
      out[e] = (uint16_t)f2bf(acc);
    } else {
      float* out = (float*)a.one[g];
      float acc = 0.f;
      for (int i = 0; i < k; ++i) {
        acc += ((const float*)rep[i])[e];
        if (clear) ((float*)rep[i])[e] = 0.f;
      }
      out[e] = acc;
    }
  }
}

// Device copies of pointer arrays of groups wider than kMaxPtrs, one cache per device.
static PtrTable g_wide_ptrs[64];
// Plain streaming copy, one 16-byte vector per thread: the yardstick the movement kernels are measured against.
// A kernel of its own so that traces and counters list it under its own name.
__global__ __launch_bounds__(kCollThreads) void copy_ref_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                                int64_t nvec) {
  const int64_t stride = (int64_t)gridDim.x * kCollThreads;
  for (int64_t u = (int64_t)blockIdx.x * kCollThreads + threadIdx.x; u < nvec; u += stride)
    dst[u] = __builtin_nontemporal_load(src + u);
}

static unsigned blocks_for(int64_t max_count, int vec) {
  int64_t units = (max_count + vec - 1) / vec;  // one unit per thread
  int64_t b = (units + kCollThreads - 1) / kCollThreads;
  if (b < 1) b = 1;
  if (b > (int64_t(1) << 22)) b = int64_t(1) << 22;
  return (unsigned)b;
}

// Shared driver: reduce == false is the broadcast direction.
static int run_collective(bool reduce, void* const one[], void* const many[], const int64_t count[], int G, int k,
                          distdl_dtype dtype, int clear_inputs, hipStream_t st) {
  if (!one || !many || !count) return set_error(DISTDL_ERR_NULL, "collective: null argument");
  if (G < 1 || k < 1) return set_error(DISTDL_ERR_INVALID_ARG, "collective: G = %d, k = %d", G, k);
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  const size_t esz = dtype_size(dtype);
  for (int g = 0; g < G; ++g) {
    if (count[g] < 0) return set_error(DISTDL_ERR_INVALID_ARG, "group %d: negative count", g);
    if (count[g] == 0) continue;
    if (!one[g] || (uintptr_t)one[g] % esz) return set_error(DISTDL_ERR_NULL, "group %d: null or misaligned array", g);
    for (int i = 0; i < k; ++i)
      if (!many[(size_t)g * k + i] || (uintptr_t)many[(size_t)g * k + i] % esz)
        return set_error(DISTDL_ERR_NULL, "group %d replica %d: null or misaligned array", g, i);
  }
  const int vec = dtype == DISTDL_F32 ? 4 : 8;
  const bool tab = k > kMaxPtrs;
  void* const* many_dev = nullptr;
  if (tab) {
    int dev = 0;
    DISTDL_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return set_error(DISTDL_ERR_UNSUPPORTED, "device index %d", dev);
    int rc = g_wide_ptrs[dev].upload((const void* const*)many, (size_t)G * k, st);
    if (rc) return rc;
    many_dev = g_wide_ptrs[dev].dev;
  }
  const int groups_per_launch = tab ? kMaxGroups : std::max(1, std::min(kMaxGroups, kMaxPtrs / k));
  for (int g0 = 0; g0 < G; g0 += groups_per_launch) {
    CollArgs a{};
    int ng = 0, np = 0;
    int64_t max_count = 0;
    for (int g = g0; g < std::min(G, g0 + groups_per_launch); ++g) {
      if (count[g] == 0) continue;
      a.one[ng] = one[g];
      a.count[ng] = count[g];
      a.first[ng] = tab ? g * k : np;
      a.k[ng] = k;
      bool wide = (uintptr_t)one[g] % 16 == 0;
      for (int i = 0; i < k; ++i) {
        void* rep = many[(size_t)g * k + i];
        if (!tab) a.many[np++] = rep;
        wide &= (uintptr_t)rep % 16 == 0;
      }
      a.wide[ng] = wide;
      max_count = std::max(max_count, count[g]);
      ++ng;
    }
    if (ng == 0) continue;
    a.many_dev = many_dev;
    a.clear_inputs = clear_inputs;
    dim3 grid(blocks_for(max_count, vec), ng), block(kCollThreads);
    ProfScope prof(reduce ? "sumreduce" : "bcast", st);
    const bool bf = dtype != DISTDL_F32;
    if (reduce) {
      if (tab) {
        if (bf) hipLaunchKernelGGL((reduce_kernel<true, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((reduce_kernel<false, true>), grid, block, 0, st, a);
      } else {
        if (bf) hipLaunchKernelGGL((reduce_kernel<true, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((reduce_kernel<false, false>), grid, block, 0, st, a);
      }
    } else {
      if (tab) {
        if (bf) hipLaunchKernelGGL((bcast_kernel<true, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((bcast_kernel<false, true>), grid, block, 0, st, a);
      } else {
        if (bf) hipLaunchKernelGGL((bcast_kernel<true, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((bcast_kernel<false, false>), grid, block, 0, st, a);
      }
    }
  }
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

// ---- inner product ----------------------------------------------------------
constexpr int kDotBlocks = kDotPartials;
constexpr int kDotArrays = 24;
struct DotArgs {
  const void* a[kDotArrays];
  const void* b[kDotArrays];
  int64_t count[kDotArrays];
  int32_t n;
  int32_t accumulate;
};

__device__ inline double wave_sum(double v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

template <bool BF16>
__global__ __launch_bounds__(256) void dot_partial_kernel(DotArgs d, double* partial) {
  double acc = 0.0;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int j = 0; j < d.n; ++j) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < d.count[j]; e += stride) {
      double x, y;
      if (BF16) {
        x = bf2f(((const uint16_t*)d.a[j])[e]);
        y = bf2f(((const uint16_t*)d.b[j])[e]);
      } else {
        x = ((const float*)d.a[j])[e];
        y = ((const float*)d.b[j])[e];
      }
      acc += x * y;
    }
  }
  __shared__ double red[4];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = red[0] + red[1] + red[2] + red[3];
    partial[blockIdx.x] = d.accumulate ? partial[blockIdx.x] + s : s;
  }
}

__global__ __launch_bounds__(256) void dot_final_kernel(const double* partial, int n, double* out) {
  double acc = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) acc += partial[i];
  __shared__ double red[4];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) *out = red[0] + red[1] + red[2] + red[3];
}

static double* g_dot_partial[64] = {};

// The launches of an inner product; `partial` holds kDotPartials doubles, every one of which is overwritten by
// the first launch, so stale contents never matter.
int launch_dot(const void* const a_dev[], const void* const b_dev[], const int64_t count[], int n_arrays,
                      distdl_dtype dtype, double* partial, double* result_dev, hipStream_t st) {
  for (int j = 0; j < n_arrays; ++j) {
    if (count[j] < 0) return set_error(DISTDL_ERR_INVALID_ARG, "dot: negative count");
    if (count[j] > 0 && (!a_dev[j] || !b_dev[j])) return set_error(DISTDL_ERR_NULL, "dot: null array");
  }
  for (int j0 = 0; j0 < n_arrays; j0 += kDotArrays) {
    DotArgs d{};
    d.n = std::min(kDotArrays, n_arrays - j0);
    d.accumulate = j0 > 0;
    for (int j = 0; j < d.n; ++j) {
      d.a[j] = a_dev[j0 + j];
      d.b[j] = b_dev[j0 + j];
      d.count[j] = count[j0 + j];
    }
    if (dtype == DISTDL_F32) hipLaunchKernelGGL(dot_partial_kernel<false>, dim3(kDotBlocks), dim3(256), 0, st, d, partial);
    else hipLaunchKernelGGL(dot_partial_kernel<true>, dim3(kDotBlocks), dim3(256), 0, st, d, partial);
  }
  hipLaunchKernelGGL(dot_final_kernel, dim3(1), dim3(256), 0, st, partial, kDotBlocks, result_dev);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_bcast_fwd(const void* const src_dev[], void* const dst_dev[], const int64_t count[], int G, int k,
                     distdl_dtype dtype, void* stream) {
  return run_collective(false, (void* const*)src_dev, dst_dev, count, G, k, dtype, 0, (hipStream_t)stream);
}

int distdl_sumreduce_adj(const void* const gdst_dev[], void* const gsrc_dev[], const int64_t count[], int G, int k,
                         distdl_dtype dtype, void* stream) {
  return run_collective(false, (void* const*)gdst_dev, gsrc_dev, count, G, k, dtype, 0, (hipStream_t)stream);
}

int distdl_bcast_adj(void* const gsrc_dev[], void* const gdst_dev[], const int64_t count[], int G, int k,
                     distdl_dtype dtype, int clear_inputs, void* stream) {
  return run_collective(true, gsrc_dev, gdst_dev, count, G, k, dtype, clear_inputs, (hipStream_t)stream);
}

int distdl_sumreduce_fwd(void* const src_dev[], void* const dst_dev[], const int64_t count[], int G, int k,
                         distdl_dtype dtype, int clear_inputs, void* stream) {
  return run_collective(true, dst_dev, src_dev, count, G, k, dtype, clear_inputs, (hipStream_t)stream);
}

int distdl_copy_ref(const void* src_dev, void* dst_dev, size_t bytes, void* stream) {
  if (!src_dev || !dst_dev) return set_error(DISTDL_ERR_NULL, "copy_ref: null argument");
  if ((uintptr_t)src_dev % 16 || (uintptr_t)dst_dev % 16 || bytes % 16)
    return set_error(DISTDL_ERR_INVALID_ARG, "copy_ref: pointers and size must be multiples of 16 bytes");
  if (bytes == 0) return DISTDL_OK;
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof("copy_ref", st);
  hipLaunchKernelGGL(copy_ref_kernel, dim3(blocks_for((int64_t)(bytes / 16), 1)), dim3(kCollThreads), 0, st,
                     (const u32x4*)src_dev, (u32x4*)dst_dev, (int64_t)(bytes / 16));
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

int distdl_allreduce(void* const bufs_dev[], const int64_t count[], int G, int k, distdl_dtype dtype, void* stream) {
  if (!bufs_dev || !count) return set_error(DISTDL_ERR_NULL, "allreduce: null argument");
  if (G < 1 || k < 1) return set_error(DISTDL_ERR_INVALID_ARG, "allreduce: G = %d, k = %d", G, k);
  // A = B R: the sum lands in replica 0 of each group (a thread reads all replicas of its elements before it
  // writes, so reducing in place is safe), then replica 0 is broadcast to the other k - 1
  std::vector<void*> first(G), rest((size_t)G * std::max(k - 1, 1));
  for (int g = 0; g < G; ++g) {
    first[g] = bufs_dev[(size_t)g * k];
    for (int i = 1; i < k; ++i) rest[(size_t)g * (k - 1) + i - 1] = bufs_dev[(size_t)g * k + i];
  }
  int rc = run_collective(true, first.data(), bufs_dev, count, G, k, dtype, 0, (hipStream_t)stream);
  if (rc || k == 1) return rc;
  return run_collective(false, first.data(), rest.data(), count, G, k - 1, dtype, 0, (hipStream_t)stream);
}

int distdl_dot(const void* const a_dev[], const void* const b_dev[], const int64_t count[], int n_arrays,
               distdl_dtype dtype, double* result_dev, void* stream) {
  if (!a_dev || !b_dev || !count || !result_dev) return set_error(DISTDL_ERR_NULL, "dot: null argument");
  if (n_arrays < 1) return set_error(DISTDL_ERR_INVALID_ARG, "dot: n_arrays = %d", n_arrays);
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  int dev = 0;
  DISTDL_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(DISTDL_ERR_UNSUPPORTED, "device index %d", dev);
  if (!g_dot_partial[dev]) DISTDL_HIP_TRY(hipMalloc((void**)&g_dot_partial[dev], kDotBlocks * sizeof(double)));
  return launch_dot(a_dev, b_dev, count, n_arrays, dtype, g_dot_partial[dev], result_dev, (hipStream_t)stream);
}

}  // extern "C"
