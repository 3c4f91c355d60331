// Halo exchange H and adjoint H* (Sec. 3 "Halo exchange") as one-pass box
// kernels over all workers, dimensions, faces, edges and corners.
//
// The nested per-dimension exchange of the paper leaves every in-domain
// non-owned cell equal to its owner's bulk value; since all partitions share
// one address space that end state is written directly: each box of halo
// cells is one strided copy from the owner's buffer (pack + exchange + unpack
// collapsed, exchange buffers never materialised), each box of padding cells
// a zero fill.  The adjoint runs in gather form: the thread that owns a bulk
// cell reads every halo copy of it (fixed ascending worker order), adds them
// and clears them -- the "add into the bulk" of C* = K_b S_{b->a} without
// atomics, so results are run-to-run identical.
#include "common.h"
#include "profile.h"

namespace distdl {

extern const int kHaloUnitsPerBlock = 1024;  // 256 threads x 4 vector units
constexpr int kThreads = 256;
constexpr int kUnroll = 4;

// ---- element helpers --------------------------------------------------------
__device__ inline float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                // round to nearest even
  return u >> 16;
}

struct F32x4 {
  using Store = float4;
  static constexpr int N = 4;
  __device__ static void unpack(const Store& s, float* a) { a[0] = s.x; a[1] = s.y; a[2] = s.z; a[3] = s.w; }
  __device__ static Store pack(const float* a) { return make_float4(a[0], a[1], a[2], a[3]); }
  __device__ static Store zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
};
struct F32x1 {
  using Store = float;
  static constexpr int N = 1;
  __device__ static void unpack(const Store& s, float* a) { a[0] = s; }
  __device__ static Store pack(const float* a) { return a[0]; }
  __device__ static Store zero() { return 0.f; }
};
struct BF16x8 {
  using Store = uint4;
  static constexpr int N = 8;
  __device__ static void unpack(const Store& s, float* a) {
    const uint32_t w[4] = {s.x, s.y, s.z, s.w};
    for (int i = 0; i < 4; ++i) {
      a[2 * i] = bf16_to_f32(w[i] & 0xffffu);
      a[2 * i + 1] = bf16_to_f32(w[i] >> 16);
    }
  }
  __device__ static Store pack(const float* a) {
    uint32_t w[4];
    for (int i = 0; i < 4; ++i) w[i] = f32_to_bf16(a[2 * i]) | (f32_to_bf16(a[2 * i + 1]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
  __device__ static Store zero() { return make_uint4(0, 0, 0, 0); }
};
struct BF16x1 {
  using Store = uint16_t;
  static constexpr int N = 1;
  __device__ static void unpack(const Store& s, float* a) { a[0] = bf16_to_f32(s); }
  __device__ static Store pack(const float* a) { return (uint16_t)f32_to_bf16(a[0]); }
  __device__ static Store zero() { return 0; }
};

// Every halo, padding and band cell is touched once per call, so loads carry the
// non-temporal hint.  Stores: the ones that carry data (halo copies, band sums)
// are plain, the zero fills (padding cells, cleared halo cells) non-temporal.
// Measured on the 64-worker volumetric geometry, that mix runs the forward
// kernel at 6.3 TB/s and the adjoint at 6.0 TB/s; with every store non-temporal
// both stay at 4.9-5.0 TB/s, with every store plain at 5.4 / 4.7 TB/s, and the
// opposite mix is as fast only when a plan has padding to clear.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// The buffers are device allocations: the address-space cast makes these
// global_load / global_store instead of flat accesses.
#define DISTDL_GLOBAL __attribute__((address_space(1)))
template <class S>
__device__ inline S nt_load(const S* p) {
  if constexpr (sizeof(S) == 16) {
    u32x4 v = __builtin_nontemporal_load((const DISTDL_GLOBAL u32x4*)p);
    S out;
    __builtin_memcpy(&out, &v, 16);
    return out;
  } else {
    return __builtin_nontemporal_load((const DISTDL_GLOBAL S*)p);
  }
}
template <class S>
__device__ inline void plain_store(S* p, const S& val) {
  if constexpr (sizeof(S) == 16) {
    u32x4 v;
    __builtin_memcpy(&v, &val, 16);
    *(DISTDL_GLOBAL u32x4*)p = v;
  } else {
    *(DISTDL_GLOBAL S*)p = val;
  }
}
template <class S>
__device__ inline void nt_store(S* p, const S& val) {
  if constexpr (sizeof(S) == 16) {
    u32x4 v;
    __builtin_memcpy(&v, &val, 16);
    __builtin_nontemporal_store(v, (DISTDL_GLOBAL u32x4*)p);
  } else {
    __builtin_nontemporal_store(val, (DISTDL_GLOBAL S*)p);
  }
}

struct UnitPos {
  uint32_t n, c0, c1, col;
};
__device__ inline UnitPos decode(uint32_t u, const HaloTaskDev& t) {
  UnitPos p;
  uint32_t row = fd_div(u, t.div_row);
  p.col = u - row * t.div_row.d;
  uint32_t r1 = fd_div(row, t.div_e1);
  p.c1 = row - r1 * t.div_e1.d;
  p.n = fd_div(r1, t.div_e0);
  p.c0 = r1 - p.n * t.div_e0.d;
  return p;
}
__device__ inline size_t view_offset(const HaloView& v, const UnitPos& p) {
  return v.base + p.n * v.sn + (size_t)(p.c0 * v.s0 + p.c1 * v.s1 + p.col);
}

// Forward: copy boxes (nsrc == 1) and zero boxes (nsrc == 0).  A thread
// handles kUnroll units: all loads are issued before the first store.
template <class E>
__global__ __launch_bounds__(kThreads) void halo_fwd_kernel(const BlockRef* __restrict__ blocks,
                                                            const HaloTaskDev* __restrict__ tasks,
                                                            void* const* __restrict__ bufs) {
  using S = typename E::Store;
  const BlockRef br = blocks[blockIdx.x];
  const HaloTaskDev t = tasks[br.task];  // by value: the record is read once into scalar registers
  const uint32_t total = t.total;
  S* __restrict__ dst = (S*)bufs[t.dst.worker];
  if (t.nsrc == 0) {
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      uint32_t u = br.unit0 + threadIdx.x + i * kThreads;
      if (u < total) nt_store(dst + view_offset(t.dst, decode(u, t)), E::zero());
    }
    return;
  }
  const S* __restrict__ src = (const S*)bufs[t.src0.worker];
  S vals[kUnroll];
  size_t doff[kUnroll];
  bool live[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    uint32_t u = br.unit0 + threadIdx.x + i * kThreads;
    live[i] = u < total;
    UnitPos p = decode(live[i] ? u : total - 1, t);  // clamped: loads need no branch
    doff[i] = view_offset(t.dst, p);
    vals[i] = nt_load(src + view_offset(t.src0, p));
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i)
    if (live[i]) plain_store(dst + doff[i], vals[i]);
}

// Adjoint: bulk boxes gather-add their halo copies and clear them; padding
// boxes are cleared.  Per source, the loads of all kUnroll units are issued
// before the clears, and the destination is loaded together with the first
// source, so that a thread has 2 * kUnroll requests in flight.
template <class E>
__global__ __launch_bounds__(kThreads) void halo_adj_kernel(const BlockRef* __restrict__ blocks,
                                                            const HaloTaskDev* __restrict__ tasks,
                                                            const HaloView* __restrict__ views,
                                                            void* const* __restrict__ bufs) {
  using S = typename E::Store;
  const BlockRef br = blocks[blockIdx.x];
  const HaloTaskDev t = tasks[br.task];  // by value: the record is read once into scalar registers
  const uint32_t total = t.total;
  S* dst = (S*)bufs[t.dst.worker];
  if (t.nsrc == 0) {
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      uint32_t u = br.unit0 + threadIdx.x + i * kThreads;
      if (u < total) nt_store(dst + view_offset(t.dst, decode(u, t)), E::zero());
    }
    return;
  }
  UnitPos pos[kUnroll];
  bool live[kUnroll];
  S dv[kUnroll], sv[kUnroll];
  float acc[kUnroll][E::N];
  S* src = (S*)bufs[t.src0.worker];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    uint32_t u = br.unit0 + threadIdx.x + i * kThreads;
    live[i] = u < total;
    pos[i] = decode(live[i] ? u : total - 1, t);  // clamped: loads need no branch
    dv[i] = nt_load(dst + view_offset(t.dst, pos[i]));
    sv[i] = nt_load(src + view_offset(t.src0, pos[i]));
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    float v[E::N];
    E::unpack(dv[i], acc[i]);
    E::unpack(sv[i], v);
    if (live[i]) nt_store(src + view_offset(t.src0, pos[i]), E::zero());
#pragma unroll
    for (int e = 0; e < E::N; ++e) acc[i][e] += v[e];
  }
  for (int s = 1; s < t.nsrc; ++s) {  // ascending source-worker order
    const HaloView sr = views[t.src_begin + s];
    src = (S*)bufs[sr.worker];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) sv[i] = nt_load(src + view_offset(sr, pos[i]));
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      float v[E::N];
      E::unpack(sv[i], v);
      if (live[i]) nt_store(src + view_offset(sr, pos[i]), E::zero());
#pragma unroll
      for (int e = 0; e < E::N; ++e) acc[i][e] += v[e];
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i)
    if (live[i]) plain_store(dst + view_offset(t.dst, pos[i]), E::pack(acc[i]));
}

int plan_prepare_device(distdl_plan* p);

template <class E>
static void launch(bool adjoint, const TaskTable& tt, const distdl_plan* p, void* const* bufs, hipStream_t st) {
  dim3 grid((unsigned)tt.blocks.size()), block(kThreads);
  (void)p;
  ProfScope prof(adjoint ? "halo_adj" : "halo_fwd", st);
  if (adjoint)
    hipLaunchKernelGGL(halo_adj_kernel<E>, grid, block, 0, st, tt.d_blocks, tt.d_tasks, tt.d_views, bufs);
  else
    hipLaunchKernelGGL(halo_fwd_kernel<E>, grid, block, 0, st, tt.d_blocks, tt.d_tasks, bufs);
}

// Copy boxes between arbitrary buffers with the forward kernel (used by the generalized repartition): the
// tasks' views index one pointer table that holds sources and destinations; unit_bytes is 16, 4 or 2.
int run_box_copy(int unit_bytes, const BlockRef* d_blocks, const HaloTaskDev* d_tasks, size_t nblocks, void* const* d_bufs,
                 const char* name, hipStream_t st) {
  if (nblocks == 0) return DISTDL_OK;
  dim3 grid((unsigned)nblocks), block(kThreads);
  ProfScope prof(name, st);
  if (unit_bytes == 16) hipLaunchKernelGGL(halo_fwd_kernel<F32x4>, grid, block, 0, st, d_blocks, d_tasks, d_bufs);
  else if (unit_bytes == 4) hipLaunchKernelGGL(halo_fwd_kernel<F32x1>, grid, block, 0, st, d_blocks, d_tasks, d_bufs);
  else if (unit_bytes == 2) hipLaunchKernelGGL(halo_fwd_kernel<BF16x1>, grid, block, 0, st, d_blocks, d_tasks, d_bufs);
  else return set_error(DISTDL_ERR_INVALID_ARG, "internal: box copy unit of %d bytes", unit_bytes);
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

// Shared by the public halo calls and by conv_fwd / conv_bwd.
int run_halo(distdl_plan* p, bool adjoint, PtrTable& tab, void* const* bufs_host, hipStream_t st) {
  int rc = plan_prepare_device(p);
  if (rc) return rc;
  const size_t esz = dtype_size(p->dtype);
  bool aligned16 = true;
  for (int w = 0; w < p->n_workers; ++w) {
    if (!bufs_host[w]) return set_error(DISTDL_ERR_NULL, "buffer of worker %d is null", w);
    if ((uintptr_t)bufs_host[w] % esz) return set_error(DISTDL_ERR_INVALID_ARG, "buffer of worker %d is misaligned", w);
    aligned16 &= ((uintptr_t)bufs_host[w] % 16) == 0;
  }
  const bool wide = aligned16 && !p->fwd16.tasks.empty();
  const TaskTable& tt = adjoint ? (wide ? p->adj16 : p->adj1) : (wide ? p->fwd16 : p->fwd1);
  if (tt.blocks.empty()) return DISTDL_OK;  // a single worker with no padding: H is the identity
  if ((rc = tab.upload((const void* const*)bufs_host, p->n_workers, st))) return rc;
  if (p->dtype == DISTDL_F32) {
    if (wide) launch<F32x4>(adjoint, tt, p, tab.dev, st);
    else launch<F32x1>(adjoint, tt, p, tab.dev, st);
  } else {
    if (wide) launch<BF16x8>(adjoint, tt, p, tab.dev, st);
    else launch<BF16x1>(adjoint, tt, p, tab.dev, st);
  }
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_halo_fwd(distdl_plan* plan, void* const bufs_dev[], void* stream) {
  if (!plan || !bufs_dev) return set_error(DISTDL_ERR_NULL, "halo_fwd: null argument");
  return run_halo(plan, false, plan->tab_x, bufs_dev, (hipStream_t)stream);
}

int distdl_halo_adj(distdl_plan* plan, void* const gbufs_dev[], void* stream) {
  if (!plan || !gbufs_dev) return set_error(DISTDL_ERR_NULL, "halo_adj: null argument");
  return run_halo(plan, true, plan->tab_dx, gbufs_dev, (hipStream_t)stream);
}

}  // extern "C"
