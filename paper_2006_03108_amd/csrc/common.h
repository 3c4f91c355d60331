// Internal declarations shared by the translation units of libdistdl.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "distdl.h"

namespace distdl {

// ---- error reporting ------------------------------------------------------
int set_error(int code, const char* fmt, ...);
#define DISTDL_HIP_TRY(expr)                                                                  \
  do {                                                                                        \
    hipError_t e__ = (expr);                                                                  \
    if (e__ != hipSuccess)                                                                    \
      return ::distdl::set_error(DISTDL_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

inline size_t dtype_size(distdl_dtype t) { return t == DISTDL_F32 ? 4 : 2; }

// Lets kernel `Kernel` be launched with more than 64 KB of dynamic LDS (up to the 160 KB of a compute unit).
// The attribute is set once per kernel and device: the call is not cheap, and a launch path that made it every
// time would pay for it on each step.
template <auto Kernel>
inline int allow_large_lds() {
  static std::atomic<uint64_t> done{0};  // one bit per device
  int dev = 0;
  DISTDL_HIP_TRY(hipGetDevice(&dev));
  const uint64_t bit = uint64_t(1) << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return DISTDL_OK;
  DISTDL_HIP_TRY(hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  done.fetch_or(bit, std::memory_order_release);
  return DISTDL_OK;
}

// ---- exact unsigned division by a runtime constant ------------------------
// Granlund & Montgomery, "Division by invariant integers using
// multiplication" (PLDI 1994), unsigned round-up variant:
//   l = ceil(log2 d), m' = floor(2^32 (2^l - d) / d) + 1,
//   t = mulhi(m', n), q = (t + ((n - t) >> min(l,1))) >> max(l-1,0).
struct FastDiv {
  uint32_t mul, sh1, sh2, d;
};
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t l = 0;
  while ((uint64_t(1) << l) < d) ++l;
  f.mul = uint32_t(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}
__host__ __device__ inline uint32_t fd_div(uint32_t n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t t = __umulhi(f.mul, n);
#else
  uint32_t t = uint32_t((uint64_t(f.mul) * n) >> 32);
#endif
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// ---- inner product -----------------------------------------------------------
// Enqueues <a, b> over n_arrays array pairs into *result_dev; `partial` is device scratch of kDotPartials doubles.
constexpr int kDotPartials = 1024;
int launch_dot(const void* const a_dev[], const void* const b_dev[], const int64_t count[], int n_arrays,
               distdl_dtype dtype, double* partial, double* result_dev, hipStream_t st);

// ---- geometry -------------------------------------------------------------
struct DimGeom {
  int64_t in_start, in_size, out_start, out_size;
  int32_t halo[2], pad[2], extra[2];
  int64_t buf, bulk_off, origin;
};

// Element access by storage type (uint16_t holds bf16: widened on load, rounded to nearest even on store).
__device__ inline float ld(const float* p, size_t i) { return p[i]; }
__device__ inline float ld(const uint16_t* p, size_t i) { return __uint_as_float((uint32_t)p[i] << 16); }
__device__ inline void st(float* p, size_t i, float v) { p[i] = v; }
__device__ inline void st(uint16_t* p, size_t i, float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) {
    p[i] = (uint16_t)((u >> 16) | 0x40u);
    return;
  }
  u += 0x7fffu + ((u >> 16) & 1u);
  p[i] = (uint16_t)(u >> 16);
}

// Per-worker geometry as the kernels read it (3 feature dims, leading dims of
// extent 1 when D < 3).
struct WorkerDev {
  int32_t buf[3];     // buffer extent in cells
  int32_t out[3];     // owned output extent
  int32_t origin[3];  // buffer coordinate of the first tap of the first output
  int32_t bulk_off[3];
  int32_t in_size[3];
  int32_t dom_lo[3], dom_hi[3];  // buffer coordinates [lo, hi) of the cells inside the global domain (the rest is zero padding)
  int32_t pad_[2];
};

// One source of a box task: the same box seen in another worker's buffer.
struct BoxSrc {
  int32_t worker;
  int32_t org[3];
};

// A rectangular box of cells in one worker's buffer that is zero-filled
// (nsrc == 0), copied from src[0] (halo forward) or that gathers its sources,
// adds them and clears them (halo adjoint).
struct BoxTask {
  int32_t dst_worker;
  int32_t nsrc;
  int32_t src_begin;  // index into the flat BoxSrc array
  int32_t org[3];     // origin in the destination buffer (cells)
  int32_t ext[3];     // extent (cells)
  FastDiv div_row;    // by ext[2] * C / V  (vector units per contiguous run)
  FastDiv div_e1;     // by ext[1]
  FastDiv div_e0;     // by ext[0]
};

struct BlockRef {
  int32_t task;
  uint32_t unit0;  // first vector unit of the task this block handles
};

// Device form of a box: the same box as one worker's buffer addresses it, in
// vector units (offset of a unit = base + n * sn + c0 * s0 + c1 * s1 + col).
struct HaloView {
  int32_t worker;
  uint32_t s1, s0;
  uint32_t pad_;
  uint64_t sn;
  uint64_t base;
};
// Device form of a task: everything a workgroup needs in one record, so that
// the only dependent loads before the data are block -> task -> pointer.
struct HaloTaskDev {
  HaloView dst;
  HaloView src0;     // first source (nsrc >= 1)
  int32_t nsrc;
  int32_t src_begin;  // sources 1 .. nsrc-1 are views[src_begin + 1 ...]
  uint32_t total;     // vector units of the task
  uint32_t pad_;
  FastDiv div_row, div_e1, div_e0;
};

struct TaskTable {
  std::vector<BoxTask> tasks;
  std::vector<BoxSrc> srcs;
  std::vector<BlockRef> blocks;
  HaloTaskDev* d_tasks = nullptr;
  HaloView* d_views = nullptr;  // one per BoxSrc, same indexing
  BlockRef* d_blocks = nullptr;
  int vec = 1;  // elements per vector unit the tables were built for
  int64_t cells_copied = 0, cells_zeroed = 0, cells_band = 0;
};

// Device copies of small host tables (a caller's pointer arrays, the block descriptors of a GEMM launch).  A call
// site sees a few tables in turn (the activations of the forward pass, the gradients of the backward pass, ...):
// the cache keeps the last kSlots of them per stream, each in its own device block, so that in steady state
// upload() finds its table and copies nothing -- which also keeps a warmed-up call free of copies when the caller
// records it into a graph.  Rules that keep a block from changing under a reader:
//   - a block is only ever rewritten (or freed and re-allocated) for a call on the stream it was last used on, so
//     the copy is ordered behind every kernel that reads the old contents;
//   - a block that was selected while its stream was being captured is pinned: the graph's kernel nodes hold its
//     address, so it is never rewritten or freed before release();
//   - a table that is not cached cannot be uploaded during capture (the copy would read host memory at replay):
//     that call fails, the caller has to make it once eagerly first;
//   - at most kMaxSlots blocks exist; when none may be reused the call fails instead of evicting a live one.
struct SlotCache {
  static constexpr int kSlots = 8;
  static constexpr int kMaxSlots = 64;
  struct Entry {
    std::vector<unsigned char> host;
    void* dev = nullptr;
    size_t cap = 0;
    hipStream_t stream = nullptr;
    uint64_t used = 0;
    bool live = false, pinned = false;
  };
  std::vector<Entry> entries;
  uint64_t clock = 0;
  int selected = -1;  // entry chosen by the last upload()
  // capturing: 1 / 0, or -1 to ask the runtime about `stream`.  simulate: apply the policy only, no HIP call
  // (host-side tests of the policy).
  int upload(const void* bytes, size_t nbytes, hipStream_t stream, int capturing = -1, bool simulate = false);
  void* dev() const { return selected < 0 ? nullptr : entries[selected].dev; }
  void release();
};

struct PtrTable {
  SlotCache cache;
  std::vector<const void*> host;  // the array selected by the last upload()
  void** dev = nullptr;           // its device copy
  int upload(const void* const* ptrs, size_t n, hipStream_t stream) {
    int rc = cache.upload(ptrs, n * sizeof(void*), stream);
    if (rc) return rc;
    dev = (void**)cache.dev();
    host.assign(ptrs, ptrs + n);
    return DISTDL_OK;
  }
  void release() {
    cache.release();
    dev = nullptr;
  }
};

template <class T>
struct DevArray {
  SlotCache cache;
  T* dev = nullptr;  // the block selected by the last upload()
  int upload(const std::vector<T>& v, hipStream_t st) {
    int rc = cache.upload(v.data(), v.size() * sizeof(T), st);
    if (rc) return rc;
    dev = (T*)cache.dev();
    return DISTDL_OK;
  }
  void release() {
    cache.release();
    dev = nullptr;
  }
};

}  // namespace distdl

struct distdl_plan {
  int D = 0;
  int64_t n_b = 0, n_ci = 0, n_co = 0;
  distdl_dtype dtype = DISTDL_F32;
  bool explicit_halo = false;
  int32_t P[3] = {1, 1, 1};
  int32_t ksize[3] = {1, 1, 1}, stride[3] = {1, 1, 1}, padding[3] = {0, 0, 0}, dilation[3] = {1, 1, 1};
  int64_t in_shape[3] = {1, 1, 1}, out_shape[3] = {1, 1, 1};
  std::vector<distdl::DimGeom> dims[3];  // index d in [0, D)
  int n_workers = 0;
  int device = 0;

  // device-side tables
  distdl::WorkerDev* d_workers = nullptr;
  std::vector<distdl::WorkerDev> workers;
  distdl::TaskTable fwd16, fwd1, adj16, adj1;  // 16-byte-vector and scalar variants
  distdl::PtrTable tab_x, tab_y, tab_dx, tab_dy;
  int64_t max_out_cells = 0, max_buf_cells = 0;

  // weight re-layout scratch for the convolution kernels (library-owned)
  float* d_wt = nullptr;
  distdl::FastDiv* d_pooldiv = nullptr;  // per worker: division by buf[1], buf[2], out[1], out[2] (pooling kernels)
  size_t wt_elems = 0;
  mutable int maxpool_ok = -1;    // 1 once every max-pool window is known to hold an in-domain cell
  mutable int corr_mfma_ok = -1;  // cached answer of corr_mfma_supported(): -1 not asked yet

  int coords(int w, int d) const {
    int c[3];
    int t = w;
    for (int k = 2; k >= 0; --k) {
      c[k] = t % P[k];
      t /= P[k];
    }
    return c[d];
  }
};
