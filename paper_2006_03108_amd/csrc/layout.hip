// Conversion between the paper's logical tensor order and the library's.
// Sec. 4 "Sparse layers" writes a worker's tensors as n_b x n_c x m_0 x ... (one
// plane of feature-space cells per channel); the kernels of this library keep
// channels last.  A caller that holds planes-first tensors converts them
// here: per (worker, sample) this is the transpose of an n_c x cells matrix,
// staged through LDS in tiles of 32 channels x 128 cells so that both sides
// are read and written in contiguous runs (256-byte runs of one channel's
// plane; whole cells, as 16-byte pieces, on the channels-last side).
#include <algorithm>

#include "common.h"
#include "profile.h"

namespace distdl {

constexpr int kLayoutWorkers = 32;  // workers per launch (pointers travel as kernel arguments)
constexpr int kTileCells = 256, kTileCh = 32;

struct LayoutArgs {
  const void* src[kLayoutWorkers];
  void* dst[kLayoutWorkers];
  int32_t cells[kLayoutWorkers];
  int32_t n_c, cell_tiles_max, ch_tiles;
  int32_t vec;  // channels-last side may use 16-byte pieces (n_c % 4 == 0, aligned pointers, 4-byte elements)
};

// T: storage type of an element (uint32_t for fp32, uint16_t for bf16); TO_CL: planes-first -> channels-last.
template <class T, bool TO_CL>
__global__ __launch_bounds__(256) void layout_kernel(LayoutArgs a) {
  __shared__ T tile[kTileCells][kTileCh + 1];  // [cell][channel], odd pitch: the cell-major side is conflict-free
  const int w = blockIdx.z, n = blockIdx.y;
  const int cells = a.cells[w];
  // Workgroups are dealt to the eight XCDs round-robin by their index.  Tiles that are neighbours along a plane
  // share the cache lines their 4-byte-aligned runs straddle, so consecutive tiles are given to one XCD (one L2):
  // the shared line is fetched once, and the two halves of a written line meet in one cache.
  const uint32_t r = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (r >= (uint32_t)a.cell_tiles_max * a.ch_tiles) return;
  const int ct = r / a.ch_tiles, cht = r - ct * a.ch_tiles;
  const int cell0 = ct * kTileCells, ch0 = cht * kTileCh;
  if (cell0 >= cells) return;
  const int tid = threadIdx.x;
  const size_t sample = (size_t)n * a.n_c * cells;
  // planes-first side: lane = cell, four channel rows per pass
  const T* pf_src = (const T*)a.src[w] + sample;
  T* pf_dst = (T*)a.dst[w] + sample;
  // channels-last side: 32 channels of a cell are contiguous
  const T* cl_src = (const T*)a.src[w] + sample;
  T* cl_dst = (T*)a.dst[w] + sample;
  // planes-first side: a wave covers 64 consecutive cells of one channel (256 bytes), all loads of a thread are
  // issued before the first LDS write so that a block has its whole 16 KB tile in flight
  const int pc = tid & 63, pr = tid >> 6;
  constexpr int kPasses = (kTileCells / 64) * (kTileCh / 4);
  if (TO_CL) {
    T v[kPasses];
#pragma unroll
    for (int i = 0; i < kPasses; ++i) {
      const int ch = pr + 4 * (i % (kTileCh / 4)), c = pc + 64 * (i / (kTileCh / 4));
      v[i] = 0;
      if (cell0 + c < cells && ch0 + ch < a.n_c)
        v[i] = __builtin_nontemporal_load(pf_src + (size_t)(ch0 + ch) * cells + cell0 + c);
    }
#pragma unroll
    for (int i = 0; i < kPasses; ++i) tile[pc + 64 * (i / (kTileCh / 4))][pr + 4 * (i % (kTileCh / 4))] = v[i];
  } else if (sizeof(T) == 4 && a.vec) {
    const int k4 = (tid & 7) * 4, cc0 = tid >> 3;  // 8 pieces per cell, 32 cells per pass
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 v[kTileCells / 32];
#pragma unroll
    for (int i = 0; i < kTileCells / 32; ++i) {
      const int cc = cc0 + 32 * i;
      v[i] = u32x4{0, 0, 0, 0};
      if (cell0 + cc < cells && ch0 + k4 < a.n_c)
        v[i] = __builtin_nontemporal_load((const u32x4*)(cl_src + (size_t)(cell0 + cc) * a.n_c + ch0 + k4));
    }
#pragma unroll
    for (int i = 0; i < kTileCells / 32; ++i) {
      const int cc = cc0 + 32 * i;
      tile[cc][k4] = (T)v[i][0], tile[cc][k4 + 1] = (T)v[i][1], tile[cc][k4 + 2] = (T)v[i][2], tile[cc][k4 + 3] = (T)v[i][3];
    }
  } else {
    const int k = tid & 31, cc0 = tid >> 5;
#pragma unroll
    for (int i = 0; i < kTileCells / 8; ++i) {
      const int cc = cc0 + 8 * i;
      if (cell0 + cc < cells && ch0 + k < a.n_c) tile[cc][k] = cl_src[(size_t)(cell0 + cc) * a.n_c + ch0 + k];
    }
  }
  __syncthreads();
  if (!TO_CL) {
#pragma unroll
    for (int i = 0; i < kPasses; ++i) {
      const int ch = pr + 4 * (i % (kTileCh / 4)), c = pc + 64 * (i / (kTileCh / 4));
      if (cell0 + c < cells && ch0 + ch < a.n_c) pf_dst[(size_t)(ch0 + ch) * cells + cell0 + c] = tile[c][ch];
    }
  } else if (sizeof(T) == 4 && a.vec) {
    const int k4 = (tid & 7) * 4, cc0 = tid >> 3;
#pragma unroll
    for (int i = 0; i < kTileCells / 32; ++i) {
      const int cc = cc0 + 32 * i;
      if (cell0 + cc < cells && ch0 + k4 < a.n_c) {
        uint4 v;
        v.x = tile[cc][k4], v.y = tile[cc][k4 + 1], v.z = tile[cc][k4 + 2], v.w = tile[cc][k4 + 3];
        *(uint4*)(cl_dst + (size_t)(cell0 + cc) * a.n_c + ch0 + k4) = v;
      }
    }
  } else {
    const int k = tid & 31, cc0 = tid >> 5;
#pragma unroll
    for (int i = 0; i < kTileCells / 8; ++i) {
      const int cc = cc0 + 8 * i;
      if (cell0 + cc < cells && ch0 + k < a.n_c) cl_dst[(size_t)(cell0 + cc) * a.n_c + ch0 + k] = tile[cc][k];
    }
  }
}

}  // namespace distdl

using namespace distdl;

extern "C" int distdl_layout_convert(const distdl_plan* plan, int what, int to_channels_last,
                                     const void* const src_dev[], void* const dst_dev[], void* stream) {
  if (!plan || !src_dev || !dst_dev) return set_error(DISTDL_ERR_NULL, "layout_convert: null argument");
  if (what != 0 && what != 1) return set_error(DISTDL_ERR_INVALID_ARG, "layout_convert: what = %d (0: padded buffers, 1: outputs)", what);
  const size_t esz = dtype_size(plan->dtype);
  const int64_t n_c = what == 0 ? plan->n_ci : plan->n_co;
  if (plan->n_b > 65535) return set_error(DISTDL_ERR_UNSUPPORTED, "layout_convert: more than 65535 samples");
  hipStream_t st = (hipStream_t)stream;
  for (int w = 0; w < plan->n_workers; ++w) {
    if (!src_dev[w] || !dst_dev[w]) return set_error(DISTDL_ERR_NULL, "layout_convert: array of worker %d is null", w);
    if ((uintptr_t)src_dev[w] % esz || (uintptr_t)dst_dev[w] % esz)
      return set_error(DISTDL_ERR_INVALID_ARG, "layout_convert: array of worker %d is misaligned", w);
  }
  for (int w0 = 0; w0 < plan->n_workers; w0 += kLayoutWorkers) {
    LayoutArgs a{};
    const int nw = std::min(kLayoutWorkers, plan->n_workers - w0);
    int64_t max_cells = 0;
    bool vec = esz == 4 && n_c % 4 == 0;
    for (int i = 0; i < nw; ++i) {
      const WorkerDev& wd = plan->workers[w0 + i];
      const int64_t cells = what == 0 ? (int64_t)wd.buf[0] * wd.buf[1] * wd.buf[2] : (int64_t)wd.out[0] * wd.out[1] * wd.out[2];
      a.src[i] = src_dev[w0 + i];
      a.dst[i] = dst_dev[w0 + i];
      a.cells[i] = (int32_t)cells;  // the planner bounds a sample of a partition to 2^31 elements
      max_cells = std::max(max_cells, cells);
      const void* cl = to_channels_last ? (const void*)dst_dev[w0 + i] : src_dev[w0 + i];
      vec &= (uintptr_t)cl % 16 == 0;
    }
    a.n_c = (int32_t)n_c;
    a.cell_tiles_max = (int32_t)((max_cells + kTileCells - 1) / kTileCells);
    a.ch_tiles = (int32_t)((n_c + kTileCh - 1) / kTileCh);
    a.vec = vec;
    const int64_t gx = (int64_t)a.cell_tiles_max * a.ch_tiles;
    if (gx >= (int64_t(1) << 31)) return set_error(DISTDL_ERR_UNSUPPORTED, "layout_convert: tensor too large");
    const dim3 grid((unsigned)((gx + 7) / 8 * 8), (unsigned)plan->n_b, (unsigned)nw), block(256);
    ProfScope prof(to_channels_last ? "layout_to_cl" : "layout_from_cl", st);
    if (esz == 4) {
      if (to_channels_last) hipLaunchKernelGGL((layout_kernel<uint32_t, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((layout_kernel<uint32_t, false>), grid, block, 0, st, a);
    } else {
      if (to_channels_last) hipLaunchKernelGGL((layout_kernel<uint16_t, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((layout_kernel<uint16_t, false>), grid, block, 0, st, a);
    }
  }
  DISTDL_HIP_TRY(hipGetLastError());
  return DISTDL_OK;
}
