// Argument blocks and entry points of the MFMA convolution kernels.
#pragma once
#include <cstddef>
#include <cstdint>

#include "common.h"

namespace distdl {

struct CorrArgs {
  int32_t mode;  // 0: forward (x^ -> y), 1: one stride-parity class of the data gradient (dy -> dx^)
  int32_t n_b, kc, nc;  // batch, contraction channels (input tensor), output channels
  int32_t ntn;          // 32-wide output-channel tiles
  int32_t n_workers;
  int32_t nt[3];         // taps per dimension in this launch
  int32_t tapoff[3][8];  // input offset of tap i along dimension d
  int32_t tapid[3][8];   // index of that tap in the layer's kernel
  int32_t tapmin[3], tapspan[3];
  int32_t is[3];   // input step per output step
  int32_t s[3];    // layer stride
  int32_t par[3];  // parity class (mode 1)
  int32_t tr, tc;  // rows x columns (dimensions 1, 2) of a workgroup's output window
  int32_t g0;      // output planes (dimension 0) a workgroup walks through
  int32_t ck;      // contraction channels per chunk: 8, or 16 when the launch multiplies in bf16
  int32_t R, Cw, CwQ;  // patch rows, cells per row, cells per residue class of the row
  int32_t a_vec4;      // patch size in 16-byte units
  int32_t a_pad;       // the same, rounded up to whole 64-lane loads (the variant that loads straight into LDS)
  int32_t bufb;        // bytes of one staging buffer of that variant: patch (a_pad units), then the weights
  FastDiv div_cw, div_tc, div_is2, div_cwq;  // exact division by Cw, tc, is[2], CwQ in the per-workgroup set-up
  int32_t tiles_max;   // tiles of the largest worker
  const float* wt;     // weights in staging order
  const int* tapinfo;  // device tables behind the weights: 8 plane offsets, then one patch offset per (t1, t2)
  const void* bias;    // may be null; element type of the tensors
};

struct WgradArgs {
  int32_t n_b, ci, co;
  int32_t k[3], s[3], dil[3];
  int32_t nchunks;  // position chunks per worker
  int32_t ncell;    // input cells the taps of 32 consecutive output columns read
  int32_t span;     // input rows the taps of one output row cover: (rows - 1) * dil1 + 1
  int32_t ob;       // output rows per work unit of the plane-per-workgroup kernel
  int64_t slot;     // floats per (worker, chunk) partial: taps*ci*co + co
};

// Geometry of one worker as a correlation launch sees it: extent and first cell of the tensor it reads,
// number of output positions per dimension, extent / first cell / step of the tensor it writes.
struct PerWorker {
  int32_t in_ext[3], in_base[3], nq[3], out_ext[3], out_base[3], os[3];
};

__host__ __device__ inline PerWorker derive(const WorkerDev& wd, const CorrArgs& a) {
  PerWorker g;
  for (int d = 0; d < 3; ++d) {
    if (a.mode == 0) {
      g.in_ext[d] = wd.buf[d];
      g.in_base[d] = wd.origin[d];
      g.nq[d] = wd.out[d];
      g.out_ext[d] = wd.out[d];
      g.out_base[d] = 0;
      g.os[d] = 1;
    } else {
      const int s = a.s[d], op = wd.origin[d] + a.par[d];
      const int first = op % s;  // first buffer cell of this parity class
      g.in_ext[d] = wd.out[d];
      g.in_base[d] = -(op / s);
      g.nq[d] = first < wd.buf[d] ? (wd.buf[d] - 1 - first) / s + 1 : 0;
      g.out_ext[d] = wd.buf[d];
      g.out_base[d] = first;
      g.os[d] = s;
    }
  }
  return g;
}

// Arguments of the forward correlation and of one stride-parity class of the data gradient (taps, steps).
CorrArgs forward_args(const distdl_plan* p);
CorrArgs class_args(const distdl_plan* p, const int par[3]);
// Grows the plan's weight re-layout scratch to at least `elems` floats.
int ensure_wscratch(distdl_plan* p, size_t elems);

bool corr_mfma_supported(const distdl_plan* p);
bool wgrad_mfma_supported(const distdl_plan* p);
size_t bwd_scratch_elems(const distdl_plan* p);
int wgrad_chunks(const distdl_plan* p);
// All three expect the plan's pointer tables (tab_x, tab_y, tab_dy, tab_dx) to be uploaded.
int conv_fwd_mfma(distdl_plan* p, const void* w, const void* bias, hipStream_t st);
int conv_bwd_data_mfma(distdl_plan* p, const void* w, hipStream_t st);
int conv_wgrad_mfma(distdl_plan* p, float* partial, hipStream_t st);

// Kernels for layers with at most 16 input and 16 output channels (16 x 16 MFMA tiles).  `vec`: channel counts
// are multiples of 4 and every array is 16-byte aligned.
bool corr16_fwd_supported(const distdl_plan* p, bool vec);
bool corr16_bwd_supported(const distdl_plan* p, bool vec);
int conv_fwd16(distdl_plan* p, const float* w, const float* bias, bool vec, hipStream_t st);
int conv_bwd_data16(distdl_plan* p, const float* w, bool vec, hipStream_t st);
bool wgrad16_supported(const distdl_plan* p, bool vec);
int wgrad16_chunks(const distdl_plan* p, bool vec);
int conv_wgrad16(distdl_plan* p, float* partial, bool vec, hipStream_t st);

}  // namespace distdl
