// Weight gradient of the local convolution (Sec. 4, "[dConv]*" with respect to w and b) for layers with at
// most 16 input and 16 output channels, fp32, channels-last, unit stride in the last two feature dimensions.
//
//   dw^[tap][ci][co] = sum_pos x^[cell(pos) + tap][ci] * dy[pos][co],      db^[co] = sum_pos dy[pos][co]
//
// v_mfma_f32_16x16x4_f32 makes a 16 x 16 (ci x co) tile from 4 positions per instruction, so a layer with few
// channels does not pay for the 32 x 32 tile of the wide kernels.  Operand layout: A lane l holds
// A[i = l % 16][k = l / 16], B lane l holds B[k = l / 16][j = l % 16], D register v of lane l holds
// D[i = 4 * (l / 16) + v][j = l % 16].
//
// A workgroup walks through units of G planes x RB output rows.  It copies the input rows and the dy rows of a
// unit into LDS with 16 floats per cell, the dy rows at the *input* row pitch and plane pitch (columns and rows
// that are no output stay zero): then the cell a tap reads is position + a per-tap constant for every
// position of the unit, rows, planes and all, so a wave multiplies 16 consecutive padded positions at a time and
// the 64 lanes of an operand read are 64 consecutive floats.  Zero dy entries cancel the padded positions.
#include <algorithm>

#include "common.h"
#include "conv_mfma.h"
#include "profile.h"

namespace distdl {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr uint32_t kOobS = 0x7ffffff0u;  // buffer offset that always fails the range check (buffers are < 2 GiB)
constexpr int kPAX = 12, kPAD = 6;       // input / dy pieces per thread and unit

struct Wgrad16Args {
  int32_t n_b, ci, co;
  int32_t k[3], s0, dil[3];
  int32_t t1d[32], t2d[32];  // row / column offset of tap t of a kernel plane (already times the dilation)
  int32_t G, RB;             // planes and output rows per unit (G > 1 only when every plane is one sample)
  int32_t nchunks;           // unit chunks per worker
  int32_t xcells, dcells;    // LDS cells of the input / dy staging areas
  int64_t slot;              // floats per partial: taps * ci * co + co
};

__device__ inline __amdgpu_buffer_rsrc_t rsrc_of(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// n / d for n < 2^20 through the reciprocal (set-up code: a few divisions per thread)
__device__ inline uint32_t div_small(uint32_t n, uint32_t d, float rcp) {
  uint32_t q = (uint32_t)((float)n * rcp);
  if (q * d > n) --q;
  else if ((q + 1) * d <= n) ++q;
  return q;
}

template <int V>
struct Piece;
template <>
struct Piece<4> {
  typedef u32x4 T;
  static __device__ inline T load(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, v, s, 0);
  }
};
template <>
struct Piece<1> {
  typedef uint32_t T;
  static __device__ inline T load(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, v, s, 0);
  }
};

// grid: (k0, chunks, workers).  NT = taps of a kernel plane, V = floats per staged piece (4 needs channel counts
// that are multiples of 4 and 16-byte aligned arrays).
template <int NT, int V>
__global__ __launch_bounds__(256, (NT > 9 && V == 4) ? 1 : 2) void wgrad16_kernel(const WorkerDev* __restrict__ workers, void* const* x_bufs,
                                                         void* const* dy_bufs, float* __restrict__ partial,
                                                         Wgrad16Args a) {
  extern __shared__ float lds[];
  typedef typename Piece<V>::T PT;
  const int t0 = blockIdx.x, chunk = blockIdx.y, worker = blockIdx.z;
  const WorkerDev wd = workers[worker];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kg = lane >> 4, ij = lane & 15;
  const int out0 = wd.out[0], out1 = wd.out[1], out2 = wd.out[2];
  const int span1 = (a.k[1] - 1) * a.dil[1] + 1, span2 = (a.k[2] - 1) * a.dil[2] + 1;
  const int G = a.G, RB = a.RB, Rx = RB + span1 - 1, Cx = out2 + span2 - 1;
  const int planes = a.n_b * out0;
  const int nrb = (out1 + RB - 1) / RB;
  const int units = ((planes + G - 1) / G) * nrb;
  const int per = (units + a.nchunks - 1) / a.nchunks;
  const int u_begin = chunk * per, u_end = min(units, u_begin + per);

  const uint32_t sx2 = a.ci, sx1 = wd.buf[2] * sx2, sx0 = wd.buf[1] * sx1, sxn = wd.buf[0] * sx0;
  const uint32_t sy2 = a.co, sy1 = out2 * sy2, sy0 = out1 * sy1, syn = out0 * sy0;
  const __amdgpu_buffer_rsrc_t rx = rsrc_of(x_bufs[worker], (uint32_t)a.n_b * sxn * 4u);
  const __amdgpu_buffer_rsrc_t rdy = rsrc_of(dy_bufs[worker], (uint32_t)a.n_b * syn * 4u);

  char* const ldsb = (char*)lds;
  const uint32_t dy_lds = (uint32_t)a.xcells * 64u;
  // everything that is not staged must read as zero: channel padding, dy columns / rows that are no output,
  // the cells behind the last row
  for (int i = tid; i < (a.xcells + a.dcells) * 4; i += 256) ((float4*)lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

  // per-thread pieces of a unit: global byte offset relative to the unit's first cell; LDS byte offset (the
  // staging areas are at most 64 KiB) with the piece's row in bits 16-23 and its plane in bits 24-29, by which
  // the rows and planes a ragged last unit does not have are switched off
  uint32_t xg[kPAX], xl[kPAX], dg[kPAD], dl[kPAD];
  {
    const uint32_t cpp = a.ci / V, ppr = Cx * cpp, npieces = G * Rx * ppr;  // pieces per cell, row, unit
    const float r_ppr = 1.0f / (float)ppr, r_cpp = 1.0f / (float)cpp, r_rx = 1.0f / (float)Rx;
#pragma unroll
    for (int i = 0; i < kPAX; ++i) {
      const uint32_t q = tid + i * 256;
      xg[i] = kOobS;
      xl[i] = 0;
      if (q < npieces) {
        const uint32_t row = div_small(q, ppr, r_ppr), within = q - row * ppr;
        const uint32_t gi = div_small(row, Rx, r_rx), r = row - gi * Rx;
        const uint32_t cell = div_small(within, cpp, r_cpp), part = within - cell * cpp;
        xg[i] = (gi * sxn + r * sx1 + within * V) * 4u;
        xl[i] = ((((gi * Rx + r) * Cx + cell) * 16u + part * V) * 4u) | (r << 16) | (gi << 24);
      }
    }
  }
  {
    const uint32_t cpp = a.co / V, ppr = out2 * cpp, npieces = G * RB * ppr;
    const float r_ppr = 1.0f / (float)max(ppr, 1u), r_cpp = 1.0f / (float)cpp, r_rb = 1.0f / (float)RB;
#pragma unroll
    for (int i = 0; i < kPAD; ++i) {
      const uint32_t q = tid + i * 256;
      dg[i] = kOobS;
      dl[i] = dy_lds;
      if (q < npieces) {
        const uint32_t row = div_small(q, ppr, r_ppr), within = q - row * ppr;
        const uint32_t gi = div_small(row, RB, r_rb), r = row - gi * RB;
        const uint32_t cell = div_small(within, cpp, r_cpp), part = within - cell * cpp;
        dg[i] = (gi * syn + r * sy1 + within * V) * 4u;
        dl[i] = (dy_lds + (((gi * Rx + r) * Cx + cell) * 16u + part * V) * 4u) | (r << 16) | (gi << 24);
      }
    }
  }

  // operand addresses: lane l reads float l of the 64 that four consecutive cells hold
  uint32_t tc[NT];  // wave-uniform, so these live in scalar registers
#pragma unroll
  for (int t = 0; t < NT; ++t) tc[t] = (uint32_t)__builtin_amdgcn_readfirstlane((a.t1d[t] * Cx + a.t2d[t]) * 64);
  const uint32_t vb = dy_lds + lane * 4u;
  const int ngroups = (((G - 1) * Rx + RB) * Cx + 15) >> 4;

  floatx4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  float bsum = 0.f;

  PT rxv[kPAX], rdv[kPAD];
  auto load_unit = [&](int u) {
    const int pg = u / nrb, rb = u - pg * nrb;
    const int p0 = pg * G;  // first plane; with G > 1 a plane is a sample
    const int n = p0 / out0, o0 = p0 - n * out0;
    const uint32_t xbase = ((uint32_t)n * sxn + (uint32_t)(wd.origin[0] + o0 * a.s0 + t0 * a.dil[0]) * sx0 +
                            (uint32_t)(wd.origin[1] + rb * RB) * sx1 + (uint32_t)wd.origin[2] * sx2) * 4u;
    const uint32_t ybase = ((uint32_t)n * syn + (uint32_t)o0 * sy0 + (uint32_t)(rb * RB) * sy1) * 4u;
    const uint32_t rows_valid = (uint32_t)min(RB, out1 - rb * RB), planes_valid = (uint32_t)min(G, planes - p0);
#pragma unroll
    for (int i = 0; i < kPAX; ++i) {
      const bool ok = ((xl[i] >> 16) & 255u) < rows_valid + span1 - 1 && (xl[i] >> 24) < planes_valid;
      rxv[i] = Piece<V>::load(rx, ok ? xg[i] : kOobS, xbase);
    }
#pragma unroll
    for (int i = 0; i < kPAD; ++i) {
      const bool ok = ((dl[i] >> 16) & 255u) < rows_valid && (dl[i] >> 24) < planes_valid;
      rdv[i] = Piece<V>::load(rdy, ok ? dg[i] : kOobS, ybase);
    }
  };
  auto write_unit = [&]() {
#pragma unroll
    for (int i = 0; i < kPAX; ++i)
      if (xg[i] != kOobS) *(PT*)(ldsb + (xl[i] & 0xffffu)) = rxv[i];
#pragma unroll
    for (int i = 0; i < kPAD; ++i)
      if (dg[i] != kOobS) *(PT*)(ldsb + (dl[i] & 0xffffu)) = rdv[i];
  };
  auto read4 = [&](uint32_t addr, float (&v)[4]) {
#pragma unroll
    for (int g = 0; g < 4; ++g) v[g] = *(const float*)(ldsb + addr + g * 256);
  };

  __syncthreads();  // the zero fill is complete
  if (u_begin < u_end) load_unit(u_begin);
  for (int u = u_begin; u < u_end; ++u) {
    write_unit();
    __syncthreads();
    if (u + 1 < u_end) load_unit(u + 1);  // in flight while this unit multiplies
    for (int gidx = wave; gidx < ngroups; gidx += 4) {
      const uint32_t fo = (uint32_t)gidx * 1024u;  // 16 positions of 64 bytes
      float b[4], a0[4], a1[4];
      const uint32_t xo = fo + lane * 4u;
      read4(vb + fo, b);
      read4(xo + tc[0], a0);
      bsum += (b[0] + b[1]) + (b[2] + b[3]);
#pragma unroll
      for (int t = 0; t < NT; t += 2) {
        if (t + 1 < NT) read4(xo + tc[t + 1], a1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[g], b[g], acc[t], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < NT) read4(xo + tc[t + 2], a0);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < NT) {
#pragma unroll
          for (int g = 0; g < 4; ++g) acc[t + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[g], b[g], acc[t + 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();  // everyone is done reading this unit
  }

  // sum over the four waves in wave order through LDS (NT * 64 float4 + 64 floats), wave 3 writes the partial
  float4* red = (float4*)lds;
  float* bred = (float*)(red + NT * 64);
  bsum += __shfl_xor(bsum, 16);
  bsum += __shfl_xor(bsum, 32);
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (w > 0) {
          const float4 r = red[t * 64 + lane];
          acc[t][0] += r.x, acc[t][1] += r.y, acc[t][2] += r.z, acc[t][3] += r.w;
        }
        if (w < 3) red[t * 64 + lane] = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
      }
      if (w > 0) bsum += bred[lane];
      if (w < 3) bred[lane] = bsum;
    }
    __syncthreads();
  }
  if (wave != 3) return;
  float* slot = partial + ((size_t)worker * a.nchunks + chunk) * a.slot;
  if (ij < a.co) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ci = 4 * kg + v;
        if (ci < a.ci) slot[((size_t)(t0 * NT + t) * a.ci + ci) * a.co + ij] = acc[t][v];
      }
    if (t0 == 0 && kg == 0) slot[(size_t)a.k[0] * NT * a.ci * a.co + ij] = bsum;
  }
}

struct Wgrad16Shape {
  int G, RB, nchunks, xcells, dcells, lds;
};

bool wgrad16_shape(const distdl_plan* p, bool vec, Wgrad16Shape& s) {
  const int nt = p->ksize[1] * p->ksize[2];
  if (p->dtype != DISTDL_F32 || p->explicit_halo) return false;
  if (p->n_ci > 16 || p->n_co > 16 || p->stride[1] != 1 || p->stride[2] != 1) return false;
  if (nt != 1 && nt != 3 && nt != 5 && nt != 7 && nt != 9 && nt != 25) return false;
  if ((double)p->n_b * p->max_buf_cells * std::max(p->n_ci, p->n_co) * 4.0 >= 2147480000.0) return false;
  const int V = vec ? 4 : 1;
  if (vec && (p->n_ci % 4 || p->n_co % 4)) return false;
  const int span1 = (p->ksize[1] - 1) * p->dilation[1] + 1, span2 = (p->ksize[2] - 1) * p->dilation[2] + 1;
  int out0 = 0, out1 = 0, out2 = 0;
  int64_t units_plane = 0;
  for (const WorkerDev& wd : p->workers) {
    out0 = std::max(out0, wd.out[0]);
    out1 = std::max(out1, wd.out[1]);
    out2 = std::max(out2, wd.out[2]);
  }
  if (out1 < 1 || out2 < 1) return false;
  const int Cx = out2 + span2 - 1;
  const int64_t tapmax = (int64_t)(span1 - 1) * Cx + span2 - 1;
  auto fits = [&](int G, int RB, Wgrad16Shape& o) {
    const int Rx = RB + span1 - 1;
    const int64_t xpieces = (int64_t)G * Rx * Cx * (p->n_ci / V), dpieces = (int64_t)G * RB * out2 * (p->n_co / V);
    if (xpieces > kPAX * 256 || dpieces > kPAD * 256 || Rx > 255 || G > 63) return false;
    const int64_t F = ((int64_t)(G - 1) * Rx + RB) * Cx, F16 = (F + 15) / 16 * 16;
    const int64_t xcells = std::max<int64_t>(F16 + tapmax + 1, (int64_t)G * Rx * Cx), dcells = F16;
    const int64_t lds = std::max<int64_t>((xcells + dcells) * 64, (int64_t)nt * 1024 + 256);
    if (lds > 64 * 1024) return false;
    o.G = G, o.RB = RB, o.xcells = (int)xcells, o.dcells = (int)dcells, o.lds = (int)lds;
    return true;
  };
  // whole planes, several of them when a plane is one sample and small; else blocks of rows
  bool found = false;
  const bool plane_is_sample = out0 == 1 && p->ksize[0] == 1;
  if (fits(1, out1, s)) {
    found = true;
    if (plane_is_sample)
      for (int G = 2; G <= p->n_b && G <= 63; ++G) {
        Wgrad16Shape t;
        if (!fits(G, out1, t)) break;
        s = t;
        if ((int64_t)G * (out1 + span1 - 1) * Cx >= 1024) break;  // 16 groups per wave are plenty
      }
  } else {
    for (int RB = std::min(out1, 255); RB >= 1; --RB)
      if (fits(1, RB, s)) {
        found = true;
        break;
      }
  }
  if (!found) return false;
  for (const WorkerDev& wd : p->workers) {
    const int64_t planes = p->n_b * wd.out[0];
    units_plane = std::max<int64_t>(units_plane, (planes + s.G - 1) / s.G * ((wd.out[1] + s.RB - 1) / s.RB));
  }
  const int64_t blocks = (int64_t)p->ksize[0] * p->n_workers;
  s.nchunks = (int)std::max<int64_t>(1, std::min<int64_t>(units_plane, (512 + blocks - 1) / blocks));
  return s.nchunks <= 65535 && p->n_workers <= 65535;
}


// ---- correlation (forward, data gradient) with 16 x 16 tiles -------------------------------------------------
//
//   out[q][n] = sum_taps sum_k W[tap][k][n] * in[base + q * step + tapoff][k],   k < kc <= 16, n < nc <= 16
//
// the same implicit GEMM as corr_mfma_kernel (forward: in = x^, out = y; data gradient: in = dy, out = one
// stride-parity class of dx^), with all contraction channels staged at once (no channel chunks) and, for
// layers whose planes are single samples, tp samples stacked in one window so that small images still fill
// the 256 positions of a workgroup.  A lane reads KM consecutive channels of its cell (KM = 1, 2, 4 for
// kc <= 4, 8, 16) and issues KM MFMAs per tap.  The patch is kept in LDS as four channel groups (group kg =
// channels KM * kg ... of every cell, groups a.ps bytes apart), so that the 16 lanes of a group read
// consecutive addresses.  The tile is accumulated transposed (the weights are the first MFMA operand): a lane
// then holds four consecutive output channels of one position and stores them as 16 bytes when the output
// channel count is a multiple of 4 (sixteen 4-byte stores per step and lane before: the store instructions of
// a step took about as long to issue as half of its MFMAs), and its set-up needs 4 store offsets, not 16.

struct Corr16Args {
  CorrArgs c;                  // taps, steps and parity class of the launch
  int32_t tp, tr, tc;          // window: planes x rows x columns (tp * tr * tc <= 256)
  int32_t R, Cw;               // patch rows and cells per row of one plane
  int32_t ps;                  // bytes between the four channel groups of the patch in LDS
  int32_t tapmin1, tapmin2;    // smallest tap offset along dimensions 1, 2
  int32_t wpw, g0, ntaps;      // workgroups per worker; steps per workgroup (large patches); taps per kernel plane
  int32_t tapo[64];            // patch byte offset of tap (t1, t2)
  const float* wt;             // weights: [t0][tap][lane][KM]
  const float* bias;           // may be null
};

template <int KM>
struct VecK;
template <>
struct VecK<1> {
  typedef float T;
};
template <>
struct VecK<2> {
  typedef float2 T;
};
template <>
struct VecK<4> {
  typedef float4 T;
};
__device__ inline float comp(const float& v, int) { return v; }
__device__ inline float comp(const float2& v, int g) { return g == 0 ? v.x : v.y; }
__device__ inline float comp(const float4& v, int g) { return g == 0 ? v.x : g == 1 ? v.y : g == 2 ? v.z : v.w; }

constexpr int kPA16 = 14, kPB16 = 7;
constexpr uint32_t kSkip = 0xffffffffu;

// NT: taps per kernel plane known at compile time (tap loop unrolled, offsets in scalar registers), or 0.
template <int KM, int V, int NT, int PA>
__global__ __launch_bounds__(256, 2) void corr16_kernel(const WorkerDev* __restrict__ workers, void* const* in_bufs,
                                                        void* const* out_bufs, Corr16Args a) {
  extern __shared__ float lds[];
  typedef typename VecK<KM>::T OT;
  typedef typename Piece<V>::T PT;
  constexpr uint32_t CG = KM * 4;  // bytes per cell and channel group in LDS
  const CorrArgs& c = a.c;
  // XCD-aware order: consecutive tiles stay behind one L2
  const uint32_t nblk = gridDim.x;
  const uint32_t rblk = (blockIdx.x & 7u) * (nblk >> 3) + (blockIdx.x >> 3);
  const uint32_t worker = rblk / (uint32_t)a.wpw, slice = rblk - worker * (uint32_t)a.wpw;
  if (worker >= (uint32_t)c.n_workers) return;
  const WorkerDev wd = workers[worker];
  const PerWorker g = derive(wd, c);
  const int nq0 = g.nq[0], planes = c.n_b * nq0;
  const int n2 = (g.nq[2] + a.tc - 1) / a.tc, n1 = (g.nq[1] + a.tr - 1) / a.tr;
  const int nsteps = (planes + a.tp - 1) / a.tp;
  // The worker's (window, step) pairs, window-major, are dealt to its a.wpw workgroups.  Small patches (MULTI):
  // in contiguous, balanced runs; a run that crosses into the next window sets its address tables up again.
  // Large patches: a.g0 steps of one window per workgroup (the loop over windows costs registers these variants
  // do not have).
  constexpr bool MULTI = PA <= 6;
  const int64_t total = (int64_t)n1 * n2 * nsteps;
  int64_t f, f_end;
  if constexpr (MULTI) {
    f = total * slice / a.wpw;
    f_end = total * (slice + 1) / a.wpw;
  } else {
    const int ngrp = (nsteps + a.g0 - 1) / a.g0;
    const int64_t window = slice / (uint32_t)ngrp;
    f = window * nsteps + (int64_t)(slice - (uint32_t)window * (uint32_t)ngrp) * a.g0;
    f_end = min(f + a.g0, (window + 1) * nsteps);
    if (window >= (int64_t)n1 * n2) return;
  }
  if (f >= f_end) return;
  int q1_0 = 0, q2_0 = 0, step_begin = 0, step_end = 0;

  const uint32_t si2 = c.kc, si1 = g.in_ext[2] * si2, si0 = g.in_ext[1] * si1, sin = g.in_ext[0] * si0;
  const uint32_t so2 = c.nc, so1 = g.out_ext[2] * so2, so0 = g.out_ext[1] * so1, son = g.out_ext[0] * so0;
  const __amdgpu_buffer_rsrc_t rin = rsrc_of(in_bufs[worker], (uint32_t)c.n_b * sin * 4u);
  const __amdgpu_buffer_rsrc_t rout = rsrc_of(out_bufs[worker], (uint32_t)c.n_b * son * 4u);
  const int nt0 = c.nt[0], ntaps = a.ntaps;
  const uint32_t wfloats = (uint32_t)ntaps * 64u * KM;  // weights of one kernel plane
  const __amdgpu_buffer_rsrc_t rw = rsrc_of(a.wt, (uint32_t)max(nt0, 1) * wfloats * 4u);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kg = lane >> 4, ij = lane & 15;
  char* const ldsb = (char*)lds;
  const uint32_t plane_cells = (uint32_t)a.R * a.Cw, ncells = a.tp * plane_cells;
  const uint32_t ps = (uint32_t)a.ps, wl = 4u * ps;  // weights behind the patch
  // channel padding of the patch must read as zero
  for (uint32_t i = tid; i < ps / 4u; i += 256) ((float4*)lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

  // per-thread patch pieces: global byte offset inside the first plane of a stage (kOobS: the cell lies outside
  // the input and reads as zero) and LDS byte offset with the piece's plane in bits 24-29
  uint32_t goff[PA], loff[PA];
  uint32_t abase[4], soff[4];
  const int trtc = a.tr * a.tc, npos = a.tp * trtc;
  auto setup_pieces = [&]() {
    const uint32_t ppc = c.kc / V, npieces = ncells * ppc;
    const float r_ppc = 1.0f / (float)ppc, r_pc = 1.0f / (float)plane_cells, r_cw = 1.0f / (float)a.Cw;
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      const uint32_t q = tid + i * 256;
      goff[i] = kOobS;
      loff[i] = kSkip;
      if (q < npieces) {
        const uint32_t cell = div_small(q, ppc, r_ppc), part = q - cell * ppc;
        const uint32_t wp = div_small(cell, plane_cells, r_pc), rem = cell - wp * plane_cells;
        const uint32_t rr = div_small(rem, a.Cw, r_cw), cc = rem - rr * a.Cw;
        const int i1 = g.in_base[1] + q1_0 * c.is[1] + a.tapmin1 + (int)rr;
        const int i2 = g.in_base[2] + q2_0 * c.is[2] + a.tapmin2 + (int)cc;
        const uint32_t ch = part * V;  // first channel of the piece
        loff[i] = (cell * CG + (ch / KM) * ps + (ch % KM) * 4u) | (wp << 24);
        if (i1 >= 0 && i1 < g.in_ext[1] && i2 >= 0 && i2 < g.in_ext[2])
          goff[i] = (wp * sin + (uint32_t)i1 * si1 + (uint32_t)i2 * si2 + part * V) * 4u;
      }
    }
  };
  // operand addresses and store offsets: lane (ij, kg) multiplies window position (wave * 4 + mt) * 16 + ij.  The
  // products are accumulated transposed (weights as the first MFMA operand), so accumulator register v of that lane
  // is output channel 4 * kg + v of the same position: four consecutive channels, one 16-byte store.
  auto setup_operands = [&]() {
  const float r_trtc = 1.0f / (float)trtc, r_tc = 1.0f / (float)a.tc;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    const uint32_t pidx = (wave * 4 + mt) * 16 + ij;
    const bool live = pidx < (uint32_t)npos;
    const uint32_t pp = live ? pidx : 0;  // idle position: multiplies something in range, never stored
    const uint32_t wp = div_small(pp, trtc, r_trtc), rem = pp - wp * trtc;
    const uint32_t wr = div_small(rem, a.tc, r_tc), wc = rem - wr * a.tc;
    abase[mt] = ((wp * a.R + wr * c.is[1]) * a.Cw + wc * c.is[2]) * CG + kg * ps;
    const int q1 = q1_0 + (int)wr, q2 = q2_0 + (int)wc;
    soff[mt] = kOobS;
    if (live && q1 < g.nq[1] && q2 < g.nq[2] && 4 * kg < c.nc)
      soff[mt] = (wp * son + (uint32_t)(g.out_base[1] + g.os[1] * q1) * so1 +
                  (uint32_t)(g.out_base[2] + g.os[2] * q2) * so2 + 4 * kg) * 4u;
  }
  };
  const uint32_t ppos = (wave * 4) * 16 + ij;  // this lane's window position in M-tile 0
  // 16-byte stores need whole channel quads (V == 4 vouches for the alignment of the arrays, and for the input
  // channel count only)
  const bool wide = V == 4 && (c.nc & 3) == 0;
  float bias[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) bias[v] = (a.bias && 4 * kg + v < c.nc) ? a.bias[4 * kg + v] : 0.f;
  const uint32_t bread = wl + lane * KM * 4u;

  // a stage is (window step, kernel plane t0); stages whose input plane lies outside the input are skipped
  // A stage position carries its sample and output plane along (stepped, not divided out of the step number: a
  // division on the scalar unit is some thirty instructions, and there were three on the path of every step), and
  // the plane offset of tap t0 is an arithmetic progression in t0 (see corr_mfma_kernel), not a table look-up.
  struct StagePos {
    int step, n, q0, t0;
  };
  const int toff0 = c.tapoff[0][0], tstep = c.nt[0] > 1 ? c.tapoff[0][1] - c.tapoff[0][0] : 0;
  auto in_plane = [&](int q0, int t0) { return g.in_base[0] + q0 * c.is[0] + toff0 + t0 * tstep; };
  auto pos_of = [&](int step) {  // (set-up: once per window)
    return a.tp > 1 ? StagePos{step, step * a.tp, 0, 0} : StagePos{step, step / nq0, step % nq0, 0};
  };
  auto next_step = [&](StagePos& sp) {
    ++sp.step;
    sp.t0 = 0;
    if (a.tp > 1) sp.n += a.tp;
    else if (++sp.q0 == nq0) sp.q0 = 0, ++sp.n;
  };
  auto next_valid = [&](StagePos& sp) {  // the first stage at or behind sp whose input plane exists
    while (sp.step < step_end) {
      while (sp.t0 < nt0) {
        const int i0 = in_plane(sp.q0, sp.t0);
        if (i0 >= 0 && i0 < g.in_ext[0]) return;
        ++sp.t0;
      }
      next_step(sp);
    }
  };
  PT ra[PA];
  u32x4 rb[kPB16];
  auto load_stage = [&](const StagePos& sp, bool weights) {
    const int t0 = sp.t0;
    const uint32_t pmax = (uint32_t)min(a.tp, planes - sp.step * a.tp);
    const uint32_t sbase = ((uint32_t)sp.n * sin + (uint32_t)in_plane(sp.q0, t0) * si0) * 4u;
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[i] = Piece<V>::load(rin, (loff[i] >> 24) < pmax ? goff[i] : kOobS, sbase);
    if (weights) {
#pragma unroll
      for (int i = 0; i < kPB16; ++i) {
        const uint32_t piece = tid + i * 256;
        rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rw, piece * 4u < wfloats ? piece * 16u : kOobS,
                                                      (uint32_t)t0 * wfloats * 4u, 0);
      }
    }
  };
  auto write_stage = [&](bool weights) {
#pragma unroll
    for (int i = 0; i < PA; ++i)
      if (loff[i] != kSkip) {
        const uint32_t o = loff[i] & 0xffffu;
        if constexpr (V == 1 || KM == 4) {
          *(PT*)(ldsb + o) = ra[i];
        } else if constexpr (KM == 2) {  // a 16-byte piece covers two channel groups
          *(uint2*)(ldsb + o) = make_uint2(ra[i][0], ra[i][1]);
          *(uint2*)(ldsb + o + ps) = make_uint2(ra[i][2], ra[i][3]);
        } else {  // KM == 1: four groups of one channel
#pragma unroll
          for (int j = 0; j < 4; ++j) *(uint32_t*)(ldsb + o + j * ps) = ra[i][j];
        }
      }
    if (weights) {
#pragma unroll
      for (int i = 0; i < kPB16; ++i) {
        const uint32_t piece = tid + i * 256;
        if (piece * 4u < wfloats) *(u32x4*)(ldsb + wl + piece * 16u) = rb[i];
      }
    }
  };

  floatx4 acc[4];
  auto store_tile = [&](const floatx4 (&t)[4], uint32_t obase, uint32_t plimit) {
    // The step's offset is added into the per-lane offset: a 16-byte buffer store that takes it from a scalar
    // register has been seen to pick up, in its first data register, a value written there two instructions
    // later (the compiler inserts the wait states only for stores without a scalar offset).
    uint32_t off[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) off[mt] = (ppos + mt * 16 < plimit ? soff[mt] : kOobS) + obase;
    if (wide) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        u32x4 o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = __float_as_uint(t[mt][v] + bias[v]);
        __builtin_amdgcn_raw_buffer_store_b128(o, rout, off[mt], 0, 0);
      }
    } else {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(t[mt][v] + bias[v]), rout,
                                                4 * kg + v < c.nc ? off[mt] + 4u * v : kOobS, 0, 0);
    }
  };
  auto read_ops = [&](int tap, OT& b, OT (&av)[4]) {
    const uint32_t tapo = NT > 0 ? (uint32_t)a.tapo[tap] : (uint32_t)__builtin_amdgcn_readfirstlane(a.tapo[tap]);
    b = *(const OT*)(ldsb + bread + tap * (64 * KM * 4));
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) av[mt] = *(const OT*)(ldsb + abase[mt] + tapo);
  };
  auto multiply = [&](const OT& b, const OT (&av)[4]) {
#pragma unroll
    for (int gk = 0; gk < KM; ++gk)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(comp(b, gk), comp(av[mt], gk), acc[mt], 0, 0, 0);
  };
  // operands of tap t + 1 are read while tap t multiplies (scheduling barriers keep the reads where they are)
  auto compute = [&]() {
    OT b0, b1, a0[4], a1[4];
    read_ops(0, b0, a0);
    if constexpr (NT > 0) {
#pragma unroll
      for (int tap = 0; tap < NT; tap += 2) {
        if (tap + 1 < NT) read_ops(tap + 1, b1, a1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(b0, a0);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 2 < NT) read_ops(tap + 2, b0, a0);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 1 < NT) multiply(b1, a1);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      for (int tap = 0; tap < ntaps; tap += 2) {
        if (tap + 1 < ntaps) read_ops(tap + 1, b1, a1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(b0, a0);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 2 < ntaps) read_ops(tap + 2, b0, a0);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 1 < ntaps) multiply(b1, a1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  __syncthreads();  // the zero fill is complete
  int staged_t0 = -1;  // kernel plane whose weights are in LDS (they stay valid from window to window)
  do {
  {
    const int64_t window = f / nsteps;
    step_begin = (int)(f - window * nsteps);
    step_end = (int)min((int64_t)nsteps, step_begin + (f_end - f));
    q2_0 = (int)(window % n2) * a.tc;
    q1_0 = (int)(window / n2) * a.tr;
    f += step_end - step_begin;
  }
  setup_pieces();
  StagePos cur = pos_of(step_begin), out = cur;  // the stage in flight; the step that is being accumulated
  if (ntaps == 0) cur.step = step_end;           // a parity class no tap reaches: zeros
  next_valid(cur);
  if (cur.step < step_end) load_stage(cur, cur.t0 != staged_t0);
  setup_operands();  // while the first stage is on its way
  for (int step = step_begin; step < step_end; ++step) {
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    while (cur.step == step) {
      const bool wnow = cur.t0 != staged_t0;
      write_stage(wnow);
      staged_t0 = cur.t0;
      __syncthreads();
      ++cur.t0;
      next_valid(cur);
      if (cur.step < step_end) load_stage(cur, cur.t0 != staged_t0);  // in flight while this stage multiplies
      compute();
      __syncthreads();  // everyone is done reading this stage
    }
    store_tile(acc, ((uint32_t)out.n * son + (uint32_t)(g.out_base[0] + g.os[0] * out.q0) * so0) * 4u,
               (uint32_t)min(a.tp, planes - step * a.tp) * trtc);
    next_step(out);
  }
  } while (MULTI && f < f_end);
}

// weights in staging order: dst[t0][tap][lane = kg * 16 + j][gk] = W[tap(t0, t1, t2)][k = KM * kg + gk][n = j], with
// W[tap][k][n] = w[n][k][tap] (forward) or w[k][n][tap] (data gradient), zero beyond the channel counts
__global__ __launch_bounds__(256) void corr16_weights_kernel(const float* __restrict__ w, float* __restrict__ dst,
                                                             CorrArgs c, int km, int ci_n, int taps, int k1, int k2) {
  const int ntaps = c.nt[1] * c.nt[2];
  const int total = c.nt[0] * ntaps * 64 * km;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int gk = idx % km;
  int r = idx / km;
  const int lane = r & 63;
  r >>= 6;
  const int tap = r % ntaps, t0 = r / ntaps;
  const int t1 = tap / c.nt[2], t2 = tap - t1 * c.nt[2];
  const int k = km * (lane >> 4) + gk, nch = lane & 15;
  float v = 0.f;
  if (k < c.kc && nch < c.nc) {
    const int ftap = (c.tapid[0][t0] * k1 + c.tapid[1][t1]) * k2 + c.tapid[2][t2];
    const int co = c.mode == 0 ? nch : k, ci = c.mode == 0 ? k : nch;
    v = w[((size_t)co * ci_n + ci) * taps + ftap];
  }
  dst[idx] = v;
}

struct Corr16Shape {
  int km, tp, tr, tc, R, Cw, ps, tapmin1, tapmin2, wpw, g0, lds;
  int pieces;     // 16-byte (or 4-byte) patch pieces of a stage
  int64_t steps;  // (window, step) pairs of the largest worker
};

bool corr16_shape(const distdl_plan* p, const CorrArgs& c, bool vec, Corr16Shape& s) {
  if (c.kc > 16 || c.nc > 16 || c.kc < 1 || c.nc < 1) return false;
  if (vec && c.kc % 4) return false;
  const int V = vec ? 4 : 1;
  const int ntaps = c.nt[1] * c.nt[2];
  if (ntaps > 64) return false;
  s.km = c.kc <= 4 ? 1 : c.kc <= 8 ? 2 : 4;
  if ((ntaps * s.km + 15) / 16 > kPB16) return false;
  int span[3] = {0, 0, 0}, tmin[3] = {0, 0, 0};
  for (int d = 1; d < 3; ++d) {
    int lo = 0, hi = 0;
    for (int i = 0; i < c.nt[d]; ++i) {
      lo = i == 0 ? c.tapoff[d][i] : std::min(lo, c.tapoff[d][i]);
      hi = i == 0 ? c.tapoff[d][i] : std::max(hi, c.tapoff[d][i]);
    }
    tmin[d] = lo;
    span[d] = hi - lo;
  }
  s.tapmin1 = tmin[1];
  s.tapmin2 = tmin[2];
  int nq0max = 0, nq1max = 0, nq2max = 0;
  int64_t planes_max = 0;
  for (const WorkerDev& wd : p->workers) {
    const PerWorker g = derive(wd, c);
    nq0max = std::max(nq0max, g.nq[0]);
    nq1max = std::max(nq1max, g.nq[1]);
    nq2max = std::max(nq2max, g.nq[2]);
    planes_max = std::max<int64_t>(planes_max, (int64_t)p->n_b * g.nq[0]);
  }
  if (nq1max < 1 || nq2max < 1 || planes_max < 1) return false;
  const bool stack = c.nt[0] <= 1 && nq0max == 1 && p->n_b > 1;
  double best = -1.0;
  for (int tc = 1; tc <= std::min(nq2max, 256); ++tc)
    for (int tr = 1; tr <= std::min(nq1max, 256 / tc); ++tr) {
      int tp = 1;
      if (stack) tp = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(256 / (tr * tc), planes_max), 63));
      for (; tp >= 1; --tp) {
        const int R = (tr - 1) * c.is[1] + span[1] + 1, Cw = (tc - 1) * c.is[2] + span[2] + 1;
        const int64_t cells = (int64_t)tp * R * Cw;
        // dwords between channel groups: at least the cells of a group, congruent to 16 * km modulo 64 so that
        // the four groups of an operand read fall on different banks
        int64_t psd = cells * s.km;
        psd += ((16 * s.km - psd) % 64 + 64) % 64;
        const int64_t lds = 16 * psd + (int64_t)ntaps * 64 * s.km * 4;
        if (cells * (c.kc / V) > kPA16 * 256 || lds > 64 * 1024) continue;
        const double used = (double)(tp * tr * tc) / 256.0;
        const double cols = (double)nq2max / ((double)((nq2max + tc - 1) / tc) * tc);
        const double rows = (double)nq1max / ((double)((nq1max + tr - 1) / tr) * tr);
        const double pl = (double)planes_max / ((double)((planes_max + tp - 1) / tp) * tp);
        const double ratio = (double)cells / ((double)tp * tr * tc * c.is[1] * c.is[2]);
        const double score = used * cols * rows * pl / (1.0 + 0.3 * std::max(0.0, ratio - 1.0));
        if (score > best + 1e-12) {
          best = score;
          s.tp = tp, s.tr = tr, s.tc = tc, s.R = R, s.Cw = Cw, s.ps = (int)(4 * psd), s.lds = (int)lds;
          s.pieces = (int)(cells * (c.kc / V));
        }
        break;  // the largest plane count that fits is the one to score
      }
    }
  if (best < 0.0) return false;
  // Workgroups per worker.  Small patches: a worker's (window, step) pairs are dealt to them in balanced
  // contiguous runs, so the launch is one even round of two workgroups per compute unit whatever the window
  // count (a workgroup's set-up, its address tables, costs about as much as two steps of a 3 x 3 kernel).
  // Large patches: g0 steps of one window per workgroup, g0 from the estimate rounds x (set-up + steps) with
  // the steps dealt evenly to the groups and about 512 workgroups running at a time.
  int64_t t_max = 0, windows_max = 0;
  for (const WorkerDev& wd : p->workers) {
    const PerWorker g = derive(wd, c);
    const int64_t steps = ((int64_t)p->n_b * g.nq[0] + s.tp - 1) / s.tp;
    const int64_t windows = (int64_t)((g.nq[1] + s.tr - 1) / s.tr) * ((g.nq[2] + s.tc - 1) / s.tc);
    t_max = std::max(t_max, steps * windows);
    windows_max = std::max(windows_max, windows);
  }
  const int64_t steps_max = (planes_max + s.tp - 1) / s.tp;
  s.g0 = 0;
  if (s.pieces <= 6 * 256) {
    // (measured on the 2-D 16-channel layer: 256, 384, 768 and 1024 workgroups in all are 5 to 35 % slower than 512)
    s.wpw = (int)std::max<int64_t>(1, std::min<int64_t>(std::max<int64_t>(1, 512 / p->n_workers), t_max));
  } else {
    const int64_t per_step = std::max<int64_t>(1, windows_max) * p->n_workers;
    double best_cost = 1e300;
    s.g0 = 1;
    for (int64_t g0 = 1; g0 <= steps_max; ++g0) {
      const int64_t groups = (steps_max + g0 - 1) / g0, even = (steps_max + groups - 1) / groups;
      if (even != g0) continue;
      const double cost = (double)((groups * per_step + 511) / 512) * (2.0 + (double)g0);
      if (cost < best_cost - 1e-9) best_cost = cost, s.g0 = (int)g0;
    }
    const int64_t wpw = windows_max * ((steps_max + s.g0 - 1) / s.g0);
    if (wpw * p->n_workers > 0x7fffff00) return false;
    s.wpw = (int)wpw;
  }
  s.steps = t_max;
  return true;
}

size_t corr16_weight_elems(const CorrArgs& c) {
  const int km = c.kc <= 4 ? 1 : c.kc <= 8 ? 2 : 4;
  return (size_t)std::max(c.nt[0], 1) * c.nt[1] * c.nt[2] * 64 * km + 64;
}

int launch_corr16(distdl_plan* p, const CorrArgs& c, bool vec, const float* w, float* wscratch, const float* bias,
                  void** in_tab, void** out_tab, const char* name, hipStream_t st) {
  Corr16Shape s;
  if (!corr16_shape(p, c, vec, s)) return set_error(DISTDL_ERR_UNSUPPORTED, "conv: shape not covered by the small-channel kernel");
  if (s.steps == 0) return DISTDL_OK;
  Corr16Args a{};
  a.c = c;
  a.tp = s.tp, a.tr = s.tr, a.tc = s.tc, a.R = s.R, a.Cw = s.Cw, a.ps = s.ps;
  a.tapmin1 = s.tapmin1, a.tapmin2 = s.tapmin2;
  a.wpw = s.wpw;
  a.g0 = s.g0;
  a.ntaps = c.nt[1] * c.nt[2];
  for (int t1 = 0; t1 < c.nt[1]; ++t1)
    for (int t2 = 0; t2 < c.nt[2]; ++t2)
      a.tapo[t1 * c.nt[2] + t2] = ((c.tapoff[1][t1] - s.tapmin1) * s.Cw + (c.tapoff[2][t2] - s.tapmin2)) * s.km * 4;
  a.wt = wscratch;
  a.bias = bias;
  const int taps = p->ksize[0] * p->ksize[1] * p->ksize[2];
  const int wtotal = c.nt[0] * a.ntaps * 64 * s.km;
  if (wtotal > 0) {
    ProfScope prof("conv_relayout_w", st);
    hipLaunchKernelGGL(corr16_weights_kernel, dim3((unsigned)((wtotal + 255) / 256)), dim3(256), 0, st, w, wscratch, c,
                       s.km, (int)p->n_ci, taps, p->ksize[1], p->ksize[2]);
  }
  int64_t blocks = (int64_t)s.wpw * p->n_workers;
  blocks = (blocks + 7) / 8 * 8;
  ProfScope prof(name, st);
  // patch pieces per thread held in registers between a stage's loads and its LDS writes: 6 covers windows of
  // 3 x 3 kernels with up to 16 channels; the tables sized for 14 cost 48 registers more
#define DISTDL_LAUNCH_C16(KM_, V_, NT_)                                                                             \
  do {                                                                                                               \
    if (s.pieces <= 6 * 256)                                                                                         \
      hipLaunchKernelGGL((corr16_kernel<KM_, V_, NT_, 6>), dim3((unsigned)blocks), dim3(256), s.lds, st,             \
                         p->d_workers, in_tab, out_tab, a);                                                          \
    else                                                                                                             \
      hipLaunchKernelGGL((corr16_kernel<KM_, V_, NT_, kPA16>), dim3((unsigned)blocks), dim3(256), s.lds, st,         \
                         p->d_workers, in_tab, out_tab, a);                                                          \
  } while (0)
#define DISTDL_LAUNCH_C16_NT(KM_, V_)                                                                               \
  do {                                                                                                               \
    if (a.ntaps == 9) DISTDL_LAUNCH_C16(KM_, V_, 9);                                                                \
    else if (a.ntaps == 25) DISTDL_LAUNCH_C16(KM_, V_, 25);                                                         \
    else DISTDL_LAUNCH_C16(KM_, V_, 0);                                                                             \
  } while (0)
  if (vec) {
    if (s.km == 1) DISTDL_LAUNCH_C16_NT(1, 4);
    else if (s.km == 2) DISTDL_LAUNCH_C16_NT(2, 4);
    else DISTDL_LAUNCH_C16_NT(4, 4);
  } else {
    if (s.km == 1) DISTDL_LAUNCH_C16_NT(1, 1);
    else if (s.km == 2) DISTDL_LAUNCH_C16_NT(2, 1);
    else DISTDL_LAUNCH_C16_NT(4, 1);
  }
#undef DISTDL_LAUNCH_C16_NT
#undef DISTDL_LAUNCH_C16
  return DISTDL_OK;
}

}  // namespace

bool wgrad16_supported(const distdl_plan* p, bool vec) {
  Wgrad16Shape s;
  return wgrad16_shape(p, vec, s);
}

int wgrad16_chunks(const distdl_plan* p, bool vec) {
  Wgrad16Shape s;
  return wgrad16_shape(p, vec, s) ? s.nchunks : 0;
}


// ---- entry points of the 16 x 16 correlation -------------------------------------------------------------------

static bool corr16_plan_ok(const distdl_plan* p) {
  if (p->dtype != DISTDL_F32 || p->explicit_halo) return false;
  if (p->n_ci > 16 || p->n_co > 16) return false;
  if ((double)p->n_b * p->max_buf_cells * std::max(p->n_ci, p->n_co) * 4.0 >= 2147480000.0) return false;
  for (int d = 0; d < 3; ++d)
    if (p->ksize[d] > 8) return false;
  return true;
}

bool corr16_fwd_supported(const distdl_plan* p, bool vec) {
  if (!corr16_plan_ok(p)) return false;
  Corr16Shape s;
  return corr16_shape(p, forward_args(p), vec && p->n_ci % 4 == 0, s);
}

bool corr16_bwd_supported(const distdl_plan* p, bool vec) {
  if (!corr16_plan_ok(p)) return false;
  for (int p0 = 0; p0 < p->stride[0]; ++p0)
    for (int p1 = 0; p1 < p->stride[1]; ++p1)
      for (int p2 = 0; p2 < p->stride[2]; ++p2) {
        const int par[3] = {p0, p1, p2};
        Corr16Shape s;
        const CorrArgs c = class_args(p, par);
        if (c.nt[0] * c.nt[1] * c.nt[2] == 0) continue;  // no tap reaches this class: the launch only writes zeros
        if (!corr16_shape(p, c, vec && p->n_co % 4 == 0, s)) return false;
      }
  return true;
}

static size_t corr16_scratch_total(const distdl_plan* p) {
  size_t total = corr16_weight_elems(forward_args(p));
  size_t bwd = 0;
  for (int p0 = 0; p0 < p->stride[0]; ++p0)
    for (int p1 = 0; p1 < p->stride[1]; ++p1)
      for (int p2 = 0; p2 < p->stride[2]; ++p2) {
        const int par[3] = {p0, p1, p2};
        bwd += corr16_weight_elems(class_args(p, par));
      }
  return std::max(total, bwd);
}

int conv_fwd16(distdl_plan* p, const float* w, const float* bias, bool vec, hipStream_t st) {
  int rc = ensure_wscratch(p, corr16_scratch_total(p));
  if (rc) return rc;
  return launch_corr16(p, forward_args(p), vec && p->n_ci % 4 == 0, w, p->d_wt, bias, p->tab_x.dev, p->tab_y.dev,
                       "conv_fwd_mfma16", st);
}

int conv_bwd_data16(distdl_plan* p, const float* w, bool vec, hipStream_t st) {
  int rc = ensure_wscratch(p, corr16_scratch_total(p));
  if (rc) return rc;
  size_t at = 0;
  for (int p0 = 0; p0 < p->stride[0]; ++p0)
    for (int p1 = 0; p1 < p->stride[1]; ++p1)
      for (int p2 = 0; p2 < p->stride[2]; ++p2) {
        const int par[3] = {p0, p1, p2};
        const CorrArgs c = class_args(p, par);
        if ((rc = launch_corr16(p, c, vec && p->n_co % 4 == 0, w, p->d_wt + at, nullptr, p->tab_dy.dev, p->tab_dx.dev,
                                "conv_bwd_data_mfma16", st)))
          return rc;
        at += corr16_weight_elems(c);
      }
  return DISTDL_OK;
}

// Partials of dw^ and db^ for every (worker, chunk) in `partial` (slots of taps * ci * co + co floats).
int conv_wgrad16(distdl_plan* p, float* partial, bool vec, hipStream_t st) {
  Wgrad16Shape s;
  if (!wgrad16_shape(p, vec, s)) return set_error(DISTDL_ERR_UNSUPPORTED, "conv: shape not covered by the small-channel kernel");
  Wgrad16Args a{};
  a.n_b = (int32_t)p->n_b;
  a.ci = (int32_t)p->n_ci;
  a.co = (int32_t)p->n_co;
  for (int d = 0; d < 3; ++d) {
    a.k[d] = p->ksize[d];
    a.dil[d] = p->dilation[d];
  }
  a.s0 = p->stride[0];
  const int nt = a.k[1] * a.k[2];
  for (int t = 0; t < nt; ++t) {
    a.t1d[t] = (t / a.k[2]) * a.dil[1];
    a.t2d[t] = (t % a.k[2]) * a.dil[2];
  }
  a.G = s.G;
  a.RB = s.RB;
  a.nchunks = s.nchunks;
  a.xcells = s.xcells;
  a.dcells = s.dcells;
  a.slot = (int64_t)a.k[0] * nt * a.ci * a.co + a.co;
  const dim3 grid((unsigned)a.k[0], (unsigned)a.nchunks, (unsigned)p->n_workers);
  ProfScope prof("conv_bwd_weight_mfma16", st);
#define DISTDL_LAUNCH_WG16(NT_)                                                                                     \
  do {                                                                                                               \
    if (vec)                                                                                                         \
      hipLaunchKernelGGL((wgrad16_kernel<NT_, 4>), grid, dim3(256), s.lds, st, p->d_workers, p->tab_x.dev,           \
                         p->tab_dy.dev, partial, a);                                                                 \
    else                                                                                                             \
      hipLaunchKernelGGL((wgrad16_kernel<NT_, 1>), grid, dim3(256), s.lds, st, p->d_workers, p->tab_x.dev,           \
                         p->tab_dy.dev, partial, a);                                                                 \
  } while (0)
  switch (nt) {
    case 1: DISTDL_LAUNCH_WG16(1); break;
    case 3: DISTDL_LAUNCH_WG16(3); break;
    case 5: DISTDL_LAUNCH_WG16(5); break;
    case 7: DISTDL_LAUNCH_WG16(7); break;
    case 9: DISTDL_LAUNCH_WG16(9); break;
    default: DISTDL_LAUNCH_WG16(25); break;
  }
#undef DISTDL_LAUNCH_WG16
  return DISTDL_OK;
}

}  // namespace distdl
