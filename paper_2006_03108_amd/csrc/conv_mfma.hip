// MFMA (matrix-core) kernels for the local convolution of the partitioned
// layer (Sec. 4, "Conv" and "[dConv]*" steps), fp32, channels-last.
//
// corr_mfma_kernel: a strided correlation written as an implicit GEMM
//     out[q][n] = sum_taps sum_k  W[tap][k][n] * in[base + q*step + tapoff][k]
//   used (a) for the forward pass (in = x^, out = y) and (b) once per stride
//   parity class for the data gradient (in = dy, out = the cells of dx^ whose
//   coordinate is congruent to that class; out-of-range dy reads as zero).
//   A workgroup owns a window of tr x tc output positions (128 or 256); per
//   (tap plane, 8-channel chunk) it stages the input patch and the weights in
//   LDS once and all taps of that plane read it from there.
// wgrad_mfma_kernel: dw^[tap][ci][co] = sum_pos x^[cell(pos,tap)][ci] dy[pos][co]
//   per worker; both MFMA operands are read straight from global memory in
//   their register layout (channels-last makes 32 channels one 128-byte row).
//   wgrad_lds_kernel stages the row segments in wave-private LDS; wgrad_taps_kernel
//   (the fast path) gives a workgroup all taps of one kernel plane and shares the
//   input rows between its waves through an LDS ring.
//
// v_mfma_f32_32x32x2_f32 operand layout: A lane l holds A[i = l%32][k = l/32],
// B lane l holds B[k = l/32][j = l%32], D register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "common.h"
#include "conv_mfma.h"
#include "lds_direct.h"
#include "profile.h"

namespace distdl {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__host__ __device__ inline int64_t tiles_of(const PerWorker& g, const CorrArgs& a) {
  // chunks of g0 consecutive (sample, dimension-0 position) planes x windows x channel tiles
  return (((int64_t)a.n_b * g.nq[0] + a.g0 - 1) / a.g0) * ((g.nq[1] + a.tr - 1) / a.tr) *
         ((g.nq[2] + a.tc - 1) / a.tc) * a.ntn;
}

constexpr int kMaxPieces = 14;
constexpr int kMaxBPieces = 8;  // weight pieces per thread held in registers (32 taps per plane)
constexpr uint32_t kOob = 0x7ffffff0u;  // buffer offset that always fails the range check (buffers are < 2 GiB)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Four consecutive channels as fp32 bit patterns: a 16-byte piece of an fp32 tensor, or an 8-byte piece of a
// bf16 tensor widened on the way (bf16 tensors are multiplied in fp32 on the matrix cores).
template <bool BF16>
__device__ inline u32x4 load4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  if constexpr (BF16) {
    const auto t = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
    return u32x4{t[0] << 16, t[0] & 0xffff0000u, t[1] << 16, t[1] & 0xffff0000u};
  } else {
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
  }
}

// fp32 -> bf16, round to nearest even, NaN kept quiet
__device__ inline uint16_t to_bf16(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// the same rounding by the hardware conversion (one instruction; the epilogues of the bf16 kernels are short of
// vector-ALU slots: those do not overlap with the matrix instructions of a SIMD)
__device__ inline uint16_t bf16_bits(float v) {
  const __bf16 b = (__bf16)v;
  uint16_t u;
  __builtin_memcpy(&u, &b, 2);
  return u;
}

template <bool BF16>
__device__ inline float load_scalar(const void* p, size_t i) {
  if constexpr (BF16) return __uint_as_float((uint32_t)((const uint16_t*)p)[i] << 16);
  else return ((const float*)p)[i];
}

// On this target VALU instructions do not overlap with MFMA execution on the same SIMD, so the loops
// below are written to issue as few of them as possible: every global access is a buffer instruction
// with a precomputed per-lane offset (out-of-range pieces carry an offset that fails the range check:
// loads return zero, stores are dropped), LDS addresses are precomputed, and the operands of tap i+1
// are read from LDS into a second register set while tap i multiplies.
//
// MT: 32-position M-tiles per wave; PA / PB: 16-byte patch / weight pieces per thread and stage.
// NT: taps per plane (nt[1] * nt[2]) known at compile time, or 0: with NT > 0 the tap loop is unrolled,
// the LDS address of every (M-tile, tap) operand is computed once per workgroup and the weight operand
// of tap t is an immediate offset, which removes the per-tap address arithmetic from the stage loop.
// MODE 0: fp32 tensors.  MODE 1: bf16 tensors (input, output, bias) widened to fp32 while they are staged; the
// weights were widened by the re-layout kernel.  MODE 2: bf16 tensors multiplied as bf16 on
// v_mfma_f32_32x32x16_bf16 (fp32 accumulation): a chunk is 16 channels, a 16-byte piece holds 8 of them and is one
// MFMA operand (A lane l holds A[i = l % 32][k = 8 * (l / 32) ... + 7]); needs channel counts that are multiples of 8.
// DMA (small patches with NT > 0, MODE 0 or 2): a stage goes from memory straight into LDS (global -> LDS loads, no
// staging registers, no ds_write) into one of two staging buffers, the next stage landing while this one is
// multiplied, one barrier per stage.  Thread (i, tid) fetches the piece whose slot is i * 256 + tid (a wave's load
// fills 64 consecutive slots); the patch is laid out in blocks of 32 cells so that such a load reads 32 contiguous
// bytes per cell.
// Registers: the fp32 variants with small patches and compile-time taps (the parity classes of the data gradient)
// are held to 128 (two M-tiles; they need 132 without the limit) or 168 (three) so that four or three workgroups
// share a compute unit (0.684 -> 0.666 ms per class on the 5^3 stride-2 layer with two M-tiles).
template <int MT, int PA, int PB, int NT, int MODE, bool DMA = false>
__global__ __launch_bounds__(256, (PA <= 4 && MT == 2 && MODE == 0 && NT > 0) ? 4 : (PA <= 4 && MT == 3 && (MODE == 0 || DMA) && NT > 0) ? 3 : 2) void corr_mfma_kernel(const WorkerDev* __restrict__ workers,
                                                           void* const* in_bufs, void* const* out_bufs, CorrArgs a) {
  extern __shared__ float4 lds[];
  constexpr bool BF16 = MODE != 0, BFM = MODE == 2;
  constexpr uint32_t ES = BF16 ? 2u : 4u;  // bytes per element in memory
  constexpr int CK = BFM ? 16 : 8;         // channels per chunk (two 16-byte pieces per cell in LDS)
  static_assert(!DMA || (NT > 0 && MODE != 1), "the direct-to-LDS variant needs compile-time taps and 16-byte pieces");
  // LDS: patch (a_vec4 16-byte units), weights (nb_vec4), one spare unit that absorbs the pieces nobody
  // needs, then the tap table.  DMA: two buffers of (a_pad + nb_vec4) units, the second one at the compile-time
  // offset kBufPitch (the most a buffer of this variant can hold), so that the operand reads of either buffer are
  // the same address registers with a different immediate offset; then the spare unit and the table.
  constexpr uint32_t kBufPitch = (uint32_t)(PA * 256 + (NT > 0 ? NT : PB * 4) * 64) * 16u;
  const int nb_vec4 = a.nt[1] * a.nt[2] * 64;
  const int a_units = DMA ? a.a_pad : a.a_vec4;  // where the weights of a buffer start
  const int dummy = DMA ? (int)(kBufPitch / 16) + a.a_pad + nb_vec4 : a.a_vec4 + nb_vec4;
  uint32_t* tap_tab = (uint32_t*)(lds + dummy + 1);  // byte offset into the patch per (t1, t2), read as a broadcast

  // XCD-aware order: consecutive tiles (which share input rows) stay on one XCD, i.e. behind one L2
  const uint32_t nblk = gridDim.x;
  const uint32_t r = (blockIdx.x & 7u) * (nblk >> 3) + (blockIdx.x >> 3);
  const uint32_t worker = r / a.tiles_max;
  uint32_t tile = r - worker * a.tiles_max;
  if (worker >= (uint32_t)a.n_workers) return;
  const WorkerDev wd = workers[worker];
  const PerWorker g = derive(wd, a);
  if ((int64_t)tile >= tiles_of(g, a)) return;

  const int nt2tiles = (g.nq[2] + a.tc - 1) / a.tc, nt1tiles = (g.nq[1] + a.tr - 1) / a.tr;
  const int q2_0 = (tile % nt2tiles) * a.tc; tile /= nt2tiles;
  const int q1_0 = (tile % nt1tiles) * a.tr; tile /= nt1tiles;
  const int ntile = tile % a.ntn; tile /= a.ntn;
  // output planes p = n * nq[0] + q0 of the worker; `tile` is now this workgroup's place among the plane groups
  const int nq0 = g.nq[0];
  const int ptotal = a.n_b * nq0, ngroups = (ptotal + a.g0 - 1) / a.g0;

  const int si2 = a.kc, si1 = g.in_ext[2] * si2, si0 = g.in_ext[1] * si1;
  const uint32_t sin = (uint32_t)g.in_ext[0] * si0;
  const uint32_t so2 = a.nc, so1 = g.out_ext[2] * so2, so0 = g.out_ext[1] * so1, son = g.out_ext[0] * so0;
  const __amdgpu_buffer_rsrc_t rin = make_rsrc(in_bufs[worker], (uint32_t)a.n_b * sin * ES);
  const __amdgpu_buffer_rsrc_t rout = make_rsrc(out_bufs[worker], (uint32_t)a.n_b * son * ES);
  const int ncc = (a.kc + CK - 1) / CK;
  const int nt0 = a.nt[0];
  const __amdgpu_buffer_rsrc_t rw =
      make_rsrc(a.wt + (size_t)ntile * nt0 * ncc * nb_vec4 * 4, (uint32_t)(nt0 * ncc * nb_vec4) * 16u);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, m = lane & 31;

  // per-thread patch pieces: byte offset inside an input plane and LDS slot, fixed for the whole tile.
  // When the channel count is not a multiple of 8, bit 0 marks the pieces of the upper half of a chunk:
  // in the last chunk they lie beyond the channels and must read as zero.
  uint32_t goff[PA], loff[DMA ? 1 : PA];
  const int npieces = a.R * a.Cw * 2;
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    goff[i] = kOob;
    int ph, rr, c;
    bool live;
    if constexpr (DMA) {
      // The piece that lives in slot tid + i * 256.  The patch's cells, row-major, are cut into blocks of 32; a block
      // is 64 slots, the first halves (ph = 0) of its cells, then the second halves: the 64 lanes of a load fetch 32
      // contiguous bytes from each of 32 neighbouring cells (with the halves in planes of their own a load touched
      // 64 cells, 16 bytes each, and issuing a stage's loads took half of a workgroup's life), and the 32 positions
      // of an operand read fall into consecutive 16-byte slots.
      const uint32_t slot = (uint32_t)(tid + i * 256);
      const uint32_t x = (slot >> 6) * 32u + (slot & 31u);  // cell
      ph = (int)((slot >> 5) & 1u);
      rr = (int)fd_div(x, a.div_cw), c = (int)x - rr * a.Cw;
      live = x < (uint32_t)(a.R * a.Cw);
    } else {
      const int piece = tid + i * 256;
      loff[i] = dummy * 16;
      ph = piece & 1;
      const int cell = piece >> 1;
      rr = (int)fd_div((uint32_t)cell, a.div_cw), c = cell - rr * a.Cw;
      live = piece < npieces;
      if (live) {
        const int cq = (int)fd_div((uint32_t)c, a.div_is2), cr = c - cq * a.is[2];
        loff[i] = (((rr * 2 + ph) * a.is[2] + cr) * a.CwQ + cq) * 16;
      }
    }
    if (live) {
      const int i1 = g.in_base[1] + q1_0 * a.is[1] + a.tapmin[1] + rr;
      const int i2 = g.in_base[2] + q2_0 * a.is[2] + a.tapmin[2] + c;
      if (i1 >= 0 && i1 < g.in_ext[1] && i2 >= 0 && i2 < g.in_ext[2])
        goff[i] = ((i1 * si1 + i2 * si2 + ph * (CK / 2)) * ES) | ((a.kc & (CK - 1)) ? ph : 0);
    }
  }
  uint32_t bl[DMA ? 1 : PB];
  if constexpr (!DMA) {
#pragma unroll
    for (int i = 0; i < PB; ++i) bl[i] = (tid + i * 256 < nb_vec4 ? a.a_vec4 + tid + i * 256 : dummy) * 16;
  }

  // The workgroup's 128*MT output positions form a tr x tc window, row-major; lane m of M-tile
  // (wave, mt) multiplies window position (wave*MT + mt)*32 + m.
  // The tile is accumulated transposed (the weights are the first MFMA operand), so accumulator register v of lane
  // (h, m) is channel ntile*32 + 8*(v/4) + 4*h + v%4 of that same position: a register quad is four consecutive
  // channels, and a lane needs one store offset per M-tile (sixteen with the tile the other way round: 36 - 45
  // registers and most of the set-up arithmetic).  fp32: a quad goes out as one 16-byte store.  bf16: a quad is 8
  // bytes; the lanes (0, m) and (1, m) exchange one quad of each pair (v_permlane32_swap), after which lane (h, m)
  // holds the eight channels 16*p + 8*h ... + 7 of pair p = 0, 1: two 16-byte stores per M-tile where 2-byte stores
  // took sixteen (a plane's epilogue then took as long as three of its six stages on the bf16 data-gradient classes
  // of the 5^3 stride-2 layer).  Channel counts that are not a multiple of 8 store the quads as they are, 8 bytes each.
  const bool pairs = BF16 && (a.nc & 7) == 0;
  uint32_t abase[MT];
  uint32_t soff[MT];  // of the first channel this lane stores at its position (kOob: nothing to store)
  const int ch0 = ntile * 32 + 4 * h, chs = pairs ? ntile * 32 + 8 * h : ch0;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int pidx = (wave * MT + mt) * 32 + m;
    int wr = (int)fd_div((uint32_t)pidx, a.div_tc), wc = pidx - wr * a.tc;
    const int q1 = q1_0 + wr, q2 = q2_0 + wc;
    soff[mt] = kOob;
    if (wr < a.tr && q1 < g.nq[1] && q2 < g.nq[2])
      soff[mt] = ((g.out_base[1] + g.os[1] * q1) * so1 + (g.out_base[2] + g.os[2] * q2) * so2 + chs) * ES;
    if (wr >= a.tr) wr = 0, wc = 0;  // idle position: multiplies something in range, never stored
    if constexpr (DMA) abase[mt] = wr * a.is[1] * a.Cw + wc * a.is[2];  // (the cell the position reads with a zero tap offset)
    else abase[mt] = (wr * a.is[1] * 2 * a.is[2] * a.CwQ + wc + h * a.is[2] * a.CwQ) * 16;
  }
  // the channel quads of this lane (channel counts are multiples of 4, so a quad is whole or absent)
  float bias[4][4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      bias[q][e] = (a.bias && ch0 + 8 * q + e < a.nc) ? load_scalar<BF16>(a.bias, ch0 + 8 * q + e) : 0.f;
  const uint32_t boff0 = tid * 16, bread = ((h * 32 + m) + a_units) * 16;  // weight piece / operand addresses

  const int* __restrict__ tapinfo = a.tapinfo;  // [0..7]: plane offsets, [8..]: patch offset per (t1, t2)
  const int ntaps = a.nt[1] * a.nt[2];
  if (tid < ntaps + 4) tap_tab[tid] = tid < ntaps ? (uint32_t)tapinfo[8 + tid] * 16u : 0u;  // visible after the first barrier below
  const bool ragged = (a.kc & (CK - 1)) != 0;
  char* const ldsb = (char*)lds;

  // A stage is one (output plane q0, tap plane t0, 8-channel chunk cc); stages whose input plane lies
  // outside the input contribute zero and are skipped.
  // (the table entry is the same for all lanes: saying so keeps the stage base offsets in scalar registers)
  // The plane offset of tap t0 is an arithmetic progression in t0 (forward: t0 * dilation; a parity class keeps every
  // (s / gcd(dilation, s))-th tap of the kernel, whose offsets fall by dilation / gcd(dilation, s) each), so it is
  // computed from the first two entries of the kernel arguments.  Read from the device table instead, each look-up
  // was a vector load and a full wait (s_waitcnt vmcnt(0)) on the path of every stage.
  const int toff0 = a.tapoff[0][0], tstep = a.nt[0] > 1 ? a.tapoff[0][1] - a.tapoff[0][0] : 0;
  auto plane_of = [&](int q0, int t0) { return g.in_base[0] + q0 * a.is[0] + toff0 + t0 * tstep; };
  // a stage position: plane p = (n, q0), tap plane t0, chunk cc
  // The workgroups of a worker's plane groups run side by side, and the input plane of (q0, t0) is that of
  // (q0 + 1, t0 - d), d = step / tap spacing.  So the planes are dealt to the groups in turn (group k takes planes k,
  // k + ngroups, ...: at any moment the groups work on neighbouring planes), and each plane's kernel planes are
  // walked in a rotated order, starting d * q0 behind: neighbours then stand on the same input plane at the same
  // moment and the first to touch a line fetches it for all behind that L2 (every input plane of the 5^3 stride-2
  // layer is then fetched for 2.5 output planes at once instead of 2.5 times: 7.8 GB instead of 23.1 GB per forward
  // launch).  j counts the kernel planes visited, t0 = (j + sk) mod nt0.
  const int rot_d = (nt0 > 1 && tstep != 0 && a.is[0] % tstep == 0) ? (a.is[0] / tstep) % nt0 : 0;
  const bool dealt = rot_d != 0 && ngroups > 1;
  const int pfirst = dealt ? (int)tile : (int)tile * a.g0, pstride = dealt ? ngroups : 1;
  // this workgroup's planes: pfirst + i * pstride, i in [0, pcnt)
  const int pcnt = dealt ? (ptotal - (int)tile + ngroups - 1) / ngroups : min(a.g0, ptotal - (int)tile * a.g0);
  auto skew_of = [&](int q0) {
    const int r = (int)(((int64_t)rot_d * q0) % nt0);  // (once per workgroup)
    return r == 0 ? 0 : (r > 0 ? nt0 - r : -r);          // (-d * q0) mod nt0
  };
  struct StagePos {
    int p, n, q0, t0, cc, j, sk;
  };
  auto advance = [&](StagePos& sp) {  // next valid stage after sp, or sp.p == pcnt (p counts this workgroup's planes)
    if (++sp.cc < ncc) return;  // same plane, next chunk
    sp.cc = 0;
    ++sp.j;
    while (sp.p < pcnt) {
      while (sp.j < nt0) {
        sp.t0 = sp.j + sp.sk < nt0 ? sp.j + sp.sk : sp.j + sp.sk - nt0;
        const int i0 = plane_of(sp.q0, sp.t0);
        if (i0 >= 0 && i0 < g.in_ext[0]) return;
        ++sp.j;
      }
      ++sp.p;
      sp.j = 0;
      sp.q0 += pstride;
      while (sp.q0 >= nq0) sp.q0 -= nq0, ++sp.n;
      sp.sk = rot_d ? skew_of(sp.q0) : 0;
    }
  };
  // DMA: the loads of stage sp, straight into the staging buffer at byte offset `bufoff`
  const uint32_t lds0 = lds_address(lds);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const lds_u32x4 din = lds_direct_rsrc(in_bufs[worker], (uint32_t)a.n_b * sin * ES);
  const lds_u32x4 dw = lds_direct_rsrc(a.wt + (size_t)ntile * nt0 * ncc * nb_vec4 * 4, (uint32_t)(nt0 * ncc * nb_vec4) * 16u);
  auto issue_stage = [&](const StagePos& sp, uint32_t bufoff) {
    const int t0 = sp.t0, cc = sp.cc;
    const uint32_t sbase = ((uint32_t)sp.n * sin + (uint32_t)plane_of(sp.q0, t0) * si0 + cc * CK) * ES;
    const bool last_ragged = ragged && cc == ncc - 1;
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      const int first = i * 256 + wave_u * 64;  // this wave's 64 slots of load i
      if (first < a.a_pad) {
        const uint32_t off = last_ragged ? ((goff[i] & 1u) ? kOob : goff[i]) : (ragged ? goff[i] & ~1u : goff[i]);
        load_to_lds(din, lds0 + bufoff + first * 16, off, sbase);
      }
    }
    const uint32_t wbase = (uint32_t)(t0 * ncc + cc) * nb_vec4 * 16u;
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int first = i * 256 + wave_u * 64;
      if (first < nb_vec4) load_to_lds(dw, lds0 + bufoff + (a.a_pad + first) * 16, boff0, wbase + i * 4096u);
    }
  };
  u32x4 ra[DMA ? 1 : PA], rb[DMA ? 1 : PB];
  auto load_stage = [&](const StagePos& sp) {
    if constexpr (DMA) return;  // (register staging: not this variant's path)
    const int t0 = sp.t0, cc = sp.cc;
    const uint32_t sbase = ((uint32_t)sp.n * sin + (uint32_t)plane_of(sp.q0, t0) * si0 + cc * CK) * ES;
    if (ragged && cc == ncc - 1) {
#pragma unroll
      for (int i = 0; i < PA; ++i)
        ra[i] = load4<MODE == 1>(rin, (goff[i] & 1u) ? kOob : goff[i], sbase);
    } else if (ragged) {
#pragma unroll
      for (int i = 0; i < PA; ++i) ra[i] = load4<MODE == 1>(rin, goff[i] & ~1u, sbase);
    } else {
#pragma unroll
      for (int i = 0; i < PA; ++i) ra[i] = load4<MODE == 1>(rin, goff[i], sbase);
    }
    const uint32_t wbase = (uint32_t)(t0 * ncc + cc) * nb_vec4 * 16u;
#pragma unroll
    for (int i = 0; i < PB; ++i) rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rw, boff0, wbase + i * 4096u, 0);
  };
  auto write_stage = [&]() {
    if constexpr (DMA) return;
#pragma unroll
    for (int i = 0; i < PA; ++i) *(u32x4*)(ldsb + loff[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < PB; ++i) *(u32x4*)(ldsb + bl[i]) = rb[i];
  };
  // operand addresses per (M-tile, tap), fixed for the whole workgroup (NT > 0 only)
  uint32_t aaddr[MT][NT > 0 ? NT : 1];
  if constexpr (NT > 0) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if constexpr (DMA) {  // block layout: cell x sits in block x / 32, half h of it at slot 32 * h + x % 32
        const int t1 = t / a.nt[2], t2 = t - t1 * a.nt[2];
        const uint32_t tapx = (uint32_t)((a.tapoff[1][t1] - a.tapmin[1]) * a.Cw + a.tapoff[2][t2] - a.tapmin[2]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const uint32_t x = abase[mt] + tapx;
          aaddr[mt][t] = ((x >> 5) * 64u + (uint32_t)h * 32u + (x & 31u)) * 16u;
        }
      } else {
        const uint32_t tapo = (uint32_t)tapinfo[8 + t] * 16u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) aaddr[mt][t] = abase[mt] + tapo;
      }
    }
  }

  // tapo: byte offset of the tap inside the patch (NT == 0: read from the LDS table two taps ahead of
  // its use, so that the table read is never waited for)
  // bo: byte offset of the staging buffer (DMA: 0 or kBufPitch, a compile-time constant at every call)
  auto read_ops = [&](int tap, uint32_t tapo, float4& b, float4 (&av)[MT], uint32_t bo) {
    if constexpr (NT > 0) {
      b = *(const float4*)(ldsb + bread + tap * 1024 + bo);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) av[mt] = *(const float4*)(ldsb + aaddr[mt][tap] + bo);
    } else {
      b = *(const float4*)(ldsb + bread + tap * 1024);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) av[mt] = *(const float4*)(ldsb + abase[mt] + tapo);
    }
  };
  auto multiply = [&](floatx16 (&acc)[MT], const float4& b, const float4 (&av)[MT]) {
    if constexpr (BFM) {  // one MFMA per 16-byte operand: 16 channels of the chunk at once
      union Frag {
        float4 f;
        bf16x8 v;
      };
      Frag fb;
      fb.f = b;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        Frag fa;
        fa.f = av[mt];
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb.v, fa.v, acc[mt], 0, 0, 0);
      }
      return;
    }
    // M-tiles interleaved, so that consecutive MFMAs do not depend on each other
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b.x, av[mt].x, acc[mt], 0, 0, 0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b.y, av[mt].y, acc[mt], 0, 0, 0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b.z, av[mt].z, acc[mt], 0, 0, 0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(b.w, av[mt].w, acc[mt], 0, 0, 0);
  };

  // The operands of tap t + 1 are read while tap t multiplies; the scheduling barriers keep the
  // compiler from sinking the LDS reads down to their first use, which would expose their latency.
  auto compute = [&](floatx16 (&acc)[MT], auto buf_c) {
    constexpr uint32_t bo = decltype(buf_c)::value ? kBufPitch : 0u;
    float4 b0, b1, a0[MT], a1[MT];
    if constexpr (NT > 0) {
      read_ops(0, 0, b0, a0, bo);
#pragma unroll
      for (int tap = 0; tap + 1 < NT; tap += 2) {
        read_ops(tap + 1, 0, b1, a1, bo);
        __builtin_amdgcn_sched_barrier(0);
        multiply(acc, b0, a0);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 2 < NT) read_ops(tap + 2, 0, b0, a0, bo);
        __builtin_amdgcn_sched_barrier(0);
        multiply(acc, b1, a1);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (NT & 1) multiply(acc, b0, a0);
    } else {
      // tap_tab has two spare entries behind the last tap, so the look-ahead reads stay in the table
      uint32_t o1 = tap_tab[1], o2 = tap_tab[2];
      read_ops(0, tap_tab[0], b0, a0, 0u);
      int tap = 0;
      for (; tap + 1 < ntaps; tap += 2) {
        read_ops(tap + 1, o1, b1, a1, 0u);
        o1 = tap_tab[tap + 3];
        __builtin_amdgcn_sched_barrier(0);
        multiply(acc, b0, a0);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 2 < ntaps) read_ops(tap + 2, o2, b0, a0, 0u);
        o2 = tap_tab[tap + 4];
        __builtin_amdgcn_sched_barrier(0);
        multiply(acc, b1, a1);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (tap < ntaps) multiply(acc, b0, a0);
    }
  };

  floatx16 acc[MT];
  StagePos sp{0, pfirst / nq0, pfirst % nq0, 0, ncc - 1, -1, 0};  // the stage whose loads are in flight
  sp.sk = rot_d ? skew_of(sp.q0) : 0;
  advance(sp);
  int on = pfirst / nq0, oq0 = pfirst % nq0;  // the output plane that is stored next
  auto zero_acc = [&]() {
#pragma unroll
    for (int t = 0; t < MT; ++t)
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  };
  auto store_plane = [&]() {
    const uint32_t obase = ((uint32_t)on * son + (uint32_t)(g.out_base[0] + g.os[0] * oq0) * so0) * ES;
    oq0 += pstride;
    while (oq0 >= nq0) oq0 -= nq0, ++on;
    // (the plane's offset is added into the per-lane offset: with a scalar offset the compiler leaves out the wait
    // states a 16-byte store needs before its data registers are written again)
    if constexpr (!BF16) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint32_t off = (ch0 + 8 * q < a.nc ? soff[mt] + (uint32_t)(8 * q) * ES : kOob) + obase;
          u32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = __float_as_uint(acc[mt][4 * q + e] + bias[q][e]);
          __builtin_amdgcn_raw_buffer_store_b128(o, rout, off, 0, 0);
        }
    } else {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        uint32_t pk[4][2];  // quad q as four bf16
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int d = 0; d < 2; ++d)
            pk[q][d] = (uint32_t)bf16_bits(acc[mt][4 * q + 2 * d] + bias[q][2 * d]) |
                       ((uint32_t)bf16_bits(acc[mt][4 * q + 2 * d + 1] + bias[q][2 * d + 1]) << 16);
        if (pairs) {
#pragma unroll
          for (int pr = 0; pr < 2; ++pr) {
            // the even quad's upper lanes (h = 1) change places with the odd quad's lower lanes (h = 0)
            u32x4 o;
#pragma unroll
            for (int d = 0; d < 2; ++d) {
              const auto sw = __builtin_amdgcn_permlane32_swap(pk[2 * pr][d], pk[2 * pr + 1][d], false, false);
              o[d] = sw[0];
              o[2 + d] = sw[1];
            }
            const uint32_t off = (chs + 16 * pr < a.nc ? soff[mt] + (uint32_t)(16 * pr) * ES : kOob) + obase;
            __builtin_amdgcn_raw_buffer_store_b128(o, rout, off, 0, 0);
          }
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            const uint32_t off = (ch0 + 8 * q < a.nc ? soff[mt] + (uint32_t)(8 * q) * ES : kOob) + obase;
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{pk[q][0], pk[q][1]}, rout, off, 0, 0);
          }
        }
      }
    }
  };
  if constexpr (DMA) {
    // Two stages per trip of the loop, one from each buffer, written out one behind the other: with a branch to one
    // of two copies of the tap loop the compiler kept the accumulators of the copies in different registers and
    // moved all of them across at every stage (48 - 96 moves for 18 - 27 MFMAs).
    int po = 0;
    zero_acc();
    if (sp.p < pcnt) issue_stage(sp, 0u);
    for (; po < sp.p; ++po) store_plane();  // leading planes that no stage feeds (sp.p <= pcnt)
    // At the top of a half, `sp` is the stage in flight into the half's buffer and belongs to output plane po.
    auto half = [&](auto buf_c) {
      // The only loads in flight are this stage's: wait for mine, then for everyone's.  Past the barrier every
      // wave has also finished multiplying the stage before, so the other buffer may be refilled.
      __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
      lds_barrier();
      advance(sp);
      if (sp.p < pcnt) issue_stage(sp, decltype(buf_c)::value ? 0u : kBufPitch);  // lands while this stage multiplies
      compute(acc, buf_c);
      if (sp.p != po) {  // that was the last stage of plane po
        store_plane();
        zero_acc();
        for (++po; po < sp.p; ++po) store_plane();  // planes without a stage: the bias alone
      }
    };
    while (po < pcnt) {
      half(std::false_type{});
      if (po >= pcnt) break;
      half(std::true_type{});
    }
  } else {
    if (sp.p < pcnt) load_stage(sp);
    for (int po = 0; po < pcnt; ++po) {  // output planes of this workgroup
      zero_acc();
      while (sp.p == po) {  // the stages that feed output plane po
        write_stage();
        __syncthreads();
        advance(sp);
        if (sp.p < pcnt) load_stage(sp);  // in flight while this stage multiplies
        compute(acc, std::false_type{});
        __syncthreads();  // everyone is done reading this stage
      }
      store_plane();
    }
  }
}

// Weights in the order the correlation kernel stages them:
//   dst[ntile][t0][cc][t1][t2][h][nn][j] = W[tap(t0,t1,t2)][k = cc*8 + 4h + j][n = ntile*32 + nn]
// with W[tap][k][n] = w[n][k][tap] (forward: n = co, k = ci) or w[k][n][tap]
// (data gradient: k = co, n = ci), zero beyond the channel counts.
template <int MODE>
__global__ __launch_bounds__(256) void corr_weights_kernel(const void* __restrict__ w, float* __restrict__ dst,
                                                           CorrArgs a, int ci_n, int co_n, int taps, int k1, int k2) {
  // elements per 16-byte piece: 4 floats, or 8 bf16 when the kernel multiplies in bf16
  constexpr int PE = MODE == 2 ? 8 : 4, CK = 2 * PE;
  const int ncc = (a.kc + CK - 1) / CK;
  const int64_t units = (int64_t)a.ntn * a.nt[0] * ncc * a.nt[1] * a.nt[2] * 64;  // 16-byte pieces
  const int64_t total = units * PE;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (blockIdx.x == 0) {  // the tap tables the correlation kernel reads, stored behind the weights
    int* tapinfo = (int*)(dst + units * 4);
    if (threadIdx.x < 8) tapinfo[threadIdx.x] = threadIdx.x < a.nt[0] ? a.tapoff[0][threadIdx.x] : 0;
    if ((int)threadIdx.x < a.nt[1] * a.nt[2]) {
      const int t1 = threadIdx.x / a.nt[2], t2 = threadIdx.x - t1 * a.nt[2];
      const int rel1 = a.tapoff[1][t1] - a.tapmin[1], rel2 = a.tapoff[2][t2] - a.tapmin[2];
      tapinfo[8 + threadIdx.x] = ((rel1 * 2) * a.is[2] + rel2 % a.is[2]) * a.CwQ + rel2 / a.is[2];
    }
  }
  if (idx >= total) return;
  const int j = idx % PE;
  int64_t r = idx / PE;
  const int nn = r & 31, hh = (r >> 5) & 1;
  r >>= 6;
  const int t2 = r % a.nt[2]; r /= a.nt[2];
  const int t1 = r % a.nt[1]; r /= a.nt[1];
  const int cc = r % ncc; r /= ncc;
  const int t0 = r % a.nt[0];
  const int ntile = (int)(r / a.nt[0]);
  const int k = cc * CK + PE * hh + j, nch = ntile * 32 + nn;
  float v = 0.f;
  if (k < a.kc && nch < a.nc) {
    const int tap = (a.tapid[0][t0] * k1 + a.tapid[1][t1]) * k2 + a.tapid[2][t2];
    const int co = a.mode == 0 ? nch : k, ci = a.mode == 0 ? k : nch;
    v = load_scalar<MODE != 0>(w, ((size_t)co * ci_n + ci) * taps + tap);
  }
  if constexpr (MODE == 2) ((uint16_t*)dst)[idx] = to_bf16(v);  // exact: v is a bf16 value
  else dst[idx] = v;
}

// ---- weight gradient ----------------------------------------------------------

constexpr int kMaxK2 = 8;

// grid: (tap-row groups of 4, ci tiles * co tiles, workers * nchunks); wave w of a block owns tap row
// (t0, t1) = group*4 + w and all k2 taps of that row.
template <int K2>
__global__ __launch_bounds__(256, 2) void wgrad_mfma_kernel(const WorkerDev* __restrict__ workers, void* const* x_bufs,
                                                         void* const* dy_bufs, float* __restrict__ partial,
                                                         WgradArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = lane >> 5, m = lane & 31;
  const int trow = blockIdx.x * 4 + wave;
  if (trow >= a.k[0] * a.k[1]) return;
  const int t0 = trow / a.k[1], t1 = trow - t0 * a.k[1];
  const int nco_t = (a.co + 31) / 32;
  const int ci_t = blockIdx.y / nco_t, co_t = blockIdx.y - ci_t * nco_t;
  const int worker = blockIdx.z / a.nchunks, chunk = blockIdx.z - worker * a.nchunks;
  const WorkerDev wd = workers[worker];
  const float* __restrict__ x = (const float*)x_bufs[worker];
  const float* __restrict__ dy = (const float*)dy_bufs[worker];
  const int ci = ci_t * 32 + m, co = co_t * 32 + m;
  const bool ci_ok = ci < a.ci, co_ok = co < a.co;

  floatx16 acc[K2];
#pragma unroll
  for (int t = 0; t < K2; ++t)
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  const int64_t sx2 = a.ci, sx1 = (int64_t)wd.buf[2] * sx2, sx0 = (int64_t)wd.buf[1] * sx1,
                sxn = (int64_t)wd.buf[0] * sx0;
  const int64_t sy2 = a.co, sy1 = (int64_t)wd.out[2] * sy2;
  const int nrows = a.n_b * wd.out[0] * wd.out[1];
  const int per = (nrows + a.nchunks - 1) / a.nchunks;
  const int row_begin = chunk * per, row_end = min(nrows, (chunk + 1) * per);
  const int O2 = wd.out[2], pairs = (O2 + 1) / 2;
  // two output positions per MFMA: lanes 0-31 take column 2*pr, lanes 32-63 column 2*pr + 1.
  // The loads of step i+1 are issued before the MFMAs of step i.
  int row = row_begin, pr = 0;
  const float* xrow = nullptr;
  const float* dyrow = nullptr;
  auto fetch = [&](float& b, float (&av)[K2]) {
    if (pr == 0) {
      const int o1 = row % wd.out[1];
      const int r2 = row / wd.out[1];
      const int o0 = r2 % wd.out[0], n = r2 / wd.out[0];
      xrow = x + n * sxn + (int64_t)(wd.origin[0] + o0 * a.s[0] + t0 * a.dil[0]) * sx0 +
             (int64_t)(wd.origin[1] + o1 * a.s[1] + t1 * a.dil[1]) * sx1 + (int64_t)wd.origin[2] * sx2 + ci;
      dyrow = dy + (int64_t)row * sy1 + co;
    }
    const int p = 2 * pr + h;
    const bool pos_ok = p < O2;
    b = (pos_ok && co_ok) ? dyrow[(int64_t)p * sy2] : 0.f;
#pragma unroll
    for (int t2 = 0; t2 < K2; ++t2)
      av[t2] = (pos_ok && ci_ok && t2 < a.k[2]) ? xrow[(int64_t)(p * a.s[2] + t2 * a.dil[2]) * sx2] : 0.f;
    if (++pr == pairs) pr = 0, ++row;
  };
  const int64_t steps = (int64_t)max(row_end - row_begin, 0) * pairs;
  float b0 = 0.f, b1 = 0.f, a0[K2], a1[K2];
#pragma unroll
  for (int t2 = 0; t2 < K2; ++t2) a0[t2] = a1[t2] = 0.f;
  if (steps > 0) fetch(b0, a0);
  for (int64_t it = 0; it < steps; ++it) {
    if (it + 1 < steps) fetch(b1, a1);
#pragma unroll
    for (int t2 = 0; t2 < K2; ++t2) acc[t2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[t2], b0, acc[t2], 0, 0, 0);
    b0 = b1;
#pragma unroll
    for (int t2 = 0; t2 < K2; ++t2) a0[t2] = a1[t2];
  }
  // acc[t2] register v of lane (h, m): dw^[tap][ci = ci_t*32 + 8*(v/4) + 4h + v%4][co = co_t*32 + m]
  float* pbase = partial + (size_t)blockIdx.z * a.slot;
#pragma unroll
  for (int t2 = 0; t2 < K2; ++t2) {
    if (t2 >= a.k[2]) break;
    const int tap = (t0 * a.k[1] + t1) * a.k[2] + t2;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int cir = ci_t * 32 + 8 * (v / 4) + 4 * h + (v % 4);
      if (cir < a.ci && co_ok) pbase[((size_t)tap * a.ci + cir) * a.co + co] = acc[t2][v];
    }
  }
}

// Same contraction with LDS staging: each wave copies, per 32 output columns, the input-row segment
// its taps read (ncell cells x 32 channels) and the dy segment (32 x 32) into a private LDS area with
// 16-byte loads, then feeds all K2 taps from there.  Every cell is fetched once per tap row instead of
// once per tap; no workgroup barrier is needed because a wave only reads what it wrote itself.
// Requires channel counts that are multiples of 4, 16-byte aligned buffers and ncell <= 64*XP/8.
template <int K2, int XP>
__global__ __launch_bounds__(256, 2) void wgrad_lds_kernel(const WorkerDev* __restrict__ workers, void* const* x_bufs,
                                                           void* const* dy_bufs, float* __restrict__ partial,
                                                           WgradArgs a) {
  extern __shared__ float4 wg_lds[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = lane >> 5, m = lane & 31;
  // kernel rows (t0, t1), four per workgroup
  const int trow = blockIdx.x * 4 + wave;
  if (trow >= a.k[0] * a.k[1]) return;  // no workgroup barrier below
  const int t0 = trow / a.k[1], t1 = trow - t0 * a.k[1];
  const int nco_t = (a.co + 31) / 32;
  const int ci_t = blockIdx.y / nco_t, co_t = blockIdx.y - ci_t * nco_t;
  const int worker = blockIdx.z / a.nchunks, chunk = blockIdx.z - worker * a.nchunks;
  const WorkerDev wd = workers[worker];
  const float* __restrict__ x = (const float*)x_bufs[worker];
  const float* __restrict__ dy = (const float*)dy_bufs[worker];
  const int ncell = a.ncell;
  float4* xs4 = wg_lds + (size_t)wave * (ncell + 32) * 8;  // [ncell][32 ch]
  float4* ys4 = xs4 + ncell * 8;                           // [32 pos][32 ch]
  const float* xs = (const float*)xs4;
  const float* ys = (const float*)ys4;

  floatx16 acc[K2];
#pragma unroll
  for (int t = 0; t < K2; ++t)
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  const int64_t sx2 = a.ci, sx1 = (int64_t)wd.buf[2] * sx2, sx0 = (int64_t)wd.buf[1] * sx1,
                sxn = (int64_t)wd.buf[0] * sx0;
  const int64_t sy2 = a.co, sy1 = (int64_t)wd.out[2] * sy2;
  const int nrows = a.n_b * wd.out[0] * wd.out[1];
  const int per = (nrows + a.nchunks - 1) / a.nchunks;
  const int row_begin = chunk * per, row_end = min(nrows, (chunk + 1) * per);
  const int O2 = wd.out[2], nseg = (O2 + 31) / 32;
  const int row_cells = wd.buf[2] - wd.origin[2];  // cells from the first tap of column 0 to the row end
  // this lane's 16-byte pieces: piece j = lane + 64*i covers cell (or position) j / 8, channels 4*(j % 8)..
  const int q4 = (lane & 7) * 4;
  const bool xch_ok = ci_t * 32 + q4 < a.ci, ych_ok = co_t * 32 + q4 < a.co;

  float4 rx[XP], ry[4];
  auto fetch = [&](int row, int seg) {
    const int o1 = row % wd.out[1];
    const int r2 = row / wd.out[1];
    const int o0 = r2 % wd.out[0], n = r2 / wd.out[0];
    const int c0 = seg * 32 * a.s[2];  // first cell of the segment, relative to the row's first tap
    const float* xrow = x + n * sxn + (int64_t)(wd.origin[0] + o0 * a.s[0] + t0 * a.dil[0]) * sx0 +
                        (int64_t)(wd.origin[1] + o1 * a.s[1] + t1 * a.dil[1]) * sx1 +
                        (int64_t)(wd.origin[2] + c0) * sx2 + ci_t * 32 + q4;
    const float* dyrow = dy + (int64_t)row * sy1 + (int64_t)seg * 32 * sy2 + co_t * 32 + q4;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int cell = (lane >> 3) + 8 * i;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (cell < ncell && c0 + cell < row_cells && xch_ok) v = *(const float4*)(xrow + (int64_t)cell * sx2);
      rx[i] = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int pos = (lane >> 3) + 8 * i;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (seg * 32 + pos < O2 && ych_ok) v = *(const float4*)(dyrow + (int64_t)pos * sy2);
      ry[i] = v;
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < XP; ++i)
      if ((lane >> 3) + 8 * i < ncell) xs4[lane + 64 * i] = rx[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) ys4[lane + 64 * i] = ry[i];
  };

  const int s2 = a.s[2];
  int toff[K2];  // cell offset of tap t2 (taps beyond the kernel re-read tap 0; their sums are never stored)
#pragma unroll
  for (int t2 = 0; t2 < K2; ++t2) toff[t2] = (t2 < a.k[2] ? t2 : 0) * a.dil[2];
  const int total = max(row_end - row_begin, 0) * nseg;
  if (total > 0) fetch(row_begin, 0);
  for (int it = 0; it < total; ++it) {
    __builtin_amdgcn_wave_barrier();
    stash();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (it + 1 < total) fetch(row_begin + (it + 1) / nseg, (it + 1) % nseg);
    // 16 steps of two positions: lanes 0-31 take position 2*pr, lanes 32-63 position 2*pr + 1
#pragma unroll 4
    for (int pr = 0; pr < 16; ++pr) {
      const int pl = 2 * pr + h;
      const float b = ys[pl * 32 + m];
      float av[K2];
#pragma unroll
      for (int t2 = 0; t2 < K2; ++t2) av[t2] = xs[(pl * s2 + toff[t2]) * 32 + m];
#pragma unroll
      for (int t2 = 0; t2 < K2; ++t2) acc[t2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t2], b, acc[t2], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  const int co = co_t * 32 + m;
  const bool co_ok = co < a.co;
  float* pbase = partial + (size_t)blockIdx.z * a.slot;
#pragma unroll
  for (int t2 = 0; t2 < K2; ++t2) {
    if (t2 >= a.k[2]) break;
    const int tap = (t0 * a.k[1] + t1) * a.k[2] + t2;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int cir = ci_t * 32 + 8 * (v / 4) + 4 * h + (v % 4);
      if (cir < a.ci && co_ok) pbase[((size_t)tap * a.ci + cir) * a.co + co] = acc[t2][v];
    }
  }
}

// Weight gradient with all taps of one kernel plane t0 in a workgroup of four waves (one per SIMD).
// The k1 * k2 taps of the plane, in row-major order, are split into four contiguous ranges of at most
// TW taps; a wave accumulates its taps in TW accumulator tiles.  The waves walk the output rows o1
// together: the input rows a step reads, origin + o1*s1 + [0, span), are kept in LDS as a ring of
// span + s1 rows, every step fetches only its s1 new rows plus the dy row segment (both one step ahead,
// through registers), and because the ring has s1 spare rows and the dy segment two buffers, the rows of
// step o1 + 1 can be written while slower waves still multiply step o1: one barrier per step.  Each
// input cell is read from memory once per t0.  Per step a wave issues 16 * TW MFMAs and a handful of
// vector instructions: ring slots advance in scalar registers, out-of-range rows are switched off through
// the scalar offset of the buffer load, and every LDS read of the inner loop is an immediate offset.
// A wave with TW - 1 taps repeats its last tap (never stored), so all waves stay in step.
// SH = 1 (fp32 MFMAs, T = 4 * (TW - 1) + 1 taps, e.g. 3 x 3 and 5 x 5 kernels): every wave owns TW - 1 taps and the
// last tap is shared, each wave multiplying a quarter of a step's 32 positions for it; the four partial tiles are
// summed through LDS, in wave order, when the workgroup is done.  That is 16 * (TW - 1) + 4 MFMAs per wave and
// step instead of 16 * TW.
// MODE 0: fp32 tensors.  MODE 1: bf16 tensors widened to fp32 while they are staged.  MODE 2: bf16 tensors staged as
// they are (a 16-byte piece holds 8 channels) and multiplied on v_mfma_f32_32x32x16_bf16, whose operands need 8
// consecutive *positions* per lane: ds_read_b64_tr_b16 gathers them from the channels-last rows.  Measured lane
// layout of that load: in every group of 16 lanes, lane 4 * b + a receives, as element v, the a-th 16-bit element
// of the 8 bytes addressed by lane b + 4 * v of the group.  With lane s of a group addressing channels
// 4 * (s % 4) ... + 3 of position s / 4, lane t of the group thus receives channel t of four consecutive positions.
template <int TW, int S2, int MODE, int SH>
__global__ __launch_bounds__(256, 2) void wgrad_taps_kernel(const WorkerDev* __restrict__ workers, void* const* x_bufs,
                                                            void* const* dy_bufs, float* __restrict__ partial,
                                                            WgradArgs a) {
  extern __shared__ float4 wt_lds[];
  constexpr int NX = 5;  // input-row pieces per thread and step
  constexpr bool BFM = MODE == 2;
  constexpr uint32_t ES = MODE ? 2u : 4u;   // bytes per element in memory
  constexpr int PCH = BFM ? 8 : 4;          // channels per 16-byte piece in LDS
  constexpr int PPC = 32 / PCH;             // pieces per cell of a 32-channel tile
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, m = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // The workgroups of the k0 kernel planes that share a (worker, chunk, channel tile) read the same input planes:
  // (o0, t0) and (o0 + 1, t0 - s0 / dil0) are the same plane.  They are given consecutive places in an XCD-aware
  // order (consecutive places stay on one XCD, i.e. behind one L2), and each walks its chunk's units in a rotated
  // order (below) so that at the same moment they are on the same input plane: the first to touch a line fetches it
  // for all of them.
  uint32_t bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  {
    const uint32_t nblk = gridDim.x * gridDim.y * gridDim.z;
    if ((nblk & 7u) == 0) {
      const uint32_t lin = bx + gridDim.x * (by + gridDim.y * bz);
      const uint32_t r = (lin & 7u) * (nblk >> 3) + (lin >> 3);
      bx = r % gridDim.x;
      const uint32_t rest = r / gridDim.x;
      by = rest % gridDim.y;
      bz = rest / gridDim.y;
    }
  }
  const int t0 = (int)bx;
  const int nco_t = (a.co + 31) / 32;
  const int ci_t = (int)by / nco_t, co_t = (int)by - ci_t * nco_t;
  const int worker = (int)bz / a.nchunks, chunk = (int)bz - worker * a.nchunks;
  const WorkerDev wd = workers[worker];
  const int s1 = a.s[1], span = a.span, ring = span + s1;
  const int rowp = (a.ncell * PPC + 63) & ~63;  // 16-byte pieces per staged row, rounded up to whole waves
  const uint32_t pitch = (uint32_t)rowp * 16u;
  char* const ldsb = (char*)wt_lds;
  const uint32_t ys_base = (uint32_t)ring * pitch;  // two dy segments of 4 KiB behind the ring

  static_assert(SH == 0 || (SH == 1 && MODE != 2), "the shared tap is split by position pairs of fp32 MFMAs");
  constexpr int NOWN = TW - SH;  // accumulators of taps this wave owns; the rest hold its part of the shared tap
  const int T = a.k[1] * a.k[2];
  const int tbase = T >> 2, trem = T & 3;
  const int tap_first = SH ? wave * NOWN : wave * tbase + min(wave, trem);
  const int ntw = SH ? NOWN : tbase + (wave < trem ? 1 : 0);
  int tap_t1[TW], tap_t2[TW];
#pragma unroll
  for (int i = 0; i < TW; ++i) {
    const int j = i < NOWN ? tap_first + min(i, ntw - 1) : T - 1;
    tap_t1[i] = j / a.k[2];
    tap_t2[i] = j - tap_t1[i] * a.k[2];
  }

  const uint32_t sx2 = a.ci, sx1 = wd.buf[2] * sx2, sx0 = wd.buf[1] * sx1, sxn = wd.buf[0] * sx0;
  const uint32_t sy2 = a.co, sy1 = wd.out[2] * sy2, sy0 = wd.out[1] * sy1, syn = wd.out[0] * sy0;
  const __amdgpu_buffer_rsrc_t rx = make_rsrc(x_bufs[worker], (uint32_t)a.n_b * sxn * ES);
  const __amdgpu_buffer_rsrc_t ry = make_rsrc(dy_bufs[worker], (uint32_t)a.n_b * syn * ES);

  floatx16 acc[TW];
#pragma unroll
  for (int t = 0; t < TW; ++t)
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  const int row_cells = wd.buf[2] - wd.origin[2];
  const int O1 = wd.out[1], O2 = wd.out[2], nseg = (O2 + 31) / 32;
  const int nblk1 = (O1 + a.ob - 1) / a.ob;
  const int nunits = a.n_b * wd.out[0] * nblk1;
  const int per = (nunits + a.nchunks - 1) / a.nchunks;
  const int unit_end = min(nunits, (chunk + 1) * per);

  // Slot i of a thread is piece i*256 + tid of a step's s1 * rowp input pieces; rowp is a multiple of 64,
  // so the new-row index prr[i] of a slot is the same for a whole wave.
  int prr[NX];
  uint32_t prest[NX], pg[NX], pgy;
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const int piece0 = i * 256 + wave * 64;
    prr[i] = piece0 / rowp;
    prest[i] = (uint32_t)(piece0 - prr[i] * rowp + lane);
  }
  auto setup_pieces = [&](int seg) {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int cell = prest[i] / PPC, q4 = (prest[i] % PPC) * PCH;
      pg[i] = kOob;  // pieces beyond the row's cells or channels stage zeros
      if (cell < a.ncell && seg * 32 * S2 + cell < row_cells && ci_t * 32 + q4 < a.ci)
        pg[i] = ((seg * 32 * S2 + cell) * sx2 + ci_t * 32 + q4) * ES;
    }
    const int pos = tid / PPC, q4 = (tid % PPC) * PCH;  // 32 positions; with 8-channel pieces only half the threads
    pgy = kOob;
    if (pos < 32 && seg * 32 + pos < O2 && co_t * 32 + q4 < a.co) pgy = ((seg * 32 + pos) * sy2 + co_t * 32 + q4) * ES;
  };
  u32x4 rp[NX], rpy;
  auto fetch = [&](int n, int o0, int o1) {
    const int c0 = wd.origin[0] + o0 * a.s[0] + t0 * a.dil[0];
    const int r_first = wd.origin[1] + o1 * s1 + span - s1;  // buffer row of new row 0
    const uint32_t xb = ((uint32_t)n * sxn + (uint32_t)c0 * sx0 + (uint32_t)r_first * sx1 + wd.origin[2] * sx2) * ES;
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      // rows beyond the buffer (and unused slots) read as zero: the scalar offset fails the range check
      const uint32_t so = (prr[i] < s1 && r_first + prr[i] < wd.buf[1]) ? xb + (uint32_t)prr[i] * sx1 * ES : kOob;
      rp[i] = load4<MODE == 1>(rx, pg[i], so);
    }
    rpy = load4<MODE == 1>(ry, pgy, ((uint32_t)n * syn + (uint32_t)o0 * sy0 + (uint32_t)o1 * sy1) * ES);
  };
  // db^ of this (worker, chunk): the workgroups of kernel plane 0 and input-channel tile 0 see every dy element
  // of their output-channel tile exactly once, on its way into LDS, and sum it there
  const bool bias_wg = t0 == 0 && ci_t == 0;
  float bsum[PCH];
#pragma unroll
  for (int j = 0; j < PCH; ++j) bsum[j] = 0.f;
  int nslot = 0;      // ring slot of the step's new row 0
  int tslot[TW];      // ring slot of the row each tap reads
  auto stash = [&](int o1) {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      if (prr[i] < s1) {  // uniform per wave
        int slot = nslot + prr[i];
        if (slot >= ring) slot -= ring;
        *(u32x4*)(ldsb + prest[i] * 16u + (uint32_t)slot * pitch) = rp[i];
      }
    }
    *(u32x4*)(ldsb + ys_base + (uint32_t)(o1 & 1) * 4096u + (uint32_t)tid * 16u) = rpy;
    if (bias_wg) {  // uniform: the dy piece this thread staged joins its part of db^ (pieces out of range are zero)
      if constexpr (BFM) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          bsum[2 * j] += __uint_as_float(rpy[j] << 16);
          bsum[2 * j + 1] += __uint_as_float(rpy[j] & 0xffff0000u);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) bsum[j] += __uint_as_float(rpy[j]);
      }
    }
  };

  // fp32: lane (h, m) reads channel m of position 2 * pr + h.  bf16 MFMA: lane s of 16-lane group G addresses
  // channels 16 * (G % 2) + 4 * (s % 4) ... + 3 of position 8 * (G / 2) + s / 4 (64 bytes per cell)
  const int lg = lane >> 4, ls = lane & 15;
  const uint32_t lane_x = BFM ? (uint32_t)((8 * (lg >> 1) + (ls >> 2)) * S2 * 64 + (16 * (lg & 1) + 4 * (ls & 3)) * 2)
                              : (uint32_t)(h * S2 * 32 + m) * 4u;
  const uint32_t lane_y = ys_base + (BFM ? (uint32_t)((8 * (lg >> 1) + (ls >> 2)) * 64 + (16 * (lg & 1) + 4 * (ls & 3)) * 2)
                                         : (uint32_t)(h * 32 + m) * 4u);
  // unit order of this kernel plane: rotated by the output planes that the last kernel plane is ahead of it
  const int unit_begin = chunk * per, unit_cnt = unit_end - unit_begin;
  const int skew = unit_cnt > 0 ? (((a.k[0] - 1 - t0) * a.dil[0]) / a.s[0] * nblk1) % unit_cnt : 0;
  for (int uj = 0; uj < unit_cnt; ++uj) {
    const int unit = unit_begin + (uj + skew < unit_cnt ? uj + skew : uj + skew - unit_cnt);
    const int plane = unit / nblk1, o1_begin = (unit - plane * nblk1) * a.ob, o1_end = min(O1, o1_begin + a.ob);
    const int o0 = plane % wd.out[0], n = plane / wd.out[0];
    for (int seg = 0; seg < nseg; ++seg) {
      setup_pieces(seg);
      nslot = (o1_begin * s1 + span - s1) % ring;
#pragma unroll
      for (int i = 0; i < TW; ++i) tslot[i] = (o1_begin * s1 + tap_t1[i] * a.dil[1]) % ring;
      __syncthreads();  // previous unit / segment fully consumed
      // prime the ring with the first span - s1 window rows of step o1_begin
      {
        const int c0 = wd.origin[0] + o0 * a.s[0] + t0 * a.dil[0];
        for (int rr = 0; rr < span - s1; ++rr) {
          const int wrow = o1_begin * s1 + rr;  // window row, relative to the first tap of output row 0
          const bool row_ok = wd.origin[1] + wrow < wd.buf[1];
          const uint32_t rb = ((uint32_t)n * sxn + (uint32_t)c0 * sx0 + (uint32_t)(wd.origin[1] + wrow) * sx1 +
                               (wd.origin[2] + seg * 32 * S2) * sx2 + ci_t * 32) * ES;
          for (int rest = tid; rest < rowp; rest += 256) {
            const int cell = rest / PPC, q4 = (rest % PPC) * PCH;
            uint32_t off = kOob;
            if (row_ok && cell < a.ncell && seg * 32 * S2 + cell < row_cells && ci_t * 32 + q4 < a.ci)
              off = (cell * sx2 + q4) * ES;
            *(u32x4*)(ldsb + (uint32_t)(wrow % ring) * pitch + (uint32_t)rest * 16u) = load4<MODE == 1>(rx, off, rb);
          }
        }
      }
      fetch(n, o0, o1_begin);
      for (int o1 = o1_begin; o1 < o1_end; ++o1) {
        stash(o1);
        __syncthreads();  // step o1 staged; every wave has finished step o1 - 1
        if (o1 + 1 < o1_end) fetch(n, o0, o1 + 1);  // in flight while this step multiplies
        const char* ta[TW];
#pragma unroll
        for (int i = 0; i < TW; ++i)
          ta[i] = ldsb + (uint32_t)tslot[i] * pitch + (uint32_t)(tap_t2[i] * a.dil[2]) * (BFM ? 64u : 128u) + lane_x;
        const char* yrow = ldsb + lane_y + (uint32_t)(o1 & 1) * 4096u;
        if constexpr (BFM) {
          // two groups of 16 positions; an operand is two transposing loads of four positions each
          typedef short v4i16 __attribute__((ext_vector_type(4)));
          typedef __attribute__((address_space(3))) v4i16* lds_v4;
          union Frag {
            v4i16 half[2];
            bf16x8 v;
          };
#pragma unroll
          for (int kg = 0; kg < 2; ++kg) {
            Frag fb, fa[TW];
            fb.half[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(yrow + kg * 1024));
            fb.half[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(yrow + kg * 1024 + 256));
#pragma unroll
            for (int i = 0; i < TW; ++i) {
              fa[i].half[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(ta[i] + kg * (16 * S2 * 64)));
              fa[i].half[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(ta[i] + kg * (16 * S2 * 64) + 4 * S2 * 64));
            }
#pragma unroll
            for (int i = 0; i < TW; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb.v, acc[i], 0, 0, 0);
          }
        } else {
        // 16 x two positions: lanes 0-31 take column 2*pr, lanes 32-63 column 2*pr + 1
#pragma unroll
        for (int pr = 0; pr < 16; ++pr) {
          const float b = *(const float*)(yrow + pr * 256);
          float av[NOWN];
#pragma unroll
          for (int i = 0; i < NOWN; ++i) av[i] = *(const float*)(ta[i] + pr * (2 * S2 * 128));
#pragma unroll
          for (int i = 0; i < NOWN; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], b, acc[i], 0, 0, 0);
        }
        if constexpr (SH > 0) {  // position pairs 4 * wave ... + 3 of the shared tap
          const char* tsh = ta[NOWN] + wave * (4 * 2 * S2 * 128);
          const char* ysh = yrow + wave * (4 * 256);
#pragma unroll
          for (int pr = 0; pr < 4; ++pr) {
            const float b = *(const float*)(ysh + pr * 256);
            const float av = *(const float*)(tsh + pr * (2 * S2 * 128));
            acc[NOWN] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b, acc[NOWN], 0, 0, 0);
          }
        }
        }
        nslot += s1;
        if (nslot >= ring) nslot -= ring;
#pragma unroll
        for (int i = 0; i < TW; ++i) {
          tslot[i] += s1;
          if (tslot[i] >= ring) tslot[i] -= ring;
        }
      }
    }
  }
  const int co = co_t * 32 + m;
  const bool co_ok = co < a.co;
  float* pbase = partial + (size_t)bz * a.slot;
#pragma unroll
  for (int i = 0; i < NOWN; ++i) {
    if (i >= ntw) break;
    const int tap = (t0 * a.k[1] + tap_t1[i]) * a.k[2] + tap_t2[i];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int cir = ci_t * 32 + 8 * (v / 4) + 4 * h + (v % 4);
      if (cir < a.ci && co_ok) pbase[((size_t)tap * a.ci + cir) * a.co + co] = acc[i][v];
    }
  }
  if constexpr (SH > 0) {
    // the shared tap: each wave's partial tile goes to LDS as [wave][register][lane]; thread tid then sums, over
    // the waves in order, the four elements register tid / 64 + 4 * k of lane tid % 64 and stores them
    float* red = (float*)wt_lds;
    __syncthreads();  // the ring is no longer read
#pragma unroll
    for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * 64 + lane] = acc[NOWN][v];
    __syncthreads();
    const int tap = (t0 * a.k[1] + tap_t1[NOWN]) * a.k[2] + tap_t2[NOWN];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int v = wave + 4 * k;
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) sum += red[(w * 16 + v) * 64 + lane];
      const int cir = ci_t * 32 + 8 * (v / 4) + 4 * h + (v % 4);
      if (cir < a.ci && co_ok) pbase[((size_t)tap * a.ci + cir) * a.co + co] = sum;
    }
  }
  if (bias_wg) {
    // thread tid summed channels (tid % PPC) * PCH ... of position tid / PPC of every row segment: add up the 32
    // positions, in order, and write the slot's trailing co entries
    float* red = (float*)wt_lds;
    __syncthreads();
    if (tid < 32 * PPC) {
#pragma unroll
      for (int j = 0; j < PCH; ++j) red[(tid / PPC) * 32 + (tid % PPC) * PCH + j] = bsum[j];
    }
    __syncthreads();
    if (tid < 32 && co_t * 32 + tid < a.co) {
      float sum = 0.f;
      for (int pos = 0; pos < 32; ++pos) sum += red[pos * 32 + tid];
      pbase[(size_t)a.k[0] * a.k[1] * a.k[2] * a.ci * a.co + co_t * 32 + tid] = sum;
    }
  }
}

// db^ partial of one (worker, chunk): sum of dy over the chunk's positions,
// written to the slot's trailing Co entries.  One block per slot.
template <bool BF16>
__global__ __launch_bounds__(256) void bias_partial_kernel(const WorkerDev* __restrict__ workers, void* const* dy_bufs,
                                                           float* __restrict__ partial, WgradArgs a) {
  const int worker = blockIdx.x / a.nchunks, chunk = blockIdx.x - worker * a.nchunks;
  const WorkerDev wd = workers[worker];
  const void* __restrict__ dy = dy_bufs[worker];
  const int nrows = a.n_b * wd.out[0] * wd.out[1];
  const int per = (nrows + a.nchunks - 1) / a.nchunks;
  const int64_t p0 = (int64_t)chunk * per * wd.out[2];
  const int64_t p1 = (int64_t)min(nrows, (chunk + 1) * per) * wd.out[2];
  __shared__ float red[256];
  const int nw = a.k[0] * a.k[1] * a.k[2] * a.ci * a.co;
  for (int c0 = 0; c0 < a.co; c0 += 32) {
    // 8 position lanes x 32 channels
    const int co = c0 + (threadIdx.x & 31);
    float acc = 0.f;
    if (co < a.co) {
      float part[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      int64_t p = p0 + (threadIdx.x >> 5);
      for (; p + 56 < p1; p += 64)
#pragma unroll
        for (int u = 0; u < 8; ++u) part[u] += load_scalar<BF16>(dy, (p + 8 * u) * a.co + co);
      for (; p < p1; p += 8) part[0] += load_scalar<BF16>(dy, p * a.co + co);
      acc = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < 32 && co < a.co) {
      float s = 0.f;
      for (int i = 0; i < 8; ++i) s += red[i * 32 + threadIdx.x];
      partial[(size_t)blockIdx.x * a.slot + nw + co] = s;
    }
    __syncthreads();
  }
}

// ---- host side ------------------------------------------------------------------

static int lds_bytes(const CorrArgs& a) { return (a.a_vec4 + a.nt[1] * a.nt[2] * 64 + 1) * 16 + (a.nt[1] * a.nt[2] + 4) * 4; }
// the variant that loads straight into LDS: two staging buffers
static int lds_bytes_dma(const CorrArgs& a) { return (4 * 256 + a.nt[1] * a.nt[2] * 64) * 16 + a.bufb + 16 + (a.nt[1] * a.nt[2] + 4) * 4; }  // PA = 4

// Window of tr x tc output positions (tr * tc <= 128 * mt) and everything derived from it.
static void finish_args(CorrArgs& a, int mt, int tc) {
  const int cap = 128 * mt;
  a.tc = std::max(1, std::min(tc, cap));
  a.tr = std::max(1, cap / a.tc);
  for (int d = 0; d < 3; ++d) {
    int lo = 0, hi = 0;
    for (int i = 0; i < a.nt[d]; ++i) {
      lo = i == 0 ? a.tapoff[d][i] : std::min(lo, a.tapoff[d][i]);
      hi = i == 0 ? a.tapoff[d][i] : std::max(hi, a.tapoff[d][i]);
    }
    a.tapmin[d] = lo;
    a.tapspan[d] = hi - lo;
  }
  a.R = (a.tr - 1) * a.is[1] + a.tapspan[1] + 1;
  a.Cw = (a.tc - 1) * a.is[2] + a.tapspan[2] + 1;
  a.CwQ = (a.Cw + a.is[2] - 1) / a.is[2];
  a.a_vec4 = a.R * 2 * a.is[2] * a.CwQ;
  a.a_pad = std::max((a.a_vec4 + 63) / 64 * 64, (a.R * a.Cw + 31) / 32 * 64);  // (blocks of 32 cells, 64 slots each)
  a.bufb = (a.a_pad + a.nt[1] * a.nt[2] * 64) * 16;
  a.div_cwq = make_fastdiv((uint32_t)a.CwQ);
  a.div_cw = make_fastdiv((uint32_t)a.Cw);
  a.div_tc = make_fastdiv((uint32_t)a.tc);
  a.div_is2 = make_fastdiv((uint32_t)a.is[2]);
}

// Fraction of the multiplied window positions that are outputs, for an nq1 x nq2 plane cut into tr x tc windows.
static double window_efficiency(int cap, int tc, int nq1, int nq2) {
  const int tr = std::max(1, cap / tc);
  const double cols = (double)nq2 / ((double)((nq2 + tc - 1) / tc) * tc);
  const double rows = (double)nq1 / ((double)((nq1 + tr - 1) / tr) * tr);
  return (double)(tr * tc) / cap * cols * rows;
}

// Window width: full output rows when they fit (else the multiple of 32 with the least padding), unless a
// narrower window wastes clearly fewer of the multiplied positions (e.g. rows of 130 in 256 positions).
static int choose_tc(int cap, int nq1max, int nq2max) {
  int tc0 = std::max(nq2max, 1);
  if (nq2max > cap) {
    tc0 = 32;
    double best = 1e30;
    for (int c = 32; c <= cap; c += 32) {
      double waste = (double)((nq2max + c - 1) / c) * c / nq2max;
      if (waste < best - 1e-9 || (waste < best + 1e-9 && c > tc0)) best = waste, tc0 = c;
    }
  }
  const double eff0 = window_efficiency(cap, tc0, nq1max, nq2max);
  int best_tc = tc0;
  double best_eff = eff0 * 1.05;
  for (int tc = 8; tc <= std::min(cap, std::max(nq2max, 1)); ++tc) {
    const double eff = window_efficiency(cap, tc, nq1max, nq2max);
    if (eff >= best_eff - 1e-9) best_eff = eff, best_tc = tc;  // ties: the wider window
  }
  return best_tc;
}

// Chooses the rows-per-wave so that two workgroups fit in a CU's LDS when
// possible; returns 0 when the patch does not fit at all.
static int choose_mt(CorrArgs& a, int nq1max, int nq2max, bool allow3) {
  if (allow3) {
    // Three M-tiles per wave (384 positions) when that window wastes clearly fewer of the multiplied positions
    // than 256 do, e.g. planes of 33 rows: 11-row windows fill three of them exactly, 7-row windows need five.
    // Built for the small-patch variants only (the parity classes of a strided layer's data gradient), not for
    // bf16 tensors widened to fp32.  Measured on the 5^3 stride-2 layer: -9 % time in bf16, -3 % in fp32 (three
    // resident workgroups of 384 positions against four of 256; while a lane still kept 16 store offsets per
    // M-tile the third tile cost the third resident workgroup and the time went up 2 %).
    CorrArgs a3 = a, a2 = a;
    finish_args(a3, 3, choose_tc(384, nq1max, nq2max));
    finish_args(a2, 2, choose_tc(256, nq1max, nq2max));
    const bool small3 = a3.R * a3.Cw * 2 <= 4 * 256 && a3.a_pad <= 4 * 256 && a3.nt[1] * a3.nt[2] * 64 <= 3 * 256 &&
                        lds_bytes(a3) <= 80 * 1024;
    if (small3 && window_efficiency(384, a3.tc, nq1max, nq2max) > 1.04 * window_efficiency(256, a2.tc, nq1max, nq2max)) {
      a = a3;
      return 3;
    }
  }
  for (int mt : {2, 1}) {
    finish_args(a, mt, choose_tc(128 * mt, nq1max, nq2max));
    if (lds_bytes(a) <= 80 * 1024 && a.R * a.Cw * 2 <= kMaxPieces * 256) return mt;
  }
  finish_args(a, 1, choose_tc(128, nq1max, nq2max));
  if (lds_bytes(a) <= 160 * 1024 && a.R * a.Cw * 2 <= kMaxPieces * 256) return 1;
  // last resort: a 32-wide window
  finish_args(a, 1, 32);
  if (lds_bytes(a) <= 160 * 1024 && a.R * a.Cw * 2 <= kMaxPieces * 256) return 1;
  return 0;
}

static void max_nq(const distdl_plan* p, const CorrArgs& a, int& nq1, int& nq2) {
  nq1 = nq2 = 0;
  for (const WorkerDev& wd : p->workers) {
    const PerWorker g = derive(wd, a);
    nq1 = std::max(nq1, g.nq[1]);
    nq2 = std::max(nq2, g.nq[2]);
  }
}

// Arithmetic mode of a correlation launch.  0: fp32; 1: bf16 tensors widened to fp32; 2: bf16 MFMAs (contraction
// channels in 16-byte pieces of 8).
static int corr_mode(const distdl_plan* p, const CorrArgs& a) {
  return p->dtype != DISTDL_BF16 ? 0 : (a.kc % 8 == 0 ? 2 : 1);
}

// Window choice of one launch (forward, or one parity class): M-tiles per wave, 0 when no window's patch fits the
// piece slots of a thread or the LDS of a compute unit (wide dilated kernels).
static int corr_window(const distdl_plan* p, CorrArgs& a) {
  const int mode = corr_mode(p, a);
  a.ck = mode == 2 ? 16 : 8;
  int nq1max, nq2max;
  max_nq(p, a, nq1max, nq2max);
  return choose_mt(a, std::max(nq1max, 1), nq2max, mode != 1);
}

bool corr_mfma_supported(const distdl_plan* p) {
  if (p->corr_mfma_ok >= 0) return p->corr_mfma_ok != 0;
  auto decide = [&]() {
    if (p->explicit_halo) return false;
    if (p->n_ci % 4 || p->n_co % 4) return false;  // 16-byte channel pieces
    // buffer instructions address one worker's tensor with 31-bit byte offsets
    if ((double)p->n_b * p->max_buf_cells * std::max(p->n_ci, p->n_co) * 4.0 >= 2147480000.0) return false;
    for (int d = 0; d < 3; ++d)
      if (p->ksize[d] > 8) return false;
    if (p->ksize[1] * p->ksize[2] > kMaxBPieces * 4) return false;  // weight pieces held in registers per stage
    // every launch of the layer must find a window: the forward one and each parity class of the data gradient
    CorrArgs fa = forward_args(p);
    if (corr_window(p, fa) == 0) return false;
    for (int p0 = 0; p0 < p->stride[0]; ++p0)
      for (int p1 = 0; p1 < p->stride[1]; ++p1)
        for (int p2 = 0; p2 < p->stride[2]; ++p2) {
          const int par[3] = {p0, p1, p2};
          CorrArgs a = class_args(p, par);
          if (corr_window(p, a) == 0) return false;
        }
    return true;
  };
  p->corr_mfma_ok = decide() ? 1 : 0;
  return p->corr_mfma_ok != 0;
}

CorrArgs forward_args(const distdl_plan* p) {
  CorrArgs a{};
  a.mode = 0;
  a.n_b = (int32_t)p->n_b;
  a.kc = (int32_t)p->n_ci;
  a.nc = (int32_t)p->n_co;
  a.ntn = (a.nc + 31) / 32;
  a.n_workers = p->n_workers;
  for (int d = 0; d < 3; ++d) {
    a.nt[d] = p->ksize[d];
    a.is[d] = p->stride[d];
    a.s[d] = p->stride[d];
    for (int i = 0; i < p->ksize[d]; ++i) {
      a.tapoff[d][i] = i * p->dilation[d];
      a.tapid[d][i] = i;
    }
  }
  return a;
}

CorrArgs class_args(const distdl_plan* p, const int par[3]) {
  CorrArgs a{};
  a.mode = 1;
  a.n_b = (int32_t)p->n_b;
  a.kc = (int32_t)p->n_co;
  a.nc = (int32_t)p->n_ci;
  a.ntn = (a.nc + 31) / 32;
  a.n_workers = p->n_workers;
  for (int d = 0; d < 3; ++d) {
    a.is[d] = 1;
    a.s[d] = p->stride[d];
    a.par[d] = par[d];
    a.nt[d] = 0;
    for (int t = 0; t < p->ksize[d]; ++t) {
      int off = t * p->dilation[d];
      if (off % p->stride[d] != par[d] % p->stride[d]) continue;
      // cell c = origin + par + s*q reads dy[q - (off - par)/s]
      a.tapoff[d][a.nt[d]] = -((off - par[d]) / p->stride[d]);
      a.tapid[d][a.nt[d]] = t;
      ++a.nt[d];
    }
  }
  return a;
}

static int64_t max_tiles(const distdl_plan* p, const CorrArgs& a) {
  int64_t mx = 0;
  for (const WorkerDev& wd : p->workers) mx = std::max(mx, tiles_of(derive(wd, a), a));
  return mx;
}

static size_t corr_weight_elems(const CorrArgs& a) {
  const int ck = a.ck ? a.ck : 8;  // channels per chunk; sized for the smaller chunk until the launch has chosen
  return (size_t)a.ntn * a.nt[0] * ((a.kc + ck - 1) / ck) * a.nt[1] * a.nt[2] * 256;
}
// weights + the tap tables (8 + 64 ints), kept 16-byte aligned
static size_t corr_scratch_elems(const CorrArgs& a) { return corr_weight_elems(a) + 72; }

// The kernel variant of a launch: M-tiles per wave, small or large patch, taps per plane known at compile time or
// not, arithmetic mode.  `large_lds` is set to the function that raises the variant's dynamic LDS limit.
struct CorrVariant {
  const void* fn = nullptr;
  int (*large_lds)() = nullptr;
  bool dma = false;  // stages go straight into LDS (two staging buffers)
};
template <int MT, int PA, int PB, int NT, int MODE, bool DMA = false>
static CorrVariant corr_variant_of() {
  return CorrVariant{(const void*)corr_mfma_kernel<MT, PA, PB, NT, MODE, DMA>,
                     &allow_large_lds<corr_mfma_kernel<MT, PA, PB, NT, MODE, DMA>>, DMA};
}
template <int MODE>
static CorrVariant corr_variant_mode(int mt, bool small, int ntaps) {
  // Small patches with the taps known at compile time load straight into LDS when the launch multiplies in bf16.
  // Measured on the data-gradient classes of the 5^3 stride-2 layer: 0.163 -> 0.153 ms per class in bf16 (stages of
  // 576 MFMA clocks), 0.692 -> 0.698 ms in fp32 (stages of 2048-4608 clocks: what the stage change costs there is not
  // the ds_write of the staged pieces), so fp32 keeps the register-staged loop.
  constexpr bool D = MODE == 2;
  if (mt == 2 && small && ntaps == 9) return corr_variant_of<2, 4, 3, 9, MODE, D>();
  if (mt == 2 && small && ntaps == 6) return corr_variant_of<2, 4, 3, 6, MODE, D>();
  if (mt == 2 && small && ntaps == 4) return corr_variant_of<2, 4, 3, 4, MODE, D>();
  if (mt == 2 && small) return corr_variant_of<2, 4, 3, 0, MODE>();
  if constexpr (MODE == 2) {  // three M-tiles per wave
    if (mt == 3 && ntaps == 9) return corr_variant_of<3, 4, 3, 9, 2, true>();
    if (mt == 3 && ntaps == 6) return corr_variant_of<3, 4, 3, 6, 2, true>();
    if (mt == 3 && ntaps == 4) return corr_variant_of<3, 4, 3, 4, 2, true>();
    if (mt == 3) return corr_variant_of<3, 4, 3, 0, 2>();
  }
  if constexpr (MODE == 0) {
    if (mt == 3 && ntaps == 9) return corr_variant_of<3, 4, 3, 9, 0>();
    if (mt == 3 && ntaps == 6) return corr_variant_of<3, 4, 3, 6, 0>();
    if (mt == 3 && ntaps == 4) return corr_variant_of<3, 4, 3, 4, 0>();
    if (mt == 3) return corr_variant_of<3, 4, 3, 0, 0>();
  }
  if (mt == 2 && ntaps == 25) return corr_variant_of<2, kMaxPieces, kMaxBPieces, 25, MODE>();
  if (mt == 2) return corr_variant_of<2, kMaxPieces, kMaxBPieces, 0, MODE>();
  if (small) return corr_variant_of<1, 4, 3, 0, MODE>();
  return corr_variant_of<1, kMaxPieces, kMaxBPieces, 0, MODE>();
}
static CorrVariant corr_variant(int mode, int mt, bool small, int ntaps) {
  return mode == 2 ? corr_variant_mode<2>(mt, small, ntaps)
                   : mode == 1 ? corr_variant_mode<1>(mt, small, ntaps) : corr_variant_mode<0>(mt, small, ntaps);
}

// Workgroups of 256 threads of kernel `fn` that one compute unit holds at a time with `lds` bytes of dynamic LDS
// (registers and LDS decide); asked of the runtime once per (kernel, LDS size) and remembered.
static int resident_workgroups(const void* fn, int lds) {
  struct Entry {
    const void* fn;
    int lds, n;
  };
  static std::mutex mu;
  static std::vector<Entry> known;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : known)
    if (e.fn == fn && e.lds == lds) return e.n;
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, 256, (size_t)lds) != hipSuccess || n < 1) n = 2;
  known.push_back(Entry{fn, lds, n});
  return n;
}

static int launch_corr(distdl_plan* p, CorrArgs a, const void* w, float* wscratch, const void* bias, void** in_tab,
                       void** out_tab, const char* name, hipStream_t st) {
  const int mode = corr_mode(p, a);
  const int mt = corr_window(p, a);
  if (mt == 0) return set_error(DISTDL_ERR_UNSUPPORTED, "conv: kernel footprint does not fit in LDS");  // corr_mfma_supported() rules this out
  const bool small = a.R * a.Cw * 2 <= 4 * 256 && a.nt[1] * a.nt[2] * 64 <= 3 * 256 && a.a_pad <= 4 * 256;
  const CorrVariant kv = corr_variant(mode, mt, small, a.nt[1] * a.nt[2]);
  const int lds = kv.dma ? lds_bytes_dma(a) : lds_bytes(a);
  if (lds > 64 * 1024)
    if (int rc = kv.large_lds()) return rc;
  // Workgroups per compute unit that add throughput: with fp32 MFMAs two already keep the matrix pipes busy (a
  // third and fourth one resident only smooth the stage changes), with bf16 MFMAs the launch is bound by latencies
  // and every resident workgroup counts.  Measured on the 5^3 stride-2 layer: counting three or four for fp32 picks
  // chunk lengths that run 1.5 - 3.5 % slower, counting two for bf16 3 % slower.
  int resident = resident_workgroups(kv.fn, lds);
  if (mode != 2) resident = std::min(resident, 2);
  // Output planes per workgroup.  A workgroup pays a fixed set-up (its address tables, about 8 * 10^3
  // cycles) and then about `per_plane` cycles per plane, its waves sharing the SIMDs with those of the other
  // resident workgroups; the chip runs 256 * resident workgroups at a time.
  // Pick the chunk length with the smallest estimated time, preferring shorter chunks among near-ties.
  a.g0 = 1;
  {
    int64_t planes_max = 0;
    for (const WorkerDev& wd : p->workers) planes_max = std::max<int64_t>(planes_max, p->n_b * derive(wd, a).nq[0]);
    const int64_t per_plane_wgs = max_tiles(p, a) / std::max<int64_t>(planes_max, 1) * p->n_workers;  // with g0 == 1
    const double setup = 8.0e3;
    const double per_plane = (double)a.nt[0] * ((a.kc + a.ck - 1) / a.ck) * a.nt[1] * a.nt[2] * mt *
                             (a.ck == 16 ? 32.0 : 256.0) * resident;
    const int64_t slots = 256 * (int64_t)resident;
    double best = 1e300;
    // When neighbouring output planes read the same input planes (see the kernel: planes are dealt to the plane groups
    // in turn and the kernel planes walked in a rotated order), at least four groups per worker, so that the groups
    // that run side by side cover a run of neighbouring planes (bf16 forward of the 5^3 stride-2 layer: 0.68 ms with 2
    // to 8 planes per workgroup, 0.71 ms with the 16 the estimate below would pick).
    const int tstep0 = a.nt[0] > 1 ? a.tapoff[0][1] - a.tapoff[0][0] : 0;
    const bool shares = tstep0 != 0 && a.is[0] % tstep0 == 0 && (a.is[0] / tstep0) % a.nt[0] != 0;
    const int64_t g0_max = shares ? std::max<int64_t>(1, planes_max / 4) : planes_max;
    for (int64_t g0 = 1; g0 <= g0_max; ++g0) {
      const int64_t wgs = (planes_max + g0 - 1) / g0 * per_plane_wgs;
      const double cost = (double)((wgs + slots - 1) / slots) * (setup + g0 * per_plane);
      if (cost < best * 0.97) best = cost, a.g0 = (int32_t)g0;
    }
  }
  a.tiles_max = (int32_t)max_tiles(p, a);
  if (a.tiles_max == 0) return DISTDL_OK;
  a.wt = wscratch;
  a.bias = bias;
  const int taps = p->ksize[0] * p->ksize[1] * p->ksize[2];
  const size_t welems = corr_weight_elems(a);
  a.tapinfo = (const int*)(wscratch + welems);
  {
    ProfScope prof("conv_relayout_w", st);
    const dim3 wgrid((unsigned)std::max<size_t>(1, (welems * (mode == 2 ? 2 : 1) + 255) / 256));
    if (mode == 2)
      hipLaunchKernelGGL(corr_weights_kernel<2>, wgrid, dim3(256), 0, st, w, wscratch, a, (int)p->n_ci, (int)p->n_co,
                         taps, p->ksize[1], p->ksize[2]);
    else if (mode == 1)
      hipLaunchKernelGGL(corr_weights_kernel<1>, wgrid, dim3(256), 0, st, w, wscratch, a, (int)p->n_ci, (int)p->n_co,
                         taps, p->ksize[1], p->ksize[2]);
    else
      hipLaunchKernelGGL(corr_weights_kernel<0>, wgrid, dim3(256), 0, st, w, wscratch, a, (int)p->n_ci, (int)p->n_co,
                         taps, p->ksize[1], p->ksize[2]);
  }
  int64_t blocks = (int64_t)a.tiles_max * p->n_workers;
  blocks = (blocks + 7) / 8 * 8;
  ProfScope prof(name, st);
  void* kargs[] = {(void*)&p->d_workers, (void*)&in_tab, (void*)&out_tab, (void*)&a};
  DISTDL_HIP_TRY(hipLaunchKernel(kv.fn, dim3((unsigned)blocks), dim3(256), kargs, (size_t)lds, st));
  return DISTDL_OK;
}

// Scratch for the re-laid-out weights: forward needs one set, the data
// gradient one per parity class (used one after the other on the stream).
int ensure_wscratch(distdl_plan* p, size_t elems) {
  if (p->wt_elems >= elems) return DISTDL_OK;
  if (p->d_wt) (void)hipFree(p->d_wt);
  p->d_wt = nullptr;
  p->wt_elems = 0;
  DISTDL_HIP_TRY(hipMalloc((void**)&p->d_wt, elems * sizeof(float)));
  p->wt_elems = elems;
  return DISTDL_OK;
}

int conv_fwd_mfma(distdl_plan* p, const void* w, const void* bias, hipStream_t st) {
  CorrArgs a = forward_args(p);
  int rc = ensure_wscratch(p, std::max(corr_scratch_elems(a), bwd_scratch_elems(p)));
  if (rc) return rc;
  return launch_corr(p, a, w, p->d_wt, bias, p->tab_x.dev, p->tab_y.dev, "conv_fwd_mfma", st);
}

size_t bwd_scratch_elems(const distdl_plan* p) {
  size_t total = 0;
  for (int p0 = 0; p0 < p->stride[0]; ++p0)
    for (int p1 = 0; p1 < p->stride[1]; ++p1)
      for (int p2 = 0; p2 < p->stride[2]; ++p2) {
        const int par[3] = {p0, p1, p2};
        CorrArgs a = class_args(p, par);
        total += corr_scratch_elems(a);
      }
  return total;
}

int conv_bwd_data_mfma(distdl_plan* p, const void* w, hipStream_t st) {
  CorrArgs fa = forward_args(p);
  int rc = ensure_wscratch(p, std::max(corr_scratch_elems(fa), bwd_scratch_elems(p)));
  if (rc) return rc;
  size_t at = 0;
  for (int p0 = 0; p0 < p->stride[0]; ++p0)
    for (int p1 = 0; p1 < p->stride[1]; ++p1)
      for (int p2 = 0; p2 < p->stride[2]; ++p2) {
        const int par[3] = {p0, p1, p2};
        CorrArgs a = class_args(p, par);
        if ((rc = launch_corr(p, a, w, p->d_wt + at, nullptr, p->tab_dy.dev, p->tab_dx.dev, "conv_bwd_data_mfma", st)))
          return rc;
        at += corr_scratch_elems(a);
      }
  return DISTDL_OK;
}

static bool wgrad_rows_shape_ok(const distdl_plan* p);

// bf16 tensors: only the plane-per-workgroup kernel widens its operands while it stages them (it also needs
// 16-byte aligned arrays, which the caller checks).
bool wgrad_mfma_supported(const distdl_plan* p) {
  if (p->explicit_halo || p->ksize[2] > kMaxK2) return false;
  return p->dtype == DISTDL_F32 || wgrad_rows_shape_ok(p);
}

// Taps per wave of the plane-per-workgroup weight-gradient kernel (0: fewer taps than waves).
static int wgrad_taps_per_wave(const distdl_plan* p) {
  const int T = p->ksize[1] * p->ksize[2];
  return T >= 4 ? (T + 3) / 4 : 0;
}

// The plane-per-workgroup kernel needs 16-byte channel pieces, a row stride of 1 or 2, a tap count
// per wave it is instantiated for, s1 new rows per step that fit the five piece slots of a thread,
// and a ring that fits in LDS.
// 0: fp32 tensors; 1: bf16 tensors widened to fp32; 2: bf16 MFMAs (channel counts that are multiples of 8)
static int wgrad_mode(const distdl_plan* p) {
  if (p->dtype != DISTDL_BF16) return 0;
  return (p->n_ci % 8 == 0 && p->n_co % 8 == 0) ? 2 : 1;
}

static bool wgrad_rows_shape_ok(const distdl_plan* p) {
  const int span = (p->ksize[1] - 1) * p->dilation[1] + 1;
  const int ncell = 31 * p->stride[2] + (p->ksize[2] - 1) * p->dilation[2] + 1;
  const int rowp = (ncell * (wgrad_mode(p) == 2 ? 4 : 8) + 63) & ~63;
  const int tw = wgrad_taps_per_wave(p);
  if (p->n_ci % 4 || p->n_co % 4) return false;
  if (tw != 3 && tw != 4 && tw != 7) return false;
  if (p->stride[2] > 2 || p->stride[1] > span) return false;
  if (p->stride[1] * rowp > 5 * 256) return false;
  if ((size_t)(span + p->stride[1]) * rowp * 16 + 8192 > 160 * 1024) return false;
  if ((double)p->n_b * p->max_buf_cells * std::max(p->n_ci, p->n_co) * 4.0 >= 2147480000.0) return false;
  return true;
}

// Output rows per work unit of the plane-per-workgroup kernel: whole planes when there are enough of them to
// fill the chip, else blocks of rows (each block re-reads span - s1 rows to prime its ring).
static int wgrad_row_block(const distdl_plan* p) {
  int64_t planes = 0, o1max = 1;
  for (const WorkerDev& wd : p->workers) {
    planes = std::max<int64_t>(planes, p->n_b * wd.out[0]);
    o1max = std::max<int64_t>(o1max, wd.out[1]);
  }
  int64_t tiles = ((p->n_ci + 31) / 32) * ((p->n_co + 31) / 32);
  int64_t blocks = (int64_t)p->ksize[0] * tiles * p->n_workers;
  int64_t want_units = (2048 + blocks - 1) / blocks;  // per worker
  if (planes >= want_units) return (int)o1max;
  int64_t per_plane = (want_units + planes - 1) / planes;
  return (int)std::max<int64_t>(8, (o1max + per_plane - 1) / per_plane);
}

int wgrad_chunks(const distdl_plan* p) {
  int64_t tiles = ((p->n_ci + 31) / 32) * ((p->n_co + 31) / 32);
  if (wgrad_rows_shape_ok(p)) {
    // chunks of work units (plane, block of output rows); about 2048 workgroups, preferring a chunk
    // count that splits the units evenly
    int64_t units = 0;
    const int ob = wgrad_row_block(p);
    for (const WorkerDev& wd : p->workers)
      units = std::max<int64_t>(units, p->n_b * wd.out[0] * ((wd.out[1] + ob - 1) / ob));
    int64_t blocks = (int64_t)p->ksize[0] * tiles * p->n_workers;
    int64_t want = std::max<int64_t>(1, std::min<int64_t>(units, (2048 + blocks - 1) / blocks));
    int64_t best = want, best_pad = INT64_MAX;
    for (int64_t c = want; c <= std::min<int64_t>(units, want + 4); ++c) {
      int64_t pad = (units + c - 1) / c * c - units;
      if (pad < best_pad) best_pad = pad, best = c;
    }
    return (int)best;
  }
  // enough (worker, chunk) slots to fill the chip a few times over
  int64_t groups = (p->ksize[0] * p->ksize[1] + 3) / 4;
  int64_t blocks = groups * tiles * p->n_workers;
  int64_t want = (1536 + blocks - 1) / blocks;
  int64_t rows = p->n_b * p->max_out_cells;  // upper bound on rows
  return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, 32), rows));
}

int conv_wgrad_mfma(distdl_plan* p, float* partial, hipStream_t st) {
  WgradArgs a{};
  a.n_b = (int32_t)p->n_b;
  a.ci = (int32_t)p->n_ci;
  a.co = (int32_t)p->n_co;
  for (int d = 0; d < 3; ++d) {
    a.k[d] = p->ksize[d];
    a.s[d] = p->stride[d];
    a.dil[d] = p->dilation[d];
  }
  a.nchunks = wgrad_chunks(p);
  a.slot = (int64_t)a.k[0] * a.k[1] * a.k[2] * a.ci * a.co + a.co;
  dim3 grid((unsigned)((a.k[0] * a.k[1] + 3) / 4), (unsigned)(((a.ci + 31) / 32) * ((a.co + 31) / 32)),
            (unsigned)(p->n_workers * a.nchunks));
  // LDS-staged variants when 16-byte pieces are possible and the segment fits
  a.ncell = 31 * a.s[2] + (a.k[2] - 1) * a.dil[2] + 1;
  a.span = (a.k[1] - 1) * a.dil[1] + 1;
  a.ob = wgrad_row_block(p);
  bool aligned = a.ci % 4 == 0 && a.co % 4 == 0;
  for (int w = 0; w < p->n_workers && aligned; ++w)
    aligned = (uintptr_t)p->tab_x.host[w] % 16 == 0 && (uintptr_t)p->tab_dy.host[w] % 16 == 0;
  const int lds = 4 * (a.ncell + 32) * 128;
  const bool bf16 = p->dtype == DISTDL_BF16;
  const bool taps_path = aligned && wgrad_rows_shape_ok(p);
  if (taps_path) {
    const int mode = wgrad_mode(p);
    const int rowp = (a.ncell * (mode == 2 ? 4 : 8) + 63) & ~63;
    const int rlds = (a.span + a.s[1]) * rowp * 16 + 8192;
    const int tw = wgrad_taps_per_wave(p);
    dim3 rgrid((unsigned)a.k[0], grid.y, grid.z), rblock(256);
    ProfScope prof("conv_bwd_weight_mfma", st);
    // one tap left over after dealing the plane's taps to the four waves: it is shared (fp32 MFMAs only)
    const int T = a.k[1] * a.k[2];
    const bool share = mode != 2 && T % 4 == 1 && T / 4 + 1 == tw && rlds >= 4 * 16 * 64 * 4;
#define DISTDL_LAUNCH_TAPS_T(TW_, S2_, BF_, SH_)                                                                    \
  do {                                                                                                              \
    if (rlds > 64 * 1024)                                                                                           \
      if (int rc_ = allow_large_lds<wgrad_taps_kernel<TW_, S2_, BF_, SH_>>()) return rc_;                           \
    hipLaunchKernelGGL((wgrad_taps_kernel<TW_, S2_, BF_, SH_>), rgrid, rblock, rlds, st, p->d_workers,              \
                       p->tab_x.dev, p->tab_dy.dev, partial, a);                                                    \
  } while (0)
#define DISTDL_LAUNCH_TAPS(TW_, S2_)                                                                                \
  do {                                                                                                              \
    if (mode == 2) DISTDL_LAUNCH_TAPS_T(TW_, S2_, 2, 0);                                                            \
    else if (mode == 1 && share) DISTDL_LAUNCH_TAPS_T(TW_, S2_, 1, 1);                                              \
    else if (mode == 1) DISTDL_LAUNCH_TAPS_T(TW_, S2_, 1, 0);                                                       \
    else if (share) DISTDL_LAUNCH_TAPS_T(TW_, S2_, 0, 1);                                                           \
    else DISTDL_LAUNCH_TAPS_T(TW_, S2_, 0, 0);                                                                      \
  } while (0)
    if (tw == 3 && a.s[2] == 1) DISTDL_LAUNCH_TAPS(3, 1);
    else if (tw == 3) DISTDL_LAUNCH_TAPS(3, 2);
    else if (tw == 4 && a.s[2] == 1) DISTDL_LAUNCH_TAPS(4, 1);
    else if (tw == 4) DISTDL_LAUNCH_TAPS(4, 2);
    else if (a.s[2] == 1) DISTDL_LAUNCH_TAPS(7, 1);
    else DISTDL_LAUNCH_TAPS(7, 2);
#undef DISTDL_LAUNCH_TAPS
#undef DISTDL_LAUNCH_TAPS_T
  } else {
    if (bf16) return set_error(DISTDL_ERR_UNSUPPORTED, "conv: bf16 weight gradient needs 16-byte aligned arrays");
    ProfScope prof("conv_bwd_weight_mfma", st);
    if (aligned && a.ncell <= 72 && a.k[2] <= 3)
      hipLaunchKernelGGL((wgrad_lds_kernel<3, 9>), grid, dim3(256), lds, st, p->d_workers, p->tab_x.dev,
                         p->tab_dy.dev, partial, a);
    else if (aligned && a.ncell <= 72 && a.k[2] <= 5)
      hipLaunchKernelGGL((wgrad_lds_kernel<5, 9>), grid, dim3(256), lds, st, p->d_workers, p->tab_x.dev,
                         p->tab_dy.dev, partial, a);
    else if (a.k[2] <= 3)
      hipLaunchKernelGGL(wgrad_mfma_kernel<3>, grid, dim3(256), 0, st, p->d_workers, p->tab_x.dev, p->tab_dy.dev,
                         partial, a);
    else if (a.k[2] <= 5)
      hipLaunchKernelGGL(wgrad_mfma_kernel<5>, grid, dim3(256), 0, st, p->d_workers, p->tab_x.dev, p->tab_dy.dev,
                         partial, a);
    else
      hipLaunchKernelGGL(wgrad_mfma_kernel<8>, grid, dim3(256), 0, st, p->d_workers, p->tab_x.dev, p->tab_dy.dev,
                         partial, a);
  }
  if (!taps_path) {  // the plane-per-workgroup kernel sums db^ itself
    ProfScope prof("conv_bias_partial", st);
    if (bf16)
      hipLaunchKernelGGL(bias_partial_kernel<true>, dim3((unsigned)(p->n_workers * a.nchunks)), dim3(256), 0, st,
                         p->d_workers, p->tab_dy.dev, partial, a);
    else
      hipLaunchKernelGGL(bias_partial_kernel<false>, dim3((unsigned)(p->n_workers * a.nchunks)), dim3(256), 0, st,
                         p->d_workers, p->tab_dy.dev, partial, a);
  }
  return DISTDL_OK;
}

}  // namespace distdl
