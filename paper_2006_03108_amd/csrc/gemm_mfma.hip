// MFMA GEMM for the partitioned affine layer (Sec. 4 "Dense layers"): one launch computes, for a
// list of output blocks,
//       C_o[M_o x N_o] = sum over segments s of  A_{o,s}[M_o x K_s] * B_{o,s}[K_s x N_o]  (+ bias_o[N_o])
// The segment loop is where the paper's sum-reduce R lives: forward y_i sums over the P_fi column
// workers (A = x_j, B = W_ij^T), the data gradient dx_j over the P_fo row workers (A = dy_i,
// B = W_ij), the weight gradient dW_ij has one segment (A = dy_i^T, B = x_j).  The broadcast B x
// is a shared read of the same x_j by every block that needs it.
//
// Operands are addressed by (pointer, leading dimension, which index is contiguous):
//   A "K-contiguous":  A[m][k] at a[m*lda + k];   "M-contiguous": a[k*lda + m]
//   B "K-contiguous":  B[k][n] at b[n*ldb + k];   "N-contiguous": b[k*ldb + n]
// Tiles are 64 x 64 or 128 x 128 per workgroup (4 waves, 1 or 2 x 2 MFMA tiles of 32 x 32 each), staged through LDS with
// 16-byte buffer loads (rows beyond the matrix fail the range check and read as zero) that run one or two
// stages ahead in registers; LDS is double buffered: one barrier per stage.
//
// fp32: v_mfma_f32_32x32x2_f32, A lane l holds A[i = l%32][k = l/32]; a 16-byte LDS read gives a lane
//       4 consecutive k, used by 4 MFMAs whose k-pairs are (j, 4+j) -- the same pairing on both operands.
// bf16: v_mfma_f32_32x32x16_bf16, A lane l holds A[i = l%32][k = 8*(l/32) .. +7], one 16-byte read.
// D register v of lane l is D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32] for both.
#include <algorithm>
#include <cstring>
#include <type_traits>

#include "common.h"
#include "gemm_mfma.h"
#include "profile.h"

namespace distdl {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr uint32_t kGemmOob = 0x7ffffff0u;

__device__ inline __amdgpu_buffer_rsrc_t gemm_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ inline uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// Calls f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N - 1>): a loop whose index is a
// compile-time constant in the body (register arrays indexed by it stay in registers).
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// BF16 = false: T is float, BK = 32 floats per stage.  BF16 = true: T is bf16 bits, BK = 64 per stage.
// TM x TN: 32 x 32 MFMA tiles per wave; the workgroup tile is 64*TM x 64*TN (4 waves, 2 x 2).
// Row pitch in LDS is BK + 16 bytes for the K-contiguous layout, tile extent + 16 (bf16: 32) bytes for the other.
//
// D: stages the global loads run ahead of the multiplication (a ring of D register sets).
// SB: one LDS buffer and two barriers per stage instead of two buffers and one barrier.
//
// nsplit > 1 (grid.y): the K stages of all segments, taken as one sequence, are cut into nsplit contiguous runs,
// one workgroup per tile and run, each of which
// writes its fp32 partial tile to `partial` ([block][split][M][N]); gemm_reduce_kernel then sums the splits
// in ascending order, adds the bias and rounds.  This is the sum-reduce R of the layer left un-fused: with a
// small batch a launch has too few tiles to fill the chip, and the splits supply the missing workgroups.
template <bool BF16, bool A_KC, bool B_KC, int TM, int TN, int D, bool SB>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const GemmBlock* __restrict__ blocks, float* __restrict__ partial,
                                                        int64_t partial_stride) {
  constexpr int ES = BF16 ? 2 : 4;             // element size
  constexpr int GK = BF16 ? 16 : 8;            // k per group: one bf16 MFMA, or four fp32 ones, per tile
  constexpr int KG = 4;                        // k groups per stage
  constexpr int BK = GK * KG;                  // k per stage
  constexpr int VE = 16 / ES;                  // elements per 16-byte piece
  constexpr int TILE_M = 64 * TM, TILE_N = 64 * TN;
  constexpr int PITCH_KC = BK * ES + 16;       // bytes per tile row, K-contiguous staging [row][k]
  constexpr int TPAD = BF16 ? 32 : 16;         // bf16: four k lines read together fall 8 banks apart
  constexpr int PITCH_TA = TILE_M * ES + TPAD;  // bytes per k line, transposed staging [k][row]
  constexpr int PITCH_TB = TILE_N * ES + TPAD;
  constexpr int A_BYTES = A_KC ? TILE_M * PITCH_KC : BK * PITCH_TA;
  constexpr int B_BYTES = B_KC ? TILE_N * PITCH_KC : BK * PITCH_TB;
  constexpr int PA = TILE_M * BK * ES / 16 / 256;  // 16-byte pieces per thread and stage
  constexpr int PB = TILE_N * BK * ES / 16 / 256;
  extern __shared__ __attribute__((aligned(16))) char smem[];  // A0 B0 A1 B1 (SB: A0 B0)

  const GemmBlock& gb = blocks[blockIdx.z];
  const int tiles_n = (gb.N + TILE_N - 1) / TILE_N, tiles_m = (gb.M + TILE_M - 1) / TILE_M;
  // consecutive tiles share the B tile (weights: m walks fastest); workgroups are dealt to the 8 XCDs
  // round-robin, so give each XCD a contiguous range of tiles and keep that sharing behind one L2
  const int tile = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (tile >= tiles_m * tiles_n) return;
  const int tm = tile % tiles_m, tn = tile / tiles_m;
  const int m0 = tm * TILE_M, n0 = tn * TILE_N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ml = lane & 31;
  const int wy = wave >> 1, wx = wave & 1;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // The K stages of all segments form one sequence; this workgroup multiplies the stages [g_first, g_first + n)
  // of it.  Loads run D stages ahead of the multiplication through a ring of D register sets, so that a
  // stage's memory latency is spread over D stages of arithmetic.
  int total = 0;
  for (int s = 0; s < gb.nseg; ++s) total += (gb.seg[s].K + BK - 1) / BK;
  const int g_first = (int)((int64_t)total * blockIdx.y / gridDim.y);
  const int n = (int)((int64_t)total * (blockIdx.y + 1) / gridDim.y) - g_first;

  // piece -> (row or k line, 16-byte column) of this thread, fixed
  //   K-contiguous: rows x (BK/VE) pieces per row; transposed: BK lines x (rows/VE) pieces per line
  u32x4 ra[D][PA], rb[D][PB];
  uint32_t a_goff[PA], b_goff[PB], a_loff[PA], b_loff[PB];
  int a_k[PA], b_k[PB];  // k of the piece's first element (to cut the K tail)
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    const int piece = tid + i * 256;
    if (A_KC) {
      a_loff[i] = (piece / (BK / VE)) * PITCH_KC + (piece % (BK / VE)) * 16;
      a_k[i] = (piece % (BK / VE)) * VE;
    } else {
      a_loff[i] = (piece / (TILE_M / VE)) * PITCH_TA + (piece % (TILE_M / VE)) * 16;
      a_k[i] = piece / (TILE_M / VE);
    }
  }
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    const int piece = tid + i * 256;
    if (B_KC) {
      b_loff[i] = (piece / (BK / VE)) * PITCH_KC + (piece % (BK / VE)) * 16;
      b_k[i] = (piece % (BK / VE)) * VE;
    } else {
      b_loff[i] = (piece / (TILE_N / VE)) * PITCH_TB + (piece % (TILE_N / VE)) * 16;
      b_k[i] = piece / (TILE_N / VE);
    }
  }

  // load cursor: segment, stage within it, and what depends on the segment
  int ls = 0, lin = g_first, l_nst = 0, l_K = 0;
  uint32_t l_lda = 0, l_ldb = 0;
  __amdgpu_buffer_rsrc_t ra_rs = gemm_rsrc(nullptr, 0), rb_rs = gemm_rsrc(nullptr, 0);
  auto enter_segment = [&]() __attribute__((always_inline)) {
    const GemmSeg& sg = gb.seg[ls];
    l_K = sg.K;
    l_nst = (sg.K + BK - 1) / BK;
    l_lda = (uint32_t)sg.lda;
    l_ldb = (uint32_t)sg.ldb;
    // resources cover exactly the operand: rows beyond M / N (or k lines beyond K) read as zero
    ra_rs = gemm_rsrc(sg.a, (uint32_t)(A_KC ? gb.M : sg.K) * sg.lda * ES);
    rb_rs = gemm_rsrc(sg.b, (uint32_t)(B_KC ? gb.N : sg.K) * sg.ldb * ES);
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      const int piece = tid + i * 256;
      if (A_KC) {
        a_goff[i] = ((uint32_t)(m0 + piece / (BK / VE)) * l_lda + a_k[i]) * ES;
      } else {
        const int mq = piece % (TILE_M / VE);
        a_goff[i] = ((uint32_t)a_k[i] * l_lda + m0 + mq * VE) * ES;
        if (m0 + mq * VE >= gb.M) a_goff[i] = kGemmOob;  // columns beyond M (whole pieces: M % VE == 0)
      }
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int piece = tid + i * 256;
      if (B_KC) {
        b_goff[i] = ((uint32_t)(n0 + piece / (BK / VE)) * l_ldb + b_k[i]) * ES;
      } else {
        const int nq = piece % (TILE_N / VE);
        b_goff[i] = ((uint32_t)b_k[i] * l_ldb + n0 + nq * VE) * ES;
        if (n0 + nq * VE >= gb.N) b_goff[i] = kGemmOob;
      }
    }
  };
  // Loads the next stage of the sequence into ring slot `slot`.  With `valid` false (past the last stage) the
  // loads are still issued, with offsets that fail the range check: every path through the loop then has the
  // same number of loads in flight, which lets the compiler wait for exactly the oldest stage instead of all.
  auto load = [&](auto slot_c, bool valid) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;
    int k0 = 0;
    if (valid) {  // wave-uniform
      while (lin >= l_nst) {
        lin -= l_nst;
        ++ls;
        enter_segment();
      }
      k0 = lin * BK;
      ++lin;
    }
    const uint32_t a_base = (uint32_t)k0 * (A_KC ? 1u : l_lda) * ES;
    const uint32_t b_base = (uint32_t)k0 * (B_KC ? 1u : l_ldb) * ES;
    // K tail: pieces are whole (K % VE == 0 for K-contiguous operands), lines beyond K fail the range check
#pragma unroll
    for (int i = 0; i < PA; ++i)
      ra[slot][i] = __builtin_amdgcn_raw_buffer_load_b128(
          ra_rs, (!valid || (A_KC && k0 + a_k[i] >= l_K)) ? kGemmOob : a_goff[i], a_base, 0);
#pragma unroll
    for (int i = 0; i < PB; ++i)
      rb[slot][i] = __builtin_amdgcn_raw_buffer_load_b128(
          rb_rs, (!valid || (B_KC && k0 + b_k[i] >= l_K)) ? kGemmOob : b_goff[i], b_base, 0);
  };
  auto stash = [&](int buf, auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;
    char* sa = smem + buf * (A_BYTES + B_BYTES);
    char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < PA; ++i) *(u32x4*)(sa + a_loff[i]) = ra[slot][i];
#pragma unroll
    for (int i = 0; i < PB; ++i) *(u32x4*)(sb + b_loff[i]) = rb[slot][i];
  };
  // multiplies the stage held in LDS buffer `buf`
  auto multiply = [&](int buf) __attribute__((always_inline)) {
      const char* sa = smem + buf * (A_BYTES + B_BYTES);
      const char* sb = sa + A_BYTES;
      // The LDS reads of k group g + 1 are issued before the MFMAs of group g; the scheduling barriers
      // pin that order (left alone, the compiler sinks the reads to their first use and the LDS latency
      // is paid once per group).
      if constexpr (!BF16) {
        auto rd = [&](int kk, float (&av)[TM][4], float (&bv)[TN][4]) {
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int row = 32 * (wy * TM + i) + ml;
            if (A_KC) {
              const float4 t = *(const float4*)(sa + row * PITCH_KC + (kk + 4 * h) * 4);
              av[i][0] = t.x; av[i][1] = t.y; av[i][2] = t.z; av[i][3] = t.w;
            } else {
#pragma unroll
              for (int j = 0; j < 4; ++j) av[i][j] = *(const float*)(sa + (kk + 4 * h + j) * PITCH_TA + row * 4);
            }
          }
#pragma unroll
          for (int i = 0; i < TN; ++i) {
            const int row = 32 * (wx * TN + i) + ml;
            if (B_KC) {
              const float4 t = *(const float4*)(sb + row * PITCH_KC + (kk + 4 * h) * 4);
              bv[i][0] = t.x; bv[i][1] = t.y; bv[i][2] = t.z; bv[i][3] = t.w;
            } else {
#pragma unroll
              for (int j = 0; j < 4; ++j) bv[i][j] = *(const float*)(sb + (kk + 4 * h + j) * PITCH_TB + row * 4);
            }
          }
        };
        auto mm = [&](const float (&av)[TM][4], const float (&bv)[TN][4]) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int im = 0; im < TM; ++im)
#pragma unroll
              for (int in = 0; in < TN; ++in)
                acc[im][in] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[im][j], bv[in][j], acc[im][in], 0, 0, 0);
        };
        float av[2][TM][4], bv[2][TN][4];
        rd(0, av[0], bv[0]);
        rd(GK, av[1], bv[1]);
        static_for<KG>([&](auto g) __attribute__((always_inline)) {
          constexpr int gv = decltype(g)::value;
          __builtin_amdgcn_sched_barrier(0);
          mm(av[gv & 1], bv[gv & 1]);
          if constexpr (gv + 2 < KG) {
            __builtin_amdgcn_sched_barrier(0);
            rd((gv + 2) * GK, av[gv & 1], bv[gv & 1]);
          }
        });
      } else {
        // An operand staged [k][row] (rows contiguous) is read with ds_read_b64_tr_b16.  Measured lane layout of
        // that load: in every group of 16 lanes, lane 4 * b + a receives, as element v, the a-th 16-bit element of
        // the 8 bytes addressed by lane b + 4 * v of the group.  Lane s of group G addresses rows
        // 16 * (G % 2) + 4 * (s % 4) ... + 3 of k line 8 * (G / 2) + s / 4, so lane t of the group receives row
        // 16 * (G % 2) + t of four consecutive k: two loads make the operand of lane l = (row l % 32, k 8 * (l / 32) ...).
        typedef short v4i16 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) v4i16* lds_v4;
        union Frag { u32x4 u; bf16x8 v; v4i16 t[2]; };
        const int tk = 8 * (lane >> 5) + ((lane & 15) >> 2), tr = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        auto rd = [&](int kk, Frag (&av)[TM], Frag (&bv)[TN]) {
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int row = 32 * (wy * TM + i) + ml;
            if (A_KC) {
              av[i].u = *(const u32x4*)(sa + row * PITCH_KC + (kk + 8 * h) * 2);
            } else {
              av[i].t[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sa + (kk + tk) * PITCH_TA + (row - ml + tr) * 2));
              av[i].t[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sa + (kk + tk + 4) * PITCH_TA + (row - ml + tr) * 2));
            }
          }
#pragma unroll
          for (int i = 0; i < TN; ++i) {
            const int row = 32 * (wx * TN + i) + ml;
            if (B_KC) {
              bv[i].u = *(const u32x4*)(sb + row * PITCH_KC + (kk + 8 * h) * 2);
            } else {
              bv[i].t[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sb + (kk + tk) * PITCH_TB + (row - ml + tr) * 2));
              bv[i].t[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sb + (kk + tk + 4) * PITCH_TB + (row - ml + tr) * 2));
            }
          }
        };
        auto mm = [&](const Frag (&av)[TM], const Frag (&bv)[TN]) {
#pragma unroll
          for (int im = 0; im < TM; ++im)
#pragma unroll
            for (int in = 0; in < TN; ++in)
              acc[im][in] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[im].v, bv[in].v, acc[im][in], 0, 0, 0);
        };
        Frag av[2][TM], bv[2][TN];
        rd(0, av[0], bv[0]);
        rd(GK, av[1], bv[1]);
        static_for<KG>([&](auto g) __attribute__((always_inline)) {
          constexpr int gv = decltype(g)::value;
          __builtin_amdgcn_sched_barrier(0);
          mm(av[gv & 1], bv[gv & 1]);
          if constexpr (gv + 2 < KG) {
            __builtin_amdgcn_sched_barrier(0);
            rd((gv + 2) * GK, av[gv & 1], bv[gv & 1]);
          }
        });
      }
  };

  if (n > 0) {
    enter_segment();  // segment 0; the first load walks on to the segment that holds stage g_first
    static_for<D>([&](auto d) __attribute__((always_inline)) { load(d, decltype(d)::value < n); });
    stash(0, std::integral_constant<int, 0>{});
    load(std::integral_constant<int, 0>{}, D < n);
    __syncthreads();
    // one stage: multiply it, move stage st + 1 into the other buffer (past the end: zeros nobody reads) and
    // refill that stage's ring slot
    auto stage = [&](int st, auto d) __attribute__((always_inline)) {
      constexpr int next = (decltype(d)::value + 1) % D;
      if constexpr (SB) {  // one LDS buffer: the next stage may only be written when everyone has read this one
        multiply(0);
        __syncthreads();
        stash(0, std::integral_constant<int, next>{});
        load(std::integral_constant<int, next>{}, st + 1 + D < n);
        __syncthreads();
      } else {
        multiply(st & 1);
        stash((st + 1) & 1, std::integral_constant<int, next>{});
        load(std::integral_constant<int, next>{}, st + 1 + D < n);
        __syncthreads();
      }
    };
    int st0 = 0;
    for (; st0 + D <= n; st0 += D)  // whole turns of the ring: no branches, so the waits stay exact
      static_for<D>([&](auto d) __attribute__((always_inline)) { stage(st0 + decltype(d)::value, d); });
    static_for<D - 1>([&](auto d) __attribute__((always_inline)) {
      if (st0 + decltype(d)::value < n) stage(st0 + decltype(d)::value, d);
    });
  }

  // epilogue: D register v of lane (h, ml) of MFMA tile (im, in) is
  //   C[m0 + 32*(wy*TM + im) + 8*(v/4) + 4*h + v%4][n0 + 32*(wx*TN + in) + ml]
  float* pc = nullptr;
  if (gridDim.y > 1) pc = partial + ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * partial_stride;
  if constexpr (BF16) {
    // bf16 results: lane = column in the MFMA layout, so storing from registers is one 2-byte store per element
    // (64 per thread with 128-tiles: measured, that epilogue was 60 % of a weight-gradient workgroup's lifetime).
    // Instead the tile is rounded into LDS (the stage buffers are done with) and written out in 16-byte pieces,
    // 256 contiguous bytes per tile row.
    if (!pc && gb.ldc % 8 == 0 && gb.N % 8 == 0 && ((uintptr_t)gb.c & 15) == 0) {  // uniform
      constexpr int CP = TILE_N * 2 + 16;  // bytes per staged row
      static_assert(TILE_M * CP <= (SB ? 1 : 2) * (A_BYTES + B_BYTES), "output tile must fit the stage buffers");
      __syncthreads();
#pragma unroll
      for (int in = 0; in < TN; ++in) {
        const int cl = 32 * (wx * TN + in) + ml, col = n0 + cl;
        float bias = 0.f;
        if (gb.bias && col < gb.N) bias = __uint_as_float((uint32_t)((const uint16_t*)gb.bias)[col] << 16);
#pragma unroll
        for (int im = 0; im < TM; ++im)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int rl = 32 * (wy * TM + im) + 8 * (v / 4) + 4 * h + (v % 4);
            *(__bf16*)(smem + rl * CP + cl * 2) = (__bf16)(acc[im][in][v] + bias);  // round to nearest even
          }
      }
      __syncthreads();
      constexpr int PPR = TILE_N / 8;  // 16-byte pieces per row
#pragma unroll
      for (int p = tid; p < TILE_M * PPR; p += 256) {
        const int rl = p / PPR, q = p - rl * PPR;
        const int row = m0 + rl, col = n0 + q * 8;
        if (row < gb.M && col < gb.N)
          *(u32x4*)((uint16_t*)gb.c + (size_t)row * gb.ldc + col) = *(const u32x4*)(smem + rl * CP + q * 16);
      }
      return;
    }
  }
#pragma unroll
  for (int in = 0; in < TN; ++in) {
    const int col = n0 + 32 * (wx * TN + in) + ml;
    if (col >= gb.N) continue;
    float bias = 0.f;
    if (!pc && gb.bias)
      bias = BF16 ? __uint_as_float((uint32_t)((const uint16_t*)gb.bias)[col] << 16) : ((const float*)gb.bias)[col];
#pragma unroll
    for (int im = 0; im < TM; ++im) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + 32 * (wy * TM + im) + 8 * (v / 4) + 4 * h + (v % 4);
        if (row >= gb.M) continue;
        if (pc) {  // fp32 partial of this split
          pc[(size_t)row * gb.N + col] = acc[im][in][v];
          continue;
        }
        const float r = acc[im][in][v] + bias;
        if (BF16) ((uint16_t*)gb.c)[(size_t)row * gb.ldc + col] = (uint16_t)f32_to_bf16_rne(r);
        else ((float*)gb.c)[(size_t)row * gb.ldc + col] = r;
      }
    }
  }
}

// C_o = sum over the splits (ascending) of the fp32 partials + bias, rounded to the output type.
// grid: (ceil(max M*N / 4 / 256), blocks); M*N is a multiple of 4 whenever the MFMA path is used.
template <bool BF16>
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const GemmBlock* __restrict__ blocks,
                                                          const float* __restrict__ partial, int64_t partial_stride,
                                                          int nsplit) {
  const GemmBlock& gb = blocks[blockIdx.y];
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;  // group of 4 consecutive elements
  const int64_t e = q * 4;
  if (e >= (int64_t)gb.M * gb.N) return;
  const int row = (int)(e / gb.N), col = (int)(e - (int64_t)row * gb.N);  // N % 4 == 0: a group stays in one row
  const float* pp = partial + (size_t)blockIdx.y * nsplit * partial_stride + e;
  float4 acc = *(const float4*)pp;
  for (int s = 1; s < nsplit; ++s) {
    const float4 t = *(const float4*)(pp + (size_t)s * partial_stride);
    acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
  }
  if (gb.bias) {
    if (BF16) {
      const uint16_t* b = (const uint16_t*)gb.bias + col;
      acc.x += __uint_as_float((uint32_t)b[0] << 16); acc.y += __uint_as_float((uint32_t)b[1] << 16);
      acc.z += __uint_as_float((uint32_t)b[2] << 16); acc.w += __uint_as_float((uint32_t)b[3] << 16);
    } else {
      const float* b = (const float*)gb.bias + col;
      acc.x += b[0]; acc.y += b[1]; acc.z += b[2]; acc.w += b[3];
    }
  }
  if (BF16) {
    uint16_t* c = (uint16_t*)gb.c + (size_t)row * gb.ldc + col;
    c[0] = (uint16_t)f32_to_bf16_rne(acc.x); c[1] = (uint16_t)f32_to_bf16_rne(acc.y);
    c[2] = (uint16_t)f32_to_bf16_rne(acc.z); c[3] = (uint16_t)f32_to_bf16_rne(acc.w);
  } else {
    float* c = (float*)gb.c + (size_t)row * gb.ldc + col;
    c[0] = acc.x; c[1] = acc.y; c[2] = acc.z; c[3] = acc.w;
  }
}

// db_i[f] = sum over the batch of dy_i[n][f]: one block per 16 features, 16 batch lanes each (many small
// blocks: the matrix is short and wide, so the parallelism has to come from the feature axis).
template <bool BF16>
__global__ __launch_bounds__(256) void colsum_kernel(const ColsumBlock* __restrict__ blocks) {
  const ColsumBlock& cb = blocks[blockIdx.y];
  const int fl = threadIdx.x & 15, lanegrp = threadIdx.x >> 4;
  const int f = blockIdx.x * 16 + fl;
  __shared__ float red[16][17];
  float acc = 0.f;
  if (f < cb.n_f && cb.out) {
    float part[4] = {0.f, 0.f, 0.f, 0.f};
    int n = lanegrp;
    for (; n + 48 < cb.n_b; n += 64)
#pragma unroll
      for (int u = 0; u < 4; ++u)
        part[u] += BF16 ? __uint_as_float((uint32_t)((const uint16_t*)cb.in)[(size_t)(n + 16 * u) * cb.n_f + f] << 16)
                        : ((const float*)cb.in)[(size_t)(n + 16 * u) * cb.n_f + f];
    for (; n < cb.n_b; n += 16)
      part[0] += BF16 ? __uint_as_float((uint32_t)((const uint16_t*)cb.in)[(size_t)n * cb.n_f + f] << 16)
                      : ((const float*)cb.in)[(size_t)n * cb.n_f + f];
    acc = (part[0] + part[1]) + (part[2] + part[3]);
  }
  red[lanegrp][fl] = acc;
  __syncthreads();
  if (lanegrp == 0 && f < cb.n_f && cb.out) {
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) s += red[g][fl];
    if (BF16) ((uint16_t*)cb.out)[f] = (uint16_t)f32_to_bf16_rne(s);
    else ((float*)cb.out)[f] = s;
  }
}

// ---- host side ------------------------------------------------------------------

bool gemm_mfma_usable(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc) {
  const int ve = bf16 ? 8 : 4;
  const size_t es = bf16 ? 2 : 4;
  if (!a_kc && b_kc) return false;  // not a layout of the affine layer: not built
  for (const GemmBlock& b : blocks) {
    if (b.nseg < 1 || b.nseg > kGemmMaxSeg) return false;
    if ((uintptr_t)b.c % es) return false;
    for (int s = 0; s < b.nseg; ++s) {
      const GemmSeg& g = b.seg[s];
      // 16-byte pieces: aligned bases, leading dimensions and contiguous extents that are multiples of a piece
      if ((uintptr_t)g.a % 16 || (uintptr_t)g.b % 16 || g.lda % ve || g.ldb % ve) return false;
      if ((a_kc || b_kc) && g.K % ve) return false;
      if (!a_kc && b.M % ve) return false;
      if (!b_kc && b.N % ve) return false;
      const double a_bytes = (double)(a_kc ? b.M : g.K) * g.lda * es, b_bytes = (double)(b_kc ? b.N : g.K) * g.ldb * es;
      if (a_bytes >= 2147480000.0 || b_bytes >= 2147480000.0) return false;
    }
  }
  return true;
}

static int64_t count_tiles(const std::vector<GemmBlock>& blocks, int t) {
  int64_t tiles = 0;
  for (const GemmBlock& b : blocks) tiles += (int64_t)((b.M + t - 1) / t) * ((b.N + t - 1) / t);
  return tiles;
}

// Workgroup tile: 128 x 128 (2 x 2 MFMA tiles per wave) when every block is at least that large.  Exception: a
// launch whose 128-tiles would fill at most half the chip but whose 64-tiles fill most of it (the small-batch
// forward and data-gradient products) takes 64 x 64 tiles over the whole K range on the streaming kernel (bf16 in
// any layout it was measured in, fp32 where that kernel exists: A contiguous along K): no partial tiles, no
// second kernel.
static int gemm_tile(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc) {
  for (const GemmBlock& b : blocks)
    if (b.M < 128 || b.N < 128) return 64;
  if (blocks.empty()) return 64;
  if ((bf16 || a_kc) && count_tiles(blocks, 128) <= 128 && count_tiles(blocks, 64) >= 192) return 64;
  return 128;
}

// Number of K splits for a launch: enough workgroups for about two (large tiles) or four per compute unit,
// every split at least four stages long, at most 8.
int gemm_mfma_splits(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc) {
  const int bk = bf16 ? 64 : 32;
  const int t = gemm_tile(blocks, bf16, a_kc);
  const int64_t tiles = count_tiles(blocks, t);
  int64_t macs = 0;
  int min_stages = INT32_MAX;
  for (const GemmBlock& b : blocks) {
    int stages = 0;
    for (int s = 0; s < b.nseg; ++s) {
      stages += (b.seg[s].K + bk - 1) / bk;
      macs += (int64_t)b.M * b.N * b.seg[s].K;
    }
    min_stages = std::min(min_stages, stages);
    if (b.N % 4) return 1;  // the reduction works on groups of 4 elements of a row
  }
  if ((bf16 || a_kc) && t == 64 && tiles >= 192) return 1;  // the whole K range per tile: see gemm_tile
  const int64_t target = t == 128 ? 512 : 1024;
  if (tiles == 0 || tiles >= target * 3 / 4) return 1;
  if (macs < (int64_t(1) << 28)) return 1;  // a launch this small is latency-bound either way: no second kernel
  int64_t want = (target + tiles - 1) / tiles;
  want = std::min<int64_t>(want, std::max(1, min_stages / 4));
  return (int)std::max<int64_t>(1, std::min<int64_t>(want, 8));
}

size_t gemm_mfma_partial_floats(const std::vector<GemmBlock>& blocks, int nsplit) {
  if (nsplit <= 1) return 0;
  int64_t mx = 0;
  for (const GemmBlock& b : blocks) mx = std::max<int64_t>(mx, (int64_t)b.M * b.N);
  return (size_t)mx * nsplit * blocks.size();
}

// T: workgroup tile / 64; the 64-tiles load two stages ahead (one workgroup per compute unit has nothing else
// to cover a stage's latency with), the 128-tiles one.
template <bool BF16, bool A_KC, bool B_KC, int T>
static int launch_gemm_variant(dim3 grid, const GemmBlock* d_blocks, float* partial, int64_t max_mn, hipStream_t st) {
  constexpr int ES = BF16 ? 2 : 4, BK = BF16 ? 64 : 32, TILE = 64 * T, D = T == 1 ? 2 : 1;
  constexpr int A_BYTES = A_KC ? TILE * (BK * ES + 16) : BK * (TILE * ES + (BF16 ? 32 : 16));
  constexpr int B_BYTES = B_KC ? TILE * (BK * ES + 16) : BK * (TILE * ES + (BF16 ? 32 : 16));
  // The weight-gradient layout (both operands with their rows contiguous: short K loops, many tiles) keeps one LDS
  // buffer and pays a second barrier per stage: a third workgroup then fits a compute unit, which is worth 4-5 %
  // there; the forward and data-gradient layouts lose 1-3 % that way and keep two buffers.
  constexpr bool SB = !A_KC && !B_KC;
  constexpr int LDS = (SB ? 1 : 2) * (A_BYTES + B_BYTES);
  if (LDS > 64 * 1024)
    if (int rc = allow_large_lds<gemm_mfma_kernel<BF16, A_KC, B_KC, T, T, D, SB>>()) return rc;
  hipLaunchKernelGGL((gemm_mfma_kernel<BF16, A_KC, B_KC, T, T, D, SB>), grid, dim3(256), LDS, st, d_blocks, partial, max_mn);
  return DISTDL_OK;
}

int launch_gemm_mfma(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc,
                     int nsplit, float* partial, const char* name, hipStream_t st, GemmColsum* colsum) {
  const int t = gemm_tile(blocks, bf16, a_kc);
  int tiles = 0;
  int64_t max_mn = 0;
  for (const GemmBlock& b : blocks) {
    tiles = std::max(tiles, ((b.M + t - 1) / t) * ((b.N + t - 1) / t));
    max_mn = std::max<int64_t>(max_mn, (int64_t)b.M * b.N);
  }
  tiles = (tiles + 7) / 8 * 8;
  if (nsplit > 1 && !partial) return set_error(DISTDL_ERR_INVALID_ARG, "gemm: split launch without a partial buffer");
  if (!a_kc && b_kc) return set_error(DISTDL_ERR_UNSUPPORTED, "gemm: operand layout not built");
  dim3 grid((unsigned)tiles, (unsigned)std::max(nsplit, 1), (unsigned)blocks.size()), block(256);
  ProfScope prof(name, st);
  // launches that take 64-tiles over the whole K range (about one tile per compute unit: the small-batch forward
  // and data-gradient products) run on the streaming kernel
  if (t == 64 && nsplit <= 1 && a_kc && gemm_stream_usable(blocks, bf16, a_kc, b_kc)) return launch_gemm_stream(d_blocks, blocks, bf16, b_kc, st);
  if (t == 128 && nsplit <= 1 && !a_kc && !b_kc && gemm_stream_usable(blocks, bf16, a_kc, b_kc)) {
    if (colsum) colsum->done = true;  // M is a multiple of a piece for every block: the feature counts fit the fused column sums
    return launch_gemm_stream_tt(d_blocks, blocks, bf16, colsum ? colsum->d_blocks : nullptr,
                                 colsum ? colsum->n_blocks : 0, colsum ? colsum->max_f : 0, st);
  }
  int rc;
#define DISTDL_GEMM(BF_, A_, B_)                                                                \
  rc = t == 128 ? launch_gemm_variant<BF_, A_, B_, 2>(grid, d_blocks, partial, max_mn, st)      \
                : launch_gemm_variant<BF_, A_, B_, 1>(grid, d_blocks, partial, max_mn, st)
  // the three operand layouts of the affine layer: forward (K, K), data gradient (K, N), weight gradient (M, N)
  if (!bf16) {
    if (a_kc && b_kc) DISTDL_GEMM(false, true, true);
    else if (a_kc) DISTDL_GEMM(false, true, false);
    else DISTDL_GEMM(false, false, false);
  } else {
    if (a_kc && b_kc) DISTDL_GEMM(true, true, true);
    else if (a_kc) DISTDL_GEMM(true, true, false);
    else DISTDL_GEMM(true, false, false);
  }
#undef DISTDL_GEMM
  if (rc) return rc;
  if (nsplit > 1) {
    dim3 rgrid((unsigned)((max_mn / 4 + 255) / 256), (unsigned)blocks.size());
    if (bf16) hipLaunchKernelGGL(gemm_reduce_kernel<true>, rgrid, block, 0, st, d_blocks, partial, max_mn, nsplit);
    else hipLaunchKernelGGL(gemm_reduce_kernel<false>, rgrid, block, 0, st, d_blocks, partial, max_mn, nsplit);
  }
  return DISTDL_OK;
}

int launch_colsum(const ColsumBlock* d_blocks, int nblocks, int max_f, bool bf16, hipStream_t st) {
  dim3 grid((unsigned)((max_f + 15) / 16), (unsigned)nblocks), block(256);
  ProfScope prof("affine_bias_grad", st);
  if (bf16) hipLaunchKernelGGL(colsum_kernel<true>, grid, block, 0, st, d_blocks);
  else hipLaunchKernelGGL(colsum_kernel<false>, grid, block, 0, st, d_blocks);
  return DISTDL_OK;
}

}  // namespace distdl
