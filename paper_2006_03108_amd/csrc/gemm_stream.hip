// bf16 GEMM for the small-batch products of the partitioned affine layer (Sec. 4 "Dense layers": forward
// y_i = sum_j x_j W_ij^T + b_i and the data gradient dx_j = sum_i dy_i W_ij), where a launch has about one 64 x 64
// output tile per compute unit and the time goes into feeding the operands, not into the matrix cores.
//
// Measured on this chip: a compute unit takes in about 45 bytes per clock from L2 whatever the landing place
// (registers or LDS, 4 or 8 waves), a tile of 64 x 64 over K = 4096 needs 1 MB, and a workgroup whose waves meet at
// a barrier every 64 k spends its time in the chain load -> ds_write -> barrier -> ds_read -> MFMA instead: with one
// wave per SIMD nothing else fills the waits, and ds_write_b128 issues at ~59 clocks per wave.  So here
//   * every wave is a pipeline of its own: wave w multiplies the 64-k steps w, w + 4, ... of the whole tile
//     (2 x 2 MFMA tiles, four independent accumulators) out of a wave-private LDS area; there is no workgroup
//     barrier in the K loop, and the four partial tiles are summed through LDS at the end, in wave order;
//   * operands go from global memory straight into LDS (buffer_load_dwordx4 ... lds): no staging registers, no
//     ds_write; about 15.7 us against 19 us through registers for 256 x 4096 x 4096.  Lane L of such a load lands at (LDS base in M0) + 16 L and an out-of-range lane writes zeros
//     (both measured); which 16 bytes a lane fetches is free, so the bank-conflict-free placement is made by
//     permuting the pieces of a row on the global side:
//       K-contiguous operand (A; B of the forward product): block = 64 rows x 128 bytes, row R keeps its piece c
//         (8 k) at position c ^ ((R >> 1) & 7): the 16 lanes of a fragment read (16 rows, one piece) fall into 16
//         different 16-byte bank groups;
//       N-contiguous operand (B of the data gradient, W as it lies in memory): block = 64 k lines x 128 bytes
//         (64 n), line l keeps piece c (8 n) at position c ^ (4 * ((l >> 1) & 1)) and is read with the
//         transposing load ds_read_b64_tr_b16 (lane layout stated in gemm_mfma.hip): the four lines a half-wave
//         reads then cover each bank once.
// The sum over the partition axis (the layer's sum-reduce R) is the continuation of the K loop over the
// segments of a block, as in gemm_mfma.hip.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "gemm_mfma.h"
#include "lds_direct.h"
#include "profile.h"

namespace distdl {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16* lds_v4;

namespace {

constexpr uint32_t kOobOff = 0x7ffffff0u;  // fails the range check of every buffer (operands are < 2 GiB)
constexpr int kOperandBytes = 64 * 128;    // one operand block of a step
constexpr int kStepBytes = 2 * kOperandBytes;
constexpr int kWaveBytes = 2 * kStepBytes;  // two steps per wave: one multiplied, one landing
constexpr int kStreamLds = 4 * kWaveBytes;  // 128 KB

// f(integral_constant<int, 0>) ... f(integral_constant<int, 3>)
template <class F>
__device__ __forceinline__ void static_for4(F&& f) {
  f(std::integral_constant<int, 0>{});
  f(std::integral_constant<int, 1>{});
  f(std::integral_constant<int, 2>{});
  f(std::integral_constant<int, 3>{});
}

union Frag {
  u32x4 u;
  bf16x8 v;
  v4i16 t[2];
};

}  // namespace

// BF16: bf16 operands and output (v_mfma_f32_32x32x16_bf16, 64 k per step), else fp32 (v_mfma_f32_32x32x2_f32, 32 k
// per step; a 16-byte fragment read gives a lane four consecutive k, used by four MFMAs whose k pairs are (j, 4 + j),
// the same pairing on both operands).  Either way a staged row of a K-contiguous operand is 128 bytes (8 pieces),
// so the staging geometry and its swizzle are the same.  An N-contiguous fp32 B is staged as 32 k lines x 256 bytes
// (64 columns), line l keeping piece c at position c ^ (8 * ((l >> 2) & 1)), and read one float per lane: the 32
// lanes of a half-wave read 128 contiguous bytes, and the two half-waves (lines l, l + 4) different bank halves.
template <bool BF16, bool B_KC>
__global__ __launch_bounds__(256, 1) void gemm_stream_kernel(const GemmBlock* __restrict__ blocks) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int ES = BF16 ? 2 : 4;        // element size
  constexpr int VE = 16 / ES;             // elements per 16-byte piece
  constexpr int SK = BF16 ? 64 : 32;      // k per step: 128 bytes of a K-contiguous row
  const GemmBlock& gb = blocks[blockIdx.z];
  const int tiles_m = (gb.M + 63) / 64, tiles_n = (gb.N + 63) / 64;
  // consecutive tiles share the B rows (m walks fastest) and stay behind one L2
  const int tile = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (tile >= tiles_m * tiles_n) return;
  const int tm = tile % tiles_m, tn = tile / tiles_m;
  const int m0 = tm * 64, n0 = tn * 64;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ml = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // known uniform: keeps everything derived from it scalar
  char* const my = smem + wave * kWaveBytes;
  const uint32_t my_lds = lds_address(my);

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // The steps of all segments form one sequence; this wave takes every fourth of them.
  int total = 0;
  for (int s = 0; s < gb.nseg; ++s) total += (gb.seg[s].K + SK - 1) / SK;
  const int n = (total - wave + 3) / 4;

  // load cursor: segment, step within it (may run past the end: such steps are issued out of range and never read)
  int ls = 0, lin = wave, l_nst = 0, l_K = 0;
  uint32_t l_ldb = 0;
  u32x4 ra = lds_direct_rsrc(nullptr, 0), rb = lds_direct_rsrc(nullptr, 0);
  uint32_t goff[16];
  // K-contiguous operand, load i: row 8 i + lane / 8, position lane % 8.  N-contiguous bf16 B: the same with k
  // lines for rows; N-contiguous fp32 B: k line 4 i + lane / 16, position lane % 16.
  auto enter_segment = [&]() __attribute__((always_inline)) {
    const GemmSeg& sg = gb.seg[ls];
    l_K = sg.K;
    l_nst = (sg.K + SK - 1) / SK;
    l_ldb = (uint32_t)sg.ldb;
    // the resources end with the operand: rows beyond M / N and k lines beyond K read as zero
    ra = lds_direct_rsrc(sg.a, (uint32_t)gb.M * sg.lda * ES);
    rb = lds_direct_rsrc(sg.b, (uint32_t)(B_KC ? gb.N : sg.K) * sg.ldb * ES);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 8 * i + (lane >> 3);
      const int ca = (lane & 7) ^ ((r >> 1) & 7);
      goff[i] = ((uint32_t)(m0 + r) * sg.lda + ca * VE) * ES;
      if (B_KC) {
        goff[8 + i] = ((uint32_t)(n0 + r) * sg.ldb + ca * VE) * ES;
      } else if (BF16) {
        const int cb = (lane & 7) ^ (4 * ((r >> 1) & 1));
        goff[8 + i] = ((uint32_t)r * sg.ldb + n0 + cb * VE) * ES;
        if (n0 + cb * VE >= gb.N) goff[8 + i] = kOobOff;  // columns beyond N (whole pieces: N % 8 == 0)
      } else {
        const int l = 4 * i + (lane >> 4);
        const int cb = (lane & 15) ^ (8 * ((l >> 2) & 1));
        goff[8 + i] = ((uint32_t)l * sg.ldb + n0 + cb * VE) * ES;
        if (n0 + cb * VE >= gb.N) goff[8 + i] = kOobOff;  // whole pieces: N % 4 == 0
      }
    }
  };
  // The loads of the cursor's step into staging buffer `buf`: issue_begin moves the cursor on by four steps and
  // fixes the step's offsets, issue_part(q) issues loads 4 q ... 4 q + 3 of its 16 (A: 0-7, B: 8-15), so that the
  // fp32 loop can spread them between its MFMAs; issue does it all at once.
  uint32_t is_d = 0, is_a = 0, is_b = 0;
  int is_kleft = 0;
  bool is_tail = false;
  auto issue_begin = [&](int buf, bool valid) __attribute__((always_inline)) {
    is_d = my_lds + buf * kStepBytes;
    int k0 = 0;
    if (valid) {  // wave-uniform
      while (lin >= l_nst) {
        lin -= l_nst;
        ++ls;
        enter_segment();
      }
      k0 = lin * SK;
      lin += 4;
    }
    // (a step past the end is switched off through the scalar part of the offset, which the range check includes:
    // no per-lane select on the path of the loads)
    is_a = valid ? (uint32_t)k0 * ES : kOobOff;
    is_b = valid ? (uint32_t)k0 * (B_KC ? 1u : l_ldb) * ES : kOobOff;
    // K tail: pieces of a K-contiguous row beyond K are switched off (whole pieces: K % VE == 0); k lines beyond
    // K lie beyond the resource
    is_tail = valid && k0 + SK > l_K;
    is_kleft = l_K - k0;
  };
  auto issue_part = [&](auto q_c) __attribute__((always_inline)) {
    constexpr int q = decltype(q_c)::value;
    constexpr bool kc_op = q < 2 || B_KC;  // loads of a K-contiguous operand
    if (kc_op && is_tail) {               // (uniform: the last step of a segment; the piece test is per lane)
#pragma unroll
      for (int i = 4 * q; i < 4 * q + 4; ++i) {
        const int r = 8 * (i & 7) + (lane >> 3);
        const int ca = (lane & 7) ^ ((r >> 1) & 7);
        const uint32_t off = ca * VE >= is_kleft ? kOobOff : goff[i];
        if (i < 8) load_to_lds(ra, is_d + i * 1024, off, is_a);
        else load_to_lds(rb, is_d + kOperandBytes + (i - 8) * 1024, off, is_b);
      }
    } else {
#pragma unroll
      for (int i = 4 * q; i < 4 * q + 4; ++i) {
        if (i < 8) load_to_lds(ra, is_d + i * 1024, goff[i], is_a);
        else load_to_lds(rb, is_d + kOperandBytes + (i - 8) * 1024, goff[i], is_b);
      }
    }
  };
  // loads 2 k and 2 k + 1 of the step; TAIL (compile time) says whether the K-tail select is needed at all
  auto issue_pair = [&](auto k_c, auto tail_c) __attribute__((always_inline)) {
    constexpr int k = decltype(k_c)::value;
    constexpr bool TAIL = decltype(tail_c)::value && (k < 4 || B_KC);
#pragma unroll
    for (int i = 2 * k; i < 2 * k + 2; ++i) {
      uint32_t off = goff[i];
      if constexpr (TAIL) {
        const int r = 8 * (i & 7) + (lane >> 3);
        const int ca = (lane & 7) ^ ((r >> 1) & 7);
        if (ca * VE >= is_kleft) off = kOobOff;
      }
      if (i < 8) load_to_lds(ra, is_d + i * 1024, off, is_a);
      else load_to_lds(rb, is_d + kOperandBytes + (i - 8) * 1024, off, is_b);
    }
  };
  auto issue = [&](int buf, bool valid) __attribute__((always_inline)) {
    issue_begin(buf, valid);
    static_for4([&](auto q) __attribute__((always_inline)) { issue_part(q); });
  };

  // fragment addresses inside a staging buffer
  //   A (and B when K-contiguous): row 32 t + ml, piece 2 g + h of the step, at position piece ^ key(row)
  uint32_t rdk[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) rdk[g] = ml * 128 + (((2 * g + h) ^ ((ml >> 1) & 7)) * 16);
  //   bf16 B when N-contiguous: k line 16 g + tk (+ 4), columns 32 t + tr ... + 3 (8 bytes) at piece (4 t + tr / 8) ^ f(line)
  const int tk = 8 * (lane >> 5) + ((lane & 15) >> 2), tr = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  uint32_t rdt[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    rdt[t] = kOperandBytes + tk * 128 + ((((4 * t + (tr >> 3)) ^ (4 * ((tk >> 1) & 1)))) * 16) + (tr & 7) * 2;
  //   fp32 B when N-contiguous: k line 8 g + 4 h + j, column 32 t + ml: one float of piece (8 t + ml / 4) ^ (8 h)
  uint32_t rdn[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    rdn[t] = kOperandBytes + 4 * h * 256 + (((8 * t + (ml >> 2)) ^ (8 * h)) * 16) + (ml & 3) * 4;

  // fragments of k groups g0, g0 + 1 of the step in buffer buf.  fp32: fa / fb hold four k per lane; an N-contiguous
  // fp32 B is read float by float into the same four slots.
  auto read_half = [&](int buf, int g0, Frag (&fa)[2][2], Frag (&fb)[2][2]) __attribute__((always_inline)) {
    const char* s = my + buf * kStepBytes;
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[g][t].u = *(const u32x4*)(s + rdk[g0 + g] + t * 4096);
        if constexpr (B_KC) {
          fb[g][t].u = *(const u32x4*)(s + kOperandBytes + rdk[g0 + g] + t * 4096);
        } else if constexpr (BF16) {
          fb[g][t].t[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + rdt[t] + (g0 + g) * 16 * 128));
          fb[g][t].t[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + rdt[t] + (g0 + g) * 16 * 128 + 4 * 128));
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) fb[g][t].u[j] = *(const uint32_t*)(s + rdn[t] + ((g0 + g) * 8 + j) * 256);
        }
      }
  };
  // accumulated transposed (B fragment as the first MFMA operand): see the epilogue
  auto mm_half = [&](const Frag (&fa)[2][2], const Frag (&fb)[2][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      if constexpr (BF16) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[g][j].v, fa[g][i].v, acc[i][j], 0, 0, 0);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fb[g][j].u[e]), __uint_as_float(fa[g][i].u[e]),
                                                               acc[i][j], 0, 0, 0);
      }
    }
  };

  if (n > 0) {
    enter_segment();
    issue(0, true);
    issue(1, 1 < n);
    if constexpr (BF16) {
      Frag xa[2][2], xb[2][2], ya[2][2], yb[2][2];
      // One step: its 16 loads have landed when at most the 16 of the next step are outstanding.  The buffer is
      // handed to the loads of the step after next as soon as every fragment of it is in registers.
      auto step = [&](int st, int buf) __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt16);
        __builtin_amdgcn_sched_barrier(0);
        read_half(buf, 0, xa, xb);
        read_half(buf, 2, ya, yb);
        __builtin_amdgcn_sched_barrier(0);
        mm_half(xa, xb);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWaitLgkmcnt0);
        issue(buf, st + 2 < n);
        __builtin_amdgcn_sched_barrier(0);
        mm_half(ya, yb);
        __builtin_amdgcn_sched_barrier(0);
      };
      int st = 0;
      for (; st + 2 <= n; st += 2) {
        step(st, 0);
        step(st + 1, 1);
      }
      if (st < n) step(st, 0);
    } else {
      // fp32: a step is 64 MFMAs of 64 clocks and this wave is alone on its SIMD (512 registers), so the pipeline is
      // one step deeper in registers and everything else is issued in the shadow of the MFMAs, in 16 slots, one
      // after every four of them.  While step s multiplies out of one register set, the fragments of step s + 1 are
      // read from the other staging buffer into the other set (its loads were issued during step s - 2: at most the
      // 16 of step s + 2 are outstanding when they have landed), and when those reads are done the buffer takes the
      // loads of step s + 3.  Every load has more than a step to land and every LDS read a step before its use.
      Frag pa[4][2], pb[4][2], qa[4][2], qb[4][2];
      auto rd_a = [&](int buf, int g, Frag (&fa)[4][2]) __attribute__((always_inline)) {
        const char* s = my + buf * kStepBytes;
#pragma unroll
        for (int t = 0; t < 2; ++t) fa[g][t].u = *(const u32x4*)(s + rdk[g] + t * 4096);
      };
      auto rd_b = [&](int buf, int g, Frag (&fb)[4][2]) __attribute__((always_inline)) {
        const char* s = my + buf * kStepBytes;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          if constexpr (B_KC) {
            fb[g][t].u = *(const u32x4*)(s + kOperandBytes + rdk[g] + t * 4096);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) fb[g][t].u[j] = *(const uint32_t*)(s + rdn[t] + (g * 8 + j) * 256);
          }
        }
      };
      auto mm4 = [&](const Frag (&fa)[4][2], const Frag (&fb)[4][2], int g, int e) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fb[g][j].u[e]), __uint_as_float(fa[g][i].u[e]),
                                                             acc[i][j], 0, 0, 0);
      };
      __builtin_amdgcn_s_waitcnt(kWaitVmcnt16);  // step 0 has landed
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        rd_a(0, g, pa);
        rd_b(0, g, pb);
      }
      __builtin_amdgcn_s_waitcnt(kWaitLgkmcnt0);
      issue(0, 2 < n);
      // step st out of (ca, cb), whose buffer is buf; (na, nb) take step st + 1.  Slots: 0 waits for the loads of
      // step st + 1, 1 - 4 read its fragments, 6 - 13 issue two loads each.  The wave has about 60 clocks per slot
      // before the matrix pipe runs dry, and a taken branch costs a good part of that, so the one decision of the
      // step (does its load have a K tail) is taken once, in front of two copies of the body.
      auto body = [&](int buf, const Frag (&ca)[4][2], const Frag (&cb)[4][2], Frag (&na)[4][2], Frag (&nb)[4][2],
                      auto tail_c) __attribute__((always_inline)) {
#pragma unroll
        for (int slot = 0; slot < 16; ++slot) {
          mm4(ca, cb, slot >> 2, slot & 3);
          __builtin_amdgcn_sched_barrier(0);
          if (slot == 0) __builtin_amdgcn_s_waitcnt(kWaitVmcnt16);
          if (slot >= 1 && slot <= 4) {
            rd_a(buf ^ 1, slot - 1, na);
            rd_b(buf ^ 1, slot - 1, nb);
          }
          if (slot == 6) __builtin_amdgcn_s_waitcnt(kWaitLgkmcnt0);
          if (slot == 6) issue_pair(std::integral_constant<int, 0>{}, tail_c);
          if (slot == 7) issue_pair(std::integral_constant<int, 1>{}, tail_c);
          if (slot == 8) issue_pair(std::integral_constant<int, 2>{}, tail_c);
          if (slot == 9) issue_pair(std::integral_constant<int, 3>{}, tail_c);
          if (slot == 10) issue_pair(std::integral_constant<int, 4>{}, tail_c);
          if (slot == 11) issue_pair(std::integral_constant<int, 5>{}, tail_c);
          if (slot == 12) issue_pair(std::integral_constant<int, 6>{}, tail_c);
          if (slot == 13) issue_pair(std::integral_constant<int, 7>{}, tail_c);
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      auto step = [&](int st, int buf, const Frag (&ca)[4][2], const Frag (&cb)[4][2], Frag (&na)[4][2],
                      Frag (&nb)[4][2]) __attribute__((always_inline)) {
        issue_begin(buf ^ 1, st + 3 < n);  // (scalars only; the loads follow in the body)
        if (is_tail) body(buf, ca, cb, na, nb, std::true_type{});
        else body(buf, ca, cb, na, nb, std::false_type{});
      };
      int st = 0;
      for (; st + 2 <= n; st += 2) {
        step(st, 0, pa, pb, qa, qb);
        step(st + 1, 1, qa, qb, pa, pb);
      }
      if (st < n) step(st, 0, pa, pb, qa, qb);
    }
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // nothing may still land in LDS when the epilogue reuses it
  }

  // Sum of the four waves' partial tiles in wave order, bias, rounding, store.  The products were accumulated
  // transposed (B fragment as the first MFMA operand): register v of lane (h, ml) of tile (i, j) is
  // C[32 i + ml][32 j + 8 (v / 4) + 4 h + v % 4], four consecutive columns per register quad, so a partial tile goes
  // to LDS in 16-byte writes.  Row m keeps its float4 number s at position s ^ (m & 15): 16 lanes, 16 bank groups.
  __syncthreads();
  float4* red = (float4*)smem;  // [wave][64 rows][16 float4]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int m = 32 * i + ml, s4 = 8 * j + 2 * q + h;
        red[(wave * 64 + m) * 16 + (s4 ^ (m & 15))] =
            float4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
      }
  __syncthreads();
  const int row = tid >> 2, c0 = (tid & 3) * 16;
  float s[16];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int slot = ((c0 >> 2) + q) ^ (row & 15);
    float4 t = red[row * 16 + slot];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float4 u = red[(w * 64 + row) * 16 + slot];
      t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
    }
    s[4 * q] = t.x; s[4 * q + 1] = t.y; s[4 * q + 2] = t.z; s[4 * q + 3] = t.w;
  }
  const int grow = m0 + row, gcol = n0 + c0;
  if (grow >= gb.M || gcol >= gb.N) return;
  const bool full = gcol + 16 <= gb.N;
  if (gb.bias) {
    if constexpr (BF16) {
      const uint16_t* bp = (const uint16_t*)gb.bias + gcol;
      if (full) {
#pragma unroll
        for (int q = 0; q < 16; ++q) s[q] += __uint_as_float((uint32_t)bp[q] << 16);
      } else {
        for (int q = 0; gcol + q < gb.N; ++q) s[q] += __uint_as_float((uint32_t)bp[q] << 16);
      }
    } else {
      const float* bp = (const float*)gb.bias + gcol;
      if (full) {
#pragma unroll
        for (int q = 0; q < 16; ++q) s[q] += bp[q];
      } else {
        for (int q = 0; gcol + q < gb.N; ++q) s[q] += bp[q];
      }
    }
  }
  if constexpr (BF16) {
    union {
      __bf16 b[16];
      uint16_t h16[16];
      u32x4 u[2];
    } o;
#pragma unroll
    for (int q = 0; q < 16; ++q) o.b[q] = (__bf16)s[q];  // round to nearest even
    uint16_t* dst = (uint16_t*)gb.c + (size_t)grow * gb.ldc + gcol;
    if (full && gb.ldc % 8 == 0 && ((uintptr_t)gb.c & 15) == 0) {
      ((u32x4*)dst)[0] = o.u[0];
      ((u32x4*)dst)[1] = o.u[1];
    } else {
#pragma unroll
      for (int q = 0; q < 16; ++q)
        if (gcol + q < gb.N) dst[q] = o.h16[q];
    }
  } else {
    float* dst = (float*)gb.c + (size_t)grow * gb.ldc + gcol;
    if (full && gb.ldc % 4 == 0 && ((uintptr_t)gb.c & 15) == 0) {
#pragma unroll
      for (int q = 0; q < 4; ++q) ((float4*)dst)[q] = float4{s[4 * q], s[4 * q + 1], s[4 * q + 2], s[4 * q + 3]};
    } else {
#pragma unroll
      for (int q = 0; q < 16; ++q)
        if (gcol + q < gb.N) dst[q] = s[q];
    }
  }
}

// The weight gradient dW_ij = dy_i^T x_j (Sec. 4, adjoint affine algorithm): both operands lie in memory as k lines
// (k = sample; A[m][k] at a[k lda + m], B[k][n] at b[k ldb + n]), K is the batch (short), the output is large.
// Workgroup tile 128 x 128, four waves of 64 x 64 (2 x 2 MFMA tiles), 32-k steps.  With K = 256 a workgroup's life is
// mostly the latency of its loads and its epilogue, so what matters is how many workgroups a compute unit holds and
// that a step's loads fly while the step before is multiplied: two staging buffers of 16 KB (filled by
// global -> LDS loads, each wave fetching a quarter of a step) and at most 128 registers let four workgroups share a
// compute unit.  A staged block is 32 k lines x 256 bytes (128 rows); line l keeps its 16-byte piece c at position
// c ^ (4 * (l & 3)): the four lines a half-wave's transposing read touches (64 bytes each) then cover the 64 banks once.
// fp32: steps of 16 k (a block is 16 lines x 512 bytes), 32x32x2 MFMAs whose operand is one float per lane
// (row lane % 32 of k line 2 p + lane / 32 for k pair p): a half-wave reads 128 consecutive bytes of its line, and
// odd lines keep piece c at c ^ 8, so that the two half-waves use different halves of the banks.
namespace {
constexpr int kTtOperand = 8192;         // one operand block of a step: 32 (bf16) or 16 (fp32) k lines of 128 elements
constexpr int kTtStep = 2 * kTtOperand;  // 16 KB
constexpr int kTtLds = 2 * kTtStep;      // 32 KB
}  // namespace

// The first cs_wgs workgroups of the grid's z = 0 slice do not multiply: they are the layer's bias gradient
// db_i[f] = sum over the batch of dy_i[n][f] (R over the samples; one chunk of 256 features of one block each, a lane
// sums 4 features over every fourth row, the four waves are added in wave order), which rides along in this launch
// instead of costing one of its own: dy is the A operand here, so it is in L2 anyway.
template <bool BF16>
__global__ __launch_bounds__(256, 4) void gemm_stream_tt_kernel(const GemmBlock* __restrict__ blocks,
                                                                const ColsumBlock* __restrict__ cs, int n_cs,
                                                                int cs_chunks, int cs_wgs) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  if ((int)blockIdx.x < cs_wgs) {
    if (blockIdx.z != 0) return;
    const int b = blockIdx.x / cs_chunks, ch = blockIdx.x - b * cs_chunks;
    if (b >= n_cs) return;
    const ColsumBlock cb = cs[b];
    if (!cb.out) return;
    const int lane_ = threadIdx.x & 63, wave_ = threadIdx.x >> 6;
    const int f0 = ch * 256 + lane_ * 4;
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (!BF16) {
      if (f0 < cb.n_f) {  // whole groups of 4 features: n_f % 4 == 0 is a condition of this kernel
        const float* in = (const float*)cb.in + f0;
        int n = wave_;
        for (; n + 28 < cb.n_b; n += 32) {
          float4 v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) v[u] = *(const float4*)(in + (size_t)(n + 4 * u) * cb.n_f);
#pragma unroll
          for (int u = 0; u < 8; ++u) sum[0] += v[u].x, sum[1] += v[u].y, sum[2] += v[u].z, sum[3] += v[u].w;
        }
        for (; n < cb.n_b; n += 4) {
          const float4 v = *(const float4*)(in + (size_t)n * cb.n_f);
          sum[0] += v.x, sum[1] += v.y, sum[2] += v.z, sum[3] += v.w;
        }
      }
    } else if (f0 < cb.n_f) {  // whole groups of 4 features: n_f % 8 == 0 is a condition of this kernel
      const uint16_t* in = (const uint16_t*)cb.in + f0;
      int n = wave_;
      for (; n + 28 < cb.n_b; n += 32) {
        uint2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *(const uint2*)(in + (size_t)(n + 4 * u) * cb.n_f);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          sum[0] += __uint_as_float(v[u].x << 16); sum[1] += __uint_as_float(v[u].x & 0xffff0000u);
          sum[2] += __uint_as_float(v[u].y << 16); sum[3] += __uint_as_float(v[u].y & 0xffff0000u);
        }
      }
      for (; n < cb.n_b; n += 4) {
        const uint2 v = *(const uint2*)(in + (size_t)n * cb.n_f);
        sum[0] += __uint_as_float(v.x << 16); sum[1] += __uint_as_float(v.x & 0xffff0000u);
        sum[2] += __uint_as_float(v.y << 16); sum[3] += __uint_as_float(v.y & 0xffff0000u);
      }
    }
    float4* red = (float4*)smem;
    red[wave_ * 64 + lane_] = float4{sum[0], sum[1], sum[2], sum[3]};
    __syncthreads();
    if (wave_ == 0 && f0 < cb.n_f) {
      float4 t = red[lane_];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float4 u = red[w * 64 + lane_];
        t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
      }
      if constexpr (BF16) {
        union {
          __bf16 b[4];
          uint2 u;
        } o;
        o.b[0] = (__bf16)t.x; o.b[1] = (__bf16)t.y; o.b[2] = (__bf16)t.z; o.b[3] = (__bf16)t.w;
        *(uint2*)((uint16_t*)cb.out + f0) = o.u;
      } else {
        *(float4*)((float*)cb.out + f0) = t;
      }
    }
    return;
  }
  const GemmBlock& gb = blocks[blockIdx.z];
  const int tiles_m = (gb.M + 127) / 128, tiles_n = (gb.N + 127) / 128;
  const int bx = (int)blockIdx.x - cs_wgs, gx = (int)gridDim.x - cs_wgs;
  const int tile = (bx & 7) * (gx >> 3) + (bx >> 3);
  if (tile >= tiles_m * tiles_n) return;
  const int tm = tile % tiles_m, tn = tile / tiles_m;
  const int m0 = tm * 128, n0 = tn * 128;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ml = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wy = wave >> 1, wx = wave & 1;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  constexpr int ES = BF16 ? 2 : 4, VE = 16 / ES, SK = BF16 ? 32 : 16;  // element bytes, elements per piece, k per step
  constexpr int LB = 128 * ES;                                         // bytes of a staged k line
  const GemmSeg& sg = gb.seg[0];  // one segment (checked on the host)
  const int K = sg.K, nsteps = (K + SK - 1) / SK;
  // resources end with the operand: k lines beyond K read as zero
  const u32x4 ra = lds_direct_rsrc(sg.a, (uint32_t)K * sg.lda * ES);
  const u32x4 rb = lds_direct_rsrc(sg.b, (uint32_t)K * sg.ldb * ES);
  const uint32_t my_lds = lds_address(smem) + wave * 2048;
  // load j of this wave (1 KB): bf16 k lines 8 wave + 4 j + lane / 16, position lane % 16 of the line;
  // fp32 k lines 4 wave + 2 j + lane / 32, position lane % 32
  uint32_t goff[4];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int l = BF16 ? 8 * wave + 4 * j + (lane >> 4) : 4 * wave + 2 * j + (lane >> 5);
    const int c = BF16 ? (lane & 15) ^ (4 * (l & 3)) : (lane & 31) ^ (8 * (l & 1));
    // whole pieces: M and N are multiples of a piece
    goff[j] = (m0 + c * VE < gb.M) ? ((uint32_t)l * sg.lda + m0 + c * VE) * ES : kOobOff;
    goff[2 + j] = (n0 + c * VE < gb.N) ? ((uint32_t)l * sg.ldb + n0 + c * VE) * ES : kOobOff;
  }
  const uint32_t a_step = (uint32_t)SK * sg.lda * ES, b_step = (uint32_t)SK * sg.ldb * ES;
  auto issue = [&](int st) __attribute__((always_inline)) {
    const uint32_t d = my_lds + (st & 1) * kTtStep;
    const uint32_t sa = (uint32_t)st * a_step, sb = (uint32_t)st * b_step;
#pragma unroll
    for (int j = 0; j < 2; ++j) load_to_lds(ra, d + j * 1024, goff[j], sa);
#pragma unroll
    for (int j = 0; j < 2; ++j) load_to_lds(rb, d + kTtOperand + j * 1024, goff[2 + j], sb);
  };
  // transposing reads: k line 16 g + tk (+ 4), rows (columns) base + tr ... + 3 as 8 bytes of piece (base + tr) / 8
  const int tk = 8 * (lane >> 5) + ((lane & 15) >> 2), tr = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  // (fp32: k line 2 p + h of pair p, row (column) base + ml: one float)
  uint32_t rda[2], rdb[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    if constexpr (BF16) {
      const int ca = (64 * wy + 32 * t + tr) >> 3, cb = (64 * wx + 32 * t + tr) >> 3;
      rda[t] = tk * 256 + ((ca ^ (4 * (tk & 3))) * 16) + (tr & 7) * 2;
      rdb[t] = kTtOperand + tk * 256 + ((cb ^ (4 * (tk & 3))) * 16) + (tr & 7) * 2;
    } else {
      const int fa_ = 64 * wy + 32 * t + ml, fb_ = 64 * wx + 32 * t + ml;
      rda[t] = h * LB + (((fa_ >> 2) ^ (8 * h)) * 16) + (fa_ & 3) * 4;
      rdb[t] = kTtOperand + h * LB + (((fb_ >> 2) ^ (8 * h)) * 16) + (fb_ & 3) * 4;
    }
  }

  if (nsteps > 0) issue(0);
  if (nsteps > 1) issue(1);
  for (int st = 0; st < nsteps; ++st) {
    const char* sbuf = smem + (st & 1) * kTtStep;
    // this wave's quarter of step st has landed (the four loads of step st + 1 may be in flight)
    if (st + 1 < nsteps) __builtin_amdgcn_s_waitcnt(kWaitVmcnt4);
    else __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    lds_barrier();  // and so has everyone's
    if constexpr (BF16) {
      Frag fa[2][2], fb[2][2];
#pragma unroll
      for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int o = g * 16 * 256;
          fa[g][t].t[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sbuf + rda[t] + o));
          fa[g][t].t[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sbuf + rda[t] + o + 4 * 256));
          fb[g][t].t[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sbuf + rdb[t] + o));
          fb[g][t].t[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sbuf + rdb[t] + o + 4 * 256));
        }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(kWaitLgkmcnt0);
      lds_barrier();  // every wave has this step in registers: its buffer may be refilled
      if (st + 2 < nsteps) issue(st + 2);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[g][j].v, fa[g][i].v, acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    } else {
      float fa[8][2], fb[8][2];
#pragma unroll
      for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          fa[p][t] = *(const float*)(sbuf + rda[t] + p * 2 * LB);
          fb[p][t] = *(const float*)(sbuf + rdb[t] + p * 2 * LB);
        }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(kWaitLgkmcnt0);
      lds_barrier();  // every wave has this step in registers: its buffer may be refilled
      if (st + 2 < nsteps) issue(st + 2);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[p][j], fa[p][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // epilogue: the tile is rounded into LDS (the staging buffers are done with: the last barrier above came after
  // their last read, and nothing was loaded behind it) and written out in 16-byte pieces, 256 contiguous bytes per row.
  // The products were accumulated transposed (B fragment as the first MFMA operand): register v of lane (h, ml) of
  // tile (i, j) is C[64 wy + 32 i + ml][64 wx + 32 j + 8 (v / 4) + 4 h + v % 4], so a register quad is four
  // consecutive columns: one 8-byte LDS write.  Row m keeps its 16-byte piece c at position c ^ (m & 15).
  if constexpr (!BF16) {
    // fp32: the tile (64 KB) does not fit the staging buffers, so each wave stages its 64 x 64 part 32 rows at a
    // time in its own quarter of them (8 KB: rows of 256 bytes, row r keeps its 16-byte piece c at c ^ (r & 15)) and
    // stores it in 16-byte pieces, 256 contiguous bytes per row; no workgroup barrier is needed (the last one above
    // came after everyone's last read of the buffers).
    char* const mine = smem + wave * 8192;
    const bool vec4 = gb.ldc % 4 == 0 && ((uintptr_t)gb.c & 15) == 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = 8 * j + 2 * q + h;
          *(float4*)(mine + ml * 256 + ((c ^ (ml & 15)) * 16)) =
              float4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        }
#pragma unroll
      for (int r8 = 0; r8 < 8; ++r8) {
        const int r = 4 * r8 + (lane >> 4), c = lane & 15;
        const float4 v = *(const float4*)(mine + r * 256 + ((c ^ (r & 15)) * 16));
        const int row = m0 + 64 * wy + 32 * i + r, col = n0 + 64 * wx + 4 * c;
        if (row < gb.M && col < gb.N) {  // whole quads: N % 4 == 0
          float* dst = (float*)gb.c + (size_t)row * gb.ldc + col;
          if (vec4) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4*)dst);
          else dst[0] = v.x, dst[1] = v.y, dst[2] = v.z, dst[3] = v.w;
        }
      }
    }
    return;
  }
  constexpr int CP = 128 * 2;  // bytes per staged row
  static_assert(128 * CP <= kTtLds, "output tile must fit the staging buffer");
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int cl = 64 * wx + 32 * j + 8 * q + 4 * h, col = n0 + cl;  // first of the quad's four columns
      float bias[4] = {0.f, 0.f, 0.f, 0.f};
      if (gb.bias && col < gb.N) {  // whole quads: N % 8 == 0
#pragma unroll
        for (int e = 0; e < 4; ++e) bias[e] = __uint_as_float((uint32_t)((const uint16_t*)gb.bias)[col + e] << 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int rl = 64 * wy + 32 * i + ml;
        union {
          __bf16 b[4];
          uint2 u;
        } o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o.b[e] = (__bf16)(acc[i][j][4 * q + e] + bias[e]);  // round to nearest even
        *(uint2*)(smem + rl * CP + (((cl >> 3) ^ (rl & 15)) * 16) + (cl & 7) * 2) = o.u;
      }
    }
  __syncthreads();
  const bool vec = gb.ldc % 8 == 0 && ((uintptr_t)gb.c & 15) == 0;  // N % 8 == 0 is a condition of this kernel
#pragma unroll
  for (int p = tid; p < 128 * 16; p += 256) {
    const int rl = p >> 4, q = p & 15;
    const int row = m0 + rl, col = n0 + q * 8;
    if (row >= gb.M || col >= gb.N) continue;
    uint16_t* dst = (uint16_t*)gb.c + (size_t)row * gb.ldc + col;
    if (vec) {
      __builtin_nontemporal_store(*(const u32x4*)(smem + rl * CP + ((q ^ (rl & 15)) * 16)), (u32x4*)dst);
    } else {
      const uint16_t* src = (const uint16_t*)(smem + rl * CP + ((q ^ (rl & 15)) * 16));
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e] = src[e];
    }
  }
}

// The launches these kernels are for.  gemm_stream_kernel: bf16, A contiguous along K, 64 x 64 tiles over the whole K
// range (no K split).  gemm_stream_tt_kernel: bf16, both operands as k lines, 128 x 128 tiles, one segment.
bool gemm_stream_usable(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc) {
  const int ve = bf16 ? 8 : 4;  // elements per 16-byte piece
  if (!a_kc) {
    if (b_kc) return false;
    for (const GemmBlock& b : blocks)
      if (b.nseg != 1 || b.M % ve || b.N % ve || (!bf16 && b.bias)) return false;
    return true;
  }
  for (const GemmBlock& b : blocks) {
    if (!b_kc && b.N % ve) return false;
    for (int s = 0; s < b.nseg; ++s)
      if (b.seg[s].K % ve) return false;
  }
  return true;
}

// d_colsum (or null): n_colsum column-sum blocks of at most max_f features (multiples of 4, 8-byte aligned rows)
// computed by extra workgroups of the same launch.
int launch_gemm_stream_tt(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16,
                          const ColsumBlock* d_colsum, int n_colsum, int max_f, hipStream_t st) {
  int tiles = 0;
  for (const GemmBlock& b : blocks) tiles = std::max(tiles, ((b.M + 127) / 128) * ((b.N + 127) / 128));
  tiles = (tiles + 7) / 8 * 8;
  const int chunks = d_colsum ? std::max(1, (max_f + 255) / 256) : 1;
  const int cs_wgs = d_colsum ? (n_colsum * chunks + 7) / 8 * 8 : 0;  // a multiple of 8 keeps the tiles' XCD mapping
  const dim3 grid((unsigned)(tiles + cs_wgs), 1, (unsigned)blocks.size()), block(256);
  if (bf16)
    hipLaunchKernelGGL(gemm_stream_tt_kernel<true>, grid, block, kTtLds, st, d_blocks, d_colsum, d_colsum ? n_colsum : 0,
                       chunks, cs_wgs);
  else
    hipLaunchKernelGGL(gemm_stream_tt_kernel<false>, grid, block, kTtLds, st, d_blocks, d_colsum, d_colsum ? n_colsum : 0,
                       chunks, cs_wgs);
  return DISTDL_OK;
}

template <bool BF16, bool B_KC>
static int launch_stream_variant(dim3 grid, const GemmBlock* d_blocks, hipStream_t st) {
  if (int rc = allow_large_lds<gemm_stream_kernel<BF16, B_KC>>()) return rc;
  hipLaunchKernelGGL((gemm_stream_kernel<BF16, B_KC>), grid, dim3(256), kStreamLds, st, d_blocks);
  return DISTDL_OK;
}

int launch_gemm_stream(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16, bool b_kc,
                       hipStream_t st) {
  int tiles = 0;
  for (const GemmBlock& b : blocks) tiles = std::max(tiles, ((b.M + 63) / 64) * ((b.N + 63) / 64));
  tiles = (tiles + 7) / 8 * 8;
  const dim3 grid((unsigned)tiles, 1, (unsigned)blocks.size());
  if (bf16) return b_kc ? launch_stream_variant<true, true>(grid, d_blocks, st) : launch_stream_variant<true, false>(grid, d_blocks, st);
  return b_kc ? launch_stream_variant<false, true>(grid, d_blocks, st) : launch_stream_variant<false, false>(grid, d_blocks, st);
}

}  // namespace distdl
