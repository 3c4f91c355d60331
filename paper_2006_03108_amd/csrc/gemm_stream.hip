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
//     ds_write.  Lane L of such a load lands at (LDS base in M0) + 16 L and an out-of-range lane writes zeros
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
#include "profile.h"

namespace distdl {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void;
typedef __attribute__((address_space(3))) v4i16* lds_v4;

namespace {

constexpr uint32_t kOobOff = 0x7ffffff0u;  // fails the range check of every buffer (operands are < 2 GiB)
constexpr int kStepK = 64;                 // k per step
constexpr int kOperandBytes = 64 * 128;    // one operand block of a step
constexpr int kStepBytes = 2 * kOperandBytes;
constexpr int kWaveBytes = 2 * kStepBytes;  // two steps per wave: one multiplied, one landing
constexpr int kStreamLds = 4 * kWaveBytes;  // 128 KB
constexpr int kRedPitch = 64;               // floats per row of a partial tile in the epilogue

__device__ inline __amdgpu_buffer_rsrc_t stream_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// s_waitcnt immediates (vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; a field of all ones does not wait)
constexpr int kWaitVm0 = 0x0F70;         // vmcnt(0)
constexpr int kWaitVm16 = 0x4F70;        // vmcnt(16)
constexpr int kWaitLgkm0 = 0xC07F;       // lgkmcnt(0)

union Frag {
  u32x4 u;
  bf16x8 v;
  v4i16 t[2];
};

}  // namespace

template <bool B_KC>
__global__ __launch_bounds__(256, 1) void gemm_stream_kernel(const GemmBlock* __restrict__ blocks) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
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

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // The 64-k steps of all segments form one sequence; this wave takes every fourth of them.
  int total = 0;
  for (int s = 0; s < gb.nseg; ++s) total += (gb.seg[s].K + kStepK - 1) / kStepK;
  const int n = (total - wave + 3) / 4;

  // load cursor: segment, step within it (may run past the end: such steps are issued out of range and never read)
  int ls = 0, lin = wave, l_nst = 0, l_K = 0;
  uint32_t l_ldb = 0;
  __amdgpu_buffer_rsrc_t ra = stream_rsrc(nullptr, 0), rb = stream_rsrc(nullptr, 0);
  uint32_t goff[16];
  // piece of lane and instruction i: row (or k line) 8 i + lane / 8, position lane % 8
  auto enter_segment = [&]() __attribute__((always_inline)) {
    const GemmSeg& sg = gb.seg[ls];
    l_K = sg.K;
    l_nst = (sg.K + kStepK - 1) / kStepK;
    l_ldb = (uint32_t)sg.ldb;
    // the resources end with the operand: rows beyond M / N and k lines beyond K read as zero
    ra = stream_rsrc(sg.a, (uint32_t)gb.M * sg.lda * 2);
    rb = stream_rsrc(sg.b, (uint32_t)(B_KC ? gb.N : sg.K) * sg.ldb * 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 8 * i + (lane >> 3);
      const int ca = (lane & 7) ^ ((r >> 1) & 7);
      goff[i] = ((uint32_t)(m0 + r) * sg.lda + ca * 8) * 2;
      if (B_KC) {
        goff[8 + i] = ((uint32_t)(n0 + r) * sg.ldb + ca * 8) * 2;
      } else {
        const int cb = (lane & 7) ^ (4 * ((r >> 1) & 1));
        goff[8 + i] = ((uint32_t)r * sg.ldb + n0 + cb * 8) * 2;
        if (n0 + cb * 8 >= gb.N) goff[8 + i] = kOobOff;  // columns beyond N (whole pieces: N % 8 == 0)
      }
    }
  };
  // Issues the loads of the cursor's step into staging buffer `buf` and moves the cursor on by four steps.
  auto issue = [&](int buf, bool valid) __attribute__((always_inline)) {
    char* d = my + buf * kStepBytes;
    int k0 = 0;
    if (valid) {  // wave-uniform
      while (lin >= l_nst) {
        lin -= l_nst;
        ++ls;
        enter_segment();
      }
      k0 = lin * kStepK;
      lin += 4;
    }
    const uint32_t a_base = (uint32_t)k0 * 2, b_base = (uint32_t)k0 * (B_KC ? 1u : l_ldb) * 2;
    if (!valid || k0 + kStepK <= l_K) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void)(d + i * 1024), 16, valid ? goff[i] : kOobOff, a_base, 0, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void)(d + kOperandBytes + i * 1024), 16,
                                                 valid ? goff[8 + i] : kOobOff, b_base, 0, 0);
    } else {
      // K tail: pieces of a K-contiguous row beyond K are switched off (whole pieces: K % 8 == 0); k lines beyond
      // K lie beyond the resource
      const int kleft = l_K - k0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = 8 * i + (lane >> 3);
        const int ca = (lane & 7) ^ ((r >> 1) & 7);
        const bool in = ca * 8 < kleft;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void)(d + i * 1024), 16, in ? goff[i] : kOobOff, a_base, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = 8 * i + (lane >> 3);
        const int ca = (lane & 7) ^ ((r >> 1) & 7);
        const bool in = !B_KC || ca * 8 < kleft;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void)(d + kOperandBytes + i * 1024), 16,
                                                 in ? goff[8 + i] : kOobOff, b_base, 0, 0);
      }
    }
  };

  // fragment addresses inside a staging buffer
  //   A (and B when K-contiguous): row 32 t + ml, piece 2 g + h of the step, at position piece ^ key(row)
  uint32_t rdk[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) rdk[g] = ml * 128 + (((2 * g + h) ^ ((ml >> 1) & 7)) * 16);
  //   B when N-contiguous: k line 16 g + tk (+ 4), columns 32 t + tr ... + 3 (8 bytes) at piece (4 t + tr / 8) ^ f(line)
  const int tk = 8 * (lane >> 5) + ((lane & 15) >> 2), tr = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  uint32_t rdt[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    rdt[t] = kOperandBytes + tk * 128 + ((((4 * t + (tr >> 3)) ^ (4 * ((tk >> 1) & 1)))) * 16) + (tr & 7) * 2;

  auto read_half = [&](int buf, int g0, Frag (&fa)[2][2], Frag (&fb)[2][2]) __attribute__((always_inline)) {
    const char* s = my + buf * kStepBytes;
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[g][t].u = *(const u32x4*)(s + rdk[g0 + g] + t * 4096);
        if constexpr (B_KC) {
          fb[g][t].u = *(const u32x4*)(s + kOperandBytes + rdk[g0 + g] + t * 4096);
        } else {
          fb[g][t].t[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + rdt[t] + (g0 + g) * 16 * 128));
          fb[g][t].t[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + rdt[t] + (g0 + g) * 16 * 128 + 4 * 128));
        }
      }
  };
  auto mm_half = [&](const Frag (&fa)[2][2], const Frag (&fb)[2][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[g][i].v, fb[g][j].v, acc[i][j], 0, 0, 0);
  };

  if (n > 0) {
    enter_segment();
    issue(0, true);
    issue(1, 1 < n);
    Frag xa[2][2], xb[2][2], ya[2][2], yb[2][2];
    // One step: its 16 loads have landed when at most the 16 of the next step are outstanding.  The buffer is
    // handed to the loads of the step after next as soon as every fragment of it is in registers.
    auto step = [&](int st, int buf) __attribute__((always_inline)) {
      __builtin_amdgcn_s_waitcnt(kWaitVm16);
      __builtin_amdgcn_sched_barrier(0);
      read_half(buf, 0, xa, xb);
      read_half(buf, 2, ya, yb);
      __builtin_amdgcn_sched_barrier(0);
      mm_half(xa, xb);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
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
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // nothing may still land in LDS when the epilogue reuses it
  }

  // Sum of the four waves' partial tiles in wave order, bias, rounding, store.
  __syncthreads();
  float* red = (float*)smem;  // [wave][64][kRedPitch]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 32 * i + 8 * (v / 4) + 4 * h + (v % 4), col = 32 * j + ml;
        red[(wave * 64 + row) * kRedPitch + col] = acc[i][j][v];
      }
  __syncthreads();
  const int row = tid >> 2, c0 = (tid & 3) * 16;
  float s[16];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float4 t = *(const float4*)(red + (size_t)row * kRedPitch + c0 + 4 * q);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float4 u = *(const float4*)(red + (size_t)(w * 64 + row) * kRedPitch + c0 + 4 * q);
      t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
    }
    s[4 * q] = t.x; s[4 * q + 1] = t.y; s[4 * q + 2] = t.z; s[4 * q + 3] = t.w;
  }
  const int grow = m0 + row, gcol = n0 + c0;
  if (grow >= gb.M || gcol >= gb.N) return;
  const bool full = gcol + 16 <= gb.N;
  if (gb.bias) {
    const uint16_t* bp = (const uint16_t*)gb.bias + gcol;
    if (full) {
#pragma unroll
      for (int q = 0; q < 16; ++q) s[q] += __uint_as_float((uint32_t)bp[q] << 16);
    } else {
      for (int q = 0; gcol + q < gb.N; ++q) s[q] += __uint_as_float((uint32_t)bp[q] << 16);
    }
  }
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
}

// The launch this kernel is for: bf16, A contiguous along K, 64 x 64 tiles over the whole K range (no K split).
bool gemm_stream_usable(const std::vector<GemmBlock>& blocks, bool a_kc, bool b_kc) {
  if (!a_kc) return false;
  for (const GemmBlock& b : blocks) {
    if (!b_kc && b.N % 8) return false;
    for (int s = 0; s < b.nseg; ++s)
      if (b.seg[s].K % 8) return false;
  }
  return true;
}

int launch_gemm_stream(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool b_kc, hipStream_t st) {
  int tiles = 0;
  for (const GemmBlock& b : blocks) tiles = std::max(tiles, ((b.M + 63) / 64) * ((b.N + 63) / 64));
  tiles = (tiles + 7) / 8 * 8;
  const dim3 grid((unsigned)tiles, 1, (unsigned)blocks.size()), block(256);
  if (b_kc) {
    if (int rc = allow_large_lds<gemm_stream_kernel<true>>()) return rc;
    hipLaunchKernelGGL(gemm_stream_kernel<true>, grid, block, kStreamLds, st, d_blocks);
  } else {
    if (int rc = allow_large_lds<gemm_stream_kernel<false>>()) return rc;
    hipLaunchKernelGGL(gemm_stream_kernel<false>, grid, block, kStreamLds, st, d_blocks);
  }
  return DISTDL_OK;
}

}  // namespace distdl
