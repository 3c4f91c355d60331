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
// Tiles are 64 x 64 per workgroup (4 waves, one 32 x 32 MFMA tile each), staged through LDS with
// 16-byte buffer loads (rows beyond the matrix fail the range check and read as zero), double
// buffered: one barrier per stage.
//
// fp32: v_mfma_f32_32x32x2_f32, A lane l holds A[i = l%32][k = l/32]; a 16-byte LDS read gives a lane
//       4 consecutive k, used by 4 MFMAs whose k-pairs are (j, 4+j) -- the same pairing on both operands.
// bf16: v_mfma_f32_32x32x16_bf16, A lane l holds A[i = l%32][k = 8*(l/32) .. +7], one 16-byte read.
// D register v of lane l is D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32] for both.
#include <algorithm>
#include <cstring>

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

// BF16 = false: T is float, BK = 32 floats per stage.  BF16 = true: T is bf16 bits, BK = 64 per stage.
// Row pitch in LDS is BK + 16 bytes for the K-contiguous layout, 64 elements + 16 bytes for the other.
template <bool BF16, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const GemmBlock* __restrict__ blocks, int tiles_n_max) {
  constexpr int ES = BF16 ? 2 : 4;             // element size
  constexpr int BK = BF16 ? 64 : 32;           // k per stage
  constexpr int VE = 16 / ES;                  // elements per 16-byte piece
  constexpr int PITCH_KC = BK * ES + 16;       // bytes per tile row, K-contiguous staging [row][k]
  constexpr int PITCH_TC = 64 * ES + 16;       // bytes per k line, transposed staging [k][row]
  constexpr int TILE_BYTES = (64 * PITCH_KC > BK * PITCH_TC) ? 64 * PITCH_KC : BK * PITCH_TC;
  constexpr int PIECES = 64 * BK * ES / 16 / 256;  // 16-byte pieces per thread, operand and stage
  __shared__ __attribute__((aligned(16))) char smem[4 * TILE_BYTES];  // A0 B0 A1 B1

  const GemmBlock& gb = blocks[blockIdx.z];
  const int tiles_n = (gb.N + 63) / 64, tiles_m = (gb.M + 63) / 64;
  // consecutive tiles share the B tile (weights: m walks fastest); workgroups are dealt to the 8 XCDs
  // round-robin, so give each XCD a contiguous range of tiles and keep that sharing behind one L2
  const int tile = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (tile >= tiles_m * tiles_n) return;
  const int tm = tile % tiles_m, tn = tile / tiles_m;
  const int m0 = tm * 64, n0 = tn * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ml = lane & 31;
  const int wy = wave >> 1, wx = wave & 1;

  floatx16 acc;
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;

  // piece -> (row or k line, 16-byte column) of this thread, fixed
  //   K-contiguous: 64 rows x (BK/VE) pieces per row; transposed: BK lines x (64/VE) pieces per line
  u32x4 ra[PIECES], rb[PIECES];
  uint32_t a_goff[PIECES], b_goff[PIECES], a_loff[PIECES], b_loff[PIECES];
  int a_k[PIECES], b_k[PIECES];  // k of the piece's first element (to cut the K tail)

  for (int s = 0; s < gb.nseg; ++s) {
    const GemmSeg& sg = gb.seg[s];
    const int K = sg.K;
    // resources cover exactly the operand: rows beyond M / N (or k lines beyond K) read as zero
    const uint32_t a_bytes = (uint32_t)(A_KC ? gb.M : K) * sg.lda * ES;
    const uint32_t b_bytes = (uint32_t)(B_KC ? gb.N : K) * sg.ldb * ES;
    const __amdgpu_buffer_rsrc_t ra_rs = gemm_rsrc(sg.a, a_bytes), rb_rs = gemm_rsrc(sg.b, b_bytes);
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int piece = tid + i * 256;
      if (A_KC) {
        const int row = piece / (BK / VE), kq = piece % (BK / VE);
        a_goff[i] = ((uint32_t)(m0 + row) * sg.lda + kq * VE) * ES;
        a_loff[i] = row * PITCH_KC + kq * 16;
        a_k[i] = kq * VE;
      } else {
        const int kl = piece / (64 / VE), mq = piece % (64 / VE);
        a_goff[i] = ((uint32_t)kl * sg.lda + m0 + mq * VE) * ES;
        a_loff[i] = kl * PITCH_TC + mq * 16;
        a_k[i] = kl;
        if (m0 + mq * VE >= gb.M) a_goff[i] = kGemmOob;  // columns beyond M (whole pieces: M % VE == 0)
      }
      if (B_KC) {
        const int row = piece / (BK / VE), kq = piece % (BK / VE);
        b_goff[i] = ((uint32_t)(n0 + row) * sg.ldb + kq * VE) * ES;
        b_loff[i] = row * PITCH_KC + kq * 16;
        b_k[i] = kq * VE;
      } else {
        const int kl = piece / (64 / VE), nq = piece % (64 / VE);
        b_goff[i] = ((uint32_t)kl * sg.ldb + n0 + nq * VE) * ES;
        b_loff[i] = kl * PITCH_TC + nq * 16;
        b_k[i] = kl;
        if (n0 + nq * VE >= gb.N) b_goff[i] = kGemmOob;
      }
    }
    auto load = [&](int k0) {
      const uint32_t a_base = (uint32_t)k0 * (A_KC ? 1u : sg.lda) * ES;
      const uint32_t b_base = (uint32_t)k0 * (B_KC ? 1u : sg.ldb) * ES;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        // K tail: pieces are whole (K % VE == 0 for K-contiguous operands), lines beyond K fail the range check
        ra[i] = __builtin_amdgcn_raw_buffer_load_b128(ra_rs, (A_KC && k0 + a_k[i] >= K) ? kGemmOob : a_goff[i], a_base, 0);
        rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rb_rs, (B_KC && k0 + b_k[i] >= K) ? kGemmOob : b_goff[i], b_base, 0);
      }
    };
    auto stash = [&](int buf) {
      char* sa = smem + buf * 2 * TILE_BYTES;
      char* sb = sa + TILE_BYTES;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        *(u32x4*)(sa + a_loff[i]) = ra[i];
        *(u32x4*)(sb + b_loff[i]) = rb[i];
      }
    };
    const int nstage = (K + BK - 1) / BK;
    load(0);
    __syncthreads();  // previous segment's last stage fully consumed
    stash(0);
    __syncthreads();
    for (int st = 0; st < nstage; ++st) {
      if (st + 1 < nstage) load((st + 1) * BK);
      const char* sa = smem + (st & 1) * 2 * TILE_BYTES;
      const char* sb = sa + TILE_BYTES;
      if (!BF16) {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 8) {
          float av[4], bv[4];
          if (A_KC) {
            const float4 t = *(const float4*)(sa + (32 * wy + ml) * PITCH_KC + (kk + 4 * h) * 4);
            av[0] = t.x; av[1] = t.y; av[2] = t.z; av[3] = t.w;
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) av[j] = *(const float*)(sa + (kk + 4 * h + j) * PITCH_TC + (32 * wy + ml) * 4);
          }
          if (B_KC) {
            const float4 t = *(const float4*)(sb + (32 * wx + ml) * PITCH_KC + (kk + 4 * h) * 4);
            bv[0] = t.x; bv[1] = t.y; bv[2] = t.z; bv[3] = t.w;
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = *(const float*)(sb + (kk + 4 * h + j) * PITCH_TC + (32 * wx + ml) * 4);
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[j], bv[j], acc, 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
          union { u32x4 u; bf16x8 v; uint16_t e[8]; } av, bv;
          if (A_KC) {
            av.u = *(const u32x4*)(sa + (32 * wy + ml) * PITCH_KC + (kk + 8 * h) * 2);
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) av.e[j] = *(const uint16_t*)(sa + (kk + 8 * h + j) * PITCH_TC + (32 * wy + ml) * 2);
          }
          if (B_KC) {
            bv.u = *(const u32x4*)(sb + (32 * wx + ml) * PITCH_KC + (kk + 8 * h) * 2);
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) bv.e[j] = *(const uint16_t*)(sb + (kk + 8 * h + j) * PITCH_TC + (32 * wx + ml) * 2);
          }
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av.v, bv.v, acc, 0, 0, 0);
        }
      }
      if (st + 1 < nstage) stash((st + 1) & 1);
      __syncthreads();
    }
  }

  // epilogue: D register v of lane (h, ml) is C[m0 + 32*wy + 8*(v/4) + 4*h + v%4][n0 + 32*wx + ml]
  const int col = n0 + 32 * wx + ml;
  if (col >= gb.N) return;
  float bias = 0.f;
  if (gb.bias) bias = BF16 ? __uint_as_float((uint32_t)((const uint16_t*)gb.bias)[col] << 16) : ((const float*)gb.bias)[col];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = m0 + 32 * wy + 8 * (v / 4) + 4 * h + (v % 4);
    if (row >= gb.M) continue;
    const float r = acc[v] + bias;
    if (BF16) ((uint16_t*)gb.c)[(size_t)row * gb.ldc + col] = (uint16_t)f32_to_bf16_rne(r);
    else ((float*)gb.c)[(size_t)row * gb.ldc + col] = r;
  }
}

// db_i[f] = sum over the batch of dy_i[n][f]: one block per 64 features, 4 batch lanes each.
template <bool BF16>
__global__ __launch_bounds__(256) void colsum_kernel(const ColsumBlock* __restrict__ blocks) {
  const ColsumBlock& cb = blocks[blockIdx.y];
  const int f = blockIdx.x * 64 + (threadIdx.x & 63), lanegrp = threadIdx.x >> 6;
  __shared__ float red[4][64];
  float acc = 0.f;
  if (f < cb.n_f && cb.out)
    for (int n = lanegrp; n < cb.n_b; n += 4)
      acc += BF16 ? __uint_as_float((uint32_t)((const uint16_t*)cb.in)[(size_t)n * cb.n_f + f] << 16)
                  : ((const float*)cb.in)[(size_t)n * cb.n_f + f];
  red[lanegrp][threadIdx.x & 63] = acc;
  __syncthreads();
  if (lanegrp == 0 && f < cb.n_f && cb.out) {
    const float s = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
    if (BF16) ((uint16_t*)cb.out)[f] = (uint16_t)f32_to_bf16_rne(s);
    else ((float*)cb.out)[f] = s;
  }
}

// ---- host side ------------------------------------------------------------------

bool gemm_mfma_usable(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc) {
  const int ve = bf16 ? 8 : 4;
  const size_t es = bf16 ? 2 : 4;
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

int launch_gemm_mfma(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc,
                     const char* name, hipStream_t st) {
  int tiles = 0;
  for (const GemmBlock& b : blocks) tiles = std::max(tiles, ((b.M + 63) / 64) * ((b.N + 63) / 64));
  tiles = (tiles + 7) / 8 * 8;
  dim3 grid((unsigned)tiles, 1, (unsigned)blocks.size()), block(256);
  ProfScope prof(name, st);
#define DISTDL_GEMM(BF_, A_, B_) hipLaunchKernelGGL((gemm_mfma_kernel<BF_, A_, B_>), grid, block, 0, st, d_blocks, 0)
  if (!bf16) {
    if (a_kc && b_kc) DISTDL_GEMM(false, true, true);
    else if (a_kc) DISTDL_GEMM(false, true, false);
    else if (b_kc) DISTDL_GEMM(false, false, true);
    else DISTDL_GEMM(false, false, false);
  } else {
    if (a_kc && b_kc) DISTDL_GEMM(true, true, true);
    else if (a_kc) DISTDL_GEMM(true, true, false);
    else if (b_kc) DISTDL_GEMM(true, false, true);
    else DISTDL_GEMM(true, false, false);
  }
#undef DISTDL_GEMM
  return DISTDL_OK;
}

int launch_colsum(const ColsumBlock* d_blocks, int nblocks, int max_f, bool bf16, hipStream_t st) {
  dim3 grid((unsigned)((max_f + 63) / 64), (unsigned)nblocks), block(256);
  ProfScope prof("affine_bias_grad", st);
  if (bf16) hipLaunchKernelGGL(colsum_kernel<true>, grid, block, 0, st, d_blocks);
  else hipLaunchKernelGGL(colsum_kernel<false>, grid, block, 0, st, d_blocks);
  return DISTDL_OK;
}

}  // namespace distdl
