// Block descriptors and launchers of the MFMA GEMM used by the partitioned affine layer.
#pragma once
#include <cstdint>
#include <vector>

#include <hip/hip_runtime.h>

namespace distdl {

constexpr int kGemmMaxSeg = 8;

struct GemmSeg {
  const void* a;  // A_{o,s}
  const void* b;  // B_{o,s}
  int32_t K, lda, ldb, pad_;
};

struct GemmBlock {
  GemmSeg seg[kGemmMaxSeg];
  void* c;
  const void* bias;  // length N, or null
  int32_t M, N, ldc, nseg;
};

struct ColsumBlock {
  const void* in;  // [n_b][n_f]
  void* out;       // [n_f], or null (skip)
  int32_t n_b, n_f;
};

// True when every operand can be moved in aligned 16-byte pieces (the MFMA kernel's requirement).
bool gemm_mfma_usable(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc);
// a_kc: A[m][k] is contiguous along k (else along m); b_kc: B[k][n] is contiguous along k (else along n).
// nsplit > 1: K split over nsplit workgroups per tile through the fp32 buffer `partial`
// (gemm_mfma_partial_floats(blocks, nsplit) floats), summed by a second kernel.
int gemm_mfma_splits(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc);
size_t gemm_mfma_partial_floats(const std::vector<GemmBlock>& blocks, int nsplit);
// colsum (optional): column sums to fold into the launch when its kernel can carry them; *colsum->done says whether
// it did (otherwise the caller launches launch_colsum itself).
struct GemmColsum {
  const ColsumBlock* d_blocks;
  int n_blocks, max_f;
  bool done;
};
int launch_gemm_mfma(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc,
                     int nsplit, float* partial, const char* name, hipStream_t st, GemmColsum* colsum = nullptr);
// The small-batch path (gemm_stream.hip): 64 x 64 tiles over the whole K range, every wave its own K-slice pipeline
// fed by global -> LDS loads, bf16 or fp32.  Usable when A is contiguous along K and every K (and, for an N-contiguous
// B, N) is a multiple of a 16-byte piece (8 bf16, 4 fp32); with both operands as k lines (weight gradient, bf16 only):
// one segment, M and N multiples of 8.
bool gemm_stream_usable(const std::vector<GemmBlock>& blocks, bool bf16, bool a_kc, bool b_kc);
int launch_gemm_stream(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16, bool b_kc,
                       hipStream_t st);
// the weight-gradient layout (both operands as k lines), 128 x 128 tiles
// d_colsum (or null): column sums (the bias gradient) computed by extra workgroups of the same launch
int launch_gemm_stream_tt(const GemmBlock* d_blocks, const std::vector<GemmBlock>& blocks, bool bf16,
                          const ColsumBlock* d_colsum, int n_colsum, int max_f, hipStream_t st);
int launch_colsum(const ColsumBlock* d_blocks, int nblocks, int max_f, bool bf16, hipStream_t st);

}  // namespace distdl
