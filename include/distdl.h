/* distdl.h -- C ABI of the MI355X (gfx950) library for the data-movement
 * primitives and partitioned layers of Hewett & Grady, "A Linear Algebraic
 * Approach to Model Parallelism in Deep Learning" (arXiv 2006.03108).
 *
 * All P "workers" (the paper's parallel workers, Sec. 3) are virtual
 * partitions that live in one GPU's HBM.  A send-receive (Sec. 3 "Send and
 * Receive": a copy C_{a->b} between two workers' memories) is a strided
 * device copy between partition buffers; its adjoint adds into the source and
 * clears the destination (Sec. 2 "Copy": C* = K_b S_{b->a}).
 *
 * Conventions
 *  - C99, no C++ types, no exceptions across the boundary.
 *  - Pointers named *_dev are DEVICE pointers owned by the caller.  Arrays of
 *    pointers / sizes are HOST arrays read during the call; the library
 *    copies what it needs, the caller may free them on return.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *    the default stream); calls are asynchronous and never synchronise.
 *  - Return value: DISTDL_OK (0) or a negative error code; on error nothing
 *    has been enqueued.  distdl_last_error() gives a thread-local message.
 *  - Outputs named d* (gradients) are OVERWRITTEN, not accumulated into: each
 *    call is an out-of-place adjoint (Sec. 3, first paragraph).
 *  - Device pointers must be aligned to the element size; 16-byte alignment
 *    (what any allocator gives) enables the vectorised kernels.
 *  - One plan may be used from one host thread at a time.
 *  - A plan keeps device copies of the pointer arrays it has been called with
 *    (the last eight per argument and stream) and whatever scratch it needs;
 *    the first call with new arrays, on a new stream or with a larger problem
 *    therefore copies a table or allocates, later calls do neither.  A call
 *    that has been made once on a stream can be recorded into a HIP graph on
 *    that stream (no allocation, no host-to-device copy, no memset).  A copy
 *    that a recorded call uses is kept unchanged until the plan is destroyed;
 *    a copy is only ever replaced by a call on the stream that used it last.
 *    A call with arrays the plan has not seen on that stream fails with
 *    INVALID_ARG while the stream is being captured, and with NOMEM when all
 *    64 copies of an argument are held by other streams or recorded graphs.
 *
 * Memory layout of sliding-kernel tensors: CHANNELS-LAST.  The paper fixes
 * only the logical shape n_b x n_c x m_0 x ... x m_{D-1} (Sec. 4 "Sparse
 * layers") and leaves ordering and layout to the implementation (Sec. 2).
 * Here a worker's padded buffer is the contiguous array
 *        [n_b][buf_0]...[buf_{D-1}][n_c]          (n_c fastest)
 * so that one feature-space cell is n_c contiguous elements: every halo
 * face, edge and corner is then made of whole contiguous cells, and the
 * channel axis is the contraction axis the matrix cores read.  Along each
 * feature dimension a buffer is  [ pad_L | halo_L | bulk | halo_R | pad_R ].
 * Outputs y are dense [n_b][out_0]...[out_{D-1}][n_co]; convolution weights
 * keep the paper's shape [n_co][n_ci][k_0]...[k_{D-1}] (last fastest).
 */
#ifndef DISTDL_H
#define DISTDL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DISTDL_F32 = 0, DISTDL_BF16 = 1 } distdl_dtype;

enum {
  DISTDL_OK = 0,
  DISTDL_ERR_INVALID_ARG = -1,
  DISTDL_ERR_NULL = -2,
  DISTDL_ERR_UNSUPPORTED = -3,
  DISTDL_ERR_EMPTY_PARTITION = -4, /* some worker would own no input or no output cell */
  DISTDL_ERR_HALO_TOO_WIDE = -5,   /* a halo exceeds the adjacent worker's bulk (Sec. 3
                                      assumes directly adjacent neighbours only) */
  DISTDL_ERR_HIP = -6,
  DISTDL_ERR_NOMEM = -7
};

#define DISTDL_MAX_DIMS 3

/* ------------------------------------------------------------------------
 * Sliding-kernel plan (Sec. 3 "Halo exchange", App. B.1).
 *
 * Splits a feature space of extent in_shape over the partition vector P
 * (Sec. 4: workers per dimension; worker id is row-major over P) and derives,
 * per dimension and worker, the halo / pad / extra widths from the worker's
 * first and last output index and the kernel's size, stride, dilation and
 * padding.  Per dimension, with n = in_shape, m = floor((n+2p-dil(k-1)-1)/s)+1:
 *   balanced split of a length L: worker r gets floor(L/P)+(r < L mod P) cells;
 *   inputs and outputs are split by it independently (output drives the load
 *   balance, App. B.1);  outputs [j0,j1] need inputs [j0*s-p, j1*s-p+dil(k-1)];
 *   pad = the part outside [0,n-1], halo = the in-domain part outside the
 *   owned range, extra = owned cells outside the needed range.
 * Errors: EMPTY_PARTITION, HALO_TOO_WIDE, INVALID_ARG (D not in 1..3, sizes
 * < 1), UNSUPPORTED (dtype).
 * ---------------------------------------------------------------------- */
typedef struct distdl_plan distdl_plan; /* opaque, library-owned */

int distdl_plan_create(distdl_plan** out, int D, int64_t n_b, int64_t n_c_in, int64_t n_c_out,
                       const int64_t in_shape[], const int32_t P[], const int32_t ksize[],
                       const int32_t stride[], const int32_t padding[], const int32_t dilation[],
                       distdl_dtype dtype);

/* Halo-only plan with user-given bulk sizes and halo widths and no padding,
 * the form of the rank-2 example of App. B.2.  bulk_sizes holds, dimension
 * after dimension, P[d] sizes; halo_lr holds, in the same order, (left,
 * right) pairs.  conv_* calls reject such a plan (UNSUPPORTED). */
int distdl_plan_create_explicit(distdl_plan** out, int D, int64_t n_b, int64_t n_c, const int32_t P[],
                                const int64_t bulk_sizes[], const int32_t halo_lr[], distdl_dtype dtype);

typedef struct {
  int64_t in_start[DISTDL_MAX_DIMS], in_size[DISTDL_MAX_DIMS];   /* owned (bulk) input range   */
  int64_t out_start[DISTDL_MAX_DIMS], out_size[DISTDL_MAX_DIMS]; /* owned output range         */
  int32_t halo[DISTDL_MAX_DIMS][2], pad[DISTDL_MAX_DIMS][2], extra[DISTDL_MAX_DIMS][2]; /* [d][left,right] */
  int64_t buf_shape[DISTDL_MAX_DIMS]; /* pad_L + halo_L + bulk + halo_R + pad_R              */
  int64_t bulk_off[DISTDL_MAX_DIMS];  /* buffer coordinate of the first bulk cell           */
  int64_t conv_origin[DISTDL_MAX_DIMS]; /* buffer coordinate of the first tap of the first
                                           owned output (= extra_L)                           */
} distdl_worker_geom;

int distdl_plan_num_workers(const distdl_plan* plan); /* prod(P), or a negative error */
int distdl_plan_query(const distdl_plan* plan, int worker, distdl_worker_geom* out);
int distdl_plan_destroy(distdl_plan* plan);

/* ------------------------------------------------------------------------
 * Halo exchange H and its adjoint H* (Sec. 3 "Halo exchange", both displayed
 * operator products; App. B.2).  In place on the P padded buffers
 * bufs_dev[worker], each [n_b][buf_0..buf_{D-1}][n_c] of the plan's dtype.
 *
 * halo_fwd: every in-domain non-owned cell <- the owning worker's bulk value
 *   (a bit-exact copy), every zero-padding cell <- 0, bulk untouched.  The
 *   result does not depend on previous halo / pad contents.  This is what the
 *   nested per-dimension exchange leaves behind, computed in one pass.
 * halo_adj: every bulk cell += the sum of all halo cells (in other workers'
 *   buffers) that alias it, summed in ascending source-worker order in fp32;
 *   then every halo and pad cell <- 0.  Deterministic (no atomics).
 * ---------------------------------------------------------------------- */
int distdl_halo_fwd(distdl_plan* plan, void* const bufs_dev[], void* stream);
int distdl_halo_adj(distdl_plan* plan, void* const gbufs_dev[], void* stream);

/* ------------------------------------------------------------------------
 * Broadcast B_{a->{k}} and sum-reduce R_{{k}->a} = B* over G independent
 * groups of k replicas (Sec. 3 "Broadcast", "Sum-reduce and all-reduce").
 * Group g has count[g] elements; replica i of group g is pointer [g*k + i].
 *
 * bcast_fwd / sumreduce_adj:  dst[g*k+i][e] = src[g][e]            (bit-exact)
 * bcast_adj / sumreduce_fwd:  out[g][e] = sum_{i=0}^{k-1} in[g*k+i][e], summed
 *   in index order in fp32, overwriting out.  With clear_inputs != 0 the
 *   replicas are zeroed afterwards (the K_i of B* = sum_i K_i S_{i->a}).
 * In and out buffers must not overlap.  Groups of more than 64 replicas read
 * their pointers from a device copy of the pointer array, cached per device
 * under the rules of the plans' tables (one host thread at a time).
 * Errors: NULL, INVALID_ARG (G, k < 1, count < 0).
 * ---------------------------------------------------------------------- */
int distdl_bcast_fwd(const void* const src_dev[], void* const dst_dev[], const int64_t count[], int G, int k,
                     distdl_dtype dtype, void* stream);
int distdl_bcast_adj(void* const gsrc_dev[], void* const gdst_dev[], const int64_t count[], int G, int k,
                     distdl_dtype dtype, int clear_inputs, void* stream);
int distdl_sumreduce_fwd(void* const src_dev[], void* const dst_dev[], const int64_t count[], int G, int k,
                         distdl_dtype dtype, int clear_inputs, void* stream);
int distdl_sumreduce_adj(const void* const gdst_dev[], void* const gsrc_dev[], const int64_t count[], int G,
                         int k, distdl_dtype dtype, void* stream);

/* ------------------------------------------------------------------------
 * Partitioned convolution: the Forward / Adjoint Convolution Algorithms of
 * Sec. 4 with the feature space partitioned only (P_co = P_ci = 1).  The plan's
 * dtype is the element type of every array (x, w, b, y and all gradients):
 * fp32, or bf16 with fp32 accumulation and results rounded to nearest even.
 *
 * conv_fwd: x <- H x in place on x_bufs_dev; w and b are read by every worker
 *   directly (the broadcasts B w, B b without materialised replicas); each
 *   worker's y[n][o][co] = b[co] + sum_{ci,kappa} w[co][ci][kappa] *
 *   x^[n][origin + o*s + kappa*dil][ci] on its own buffer, no further padding.
 *   y_dev[worker] is dense [n_b][out_0..][n_co].  bias_dev may be NULL.
 * conv_bwd: x_bufs_dev must hold H x (as left by conv_fwd).  Computes the
 *   local [dConv]* into the whole padded dx buffers, dw = sum over workers of
 *   the local dw^ and db likewise (the sum-reduces R that are the adjoints of
 *   B w and B b), then dx <- H* dx: on return each dx buffer holds the
 *   gradient in its bulk and zeros in halo and pad cells.  dw_dev has the
 *   shape of w; dbias_dev may be NULL.  workspace_dev must provide
 *   distdl_conv_bwd_workspace(plan) bytes (16-byte aligned).
 *   The workspace holds fp32 partials of dw whatever the dtype.
 * Errors: UNSUPPORTED for an explicit plan; INVALID_ARG for a short workspace
 * or arrays that are not aligned to their element size.
 * ---------------------------------------------------------------------- */
int distdl_conv_fwd(distdl_plan* plan, void* const x_bufs_dev[], const void* w_dev, const void* bias_dev,
                    void* const y_dev[], void* stream);
int distdl_conv_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* w_dev,
                    const void* const dy_dev[], void* const dx_bufs_dev[], void* dw_dev, void* dbias_dev,
                    void* workspace_dev, size_t workspace_bytes, void* stream);
size_t distdl_conv_bwd_workspace(const distdl_plan* plan);

/* The local steps of the same two algorithms alone, for callers that apply H
 * and H* themselves (several layers sharing one exchange, the channel-
 * partitioned layer, tests of the step order): conv_local_fwd is y^ <-
 * Conv(w, b; x^) on buffers that already hold H x; conv_local_bwd is (dw, db,
 * dx^) <- [dConv]*(dy) with the sum-reduce of dw and db over the workers and
 * WITHOUT dx <- H* dx: every cell of the padded dx buffers, halo and padding
 * cells included, holds its local gradient.  distdl_halo_adj on the dx
 * buffers completes the step.  Arguments and errors as above. */
int distdl_conv_local_fwd(distdl_plan* plan, void* const x_bufs_dev[], const void* w_dev, const void* bias_dev,
                          void* const y_dev[], void* stream);
int distdl_conv_local_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* w_dev,
                          const void* const dy_dev[], void* const dx_bufs_dev[], void* dw_dev, void* dbias_dev,
                          void* workspace_dev, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Layout conversion.  Sec. 4 "Sparse layers" writes a worker's tensors in the
 * logical order n_b x n_c x m_0 x ... x m_{D-1}; a caller that stores them
 * that way (planes first: [n_b][n_c][cells], cells row-major) converts to and
 * from the channels-last arrays every other call of this library takes.
 *   what = 0: the padded buffers, n_c_in channels, cells = buf_0 * ... (also
 *             the dx buffers);  what = 1: the outputs, n_c_out channels,
 *             cells = out_0 * ... (also dy).
 *   to_channels_last != 0: src is planes-first, dst channels-last; 0: the
 *             reverse.  src_dev / dst_dev: one array per worker, of the
 *             plan's dtype, element-aligned, not overlapping.
 * A pure permutation (bit-exact); per sample a transpose of an n_c x cells
 * matrix staged through LDS tiles so that both sides move in contiguous runs.
 * Errors: NULL, INVALID_ARG (what, misaligned arrays), UNSUPPORTED (more than
 * 65535 samples).
 * ---------------------------------------------------------------------- */
int distdl_layout_convert(const distdl_plan* plan, int what, int to_channels_last, const void* const src_dev[],
                          void* const dst_dev[], void* stream);

/* ------------------------------------------------------------------------
 * Partitioned affine layer: the Forward / Adjoint Affine Algorithms of
 * Sec. 4 "Dense layers" on a P_fo x P_fi weight partition; worker (i, j) has
 * id i*P_fi + j and holds W_ij [fo_i][fi_j] row-major.  Feature blocks follow
 * the balanced split.  x_j is [n_b][fi_j], y_i is [n_b][fo_i], row-major.
 *
 * affine_fwd: y_i = sum_j x_j W_ij^T + b_i  -- the broadcast of x_j along
 *   P_fo is a shared read, the sum-reduce along P_fi is the continuation of
 *   the contraction over j (ascending); b_i is added once (it lives on column
 *   j = 0 only).  b_dev, or any b_dev[i], may be NULL.
 * affine_bwd: dW_ij = dy_i^T x_j;  db_i = sum_n dy_i[n][:];  dx_j = sum_i
 *   dy_i W_ij (i ascending).  db_dev may be NULL.
 * fp32: fp32 operands and accumulation.  bf16: bf16 operands, fp32
 * accumulation, outputs rounded to bf16 (nearest even); b and db are bf16.
 * ---------------------------------------------------------------------- */
typedef struct distdl_affine_plan distdl_affine_plan;
int distdl_affine_plan_create(distdl_affine_plan** out, int64_t n_b, int64_t n_fi, int64_t n_fo, int P_fo,
                              int P_fi, distdl_dtype dtype);
int distdl_affine_plan_destroy(distdl_affine_plan* plan);
int distdl_affine_fwd(distdl_affine_plan* plan, const void* const x_dev[], const void* const W_dev[],
                      const void* const b_dev[], void* const y_dev[], void* stream);
int distdl_affine_bwd(distdl_affine_plan* plan, const void* const x_dev[], const void* const W_dev[],
                      const void* const dy_dev[], void* const dx_dev[], void* const dW_dev[],
                      void* const db_dev[], void* stream);

/* ------------------------------------------------------------------------
 * Glue of the example network (Sec. 5, App. C), fp32, channels-last.  Small,
 * latency-bound calls that let a whole partitioned network step run through
 * the library; same conventions as above.  The pooling calls also take bf16
 * plans (bf16 tensors, fp32 arithmetic, results rounded to nearest even).
 *
 * relu_fwd / relu_bwd: point-wise layers need no data movement (Sec. 4):
 *   y = max(x, 0);  dx = x > 0 ? dy : 0, over n arrays of count[i] elements.
 * maxpool_fwd / maxpool_bwd: the Forward / Adjoint Pooling Algorithms of
 *   Sec. 4 on a sliding-kernel plan with n_c_in == n_c_out: x <- H x, then the
 *   local max over each window starting at the worker's origin (which skips
 *   "extra" input, App. B.1); backward routes dy to the first maximum of each
 *   window (row-major tap order) over the whole padded buffer, then dx <- H* dx.
 *   x_bufs_dev of maxpool_bwd must hold H x.  The maximum runs over the cells
 *   of the tensor itself: zero-padding cells never win it and never receive
 *   gradient (the pooling layer of the framework the paper wraps pads with
 *   -inf); a plan in which some window lies entirely in the padding
 *   (padding beyond the kernel's reach) is rejected with UNSUPPORTED.
 * avgpool_fwd / avgpool_bwd: the same two algorithms with the mean as the
 *   local pool: y = (sum of the window's taps) / window size, zero-padding
 *   cells counted as the zeros they hold; it is linear, so the backward call
 *   needs no saved input: dx <- H* ([dPool]* dy), every tap of a window
 *   receiving dy / window size.  Kernel size, stride and dilation are the
 *   plan's, any values the planner accepts (App. B.1 unbalanced cases included).
 * bulk_copy: dense [n_b][in_size..][n_c] per worker <-> the bulk of the padded
 *   buffers (to_bufs != 0: dense -> buffers), the hand-over between two layers
 *   whose partitions of the same tensor agree.
 * repartition_fwd / repartition_adj: the generalized all-to-all of Sec. 3 for
 *   the case the example needs: the plan's per-worker OUTPUT blocks
 *   [n_b][out_size..][n_c_out] -> P_f feature blocks [n_b][f_j] of the
 *   row-major flattening of [n_c][out_0..] (balanced split); the adjoint is
 *   the inverse permutation.
 * mse_fwd_bwd: loss = mean over all elements of (y - t)^2 into *loss_dev (one
 *   double in device memory), dy = 2 (y - t) / N; y, t, dy are lists of n <= 16
 *   arrays.
 * ---------------------------------------------------------------------- */
int distdl_relu_fwd(const void* const x_dev[], void* const y_dev[], const int64_t count[], int n, void* stream);
int distdl_relu_bwd(const void* const x_dev[], const void* const dy_dev[], void* const dx_dev[],
                    const int64_t count[], int n, void* stream);
int distdl_maxpool_fwd(distdl_plan* plan, void* const x_bufs_dev[], void* const y_dev[], void* stream);
int distdl_maxpool_bwd(distdl_plan* plan, const void* const x_bufs_dev[], const void* const dy_dev[],
                       void* const dx_bufs_dev[], void* stream);
int distdl_avgpool_fwd(distdl_plan* plan, void* const x_bufs_dev[], void* const y_dev[], void* stream);
int distdl_avgpool_bwd(distdl_plan* plan, const void* const dy_dev[], void* const dx_bufs_dev[], void* stream);
int distdl_bulk_copy(distdl_plan* plan, void* const dense_dev[], void* const bufs_dev[], int to_bufs, void* stream);
int distdl_repartition_fwd(distdl_plan* plan, const void* const src_dev[], int P_f, void* const dst_dev[],
                           void* stream);
int distdl_repartition_adj(distdl_plan* plan, const void* const gdst_dev[], int P_f, void* const gsrc_dev[],
                           void* stream);
int distdl_mse_fwd_bwd(const void* const y_dev[], const void* const t_dev[], void* const dy_dev[],
                       const int64_t count[], int n, double* loss_dev, void* stream);

/* ------------------------------------------------------------------------
 * Convolution with the channels partitioned as well (Sec. 4, Forward / Adjoint
 * Convolution Algorithms on a P_co x P_ci x feature-space partition; the
 * weights live on the P_co x P_ci grid, the bias on its ci = 0 column), fp32 or
 * bf16 (the partial outputs of the blocks are rounded to bf16 before they are
 * sum-reduced).
 * Channel blocks follow the balanced rule.  With S = prod P spatial workers:
 *   x_bufs_dev[j*S + s]: padded buffer [n_b][buf..][ci_j] of input block j on
 *       spatial worker s (bulk filled; holds H x afterwards, which bwd expects);
 *   w_dev[i*P_ci + j]:   [co_i][ci_j][taps]; bias_dev[i]: [co_i] or null array;
 *   y_dev[i*S + s]:      dense [n_b][out..][co_i].
 * fwd: x_j <- H x_j; y^_ij <- Conv(w_ij, b_i if j == 0; x_j) (the broadcast
 * of x along P_co is a shared read); y_i <- sum over j in ascending order.
 * bwd: (dx^_ij, dw_ij, db_i) <- [dConv]*(dy_i), dw_ij / db_i summed over the
 * spatial workers; dx_j <- sum over i ascending; dx_j <- H* dx_j.  All
 * outputs are overwritten.  Partial results and the backward workspace are
 * plan-owned device memory, allocated on first use.
 * convcp_block_plan returns the sliding-kernel plan of block (i, j) (owned by
 * the layer plan) for geometry queries; convcp_channels the channel range of
 * input block (output_side = 0) or output block (1).
 * ---------------------------------------------------------------------- */
typedef struct distdl_convcp_plan distdl_convcp_plan;
int distdl_convcp_plan_create(distdl_convcp_plan** out, int D, int64_t n_b, int64_t n_c_in, int64_t n_c_out,
                              const int64_t in_shape[], const int32_t P[], int P_co, int P_ci, const int32_t ksize[],
                              const int32_t stride[], const int32_t padding[], const int32_t dilation[],
                              distdl_dtype dtype);
int distdl_convcp_plan_destroy(distdl_convcp_plan* plan);
const distdl_plan* distdl_convcp_block_plan(const distdl_convcp_plan* plan, int i, int j);
int distdl_convcp_channels(const distdl_convcp_plan* plan, int output_side, int block, int64_t* start, int64_t* size);
int distdl_convcp_fwd(distdl_convcp_plan* plan, void* const x_bufs_dev[], const void* const w_dev[],
                      const void* const bias_dev[], void* const y_dev[], void* stream);
int distdl_convcp_bwd(distdl_convcp_plan* plan, const void* const x_bufs_dev[], const void* const w_dev[],
                      const void* const dy_dev[], void* const dx_bufs_dev[], void* const dw_dev[],
                      void* const dbias_dev[], void* stream);

/* ------------------------------------------------------------------------
 * Generalized all-to-all / repartition (Sec. 3, the "all-to-all" that
 * re-partitions a tensor; App. C uses it between the convolutional and the
 * dense layers).  A tensor of rank R <= 4 and the given shape is held as one
 * dense row-major block per worker of a partition P_src (worker id row-major
 * over P_src, every dimension split by the balanced rule: block r of a length
 * L gets floor(L / P) + (r < L mod P) entries); repart_fwd re-cuts it into
 * the blocks of partition P_dst.  It is a permutation of the elements, so
 * repart_adj (the adjoint) is the inverse: it takes blocks of P_dst and
 * writes the blocks of P_src.  Outputs are overwritten in full.
 *   repart_plan_block: start[R] / size[R] of block `worker` of side 0 (P_src)
 *   or 1 (P_dst); repart_plan_num_blocks: number of blocks of that side.
 *   src_dev / dst_dev: one device pointer per block of the respective side,
 *   element-aligned; 16-byte accesses are used when every pointer is 16-byte
 *   aligned and every block row and intersection is a whole number of
 *   16-byte vectors.  Source and destination blocks must not overlap.
 * Errors: INVALID_ARG for bad rank / extents, EMPTY_PARTITION when a dimension
 * is split into more parts than it has entries, UNSUPPORTED for blocks beyond
 * 2^32 elements per leading index, NULL for null or misaligned pointers.
 * ---------------------------------------------------------------------- */
typedef struct distdl_repart_plan distdl_repart_plan;
int distdl_repart_plan_create(distdl_repart_plan** out, int R, const int64_t shape[], const int32_t P_src[],
                              const int32_t P_dst[], distdl_dtype dtype);
int distdl_repart_plan_destroy(distdl_repart_plan* plan);
int distdl_repart_plan_num_blocks(const distdl_repart_plan* plan, int side);
int distdl_repart_plan_block(const distdl_repart_plan* plan, int side, int worker, int64_t start[], int64_t size[]);
int distdl_repart_fwd(distdl_repart_plan* plan, const void* const src_dev[], void* const dst_dev[], void* stream);
int distdl_repart_adj(distdl_repart_plan* plan, const void* const gdst_dev[], void* const gsrc_dev[], void* stream);

/* ------------------------------------------------------------------------
 * All-reduce A = B R (Sec. 3 "Sum-reduce and all-reduce": the sum-reduction
 * composed with the broadcast; self-adjoint).  In place: every one of the k
 * replicas of group g, bufs_dev[g*k + i], ends as the sum of the group's
 * replicas, added in index order i = 0 .. k-1 (so all replicas end
 * bit-identical).  Replicas of a group must not overlap.  Errors as for the
 * calls above.
 * ---------------------------------------------------------------------- */
int distdl_allreduce(void* const bufs_dev[], const int64_t count[], int G, int k, distdl_dtype dtype, void* stream);

/* ------------------------------------------------------------------------
 * Euclidean inner product over a list of device arrays (Sec. 2, second
 * displayed equation; the direct sum over workers of Sec. 3), accumulated in
 * fp64 on the device.  result_dev points to ONE double in device memory.
 * Used for the adjoint test |<Fx,y> - <x,F*y>| / max(...) (Sec. 3
 * "Implementation") on device-resident data.  The calls of one device share
 * a buffer of partial sums (as distdl_mse_fwd_bwd calls do): calls that
 * overlap in time on different streams race.
 * ---------------------------------------------------------------------- */
int distdl_dot(const void* const a_dev[], const void* const b_dev[], const int64_t count[], int n_arrays,
               distdl_dtype dtype, double* result_dev, void* stream);

/* distdl_dot for callers that cannot allocate device memory: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels, summation order and result as
 * distdl_dot; the partial sums live in a device array that is part of the
 * library's code object (8 KiB per GPU, held until the process ends), so the
 * call allocates nothing, copies no table and frees nothing.  Limit: at most
 * 96 array pairs (INVALID_ARG beyond; distdl_dot has no limit).  All calls
 * on one GPU share that array: it keeps the last call's partial sums, which
 * the next call overwrites before it reads them, and calls that overlap in
 * time on one GPU race.  The first call on a device looks the array's address
 * up; make it before a capture starts. */
int distdl_dot_static(const void* const a_dev[], const void* const b_dev[], const int64_t count[], int n_arrays,
                      distdl_dtype dtype, double* result_dev, void* stream);

/* ------------------------------------------------------------------------
 * Measurement support.  plan_stats: cell counts behind the algorithmic-bytes
 * figures of the halo kernels, summed over all workers and per sample and
 * channel: out[0] halo cells (in-domain, non-owned), out[1] zero-padding
 * cells, out[2] bulk cells of which some other worker holds a copy (the band
 * the adjoint adds into), out[3] halo cells the adjoint gathers (= out[0]).
 * profile_enable(1) makes every kernel launch of the library be bracketed by
 * two HIP events on the launch stream; profile_report waits for them and
 * writes one line "name launches total_ms" per kernel name into out (a
 * NUL-terminated text of at most cap bytes), then forgets them.  Returns the
 * text length.  Not thread-safe; meant for the benchmark.
 * ---------------------------------------------------------------------- */
int distdl_plan_stats(const distdl_plan* plan, int64_t out[4]);
/* copy_ref: a plain streaming device-to-device copy of `bytes` bytes (16-byte
 * aligned pointers, a multiple of 16 bytes), one 16-byte vector per thread:
 * the yardstick "what a copy reaches on this chip" that the benchmark quotes
 * next to the movement kernels, under a kernel name of its own. */
int distdl_copy_ref(const void* src_dev, void* dst_dev, size_t bytes, void* stream);
int distdl_profile_enable(int on);
int distdl_profile_report(char* out, size_t cap);

/* ------------------------------------------------------------------------
 * Introspection of the host planner (for tests that run without a GPU): the
 * one-pass halo kernels are driven by a table of box tasks.  Task `index` of
 * the forward (adjoint = 0) or adjoint table is written to out[] as
 *   dst_worker, nsrc, org[3], ext[3], then per source: worker, org[3]
 * in buffer-cell coordinates of 3 feature dims (leading dims of extent 1 when
 * D < 3).  nsrc = 0: zero fill; forward nsrc = 1: dst box <- source box;
 * adjoint nsrc >= 1: dst box += each source box, source boxes <- 0.
 * get_task returns the number of ints written.
 * ---------------------------------------------------------------------- */
int distdl_debug_task_count(const distdl_plan* plan, int adjoint);
/* Kernel family the convolution calls would pick for this plan when every
 * array is 16-byte aligned: out[0] forward, out[1] data gradient, out[2]
 * weight gradient; 0 = direct kernels (any shape), 1 = 32-wide matrix-core
 * tiles, 2 = 16-wide matrix-core tiles (at most 16 channels). */
int distdl_debug_conv_path(const distdl_plan* plan, int32_t out[3]);
/* Runs the replacement policy of the cached device tables (see Conventions)
 * on a sequence of n calls without touching a device: call i arrives on
 * stream stream_id[i] with table contents table_id[i], during stream capture
 * if capturing[i] != 0.  slot_out[i] is the index of the device copy the call
 * would use, or the negative error code it would fail with. */
int distdl_debug_slot_policy(const int32_t stream_id[], const int32_t table_id[], const int32_t capturing[], int n,
                             int32_t slot_out[]);
/* floor(n / d) through the multiply-shift constants the kernels use to decode
 * a flat work index (d >= 1). */
uint32_t distdl_debug_fastdiv(uint32_t n, uint32_t d);
int distdl_debug_get_task(const distdl_plan* plan, int adjoint, int index, int32_t out[], int cap);

const char* distdl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DISTDL_H */
