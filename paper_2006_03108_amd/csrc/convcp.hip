// Convolution on a P_co x P_ci x (feature space) partition: the full Forward / Adjoint Convolution Algorithms
// of Sec. 4, where the broadcast of x along P_co and the sum-reduce of y^ along P_ci are not trivial.
//   forward:  x_j <- H x_j;  y^_ij <- Conv(w_ij, b_i [j == 0]; x_j)  (every co block reads the same x_j: the
//             broadcast B along P_co is a shared read);  y_i <- R over j of y^_ij
//   adjoint:  (dx^_ij, dw_ij, db_i [j == 0]) <- [dConv]*(dy_i)  (B along P_ci of dy_i is a shared read; dw and
//             db are summed over the spatial workers inside the layer call);  dx_j <- R over i of dx^_ij;
//             dx_j <- H* dx_j
// Every (i, j) block runs the single-block layer kernels on a plan of its own channel counts; the two
// sum-reduces run on the reduce kernel in block order (j resp. i ascending).  fp32.
#include <algorithm>
#include <vector>

#include "common.h"
#include "conv_core.h"
#include "distdl.h"
#include "profile.h"

struct distdl_convcp_plan {
  int D = 0, P_co = 1, P_ci = 1, S = 0;
  int64_t n_b = 0, n_ci = 0, n_co = 0;
  std::vector<int64_t> co_start, co_size, ci_start, ci_size;
  std::vector<distdl_plan*> sub;  // [i * P_ci + j]
  char* d_tmp = nullptr;          // y^_ij (forward) or dx^_ij (adjoint) partials, in the layer's element type
  size_t tmp_floats = 0;          // its size in bytes
  distdl_dtype dtype = DISTDL_F32;
  void* d_ws = nullptr;           // workspace of the single-block backward call
  size_t ws_bytes = 0;
};

namespace distdl {

static void balanced(int64_t n, int parts, std::vector<int64_t>& start, std::vector<int64_t>& size) {
  start.resize(parts);
  size.resize(parts);
  int64_t at = 0;
  for (int r = 0; r < parts; ++r) {
    size[r] = n / parts + (r < n % parts ? 1 : 0);
    start[r] = at;
    at += size[r];
  }
}

static int ensure(void** p, size_t* have, size_t want) {
  if (*have >= want) return DISTDL_OK;
  if (*p) (void)hipFree(*p);
  *p = nullptr;
  *have = 0;
  DISTDL_HIP_TRY(hipMalloc(p, want));
  *have = want;
  return DISTDL_OK;
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_convcp_plan_create(distdl_convcp_plan** out, int D, int64_t n_b, int64_t n_c_in, int64_t n_c_out,
                              const int64_t in_shape[], const int32_t P[], int P_co, int P_ci, const int32_t ksize[],
                              const int32_t stride[], const int32_t padding[], const int32_t dilation[],
                              distdl_dtype dtype) {
  if (!out) return set_error(DISTDL_ERR_NULL, "convcp_plan_create: null argument");
  *out = nullptr;
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_INVALID_ARG, "convcp: unknown dtype");
  if (P_co < 1 || P_ci < 1) return set_error(DISTDL_ERR_INVALID_ARG, "convcp: P_co = %d, P_ci = %d", P_co, P_ci);
  if (P_co > n_c_out || P_ci > n_c_in)
    return set_error(DISTDL_ERR_EMPTY_PARTITION, "convcp: more channel blocks than channels");
  distdl_convcp_plan* p = new (std::nothrow) distdl_convcp_plan();
  if (!p) return set_error(DISTDL_ERR_NOMEM, "out of host memory");
  p->D = D;
  p->P_co = P_co;
  p->P_ci = P_ci;
  p->n_b = n_b;
  p->n_ci = n_c_in;
  p->n_co = n_c_out;
  p->dtype = dtype;
  balanced(n_c_out, P_co, p->co_start, p->co_size);
  balanced(n_c_in, P_ci, p->ci_start, p->ci_size);
  p->sub.assign((size_t)P_co * P_ci, nullptr);
  for (int i = 0; i < P_co; ++i)
    for (int j = 0; j < P_ci; ++j) {
      int rc = distdl_plan_create(&p->sub[(size_t)i * P_ci + j], D, n_b, p->ci_size[j], p->co_size[i], in_shape, P, ksize,
                                  stride, padding, dilation, dtype);
      if (rc) {
        distdl_convcp_plan_destroy(p);
        return rc;
      }
    }
  p->S = distdl_plan_num_workers(p->sub[0]);
  *out = p;
  return DISTDL_OK;
}

int distdl_convcp_plan_destroy(distdl_convcp_plan* p) {
  if (!p) return DISTDL_OK;
  for (distdl_plan* s : p->sub)
    if (s) distdl_plan_destroy(s);
  if (p->d_tmp) (void)hipFree(p->d_tmp);
  if (p->d_ws) (void)hipFree(p->d_ws);
  delete p;
  return DISTDL_OK;
}

const distdl_plan* distdl_convcp_block_plan(const distdl_convcp_plan* p, int i, int j) {
  if (!p || i < 0 || i >= p->P_co || j < 0 || j >= p->P_ci) {
    set_error(DISTDL_ERR_INVALID_ARG, "convcp_block_plan: bad argument");
    return nullptr;
  }
  return p->sub[(size_t)i * p->P_ci + j];
}

int distdl_convcp_channels(const distdl_convcp_plan* p, int output_side, int block, int64_t* start, int64_t* size) {
  if (!p || !start || !size) return set_error(DISTDL_ERR_NULL, "convcp_channels: null argument");
  const std::vector<int64_t>& st = output_side ? p->co_start : p->ci_start;
  const std::vector<int64_t>& sz = output_side ? p->co_size : p->ci_size;
  if (block < 0 || block >= (int)st.size()) return set_error(DISTDL_ERR_INVALID_ARG, "convcp_channels: block %d", block);
  *start = st[block];
  *size = sz[block];
  return DISTDL_OK;
}

int distdl_convcp_fwd(distdl_convcp_plan* p, void* const x_bufs_dev[], const void* const w_dev[],
                      const void* const bias_dev[], void* const y_dev[], void* stream) {
  if (!p || !x_bufs_dev || !w_dev || !y_dev) return set_error(DISTDL_ERR_NULL, "convcp_fwd: null argument");
  hipStream_t st = (hipStream_t)stream;
  const int S = p->S, Pco = p->P_co, Pci = p->P_ci;
  int rc;
  for (int i = 0; i < Pco * Pci; ++i)
    if (!w_dev[i]) return set_error(DISTDL_ERR_NULL, "convcp_fwd: weight block %d is null", i);
  // y^_ij partials (only when there is something to sum)
  std::vector<int64_t> ycount((size_t)Pco * S);
  size_t tmp = 0;
  for (int i = 0; i < Pco; ++i)
    for (int s = 0; s < S; ++s) {
      distdl_worker_geom g;
      if ((rc = distdl_plan_query(p->sub[(size_t)i * Pci], s, &g))) return rc;
      int64_t cells = p->n_b;
      for (int d = 0; d < p->D; ++d) cells *= g.out_size[d];
      ycount[(size_t)i * S + s] = cells * p->co_size[i];
      tmp += (size_t)ycount[(size_t)i * S + s] * Pci;
    }
  const size_t esz = p->dtype == DISTDL_BF16 ? 2 : 4;
  if (Pci > 1 && (rc = ensure((void**)&p->d_tmp, &p->tmp_floats, tmp * esz + 16 * (size_t)Pco * Pci * S))) return rc;
  for (int j = 0; j < Pci; ++j) {  // x_j <- H x_j, once per input block
    distdl_plan* pj = p->sub[j];
    if ((rc = run_halo(pj, false, pj->tab_x, x_bufs_dev + (size_t)j * S, st))) return rc;
  }
  std::vector<void*> parts((size_t)Pco * S * Pci);  // [(i, s)][j]
  char* at = p->d_tmp;
  for (int i = 0; i < Pco; ++i) {
    for (int j = 0; j < Pci; ++j) {
      std::vector<void*> target(S);
      for (int s = 0; s < S; ++s) {
        if (Pci == 1) {
          target[s] = y_dev[(size_t)i * S + s];
        } else {
          target[s] = at;
          parts[((size_t)i * S + s) * Pci + j] = at;
          at += (ycount[(size_t)i * S + s] * esz + 15) / 16 * 16;  // every partial starts 16-byte aligned
        }
      }
      const void* b = (bias_dev && j == 0) ? bias_dev[i] : nullptr;  // the bias lives on the ci = 0 sub-partition
      if ((rc = conv_fwd_core(p->sub[(size_t)i * Pci + j], x_bufs_dev + (size_t)j * S, w_dev[(size_t)i * Pci + j], b,
                              target.data(), st, false)))
        return rc;
    }
  }
  if (Pci > 1)  // y_i <- R over j
    return distdl_sumreduce_fwd(parts.data(), y_dev, ycount.data(), Pco * S, Pci, p->dtype, 0, stream);
  return DISTDL_OK;
}

int distdl_convcp_bwd(distdl_convcp_plan* p, const void* const x_bufs_dev[], const void* const w_dev[],
                      const void* const dy_dev[], void* const dx_bufs_dev[], void* const dw_dev[],
                      void* const dbias_dev[], void* stream) {
  if (!p || !x_bufs_dev || !w_dev || !dy_dev || !dx_bufs_dev || !dw_dev)
    return set_error(DISTDL_ERR_NULL, "convcp_bwd: null argument");
  hipStream_t st = (hipStream_t)stream;
  const int S = p->S, Pco = p->P_co, Pci = p->P_ci;
  int rc;
  for (int i = 0; i < Pco * Pci; ++i)
    if (!w_dev[i] || !dw_dev[i]) return set_error(DISTDL_ERR_NULL, "convcp_bwd: weight block %d is null", i);
  std::vector<int64_t> xcount((size_t)Pci * S);
  size_t tmp = 0, ws = 16;
  for (int j = 0; j < Pci; ++j)
    for (int s = 0; s < S; ++s) {
      distdl_worker_geom g;
      if ((rc = distdl_plan_query(p->sub[j], s, &g))) return rc;
      int64_t cells = p->n_b;
      for (int d = 0; d < p->D; ++d) cells *= g.buf_shape[d];
      xcount[(size_t)j * S + s] = cells * p->ci_size[j];
      tmp += (size_t)xcount[(size_t)j * S + s] * Pco;
    }
  for (distdl_plan* sp : p->sub) ws = std::max(ws, distdl_conv_bwd_workspace(sp));
  const size_t esz = p->dtype == DISTDL_BF16 ? 2 : 4;
  if (Pco > 1 && (rc = ensure((void**)&p->d_tmp, &p->tmp_floats, tmp * esz + 16 * (size_t)Pco * Pci * S))) return rc;
  if ((rc = ensure(&p->d_ws, &p->ws_bytes, ws))) return rc;
  std::vector<void*> parts((size_t)Pci * S * Pco);  // [(j, s)][i]
  char* at = p->d_tmp;
  for (int i = 0; i < Pco; ++i) {
    for (int j = 0; j < Pci; ++j) {
      std::vector<void*> target(S);
      for (int s = 0; s < S; ++s) {
        if (Pco == 1) {
          target[s] = dx_bufs_dev[(size_t)j * S + s];
        } else {
          target[s] = at;
          parts[((size_t)j * S + s) * Pco + i] = at;
          at += (xcount[(size_t)j * S + s] * esz + 15) / 16 * 16;
        }
      }
      void* db = (dbias_dev && j == 0) ? dbias_dev[i] : nullptr;
      if ((rc = conv_bwd_core(p->sub[(size_t)i * Pci + j], x_bufs_dev + (size_t)j * S, w_dev[(size_t)i * Pci + j],
                              dy_dev + (size_t)i * S, target.data(), dw_dev[(size_t)i * Pci + j], db, p->d_ws, p->ws_bytes,
                              st, false)))
        return rc;
    }
  }
  if (Pco > 1 &&  // dx_j <- R over i
      (rc = distdl_sumreduce_fwd(parts.data(), dx_bufs_dev, xcount.data(), Pci * S, Pco, p->dtype, 0, stream)))
    return rc;
  for (int j = 0; j < Pci; ++j) {  // dx_j <- H* dx_j
    distdl_plan* pj = p->sub[j];
    if ((rc = run_halo(pj, true, pj->tab_dx, dx_bufs_dev + (size_t)j * S, st))) return rc;
  }
  return DISTDL_OK;
}

}  // extern "C"
