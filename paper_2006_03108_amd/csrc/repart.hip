// Generalized all-to-all (Sec. 3 "all-to-all" / repartition; App. C uses it between the convolutional and the
// dense layers): the same tensor, held as the dense row-major blocks of one balanced partition, re-cut into
// the blocks of another.  Every (destination block, source block) pair with a non-empty intersection is one
// box copy; the boxes run on the halo exchange's copy kernel.  The operator is a permutation of the tensor's
// elements, so its adjoint is the inverse re-cut: the same table with the roles of the two sides swapped.
#include <algorithm>
#include <cstring>
#include <vector>

#include "common.h"
#include "profile.h"

namespace distdl {
extern const int kHaloUnitsPerBlock;
int run_box_copy(int unit_bytes, const BlockRef* d_blocks, const HaloTaskDev* d_tasks, size_t nblocks, void* const* d_bufs,
                 const char* name, hipStream_t st);

constexpr int kRepartDims = 4;

struct RepartSide {
  int32_t P[kRepartDims];
  int n_workers = 1;
  std::vector<int64_t> start[kRepartDims], size[kRepartDims];  // per dimension, per coordinate
  void coords(int w, int c[kRepartDims]) const {
    for (int d = kRepartDims - 1; d >= 0; --d) {
      c[d] = w % P[d];
      w /= P[d];
    }
  }
};

struct RepartTable {  // one direction, one vector width
  std::vector<HaloTaskDev> tasks;
  std::vector<BlockRef> blocks;
  HaloTaskDev* d_tasks = nullptr;
  BlockRef* d_blocks = nullptr;
};
}  // namespace distdl

struct distdl_repart_plan {
  int R = 0;
  int64_t shape[distdl::kRepartDims] = {1, 1, 1, 1};
  distdl_dtype dtype = DISTDL_F32;
  distdl::RepartSide side[2];            // 0: source partition, 1: destination partition
  distdl::RepartTable tab[2][2];         // [direction: 0 fwd, 1 adj][0: 16-byte units, 1: element units]
  bool wide_ok = false;                  // the 16-byte tables exist
  bool on_device = false;
  distdl::PtrTable ptrs;
};

namespace distdl {

static void split_side(RepartSide& s, const int64_t shape[kRepartDims]) {
  s.n_workers = 1;
  for (int d = 0; d < kRepartDims; ++d) {
    s.start[d].resize(s.P[d]);
    s.size[d].resize(s.P[d]);
    int64_t at = 0;
    for (int r = 0; r < s.P[d]; ++r) {  // balanced rule: floor(L / P) + (r < L mod P)
      const int64_t z = shape[d] / s.P[d] + (r < shape[d] % s.P[d] ? 1 : 0);
      s.start[d][r] = at;
      s.size[d][r] = z;
      at += z;
    }
    s.n_workers *= s.P[d];
  }
}

// view of box [lo, lo + ext) (global coordinates) inside block `w` of side `s`, in units of `vec` elements
static HaloView make_view(const RepartSide& s, int w, int ptr_index, const int64_t lo[kRepartDims], int vec) {
  int c[kRepartDims];
  s.coords(w, c);
  int64_t bs[kRepartDims], off[kRepartDims];
  for (int d = 0; d < kRepartDims; ++d) {
    bs[d] = s.size[d][c[d]];
    off[d] = lo[d] - s.start[d][c[d]];
  }
  HaloView v{};
  v.worker = ptr_index;
  v.s1 = (uint32_t)(bs[3] / vec);
  v.s0 = (uint32_t)(bs[2] * (bs[3] / vec));
  v.sn = (uint64_t)bs[1] * v.s0;
  v.base = (uint64_t)off[0] * v.sn + (uint64_t)off[1] * v.s0 + (uint64_t)off[2] * v.s1 + (uint64_t)(off[3] / vec);
  return v;
}

// All copy boxes from partition `from` to partition `to`; false if something does not fit the kernel's 32-bit
// strides, or (vec > 1) if a block row or an intersection is not a whole number of vectors.
static bool build_table(const distdl_repart_plan& p, int from, int to, int vec, RepartTable& out) {
  const RepartSide &S = p.side[from], &D = p.side[to];
  // pointer table: [source pointers of the call][destination pointers of the call]
  for (int wd = 0; wd < D.n_workers; ++wd) {
    int cd[kRepartDims];
    D.coords(wd, cd);
    for (int ws = 0; ws < S.n_workers; ++ws) {
      int cs[kRepartDims];
      S.coords(ws, cs);
      int64_t lo[kRepartDims], ext[kRepartDims];
      bool empty = false;
      for (int d = 0; d < kRepartDims; ++d) {
        lo[d] = std::max(S.start[d][cs[d]], D.start[d][cd[d]]);
        const int64_t hi = std::min(S.start[d][cs[d]] + S.size[d][cs[d]], D.start[d][cd[d]] + D.size[d][cd[d]]);
        ext[d] = hi - lo[d];
        empty |= ext[d] <= 0;
      }
      if (empty) continue;
      if (vec > 1) {  // rows of both blocks, the box's row and its offsets must be whole vectors
        if (S.size[3][cs[3]] % vec || D.size[3][cd[3]] % vec || ext[3] % vec || (lo[3] - S.start[3][cs[3]]) % vec ||
            (lo[3] - D.start[3][cd[3]]) % vec)
          return false;
      }
      for (const RepartSide* side : {&S, &D}) {
        const int* c = side == &S ? cs : cd;
        if ((double)side->size[1][c[1]] * side->size[2][c[2]] * side->size[3][c[3]] >= 4294967296.0) return false;
      }
      HaloTaskDev t{};
      t.src0 = make_view(S, ws, ws, lo, vec);
      t.dst = make_view(D, wd, S.n_workers + wd, lo, vec);
      t.nsrc = 1;
      t.src_begin = 0;
      const int64_t row = ext[3] / vec;
      const int64_t total = ext[0] * ext[1] * ext[2] * row;
      if (total >= (int64_t(1) << 32)) return false;
      t.total = (uint32_t)total;
      t.div_row = make_fastdiv((uint32_t)row);
      t.div_e1 = make_fastdiv((uint32_t)ext[2]);
      t.div_e0 = make_fastdiv((uint32_t)ext[1]);
      const int id = (int)out.tasks.size();
      out.tasks.push_back(t);
      for (int64_t u = 0; u < total; u += kHaloUnitsPerBlock) out.blocks.push_back(BlockRef{id, (uint32_t)u});
    }
  }
  return true;
}

template <class T>
static int to_dev(const std::vector<T>& v, T** out) {
  *out = nullptr;
  if (v.empty()) return DISTDL_OK;
  DISTDL_HIP_TRY(hipMalloc((void**)out, v.size() * sizeof(T)));
  DISTDL_HIP_TRY(hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return DISTDL_OK;
}

static int run_repart(distdl_repart_plan* p, int dir, const void* const from_dev[], void* const to_dev_[], hipStream_t st) {
  if (!p || !from_dev || !to_dev_) return set_error(DISTDL_ERR_NULL, "repart: null argument");
  const RepartSide &S = p->side[dir], &D = p->side[1 - dir];
  const size_t esz = dtype_size(p->dtype);
  bool aligned16 = true;
  std::vector<const void*> all((size_t)S.n_workers + D.n_workers);
  for (int w = 0; w < S.n_workers + D.n_workers; ++w) {
    const void* ptr = w < S.n_workers ? from_dev[w] : to_dev_[w - S.n_workers];
    if (!ptr || (uintptr_t)ptr % esz) return set_error(DISTDL_ERR_NULL, "repart: block %d null or misaligned", w);
    aligned16 &= (uintptr_t)ptr % 16 == 0;
    all[w] = ptr;
  }
  int rc;
  if (!p->on_device) {
    for (int d = 0; d < 2; ++d)
      for (int v = 0; v < 2; ++v) {
        RepartTable& t = p->tab[d][v];
        if ((rc = to_dev(t.tasks, &t.d_tasks)) || (rc = to_dev(t.blocks, &t.d_blocks))) return rc;
      }
    p->on_device = true;
  }
  if ((rc = p->ptrs.upload(all.data(), all.size(), st))) return rc;
  const bool wide = aligned16 && p->wide_ok;
  const RepartTable& t = p->tab[dir][wide ? 0 : 1];
  return run_box_copy(wide ? 16 : (int)esz, t.d_blocks, t.d_tasks, t.blocks.size(), p->ptrs.dev,
                      dir == 0 ? "repart_fwd" : "repart_adj", st);
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_repart_plan_create(distdl_repart_plan** out, int R, const int64_t shape[], const int32_t P_src[],
                              const int32_t P_dst[], distdl_dtype dtype) {
  if (!out || !shape || !P_src || !P_dst) return set_error(DISTDL_ERR_NULL, "repart_plan_create: null argument");
  *out = nullptr;
  if (R < 1 || R > kRepartDims) return set_error(DISTDL_ERR_INVALID_ARG, "repart: R = %d not in 1..%d", R, kRepartDims);
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  distdl_repart_plan* p = new (std::nothrow) distdl_repart_plan();
  if (!p) return set_error(DISTDL_ERR_NOMEM, "out of host memory");
  p->R = R;
  p->dtype = dtype;
  const int lead = kRepartDims - R;
  for (int d = 0; d < kRepartDims; ++d) p->side[0].P[d] = p->side[1].P[d] = 1;
  for (int d = 0; d < R; ++d) {
    if (shape[d] < 1 || P_src[d] < 1 || P_dst[d] < 1 || shape[d] >= (int64_t(1) << 31)) {
      delete p;
      return set_error(DISTDL_ERR_INVALID_ARG, "repart: dimension %d: bad extent or partition", d);
    }
    if (P_src[d] > shape[d] || P_dst[d] > shape[d]) {
      delete p;
      return set_error(DISTDL_ERR_EMPTY_PARTITION, "repart: dimension %d of extent %lld split %d / %d ways", d,
                       (long long)shape[d], P_src[d], P_dst[d]);
    }
    p->shape[lead + d] = shape[d];
    p->side[0].P[lead + d] = P_src[d];
    p->side[1].P[lead + d] = P_dst[d];
  }
  split_side(p->side[0], p->shape);
  split_side(p->side[1], p->shape);
  if ((int64_t)p->side[0].n_workers * p->side[1].n_workers > (int64_t(1) << 22)) {
    delete p;
    return set_error(DISTDL_ERR_UNSUPPORTED, "repart: too many block pairs");
  }
  const int vec16 = (int)(16 / dtype_size(dtype));
  RepartTable w0, w1;
  p->wide_ok = build_table(*p, 0, 1, vec16, w0) && build_table(*p, 1, 0, vec16, w1);
  if (p->wide_ok) p->tab[0][0] = w0, p->tab[1][0] = w1;
  if (!build_table(*p, 0, 1, 1, p->tab[0][1]) || !build_table(*p, 1, 0, 1, p->tab[1][1])) {
    delete p;
    return set_error(DISTDL_ERR_UNSUPPORTED, "repart: a block is too large for 32-bit strides");
  }
  *out = p;
  return DISTDL_OK;
}

int distdl_repart_plan_destroy(distdl_repart_plan* p) {
  if (!p) return DISTDL_OK;
  for (int d = 0; d < 2; ++d)
    for (int v = 0; v < 2; ++v) {
      if (p->tab[d][v].d_tasks) (void)hipFree(p->tab[d][v].d_tasks);
      if (p->tab[d][v].d_blocks) (void)hipFree(p->tab[d][v].d_blocks);
    }
  p->ptrs.release();
  delete p;
  return DISTDL_OK;
}

int distdl_repart_plan_num_blocks(const distdl_repart_plan* p, int side) {
  if (!p || side < 0 || side > 1) return set_error(DISTDL_ERR_INVALID_ARG, "repart_plan_num_blocks: bad argument");
  return p->side[side].n_workers;
}

int distdl_repart_plan_block(const distdl_repart_plan* p, int side, int worker, int64_t start[], int64_t size[]) {
  if (!p || !start || !size || side < 0 || side > 1) return set_error(DISTDL_ERR_INVALID_ARG, "repart_plan_block: bad argument");
  const RepartSide& s = p->side[side];
  if (worker < 0 || worker >= s.n_workers) return set_error(DISTDL_ERR_INVALID_ARG, "repart_plan_block: worker %d", worker);
  int c[kRepartDims];
  s.coords(worker, c);
  const int lead = kRepartDims - p->R;
  for (int d = 0; d < p->R; ++d) {
    start[d] = s.start[lead + d][c[lead + d]];
    size[d] = s.size[lead + d][c[lead + d]];
  }
  return DISTDL_OK;
}

int distdl_repart_fwd(distdl_repart_plan* plan, const void* const src_dev[], void* const dst_dev[], void* stream) {
  return run_repart(plan, 0, src_dev, dst_dev, (hipStream_t)stream);
}

int distdl_repart_adj(distdl_repart_plan* plan, const void* const gdst_dev[], void* const gsrc_dev[], void* stream) {
  return run_repart(plan, 1, gdst_dev, gsrc_dev, (hipStream_t)stream);
}

}  // extern "C"
