// Host-side planner: partition geometry (Sec. 3 "Halo exchange", App. B.1) and
// the box-task tables that drive the one-pass halo kernels.
#include <algorithm>
#include <cstring>
#include <new>

#include "common.h"

namespace distdl {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

int SlotCache::upload(const void* bytes, size_t nbytes, hipStream_t stream, int capturing, bool simulate) {
  ++clock;
  if (capturing < 0) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    DISTDL_HIP_TRY(hipStreamIsCapturing(stream, &cs));
    capturing = cs != hipStreamCaptureStatusNone;
  }
  int pick = -1;
  for (size_t i = 0; i < entries.size(); ++i) {
    const Entry& e = entries[i];
    if (e.live && e.stream == stream && e.host.size() == nbytes && std::memcmp(e.host.data(), bytes, nbytes) == 0) {
      pick = (int)i;
      break;
    }
  }
  if (pick < 0) {
    if (capturing)
      return set_error(DISTDL_ERR_INVALID_ARG,
                       "a call with new pointer arrays or shapes cannot be recorded into a graph: make it once on "
                       "this stream before the capture starts");
    // blocks this call may rewrite: unpinned ones last used on this very stream
    int lru = -1, mine = 0;
    for (size_t i = 0; i < entries.size(); ++i) {
      const Entry& e = entries[i];
      if (e.pinned || e.stream != stream) continue;
      ++mine;
      if (lru < 0 || e.used < entries[lru].used) lru = (int)i;
    }
    if (mine >= kSlots || ((int)entries.size() >= kMaxSlots && lru >= 0)) {
      pick = lru;
    } else if ((int)entries.size() < kMaxSlots) {
      entries.emplace_back();
      pick = (int)entries.size() - 1;
    } else {
      return set_error(DISTDL_ERR_NOMEM,
                       "all %d table blocks of this call site are held by other streams or recorded graphs", kMaxSlots);
    }
    Entry& e = entries[pick];
    if (!simulate) {
      if (nbytes > e.cap) {
        if (e.dev) (void)hipFree(e.dev);  // waits for the device
        e.dev = nullptr;
        e.cap = 0;
        e.live = false;
        DISTDL_HIP_TRY(hipMalloc(&e.dev, std::max<size_t>(nbytes, 16)));
        e.cap = nbytes;
      }
    }
    e.host.assign((const unsigned char*)bytes, (const unsigned char*)bytes + nbytes);
    // pageable source: the runtime stages the bytes before returning, and the copy is ordered on the stream
    // behind earlier kernels that read the block
    if (!simulate && nbytes)
      DISTDL_HIP_TRY(hipMemcpyAsync(e.dev, e.host.data(), nbytes, hipMemcpyHostToDevice, stream));
    e.stream = stream;
    e.live = true;
  }
  Entry& e = entries[pick];
  e.used = clock;
  if (capturing) e.pinned = true;
  selected = pick;
  return DISTDL_OK;
}

void SlotCache::release() {
  for (Entry& e : entries)
    if (e.dev) (void)hipFree(e.dev);
  entries.clear();
  selected = -1;
}

// ---- per-dimension geometry ------------------------------------------------

static void split_balanced(int64_t len, int parts, std::vector<int64_t>& start, std::vector<int64_t>& size) {
  start.resize(parts);
  size.resize(parts);
  int64_t q = len / parts, rem = len % parts, at = 0;
  for (int r = 0; r < parts; ++r) {
    size[r] = q + (r < rem ? 1 : 0);
    start[r] = at;
    at += size[r];
  }
}

static int check_halos(const std::vector<DimGeom>& g, int dim) {
  int parts = (int)g.size();
  for (int r = 0; r < parts; ++r) {
    if (g[r].halo[0] > 0 && (r == 0 || g[r].halo[0] > g[r - 1].in_size))
      return set_error(DISTDL_ERR_HALO_TOO_WIDE, "dim %d worker %d: left halo %d exceeds the neighbour's bulk", dim, r,
                       g[r].halo[0]);
    if (g[r].halo[1] > 0 && (r == parts - 1 || g[r].halo[1] > g[r + 1].in_size))
      return set_error(DISTDL_ERR_HALO_TOO_WIDE, "dim %d worker %d: right halo %d exceeds the neighbour's bulk", dim,
                       r, g[r].halo[1]);
  }
  return DISTDL_OK;
}

static int kernel_dim(int dim, int64_t n, int k, int s, int p, int dil, int parts, std::vector<DimGeom>& out,
                      int64_t* m_out) {
  int64_t span = (int64_t)dil * (k - 1);
  int64_t num = n + 2 * (int64_t)p - span - 1;
  int64_t m = num < 0 ? 0 : num / s + 1;
  *m_out = m;
  if (m < parts || n < parts)
    return set_error(DISTDL_ERR_EMPTY_PARTITION, "dim %d: %lld inputs / %lld outputs over %d workers", dim,
                     (long long)n, (long long)m, parts);
  std::vector<int64_t> is, iz, os, oz;
  split_balanced(n, parts, is, iz);
  split_balanced(m, parts, os, oz);
  out.resize(parts);
  for (int r = 0; r < parts; ++r) {
    DimGeom& g = out[r];
    g.in_start = is[r];
    g.in_size = iz[r];
    g.out_start = os[r];
    g.out_size = oz[r];
    int64_t own_lo = is[r], own_hi = is[r] + iz[r] - 1;
    int64_t need_lo = os[r] * s - p;
    int64_t need_hi = (os[r] + oz[r] - 1) * s - p + span;
    int64_t pl = need_lo < 0 ? -need_lo : 0;
    int64_t pr = need_hi > n - 1 ? need_hi - (n - 1) : 0;
    int64_t lo = std::max<int64_t>(need_lo, 0), hi = std::min<int64_t>(need_hi, n - 1);
    g.pad[0] = (int32_t)pl;
    g.pad[1] = (int32_t)pr;
    g.halo[0] = (int32_t)std::max<int64_t>(0, own_lo - lo);
    g.halo[1] = (int32_t)std::max<int64_t>(0, hi - own_hi);
    g.extra[0] = (int32_t)std::max<int64_t>(0, lo - own_lo);
    g.extra[1] = (int32_t)std::max<int64_t>(0, own_hi - hi);
    g.bulk_off = g.pad[0] + g.halo[0];
    g.buf = g.bulk_off + g.in_size + g.halo[1] + g.pad[1];
    g.origin = need_lo - (own_lo - g.bulk_off);  // == extra[0]
  }
  return check_halos(out, dim);
}

static void unit_dim(std::vector<DimGeom>& out) {
  DimGeom g{};
  g.in_size = g.out_size = g.buf = 1;
  out.assign(1, g);
}

// ---- box tasks ---------------------------------------------------------------

namespace {
enum SegKind { SEG_PAD, SEG_HALO_L, SEG_BULK, SEG_HALO_R };
struct Seg {
  SegKind kind;
  int32_t start, len;
};
struct Interval {  // part of a worker's bulk along one dimension (adjoint side)
  int32_t start, len;  // relative to the first bulk cell
  bool from_left, from_right;
};
}  // namespace

static void finish_task(TaskTable& tt, BoxTask t, int64_t n_b, int64_t n_c, int vec, int units_per_block) {
  int64_t row = (int64_t)t.ext[2] * n_c / vec;
  t.div_row = make_fastdiv((uint32_t)row);
  t.div_e1 = make_fastdiv((uint32_t)t.ext[1]);
  t.div_e0 = make_fastdiv((uint32_t)t.ext[0]);
  int64_t units = n_b * t.ext[0] * t.ext[1] * row;
  int id = (int)tt.tasks.size();
  tt.tasks.push_back(t);
  for (int64_t u = 0; u < units; u += units_per_block) tt.blocks.push_back(BlockRef{id, (uint32_t)u});
}

static const DimGeom& geom_of(const distdl_plan& p, int w, int d, int delta = 0) {
  return p.dims[d][p.coords(w, d) + delta];
}

static int worker_with_delta(const distdl_plan& p, int w, const int delta[3]) {
  int id = 0;
  for (int d = 0; d < 3; ++d) id = id * p.P[d] + p.coords(w, d) + delta[d];
  return id;
}

static void build_forward_table(const distdl_plan& p, TaskTable& tt, int vec, int upb, bool count) {
  for (int w = 0; w < p.n_workers; ++w) {
    std::vector<Seg> segs[3];
    for (int d = 0; d < 3; ++d) {
      const DimGeom& g = geom_of(p, w, d);
      int32_t at = 0;
      auto add = [&](SegKind k, int64_t len) {
        if (len > 0) segs[d].push_back(Seg{k, at, (int32_t)len});
        at += (int32_t)len;
      };
      add(SEG_PAD, g.pad[0]);
      add(SEG_HALO_L, g.halo[0]);
      add(SEG_BULK, g.in_size);
      add(SEG_HALO_R, g.halo[1]);
      add(SEG_PAD, g.pad[1]);
    }
    for (const Seg& s0 : segs[0])
      for (const Seg& s1 : segs[1])
        for (const Seg& s2 : segs[2]) {
          const Seg* s[3] = {&s0, &s1, &s2};
          bool all_bulk = true, any_pad = false;
          for (int d = 0; d < 3; ++d) {
            all_bulk &= s[d]->kind == SEG_BULK;
            any_pad |= s[d]->kind == SEG_PAD;
          }
          if (all_bulk) continue;
          BoxTask t{};
          t.dst_worker = w;
          t.src_begin = (int32_t)tt.srcs.size();
          int64_t cells = 1;
          for (int d = 0; d < 3; ++d) {
            t.org[d] = s[d]->start;
            t.ext[d] = s[d]->len;
            cells *= s[d]->len;
          }
          if (any_pad) {
            t.nsrc = 0;
            if (count) tt.cells_zeroed += cells;
          } else {
            t.nsrc = 1;
            BoxSrc src{};
            int delta[3];
            for (int d = 0; d < 3; ++d) {
              delta[d] = s[d]->kind == SEG_HALO_L ? -1 : s[d]->kind == SEG_HALO_R ? 1 : 0;
              const DimGeom& gn = geom_of(p, w, d, delta[d]);
              if (delta[d] < 0)  // last `len` bulk cells of the left neighbour
                src.org[d] = (int32_t)(gn.bulk_off + gn.in_size - s[d]->len);
              else  // first cells of the right neighbour's bulk, or the same bulk range
                src.org[d] = (int32_t)gn.bulk_off;
            }
            src.worker = worker_with_delta(p, w, delta);
            tt.srcs.push_back(src);
            if (count) tt.cells_copied += cells;
          }
          finish_task(tt, t, p.n_b, p.n_ci, vec, upb);
        }
  }
}

static void build_adjoint_table(const distdl_plan& p, TaskTable& tt, int vec, int upb, bool count) {
  // zero-fill of the padding cells: same boxes as the forward table's
  {
    TaskTable fwd;
    build_forward_table(p, fwd, vec, upb, false);
    for (const BoxTask& t : fwd.tasks)
      if (t.nsrc == 0) {
        BoxTask z = t;
        z.src_begin = (int32_t)tt.srcs.size();
        if (count) tt.cells_zeroed += (int64_t)t.ext[0] * t.ext[1] * t.ext[2];
        finish_task(tt, z, p.n_b, p.n_ci, vec, upb);
      }
  }
  for (int w = 0; w < p.n_workers; ++w) {
    std::vector<Interval> iv[3];
    for (int d = 0; d < 3; ++d) {
      const DimGeom& g = geom_of(p, w, d);
      int r = p.coords(w, d);
      int32_t size = (int32_t)g.in_size;
      int32_t left_cover = r > 0 ? p.dims[d][r - 1].halo[1] : 0;             // bulk cells [0, left_cover)
      int32_t right_cover = r + 1 < p.P[d] ? p.dims[d][r + 1].halo[0] : 0;  // bulk cells [size-right_cover, size)
      int32_t cuts[4] = {0, std::min(left_cover, size), std::max(size - right_cover, 0), size};
      std::sort(cuts, cuts + 4);
      for (int c = 0; c < 3; ++c) {
        int32_t a = cuts[c], b = cuts[c + 1];
        if (b <= a) continue;
        iv[d].push_back(Interval{a, b - a, b <= left_cover, a >= size - right_cover});
      }
    }
    for (const Interval& i0 : iv[0])
      for (const Interval& i1 : iv[1])
        for (const Interval& i2 : iv[2]) {
          const Interval* it[3] = {&i0, &i1, &i2};
          int nopt[3];
          int opt[3][3];  // per dim: deltas available (0 always first)
          int combos = 1;
          for (int d = 0; d < 3; ++d) {
            nopt[d] = 0;
            opt[d][nopt[d]++] = 0;
            if (it[d]->from_left) opt[d][nopt[d]++] = -1;
            if (it[d]->from_right) opt[d][nopt[d]++] = 1;
            combos *= nopt[d];
          }
          if (combos == 1) continue;  // interior: nobody else holds these cells
          BoxTask t{};
          t.dst_worker = w;
          t.src_begin = (int32_t)tt.srcs.size();
          int64_t cells = 1;
          for (int d = 0; d < 3; ++d) {
            t.org[d] = (int32_t)geom_of(p, w, d).bulk_off + it[d]->start;
            t.ext[d] = it[d]->len;
            cells *= it[d]->len;
          }
          std::vector<BoxSrc> found;
          for (int a = 0; a < nopt[0]; ++a)
            for (int b = 0; b < nopt[1]; ++b)
              for (int c = 0; c < nopt[2]; ++c) {
                int delta[3] = {opt[0][a], opt[1][b], opt[2][c]};
                if (!delta[0] && !delta[1] && !delta[2]) continue;
                BoxSrc src{};
                for (int d = 0; d < 3; ++d) {
                  const DimGeom& g = geom_of(p, w, d);
                  const DimGeom& gs = geom_of(p, w, d, delta[d]);
                  if (delta[d] == 0)
                    src.org[d] = (int32_t)gs.bulk_off + it[d]->start;
                  else if (delta[d] < 0)  // our cells sit in the left neighbour's right halo
                    src.org[d] = (int32_t)(gs.bulk_off + gs.in_size) + it[d]->start;
                  else  // ... in the right neighbour's left halo
                    src.org[d] = (int32_t)gs.bulk_off - ((int32_t)g.in_size - it[d]->start);
                }
                src.worker = worker_with_delta(p, w, delta);
                found.push_back(src);
              }
          std::sort(found.begin(), found.end(), [](const BoxSrc& x, const BoxSrc& y) { return x.worker < y.worker; });
          t.nsrc = (int32_t)found.size();
          tt.srcs.insert(tt.srcs.end(), found.begin(), found.end());
          if (count) {
            tt.cells_band += cells;
            tt.cells_copied += cells * t.nsrc;
          }
          finish_task(tt, t, p.n_b, p.n_ci, vec, upb);
        }
  }
}

template <class T>
static int to_device(const std::vector<T>& v, T** out) {
  *out = nullptr;
  if (v.empty()) return DISTDL_OK;
  DISTDL_HIP_TRY(hipMalloc((void**)out, v.size() * sizeof(T)));
  DISTDL_HIP_TRY(hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return DISTDL_OK;
}

// Resolves the box tables into the records the kernels read (strides and
// origins in vector units) and checks that the last unit of every view lies
// inside its worker's buffer.
static int upload_table(const distdl_plan& p, TaskTable& tt) {
  if (tt.tasks.empty()) return DISTDL_OK;
  const int64_t n_c = p.n_ci;
  const int64_t cv = n_c / tt.vec;
  auto view = [&](int worker, const int32_t org[3], const BoxTask& t, HaloView* out) {
    const WorkerDev& w = p.workers[worker];
    HaloView v{};
    v.worker = worker;
    v.s1 = (uint32_t)(w.buf[2] * cv);
    v.s0 = (uint32_t)(w.buf[1] * (int64_t)v.s1);
    v.sn = (uint64_t)w.buf[0] * v.s0;
    v.base = (uint64_t)org[0] * v.s0 + (uint64_t)org[1] * v.s1 + (uint64_t)org[2] * cv;
    uint64_t last = v.base + (uint64_t)(p.n_b - 1) * v.sn + (uint64_t)(t.ext[0] - 1) * v.s0 +
                    (uint64_t)(t.ext[1] - 1) * v.s1 + (uint64_t)t.ext[2] * cv - 1;
    if (last >= (uint64_t)p.n_b * v.sn) return false;
    *out = v;
    return true;
  };
  std::vector<HaloTaskDev> tasks(tt.tasks.size());
  std::vector<HaloView> views(tt.srcs.size());
  for (size_t i = 0; i < tt.tasks.size(); ++i) {
    const BoxTask& t = tt.tasks[i];
    HaloTaskDev d{};
    bool ok = view(t.dst_worker, t.org, t, &d.dst);
    for (int s = 0; s < t.nsrc && ok; ++s)
      ok = view(tt.srcs[t.src_begin + s].worker, tt.srcs[t.src_begin + s].org, t, &views[t.src_begin + s]);
    if (!ok) return set_error(DISTDL_ERR_INVALID_ARG, "internal: task view out of range");
    if (t.nsrc > 0) d.src0 = views[t.src_begin];
    d.nsrc = t.nsrc;
    d.src_begin = t.src_begin;
    int64_t total = p.n_b * t.ext[0] * t.ext[1] * (int64_t)t.div_row.d;
    if (total >= (int64_t(1) << 32)) return set_error(DISTDL_ERR_UNSUPPORTED, "internal: task too large");
    d.total = (uint32_t)total;
    d.div_row = t.div_row;
    d.div_e1 = t.div_e1;
    d.div_e0 = t.div_e0;
    tasks[i] = d;
  }
  int rc;
  if ((rc = to_device(tasks, &tt.d_tasks))) return rc;
  if ((rc = to_device(views, &tt.d_views))) return rc;
  if ((rc = to_device(tt.blocks, &tt.d_blocks))) return rc;
  return DISTDL_OK;
}

static void free_table(TaskTable& tt) {
  if (tt.d_tasks) (void)hipFree(tt.d_tasks);
  if (tt.d_views) (void)hipFree(tt.d_views);
  if (tt.d_blocks) (void)hipFree(tt.d_blocks);
  tt.d_tasks = nullptr;
  tt.d_views = nullptr;
  tt.d_blocks = nullptr;
}

extern const int kHaloUnitsPerBlock;

// Every box of every task must lie inside the buffer it addresses: checked on
// the host so that no kernel is ever launched with an out-of-range box.
static int validate_table(const distdl_plan& p, const TaskTable& tt) {
  auto inside = [&](int worker, const int32_t org[3], const int32_t ext[3]) {
    if (worker < 0 || worker >= p.n_workers) return false;
    for (int d = 0; d < 3; ++d)
      if (org[d] < 0 || ext[d] < 1 || org[d] + ext[d] > p.workers[worker].buf[d]) return false;
    return true;
  };
  for (const BoxTask& t : tt.tasks) {
    if (!inside(t.dst_worker, t.org, t.ext)) return set_error(DISTDL_ERR_INVALID_ARG, "internal: task box out of range");
    for (int s = 0; s < t.nsrc; ++s)
      if (!inside(tt.srcs[t.src_begin + s].worker, tt.srcs[t.src_begin + s].org, t.ext))
        return set_error(DISTDL_ERR_INVALID_ARG, "internal: task source box out of range");
  }
  return DISTDL_OK;
}

static int finish_plan(distdl_plan* p) {
  p->n_workers = p->P[0] * p->P[1] * p->P[2];
  p->workers.resize(p->n_workers);
  for (int w = 0; w < p->n_workers; ++w) {
    WorkerDev& wd = p->workers[w];
    int64_t bufc = 1, outc = 1;
    for (int d = 0; d < 3; ++d) {
      const DimGeom& g = geom_of(*p, w, d);
      wd.buf[d] = (int32_t)g.buf;
      wd.out[d] = (int32_t)g.out_size;
      wd.origin[d] = (int32_t)g.origin;
      wd.bulk_off[d] = (int32_t)g.bulk_off;
      wd.in_size[d] = (int32_t)g.in_size;
      wd.dom_lo[d] = g.pad[0];
      wd.dom_hi[d] = (int32_t)g.buf - g.pad[1];
      bufc *= g.buf;
      outc *= g.out_size;
    }
    wd.pad_[0] = wd.pad_[1] = 0;
    int64_t cmax = std::max(p->n_ci, p->n_co);
    if (bufc * cmax >= (int64_t(1) << 31) || outc * cmax >= (int64_t(1) << 31))
      return set_error(DISTDL_ERR_UNSUPPORTED, "worker %d: one sample of a partition exceeds 2^31 elements", w);
    if ((double)p->n_b * (double)bufc * (double)cmax >= 4294967296.0)
      return set_error(DISTDL_ERR_UNSUPPORTED, "worker %d: a partition buffer exceeds 2^32 elements", w);
    p->max_buf_cells = std::max(p->max_buf_cells, bufc);
    p->max_out_cells = std::max(p->max_out_cells, outc);
  }
  int vec16 = (int)(16 / dtype_size(p->dtype));
  if (p->n_ci % vec16 == 0) {
    build_forward_table(*p, p->fwd16, vec16, kHaloUnitsPerBlock, true);
    build_adjoint_table(*p, p->adj16, vec16, kHaloUnitsPerBlock, true);
    p->fwd16.vec = p->adj16.vec = vec16;
  }
  build_forward_table(*p, p->fwd1, 1, kHaloUnitsPerBlock, true);
  build_adjoint_table(*p, p->adj1, 1, kHaloUnitsPerBlock, true);
  for (const TaskTable* tt : {&p->fwd16, &p->adj16, &p->fwd1, &p->adj1}) {
    int rc = validate_table(*p, *tt);
    if (rc) return rc;
  }
  // device-side state is created lazily by plan_prepare_device() on first use,
  // so that plans can be built and queried on a host without a GPU
  return DISTDL_OK;
}

int plan_prepare_device(distdl_plan* p) {
  if (p->d_workers) return DISTDL_OK;
  DISTDL_HIP_TRY(hipGetDevice(&p->device));
  int rc;
  if ((rc = to_device(p->workers, &p->d_workers))) return rc;
  if ((rc = upload_table(*p, p->fwd16)) || (rc = upload_table(*p, p->adj16)) || (rc = upload_table(*p, p->fwd1)) ||
      (rc = upload_table(*p, p->adj1)))
    return rc;
  return DISTDL_OK;
}

}  // namespace distdl

using namespace distdl;

extern "C" {

const char* distdl_last_error(void) { return g_err; }

int distdl_plan_create(distdl_plan** out, int D, int64_t n_b, int64_t n_c_in, int64_t n_c_out, const int64_t in_shape[],
                       const int32_t P[], const int32_t ksize[], const int32_t stride[], const int32_t padding[],
                       const int32_t dilation[], distdl_dtype dtype) {
  if (!out || !in_shape || !P || !ksize || !stride || !padding || !dilation)
    return set_error(DISTDL_ERR_NULL, "plan_create: null argument");
  *out = nullptr;
  if (D < 1 || D > DISTDL_MAX_DIMS) return set_error(DISTDL_ERR_INVALID_ARG, "D = %d not in 1..3", D);
  if (n_b < 1 || n_c_in < 1 || n_c_out < 1) return set_error(DISTDL_ERR_INVALID_ARG, "n_b, n_c must be >= 1");
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  for (int d = 0; d < D; ++d) {
    if (in_shape[d] < 1 || P[d] < 1 || ksize[d] < 1 || stride[d] < 1 || padding[d] < 0 || dilation[d] < 1)
      return set_error(DISTDL_ERR_INVALID_ARG, "dim %d: bad size / partition / kernel parameter", d);
    if (in_shape[d] >= (int64_t(1) << 31)) return set_error(DISTDL_ERR_UNSUPPORTED, "dim %d too long", d);
  }
  distdl_plan* p = new (std::nothrow) distdl_plan();
  if (!p) return set_error(DISTDL_ERR_NOMEM, "out of host memory");
  p->D = D;
  p->n_b = n_b;
  p->n_ci = n_c_in;
  p->n_co = n_c_out;
  p->dtype = dtype;
  int lead = 3 - D;
  for (int d = 0; d < lead; ++d) unit_dim(p->dims[d]);
  for (int d = 0; d < D; ++d) {
    int i = lead + d;
    p->P[i] = P[d];
    p->ksize[i] = ksize[d];
    p->stride[i] = stride[d];
    p->padding[i] = padding[d];
    p->dilation[i] = dilation[d];
    p->in_shape[i] = in_shape[d];
    int rc = kernel_dim(d, in_shape[d], ksize[d], stride[d], padding[d], dilation[d], P[d], p->dims[i],
                        &p->out_shape[i]);
    if (rc) {
      delete p;
      return rc;
    }
  }
  int rc = finish_plan(p);
  if (rc) {
    delete p;
    return rc;
  }
  *out = p;
  return DISTDL_OK;
}

int distdl_plan_create_explicit(distdl_plan** out, int D, int64_t n_b, int64_t n_c, const int32_t P[],
                                const int64_t bulk_sizes[], const int32_t halo_lr[], distdl_dtype dtype) {
  if (!out || !P || !bulk_sizes || !halo_lr) return set_error(DISTDL_ERR_NULL, "plan_create_explicit: null argument");
  *out = nullptr;
  if (D < 1 || D > DISTDL_MAX_DIMS) return set_error(DISTDL_ERR_INVALID_ARG, "D = %d not in 1..3", D);
  if (n_b < 1 || n_c < 1) return set_error(DISTDL_ERR_INVALID_ARG, "n_b, n_c must be >= 1");
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  distdl_plan* p = new (std::nothrow) distdl_plan();
  if (!p) return set_error(DISTDL_ERR_NOMEM, "out of host memory");
  p->D = D;
  p->n_b = n_b;
  p->n_ci = p->n_co = n_c;
  p->dtype = dtype;
  p->explicit_halo = true;
  int lead = 3 - D;
  for (int d = 0; d < lead; ++d) unit_dim(p->dims[d]);
  size_t at = 0;
  for (int d = 0; d < D; ++d) {
    int i = lead + d;
    if (P[d] < 1) {
      delete p;
      return set_error(DISTDL_ERR_INVALID_ARG, "dim %d: P < 1", d);
    }
    p->P[i] = P[d];
    p->dims[i].resize(P[d]);
    int64_t start = 0;
    for (int r = 0; r < P[d]; ++r, ++at) {
      DimGeom g{};
      if (bulk_sizes[at] < 1 || halo_lr[2 * at] < 0 || halo_lr[2 * at + 1] < 0) {
        delete p;
        return bulk_sizes[at] < 1 ? set_error(DISTDL_ERR_EMPTY_PARTITION, "dim %d worker %d owns nothing", d, r)
                                  : set_error(DISTDL_ERR_INVALID_ARG, "negative halo width");
      }
      g.in_start = g.out_start = start;
      g.in_size = g.out_size = bulk_sizes[at];
      g.halo[0] = halo_lr[2 * at];
      g.halo[1] = halo_lr[2 * at + 1];
      g.bulk_off = g.halo[0];
      g.buf = g.halo[0] + g.in_size + g.halo[1];
      start += bulk_sizes[at];
      p->dims[i][r] = g;
    }
    p->in_shape[i] = p->out_shape[i] = start;
    int rc = check_halos(p->dims[i], d);
    if (rc) {
      delete p;
      return rc;
    }
  }
  int rc = finish_plan(p);
  if (rc) {
    delete p;
    return rc;
  }
  *out = p;
  return DISTDL_OK;
}

int distdl_plan_num_workers(const distdl_plan* plan) {
  if (!plan) return set_error(DISTDL_ERR_NULL, "null plan");
  return plan->n_workers;
}

int distdl_plan_query(const distdl_plan* plan, int worker, distdl_worker_geom* out) {
  if (!plan || !out) return set_error(DISTDL_ERR_NULL, "plan_query: null argument");
  if (worker < 0 || worker >= plan->n_workers) return set_error(DISTDL_ERR_INVALID_ARG, "worker %d out of range", worker);
  std::memset(out, 0, sizeof *out);
  int lead = 3 - plan->D;
  for (int d = 0; d < plan->D; ++d) {
    const DimGeom& g = geom_of(*plan, worker, lead + d);
    out->in_start[d] = g.in_start;
    out->in_size[d] = g.in_size;
    out->out_start[d] = g.out_start;
    out->out_size[d] = g.out_size;
    for (int s = 0; s < 2; ++s) {
      out->halo[d][s] = g.halo[s];
      out->pad[d][s] = g.pad[s];
      out->extra[d][s] = g.extra[s];
    }
    out->buf_shape[d] = g.buf;
    out->bulk_off[d] = g.bulk_off;
    out->conv_origin[d] = g.origin;
  }
  return DISTDL_OK;
}

int distdl_debug_slot_policy(const int32_t stream_id[], const int32_t table_id[], const int32_t capturing[], int n,
                             int32_t slot_out[]) {
  if (!stream_id || !table_id || !capturing || !slot_out) return set_error(DISTDL_ERR_NULL, "slot_policy: null argument");
  SlotCache cache;
  for (int i = 0; i < n; ++i) {
    const int32_t table = table_id[i];
    int rc = cache.upload(&table, sizeof table, (hipStream_t)(uintptr_t)(0x1000 + 16 * stream_id[i]), capturing[i] != 0,
                          true);
    slot_out[i] = rc ? rc : cache.selected;
  }
  return DISTDL_OK;
}

uint32_t distdl_debug_fastdiv(uint32_t n, uint32_t d) {
  if (d == 0) return 0;
  return fd_div(n, make_fastdiv(d));
}

int distdl_debug_task_count(const distdl_plan* plan, int adjoint) {
  if (!plan) return set_error(DISTDL_ERR_NULL, "null plan");
  return (int)(adjoint ? plan->adj1 : plan->fwd1).tasks.size();
}

int distdl_debug_get_task(const distdl_plan* plan, int adjoint, int index, int32_t out[], int cap) {
  if (!plan || !out) return set_error(DISTDL_ERR_NULL, "null argument");
  const TaskTable& tt = adjoint ? plan->adj1 : plan->fwd1;
  if (index < 0 || index >= (int)tt.tasks.size()) return set_error(DISTDL_ERR_INVALID_ARG, "task index out of range");
  const BoxTask& t = tt.tasks[index];
  int need = 8 + 4 * t.nsrc;
  if (cap < need) return set_error(DISTDL_ERR_INVALID_ARG, "output too short");
  out[0] = t.dst_worker;
  out[1] = t.nsrc;
  for (int d = 0; d < 3; ++d) {
    out[2 + d] = t.org[d];
    out[5 + d] = t.ext[d];
  }
  for (int s = 0; s < t.nsrc; ++s) {
    const BoxSrc& b = tt.srcs[t.src_begin + s];
    out[8 + 4 * s] = b.worker;
    for (int d = 0; d < 3; ++d) out[9 + 4 * s + d] = b.org[d];
  }
  return need;
}

int distdl_plan_destroy(distdl_plan* plan) {
  if (!plan) return DISTDL_OK;
  free_table(plan->fwd16);
  free_table(plan->adj16);
  free_table(plan->fwd1);
  free_table(plan->adj1);
  plan->tab_x.release();
  plan->tab_y.release();
  plan->tab_dx.release();
  plan->tab_dy.release();
  if (plan->d_workers) (void)hipFree(plan->d_workers);
  if (plan->d_wt) (void)hipFree(plan->d_wt);
  if (plan->d_pooldiv) (void)hipFree(plan->d_pooldiv);
  delete plan;
  return DISTDL_OK;
}

}  // extern "C"
