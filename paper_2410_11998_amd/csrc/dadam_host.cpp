// Host side of libdadam: the C ABI of include/dadam.h - argument validation, the segment/tile
// planner, neighbour-list slots, per-iteration scalars and launch set-up.  No arithmetic of the
// method happens here except the scalar bias corrections of Algorithm 3 line 8, which are the same
// for every element of an iteration.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "dadam_internal.h"

using namespace dadam;

namespace {

thread_local std::string g_init_error;

struct Slot {
  bool set = false;
  std::vector<int32_t> row_ptr, col;
  std::vector<float> w;
  int32_t* d_row_ptr = nullptr;
  int32_t* d_col = nullptr;
  float* d_w = nullptr;
  int32_t max_degree = 0;             // longest row
  std::vector<int32_t> order;         // rows ordered so that neighbours share sources (empty: nothing is shared)
  int32_t* d_order = nullptr;
  bool reuse = false;                 // some source is read by two or more rows
  std::vector<int32_t> sole_reader;   // per source: the only row reading it, -1 none, -2 several
};

struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t err = hipSuccess;
  explicit DeviceGuard(int dev) {
    err = hipGetDevice(&prev);
    if (err == hipSuccess && prev != dev) {
      err = hipSetDevice(dev);
      switched = (err == hipSuccess);
    }
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

}  // namespace

struct dadam_handle {
  dadam_config cfg{};
  std::vector<dadam_tensor_desc> tensors;
  std::vector<uint32_t> tensor_seg;  // segment of each non-empty tensor, UINT32_MAX for empty ones
  std::vector<Segment> segs;
  Segment* d_segs = nullptr;
  double* d_partials = nullptr;  // kConsensusPartials doubles of scratch for the consensus error
  // Handles with more than kInlineRows rows or sources: device copies of the bound pointer tables, two per
  // binding (as bound, and with x_src / x_dst exchanged), DADAM_BINDINGS_KEPT bindings in a ring.
  BoundTables* d_tables = nullptr;
  uint32_t binding = 0;  // ring position of the current binding
  bool swapped = false;  // dadam_swap_x flips between the binding's two copies
  double* d_static_partials = nullptr;  // the same in the library's device image (dadam_mix_consensus_static)
  uint32_t static_capacity = 0;         // doubles it holds
  TileShape shape{4, 1, false};
  TileShape mix_shape{4, 1, false};  // shape of the mixing-only launch (more bytes in flight per wavefront)
  uint32_t mix_tile_elems = 0, mix_lds_bytes = 0;
  uint64_t n_work_m = 0;
  bool nontemporal = false;
  int vec = 4;
  uint32_t tile_elems = 0, direct_elems = 0, lds_bytes = 0;
  bool tile_possible = false;
  uint64_t n_work_t = 0, n_work_d = 0;
  Slot slots[DADAM_MAX_SLOTS];
  bool bound = false;
  const void* x_src[kMaxRows] = {};
  void* x_dst[kMaxRows] = {};
  float* m_hat[kMaxRows] = {};
  float* v_hat[kMaxRows] = {};
  float* acc[kMaxRows] = {};
  std::vector<int32_t> inplace_cols[kMaxRows];  // every source buffer that x_dst[i] coincides with
  uint32_t lds_limit = 65536;  // LDS one workgroup may use
  uint32_t n_xcds = 8;         // dies consecutive workgroup ids are dealt over
  // Gradient tables that passed check_grads against the current outputs: a caller that cycles a few
  // gradient sets (or issues a step bucket by bucket) is checked once per set, not once per call.
  struct CheckedGrads { uint64_t gen; std::vector<const void*> ptrs; };
  std::vector<CheckedGrads> checked;
  size_t checked_next = 0;
  // Names the set of output buffers: dadam_bind moves on to the next even number, dadam_swap_x flips
  // the lowest bit (two exchanges give back the same tables).
  uint64_t outputs_gen = 0;
  std::vector<std::pair<uintptr_t, uintptr_t>> outputs_sorted[2];  // [lo, hi) of x_dst, m_hat, v_hat, b, by lo
  uint64_t outputs_sorted_gen[2] = {~0ull, ~0ull};
  float lr = 0.f;
  double betav = 0.0;
  mutable std::string err;
};

namespace {

int fail(const dadam_handle* h, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  if (h) h->err = buf; else g_init_error = buf;
  return code;
}

size_t dtype_bytes(uint32_t dt) { return dt == DADAM_BF16 ? 2 : 4; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Interval {
  uintptr_t lo, hi;
  int kind;  // 0 x_src, 1 x_dst, 2 state
  int index;
};

bool overlaps(const Interval& a, const Interval& b) { return a.lo < b.hi && b.lo < a.hi; }

// Measurement builds (-DDADAM_TUNING, never what build() makes) let the environment override kernel
// shapes when a handle is created; the shipped library has no such switches.
#ifdef DADAM_TUNING
int env_int(const char* name, int fallback) {
  const char* v = getenv(name);
  if (!v || !*v) return fallback;
  return atoi(v);
}
#else
constexpr int env_int(const char*, int fallback) { return fallback; }
#endif

// Build maximal runs of contiguous tensors and number the tiles of both tile grids.
int plan(dadam_handle* h) {
  h->segs.clear();
  h->tensor_seg.assign(h->tensors.size(), UINT32_MAX);
  for (size_t k = 0; k < h->tensors.size(); ++k) {
    const dadam_tensor_desc& t = h->tensors[k];
    if (t.numel == 0) continue;
    if (!h->segs.empty() && h->segs.back().hi == t.offset_elems && h->segs.back().weight_decay == t.weight_decay) {
      h->segs.back().hi = t.offset_elems + t.numel;
    } else {
      Segment s{};
      s.lo = t.offset_elems;
      s.hi = t.offset_elems + t.numel;
      s.weight_decay = t.weight_decay;
      h->segs.push_back(s);
    }
    h->tensor_seg[k] = (uint32_t)(h->segs.size() - 1);
  }
  uint64_t wt = 0, wd = 0, wm = 0;
  for (Segment& s : h->segs) {
    s.first_tile[kGridTile] = s.lo / h->tile_elems;
    s.first_tile[kGridDirect] = s.lo / h->direct_elems;
    s.first_tile[kGridMix] = s.lo / h->mix_tile_elems;
    if (wt > 0x7fffffffull || wd > 0x7fffffffull) break;
    s.work0[kGridTile] = (uint32_t)wt;
    s.work0[kGridDirect] = (uint32_t)wd;
    s.work0[kGridMix] = (uint32_t)wm;
    wt += (s.hi - 1) / h->tile_elems - s.first_tile[kGridTile] + 1;
    wd += (s.hi - 1) / h->direct_elems - s.first_tile[kGridDirect] + 1;
    wm += (s.hi - 1) / h->mix_tile_elems - s.first_tile[kGridMix] + 1;
  }
  h->n_work_t = wt;
  h->n_work_d = wd;
  h->n_work_m = wm;
  if (wt > 0x7fffffffull || wd * (h->cfg.n_rows + h->n_xcds) > 0x7fffffffull)  // direct mode pads rows up to the dies
    return fail(nullptr, DADAM_EINVAL, "layout too large: more than 2^31-1 work items");
  return DADAM_OK;
}

// Work-item range [w0, w1) of the tiles that intersect elements [lo, hi), which start in segment
// s0 and end in segment s1.
void work_range(const dadam_handle* h, Grid grid, uint32_t s0, uint32_t s1, uint64_t lo,
                uint64_t hi, uint32_t* w0, uint32_t* w1) {
  const uint64_t T = grid == kGridTile ? h->tile_elems : grid == kGridDirect ? h->direct_elems : h->mix_tile_elems;
  const Segment& a = h->segs[s0];
  const Segment& b = h->segs[s1];
  *w0 = a.work0[grid] + (uint32_t)(lo / T - a.first_tile[grid]);
  *w1 = b.work0[grid] + (uint32_t)((hi - 1) / T - b.first_tile[grid]) + 1;
}

int check_bound(const dadam_handle* h) {
  if (!h->bound) return fail(h, DADAM_ESTATE, "no buffers bound: call dadam_bind first");
  return DADAM_OK;
}

// The last check before a launch, after every argument has been validated (so that a host-only
// handle reports what is wrong with a call exactly as a device handle would).
int check_device(const dadam_handle* h) {
  if (h->cfg.device == DADAM_DEVICE_NONE)
    return fail(h, DADAM_ESTATE, "host-only handle (device = DADAM_DEVICE_NONE) cannot launch");
  return DADAM_OK;
}

// Gradients are read-only; what they must not overlap is anything the call writes.  The outputs are
// pairwise disjoint (dadam_bind checked that), so they are kept sorted and each gradient is located
// with a binary search; a table that passed is remembered until the outputs change.
int check_grads(dadam_handle* h, const void* const* grads) {
  if (!grads) return fail(h, DADAM_EINVAL, "grads is null");
  const uint32_t R = h->cfg.n_rows;
  for (const auto& ok : h->checked)
    if (ok.gen == h->outputs_gen && std::equal(ok.ptrs.begin(), ok.ptrs.end(), grads)) return DADAM_OK;
  const size_t gb = h->cfg.d * dtype_bytes(h->cfg.grad_dtype);
  const size_t xb = h->cfg.d * dtype_bytes(h->cfg.param_dtype);
  const size_t sb = h->cfg.d * 4;
  const int par = (int)(h->outputs_gen & 1u);
  auto& o = h->outputs_sorted[par];
  if (h->outputs_sorted_gen[par] != h->outputs_gen) {
    o.clear();
    for (uint32_t j = 0; j < R; ++j) {
      o.push_back({(uintptr_t)h->x_dst[j], (uintptr_t)h->x_dst[j] + xb});
      o.push_back({(uintptr_t)h->m_hat[j], (uintptr_t)h->m_hat[j] + sb});
      o.push_back({(uintptr_t)h->v_hat[j], (uintptr_t)h->v_hat[j] + sb});
      if (h->acc[j]) o.push_back({(uintptr_t)h->acc[j], (uintptr_t)h->acc[j] + sb});
    }
    std::sort(o.begin(), o.end());
    h->outputs_sorted_gen[par] = h->outputs_gen;
  }
  for (uint32_t i = 0; i < R; ++i) {
    if (!grads[i]) return fail(h, DADAM_EINVAL, "grads[%u] is null", i);
    if (!aligned16(grads[i])) return fail(h, DADAM_EALIGN, "grads[%u] is not 16-byte aligned", i);
    const uintptr_t lo = (uintptr_t)grads[i], hi = lo + gb;
    // first output that ends beyond lo; it overlaps iff it starts below hi
    auto it = std::upper_bound(o.begin(), o.end(), lo,
                               [](uintptr_t v, const std::pair<uintptr_t, uintptr_t>& iv) { return v < iv.second; });
    if (it != o.end() && it->first < hi)
      return fail(h, DADAM_EALIAS, "grads[%u] overlaps an output buffer (x_dst, m_hat, v_hat or acc)", i);
  }
  dadam_handle::CheckedGrads ok{h->outputs_gen, std::vector<const void*>(grads, grads + R)};
  if (h->checked.size() < 8) h->checked.push_back(std::move(ok));
  else { h->checked[h->checked_next] = std::move(ok); h->checked_next = (h->checked_next + 1) % 8; }
  return DADAM_OK;
}

void fill_args(const dadam_handle* h, const Slot* slot, const void* const* grads, StepArgs* a) {
  memset(a, 0, sizeof(*a));
  const uint32_t R = h->cfg.n_rows, C = h->cfg.n_cols;
  if (h->d_tables) {
    a->ext = h->d_tables + 2 * h->binding + (h->swapped ? 1 : 0);
  } else if (R <= (uint32_t)kInlineRows && C <= (uint32_t)kInlineRows) {
    for (uint32_t c = 0; c < C; ++c) a->x_src[c] = h->x_src[c];
    for (uint32_t i = 0; i < R; ++i) {
      a->x_dst[i] = h->x_dst[i];
      a->m_hat[i] = h->m_hat[i];
      a->v_hat[i] = h->v_hat[i];
      a->acc[i] = h->acc[i];
    }
  }
  for (uint32_t i = 0; i < R; ++i) a->grad[i] = grads ? grads[i] : nullptr;
  if (slot) {
    a->row_ptr = slot->d_row_ptr;
    a->col = slot->d_col;
    a->w = slot->d_w;
    // the dies take contiguous groups of the sharing order in turn
    if (slot->d_order && h->n_xcds > 1) {
      a->row_order = slot->d_order;
      a->order_group = (R + h->n_xcds - 1) / h->n_xcds;
    }
  }
  a->seg = h->d_segs;
  a->n_seg = (uint32_t)h->segs.size();
  a->n_rows = R;
  a->n_cols = C;
  a->n_xcd = h->n_xcds;
  a->xcd_block = (uint32_t)env_int("DADAM_XCD_BLOCK", (int)kDieBlockTiles);
}

// Scalars of iteration t (Algorithm 3 lines 4 and 8), computed in double and rounded once.
void fill_scalars(const dadam_handle* h, uint64_t t, Scalars* s) {
  const double b1 = (double)h->cfg.beta1, b2 = (double)h->cfg.beta2, bv = h->betav;
  const uint64_t S = h->cfg.accum_s;
  const double th = (double)((t + S - 1) / S);  // t_hat = ceil(t / s)
  s->beta1 = (float)b1;
  s->omb1 = (float)(1.0 - b1);
  s->beta2 = (float)b2;
  s->omb2 = (float)(1.0 - b2);
  s->betav = (float)bv;
  s->ombv = (float)(1.0 - bv);
  s->inv_c1 = (float)(1.0 / (1.0 - std::pow(b1, th)));
  s->inv_c2 = (float)(1.0 / (1.0 - std::pow(b2, th)));
  s->eps = h->cfg.eps;
  s->lr = h->lr;
  s->inv_s = (float)(1.0 / (double)S);
}

Phase fused_phase(const dadam_handle* h, uint64_t t) {
  const uint64_t S = h->cfg.accum_s;
  if (S == 1) return kAlg1;
  if (t % S == 0) return kFold;
  if ((t - 1) % S == 0) return kLoopStart;
  return kPlain;
}

// Decide tile or direct mode for this slot and these flags; checks in-place legality.
int choose_mode(const dadam_handle* h, const Slot& slot, uint32_t flags, bool* tile_mode) {
  if ((flags & DADAM_FORCE_DIRECT) && (flags & DADAM_FORCE_TILE))
    return fail(h, DADAM_EINVAL, "DADAM_FORCE_DIRECT and DADAM_FORCE_TILE are exclusive");
  bool direct_legal = true;
  // A row updated in place overwrites every source buffer that shares its memory (two source
  // entries may name one buffer); the direct kernel may do that only if nobody but the row itself
  // reads any of them.
  for (uint32_t i = 0; i < h->cfg.n_rows; ++i)
    for (int32_t c : h->inplace_cols[i]) {
      int32_t sr = slot.sole_reader[c];
      if (!(sr == -1 || sr == (int32_t)i)) direct_legal = false;
    }
  if (flags & DADAM_FORCE_TILE) {
    if (!h->tile_possible) return fail(h, DADAM_EINVAL, "tile mode needs the source tile to fit in LDS");
    *tile_mode = true;
  } else if (flags & DADAM_FORCE_DIRECT) {
    if (!direct_legal)
      return fail(h, DADAM_EALIAS, "in-place update of a source that another row reads needs tile mode");
    *tile_mode = false;
  } else {
    // Shared sources normally mean tile mode.  Two exceptions, where the rows stream directly and the dies
    // take them in the sharing order, so that the second reader of a source finds it in its die's L2:
    // (1) rows of at most two sources over more sources than the two-vector tile holds (64 replicas of a
    // one-peer graph: mixing 0.77 against 0.75 of peak, the whole step 0.792 against 0.788; with three
    // sources a row, a ring, the tile is as fast or faster);
    // (2) a tile so large that a CU holds one workgroup of it (more than 80 sources on 160 KB), with rows of
    // at most eight sources (128 replicas: the step 0.76-0.79 against 0.48-0.49, mixing 0.50-0.74 against 0.40).
    const bool ordered = slot.reuse && direct_legal && h->n_xcds > 1;
    const bool pairs_stream = ordered && slot.max_degree <= 2 && h->cfg.n_cols > 16;
    const bool lone_tile = ordered && slot.max_degree <= 8 && 2 * (uint64_t)h->lds_bytes > h->lds_limit;
    *tile_mode = h->tile_possible && ((slot.reuse && !pairs_stream && !lone_tile) || !direct_legal);
    if (!*tile_mode && !direct_legal)
      return fail(h, DADAM_EALIAS, "in-place update of a shared source is impossible: tile does not fit in LDS");
  }
  return DADAM_OK;
}

int resolve_range(const dadam_handle* h, uint32_t tb, uint32_t te, bool whole, uint64_t* lo,
                  uint64_t* hi, uint32_t* s0, uint32_t* s1, bool* empty) {
  *empty = false;
  if (whole) {
    if (h->segs.empty()) { *empty = true; return DADAM_OK; }
    *lo = h->segs.front().lo;
    *hi = h->segs.back().hi;
    *s0 = 0;
    *s1 = (uint32_t)h->segs.size() - 1;
    return DADAM_OK;
  }
  if (tb > te || te > h->tensors.size())
    return fail(h, DADAM_EINVAL, "tensor range [%u, %u) outside [0, %zu]", tb, te, h->tensors.size());
  uint32_t first = UINT32_MAX, last = UINT32_MAX;
  for (uint32_t k = tb; k < te; ++k)
    if (h->tensor_seg[k] != UINT32_MAX) { if (first == UINT32_MAX) first = k; last = k; }
  if (first == UINT32_MAX) { *empty = true; return DADAM_OK; }
  *lo = h->tensors[first].offset_elems;
  *hi = h->tensors[last].offset_elems + h->tensors[last].numel;
  *s0 = h->tensor_seg[first];
  *s1 = h->tensor_seg[last];
  return DADAM_OK;
}

int step_impl(dadam_handle* h, uint32_t slot_id, const void* const* grads, uint64_t t, uint32_t flags,
              bool whole, uint32_t tb, uint32_t te, bool mix_only, void* stream, double* consensus_out = nullptr,
              double* partials = nullptr) {
  if (!h) return DADAM_EINVAL;
  int rc = check_bound(h);
  if (rc) return rc;
  if (slot_id >= DADAM_MAX_SLOTS || !h->slots[slot_id].set)
    return fail(h, DADAM_ESTATE, "topology slot %u is not set", slot_id);
  if (flags & ~(DADAM_FUSE_ACCUM | DADAM_FORCE_DIRECT | DADAM_FORCE_TILE))
    return fail(h, DADAM_EINVAL, "unknown flag bits 0x%x", flags);
  const Slot& slot = h->slots[slot_id];
  Phase phase = kMixOnly;
  if (!mix_only) {
    if (t == 0) return fail(h, DADAM_EINVAL, "iterations are numbered from 1");
    rc = check_grads(h, grads);
    if (rc) return rc;
    phase = (flags & DADAM_FUSE_ACCUM) ? fused_phase(h, t) : kUpdateOnly;
    if (h->cfg.accum_s > 1 && (flags & DADAM_FUSE_ACCUM))
      for (uint32_t i = 0; i < h->cfg.n_rows; ++i)
        if (!h->acc[i]) return fail(h, DADAM_ESTATE, "accumulator of row %u is not bound", i);
  }
  bool tile_mode = false;
  // the consensus error is computed from the staged tile: ask for tile mode unless the caller chose
  if (consensus_out && !(flags & DADAM_FORCE_DIRECT) && h->tile_possible && slot.reuse) flags |= DADAM_FORCE_TILE;
  rc = choose_mode(h, slot, flags, &tile_mode);
  if (rc) return rc;
  if (consensus_out) {
    if (!tile_mode)
      return fail(h, DADAM_ESTATE, "the consensus error is a by-product of tile mode (shared sources that fit in LDS)");
    phase = kMixConsensus;
  }
  uint64_t lo = 0, hi = 0;
  uint32_t s0 = 0, s1 = 0;
  bool empty = false;
  rc = resolve_range(h, tb, te, whole, &lo, &hi, &s0, &s1, &empty);
  if (rc) return rc;
  rc = check_device(h);
  if (rc) return rc;
  if (!partials) partials = h->d_partials;
  DeviceGuard guard(h->cfg.device);
  if (guard.err != hipSuccess) return fail(h, DADAM_EHIP, "hipSetDevice: %s", hipGetErrorString(guard.err));
  if (consensus_out) {
    int e0 = launch_consensus_zero(partials, stream);
    if (e0 != (int)hipSuccess) return fail(h, DADAM_EHIP, "kernel launch failed: %s", hipGetErrorString((hipError_t)e0));
  }
  if (empty) {
    if (consensus_out) (void)launch_consensus_sum(partials, consensus_out, stream);
    return DADAM_OK;
  }
  uint32_t w0 = 0, w1 = 0;
  const Grid grid = !tile_mode ? kGridDirect : mix_only ? kGridMix : kGridTile;
  work_range(h, grid, s0, s1, lo, hi, &w0, &w1);
  StepArgs a;
  fill_args(h, &slot, mix_only ? nullptr : grads, &a);
  a.grid = grid;
  a.work_begin = w0;
  a.clip_lo = lo;
  a.clip_hi = hi;
  a.partials = partials;
  fill_scalars(h, mix_only ? 1 : t, &a.s);
  int e = tile_mode
              ? launch_tile((int)h->cfg.param_dtype, (int)h->cfg.grad_dtype, phase, mix_only ? h->mix_shape : h->shape, a, w1 - w0,
                            mix_only ? h->mix_lds_bytes : h->lds_bytes, stream)
              : launch_direct((int)h->cfg.param_dtype, (int)h->cfg.grad_dtype, phase,
                              // where rows share sources the re-reads must find them in the cache
                              h->nontemporal, slot.reuse, a, w1 - w0, stream);
  if (e == (int)hipSuccess && consensus_out) e = launch_consensus_sum(partials, consensus_out, stream);
  if (e != (int)hipSuccess)
    return fail(h, DADAM_EHIP, "kernel launch failed: %s", hipGetErrorString((hipError_t)e));
  return DADAM_OK;
}

// Rows in an order in which consecutive rows share as many sources as possible (greedy: from the current row
// to the unvisited row that shares most sources with it, the lowest-numbered on a tie; when nothing is shared
// any more, on to the lowest unvisited row).  A one-peer graph with hop h comes out as its chains
// 0, h, 2h, ..., a ring as 0, 1, 2, ...  The direct kernels hand contiguous groups of this order to the dies.
std::vector<int32_t> sharing_order(uint32_t R, uint32_t C, const int32_t* row_ptr, const int32_t* col) {
  std::vector<std::vector<int32_t>> readers(C);
  for (uint32_t i = 0; i < R; ++i)
    for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) readers[col[k]].push_back((int32_t)i);
  std::vector<int32_t> order;
  std::vector<char> visited(R, 0);
  std::vector<int32_t> shared(R);
  uint32_t lowest = 0;
  int32_t cur = 0;
  while (true) {
    order.push_back(cur);
    visited[cur] = 1;
    if (order.size() == R) break;
    std::fill(shared.begin(), shared.end(), 0);
    for (int32_t k = row_ptr[cur]; k < row_ptr[cur + 1]; ++k)
      for (int32_t j : readers[col[k]])
        if (!visited[j]) ++shared[j];
    int32_t best = -1;
    for (uint32_t j = 0; j < R; ++j)
      if (shared[j] > 0 && (best < 0 || shared[j] > shared[best])) best = (int32_t)j;
    if (best < 0) {
      while (visited[lowest]) ++lowest;
      best = (int32_t)lowest;
    }
    cur = best;
  }
  return order;
}

void free_slot(Slot& s) {
  if (s.d_row_ptr) (void)hipFree(s.d_row_ptr);
  if (s.d_col) (void)hipFree(s.d_col);
  if (s.d_w) (void)hipFree(s.d_w);
  if (s.d_order) (void)hipFree(s.d_order);
  s = Slot();
}

}  // namespace

// -------------------------------------------------------------------------------------------------
// C ABI
// -------------------------------------------------------------------------------------------------
extern "C" {

int dadam_init(const dadam_config* cfg, dadam_handle** out) {
  if (!cfg || !out) return fail(nullptr, DADAM_EINVAL, "cfg or out is null");
  if (cfg->abi_version != DADAM_ABI_VERSION)
    return fail(nullptr, DADAM_EINVAL, "abi_version %u, library has %u", cfg->abi_version, DADAM_ABI_VERSION);
  if (cfg->n_rows == 0 || cfg->n_rows > DADAM_MAX_ROWS || cfg->n_cols == 0 || cfg->n_cols > DADAM_MAX_ROWS)
    return fail(nullptr, DADAM_EINVAL, "n_rows and n_cols must be in [1, %u]", DADAM_MAX_ROWS);
  if (cfg->d == 0) return fail(nullptr, DADAM_EINVAL, "d is zero");
  if (cfg->d > (1ull << 40)) return fail(nullptr, DADAM_EINVAL, "d too large");
  if (cfg->param_dtype > DADAM_BF16 || cfg->grad_dtype > DADAM_BF16)
    return fail(nullptr, DADAM_EINVAL, "unknown dtype");
  if (cfg->accum_s == 0) return fail(nullptr, DADAM_EINVAL, "accum_s must be >= 1");
  if (!std::isfinite(cfg->lr)) return fail(nullptr, DADAM_EINVAL, "lr is not finite");
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
    return fail(nullptr, DADAM_EINVAL, "betas must be in [0, 1)");
  if (!(cfg->eps >= 0.f) || !std::isfinite(cfg->eps)) return fail(nullptr, DADAM_EINVAL, "eps must be finite and >= 0");
  if (cfg->n_tensors > 0 && !cfg->tensors) return fail(nullptr, DADAM_EINVAL, "tensors is null");
  if (cfg->n_tensors == 0) return fail(nullptr, DADAM_EINVAL, "the layout has no tensors");
  if (cfg->device < 0 && cfg->device != DADAM_DEVICE_NONE) return fail(nullptr, DADAM_EINVAL, "bad device ordinal");
  double betav = (double)cfg->beta2;
  if (!std::isnan(cfg->beta_vhat) && cfg->beta_vhat >= 0.f) {
    if (!(cfg->beta_vhat < 1.f)) return fail(nullptr, DADAM_EINVAL, "beta_vhat must be in [0, 1)");
    betav = (double)cfg->beta_vhat;
  }
  uint64_t prev_end = 0;
  for (uint32_t k = 0; k < cfg->n_tensors; ++k) {
    const dadam_tensor_desc& t = cfg->tensors[k];
    if (t.offset_elems < prev_end)
      return fail(nullptr, DADAM_EINVAL, "tensor %u starts before tensor %u ends (list must be ordered and disjoint)", k, k ? k - 1 : 0);
    if (t.numel > cfg->d || t.offset_elems > cfg->d - t.numel)
      return fail(nullptr, DADAM_EINVAL, "tensor %u reaches beyond d", k);
    if (!(t.weight_decay >= 0.f) || !std::isfinite(t.weight_decay))
      return fail(nullptr, DADAM_EINVAL, "tensor %u: weight_decay must be finite and >= 0", k);
    if (t.flags != 0) return fail(nullptr, DADAM_EINVAL, "tensor %u: flags is reserved and must be 0", k);
    if (t.weight_decay > 0.f && cfg->n_rows > cfg->n_cols)
      return fail(nullptr, DADAM_EINVAL, "weight decay needs source buffer i to be row i's own parameters (n_rows <= n_cols)");
    prev_end = t.offset_elems + t.numel;
  }
  dadam_handle* h = new (std::nothrow) dadam_handle();
  if (!h) return fail(nullptr, DADAM_EINVAL, "out of host memory");
  h->cfg = *cfg;
  h->tensors.assign(cfg->tensors, cfg->tensors + cfg->n_tensors);
  h->cfg.tensors = nullptr;
  h->lr = cfg->lr;
  h->betav = betav;

  // What the chip offers: LDS one workgroup may use and the number of dies (XCDs), asked of the
  // device; a host-only handle plans for 64 KB and 8 dies unless the configuration says otherwise.
  if (cfg->device != DADAM_DEVICE_NONE) {
    int lds = 0, xcc = 0;
    hipError_t e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, cfg->device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&xcc, hipDeviceAttributeNumberOfXccs, cfg->device);
    if (e != hipSuccess || lds <= 0) {
      delete h;
      return fail(nullptr, DADAM_EHIP, "cannot read the device's LDS size / die count: %s", hipGetErrorString(e));
    }
    h->lds_limit = (uint32_t)lds;
    h->n_xcds = xcc > 0 ? (uint32_t)xcc : 1u;
    if (cfg->lds_limit_bytes > h->lds_limit) {
      delete h;
      return fail(nullptr, DADAM_EINVAL, "lds_limit_bytes %u exceeds the device's %u", cfg->lds_limit_bytes, h->lds_limit);
    }
  }
  if (cfg->lds_limit_bytes) h->lds_limit = cfg->lds_limit_bytes;
  if (cfg->n_xcds) h->n_xcds = cfg->n_xcds;
  h->n_xcds = (uint32_t)env_int("DADAM_XCDS", (int)h->n_xcds);
  if (h->n_xcds > 64) { delete h; return fail(nullptr, DADAM_EINVAL, "n_xcds out of range"); }

  // tile geometry: 16 bytes per lane and vector, `ut` vectors per lane, all source buffers' slices
  // of one tile resident in LDS.  Measured on MI355X: one vector per lane (many small workgroups)
  // streams best; eight wavefronts per group, four when there are fewer than eight rows to deal out.
  h->vec = vec_elems((int)cfg->param_dtype);
  TileShape shape;
  shape.ut = 1;
  shape.waves = cfg->n_rows >= 8 ? 8 : 4;
  // Non-temporal accesses pay off when an iteration's working set cannot stay in the last-level
  // cache anyway; small problems keep ordinary accesses so that one iteration finds the previous
  // one's output on chip.
  const double touched = (double)cfg->d * cfg->n_rows * 24.0;
  h->nontemporal = env_int("DADAM_NT", touched > 512.0 * 1024 * 1024 ? 1 : 0) != 0;
  shape.nontemporal = h->nontemporal;
  shape.ut = env_int("DADAM_TILE_UT", shape.ut);
  shape.waves = env_int("DADAM_TILE_WAVES", shape.waves);
  if (!tile_shape_supported(shape)) {
    delete h;
    return fail(nullptr, DADAM_EINVAL, "unsupported tile shape (waves %d, ut %d)", shape.waves, shape.ut);
  }
  h->shape = shape;
  h->tile_elems = (uint32_t)(kWave * h->vec * shape.ut);
  h->direct_elems = (uint32_t)(kDirectThreads * h->vec * direct_unroll());
  h->lds_bytes = cfg->n_cols * (uint32_t)shape.ut * kWave * 16u;
  h->tile_possible = h->lds_bytes <= h->lds_limit;
  // The mixing-only launch moves few bytes per row, so it wants more of them in flight per
  // wavefront: two vectors per lane and four wavefronts, as long as that tile stays small enough
  // (32 KB) for five workgroups to share a CU's LDS.  Measured: 16 sources (32 KB) +3 % over the
  // step's shape; 64 sources (128 KB, one workgroup per CU) 0.68-0.75 of peak against 0.76 with the
  // step's one-vector tile, so large source counts keep that.
  h->mix_shape = shape;
  if (cfg->n_cols * 2u * kWave * 16u <= 32768u && h->lds_limit >= 32768u && env_int("DADAM_TILE_UT", 0) == 0 &&
      env_int("DADAM_TILE_WAVES", 0) == 0) {
    h->mix_shape.ut = 2;
    h->mix_shape.waves = 4;
  }
  h->mix_shape.ut = env_int("DADAM_MIX_UT", h->mix_shape.ut);
  h->mix_shape.waves = env_int("DADAM_MIX_WAVES", h->mix_shape.waves);
  if (!tile_shape_supported(h->mix_shape) || cfg->n_cols * (uint32_t)h->mix_shape.ut * kWave * 16u > h->lds_limit)
    h->mix_shape = shape;
  h->mix_tile_elems = (uint32_t)(kWave * h->vec * h->mix_shape.ut);
  h->mix_lds_bytes = cfg->n_cols * (uint32_t)h->mix_shape.ut * kWave * 16u;
  int rc = plan(h);
  if (rc) { delete h; return rc; }

  if (cfg->device != DADAM_DEVICE_NONE) {
    DeviceGuard guard(cfg->device);
    hipError_t e = guard.err;
    if (e == hipSuccess && !h->segs.empty()) {
      e = hipMalloc((void**)&h->d_segs, h->segs.size() * sizeof(Segment));
      if (e == hipSuccess)
        e = hipMemcpy(h->d_segs, h->segs.data(), h->segs.size() * sizeof(Segment), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && (cfg->n_rows > (uint32_t)kInlineRows || cfg->n_cols > (uint32_t)kInlineRows))
      e = hipMalloc((void**)&h->d_tables, 2 * DADAM_BINDINGS_KEPT * sizeof(BoundTables));
    if (e == hipSuccess) e = hipMalloc((void**)&h->d_partials, kConsensusPartials * sizeof(double));
    // the array in the device image: its address on THIS device (the guard has made it current)
    if (e == hipSuccess) e = (hipError_t)static_partials(&h->d_static_partials, &h->static_capacity);
    if (e != hipSuccess) {
      if (h->d_segs) (void)hipFree(h->d_segs);
      if (h->d_partials) (void)hipFree(h->d_partials);
      if (h->d_tables) (void)hipFree(h->d_tables);
      delete h;
      return fail(nullptr, DADAM_EHIP, "device set-up failed: %s", hipGetErrorString(e));
    }
  }
  *out = h;
  return DADAM_OK;
}

int dadam_set_topology(dadam_handle* h, uint32_t slot_id, const int32_t* row_ptr, const int32_t* col_idx,
                       const float* w, uint32_t* warn) {
  if (!h) return DADAM_EINVAL;
  if (warn) *warn = 0;
  if (slot_id >= DADAM_MAX_SLOTS) return fail(h, DADAM_EINVAL, "slot %u out of range", slot_id);
  if (!row_ptr || !col_idx || !w) return fail(h, DADAM_EINVAL, "null neighbour list");
  const uint32_t R = h->cfg.n_rows, C = h->cfg.n_cols;
  if (row_ptr[0] != 0) return fail(h, DADAM_ETOPO, "row_ptr[0] must be 0");
  for (uint32_t i = 0; i < R; ++i) {
    if (row_ptr[i + 1] <= row_ptr[i]) return fail(h, DADAM_ETOPO, "row %u is empty or row_ptr decreases", i);
    if ((uint32_t)(row_ptr[i + 1] - row_ptr[i]) > C) return fail(h, DADAM_ETOPO, "row %u has more entries than sources", i);
  }
  const int32_t nnz = row_ptr[R];
  std::vector<double> colsum(C, 0.0);
  std::vector<int32_t> sole(C, -1);
  bool reuse = false;
  for (uint32_t i = 0; i < R; ++i) {
    double sum = 0.0;
    std::vector<char> seen(C, 0);
    for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
      int32_t c = col_idx[k];
      if (c < 0 || (uint32_t)c >= C) return fail(h, DADAM_ETOPO, "row %u: column %d out of range", i, c);
      if (seen[c]) return fail(h, DADAM_ETOPO, "row %u lists source %d twice", i, c);
      seen[c] = 1;
      if (!(w[k] > 0.f) || !std::isfinite(w[k])) return fail(h, DADAM_ETOPO, "row %u: weight %d is not finite and positive", i, k);
      sum += (double)w[k];
      colsum[c] += (double)w[k];
      if (sole[c] == -1) sole[c] = (int32_t)i; else { sole[c] = -2; reuse = true; }
    }
    if (std::fabs(sum - 1.0) > 1e-5) return fail(h, DADAM_ETOPO, "row %u sums to %.9g, not 1", i, sum);
  }
  if (R == C && warn)
    for (uint32_t c = 0; c < C; ++c)
      if (std::fabs(colsum[c] - 1.0) > 1e-5) *warn |= DADAM_WARN_NOT_COLUMN_STOCHASTIC;

  Slot fresh;
  fresh.set = true;
  fresh.row_ptr.assign(row_ptr, row_ptr + R + 1);
  fresh.col.assign(col_idx, col_idx + nnz);
  fresh.w.assign(w, w + nnz);
  fresh.reuse = reuse;
  fresh.sole_reader = sole;
  for (uint32_t i = 0; i < R; ++i) fresh.max_degree = std::max(fresh.max_degree, row_ptr[i + 1] - row_ptr[i]);
  if (reuse) fresh.order = sharing_order(R, C, row_ptr, col_idx);
  if (h->cfg.device != DADAM_DEVICE_NONE) {
    DeviceGuard guard(h->cfg.device);
    hipError_t e = guard.err;
    if (e == hipSuccess) e = hipMalloc((void**)&fresh.d_row_ptr, (R + 1) * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&fresh.d_col, (size_t)nnz * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&fresh.d_w, (size_t)nnz * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(fresh.d_row_ptr, row_ptr, (R + 1) * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(fresh.d_col, col_idx, (size_t)nnz * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(fresh.d_w, w, (size_t)nnz * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess && !fresh.order.empty()) {
      e = hipMalloc((void**)&fresh.d_order, R * sizeof(int32_t));
      if (e == hipSuccess) e = hipMemcpy(fresh.d_order, fresh.order.data(), R * sizeof(int32_t), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
      free_slot(fresh);
      return fail(h, DADAM_EHIP, "uploading the neighbour list failed: %s", hipGetErrorString(e));
    }
  }
  if (h->cfg.device != DADAM_DEVICE_NONE) {
    DeviceGuard guard(h->cfg.device);
    free_slot(h->slots[slot_id]);
  }
  h->slots[slot_id] = fresh;
  return DADAM_OK;
}

int dadam_bind(dadam_handle* h, const dadam_buffers* b) {
  if (!h) return DADAM_EINVAL;
  if (!b || !b->x_src || !b->x_dst || !b->m_hat || !b->v_hat) return fail(h, DADAM_EINVAL, "null buffer table");
  const uint32_t R = h->cfg.n_rows, C = h->cfg.n_cols;
  if (!b->acc && h->cfg.accum_s > 1) return fail(h, DADAM_EINVAL, "acc table is null but accum_s > 1");
  const size_t xb = h->cfg.d * dtype_bytes(h->cfg.param_dtype);
  const size_t sb = h->cfg.d * 4;
  std::vector<Interval> iv;
  for (uint32_t c = 0; c < C; ++c) {
    if (!b->x_src[c]) return fail(h, DADAM_EINVAL, "x_src[%u] is null", c);
    if (!aligned16(b->x_src[c])) return fail(h, DADAM_EALIGN, "x_src[%u] is not 16-byte aligned", c);
    iv.push_back({(uintptr_t)b->x_src[c], (uintptr_t)b->x_src[c] + xb, 0, (int)c});
  }
  for (uint32_t i = 0; i < R; ++i) {
    const void* ps[4] = {b->x_dst[i], b->m_hat[i], b->v_hat[i], b->acc ? b->acc[i] : nullptr};
    const char* names[4] = {"x_dst", "m_hat", "v_hat", "acc"};
    for (int q = 0; q < 4; ++q) {
      if (!ps[q]) {
        if (q == 3 && h->cfg.accum_s == 1) continue;
        return fail(h, DADAM_EINVAL, "%s[%u] is null", names[q], i);
      }
      if (!aligned16(ps[q])) return fail(h, DADAM_EALIGN, "%s[%u] is not 16-byte aligned", names[q], i);
      iv.push_back({(uintptr_t)ps[q], (uintptr_t)ps[q] + (q == 0 ? xb : sb), q == 0 ? 1 : 2, (int)i});
    }
  }
  std::vector<int32_t> inplace[kMaxRows];
  for (size_t p = 0; p < iv.size(); ++p)
    for (size_t q = p + 1; q < iv.size(); ++q) {
      const Interval& a = iv[p];
      const Interval& c = iv[q];
      if (!overlaps(a, c)) continue;
      if (a.kind == 0 && c.kind == 0) continue;  // two read-only sources may coincide
      if (a.kind == 0 && c.kind == 1 && a.lo == c.lo) {  // update in place
        inplace[c.index].push_back(a.index);
        continue;
      }
      return fail(h, DADAM_EALIAS, "buffers overlap: kind %d index %d and kind %d index %d (0 x_src, 1 x_dst, 2 state)",
                  a.kind, a.index, c.kind, c.index);
    }
  if (h->d_tables) {
    // The tables do not fit the kernel arguments: two immutable device copies for this binding (as bound,
    // and as dadam_swap_x would leave it), in the ring slot after the current one, so that launches in
    // flight keep reading the copies they were given.
    std::vector<BoundTables> t(2);
    memset(t.data(), 0, 2 * sizeof(BoundTables));
    for (int v = 0; v < 2; ++v) {
      for (uint32_t c = 0; c < C; ++c) t[v].x_src[c] = (uint64_t)(uintptr_t)b->x_src[c];
      for (uint32_t i = 0; i < R; ++i) {
        t[v].x_dst[i] = (uint64_t)(uintptr_t)b->x_dst[i];
        t[v].m_hat[i] = (uint64_t)(uintptr_t)b->m_hat[i];
        t[v].v_hat[i] = (uint64_t)(uintptr_t)b->v_hat[i];
        t[v].acc[i] = b->acc ? (uint64_t)(uintptr_t)b->acc[i] : 0;
      }
    }
    if (R == C)
      for (uint32_t i = 0; i < R; ++i)
        if (inplace[i].empty()) {  // what dadam_swap_x does
          t[1].x_src[i] = (uint64_t)(uintptr_t)b->x_dst[i];
          t[1].x_dst[i] = (uint64_t)(uintptr_t)b->x_src[i];
        }
    const uint32_t next = h->bound ? (h->binding + 1) % DADAM_BINDINGS_KEPT : h->binding;
    DeviceGuard guard(h->cfg.device);
    hipError_t e = guard.err;
    if (e == hipSuccess) e = hipMemcpy(h->d_tables + 2 * next, t.data(), 2 * sizeof(BoundTables), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(h, DADAM_EHIP, "copying the pointer tables to the device failed: %s", hipGetErrorString(e));
    h->binding = next;
  }
  h->swapped = false;
  for (uint32_t c = 0; c < C; ++c) h->x_src[c] = b->x_src[c];
  for (uint32_t i = 0; i < R; ++i) {
    h->x_dst[i] = b->x_dst[i];
    h->m_hat[i] = b->m_hat[i];
    h->v_hat[i] = b->v_hat[i];
    h->acc[i] = b->acc ? b->acc[i] : nullptr;
    h->inplace_cols[i] = inplace[i];
  }
  h->bound = true;
  h->outputs_gen = (h->outputs_gen | 1u) + 1u;
  return DADAM_OK;
}

int dadam_swap_x(dadam_handle* h) {
  if (!h) return DADAM_EINVAL;
  if (!h->bound) return fail(h, DADAM_ESTATE, "no buffers bound");
  if (h->cfg.n_rows != h->cfg.n_cols) return fail(h, DADAM_ESTATE, "swap needs n_rows == n_cols");
  for (uint32_t i = 0; i < h->cfg.n_rows; ++i) {
    if (!h->inplace_cols[i].empty()) continue;  // in-place rows stay as they are
    void* s = const_cast<void*>(h->x_src[i]);
    h->x_src[i] = h->x_dst[i];
    h->x_dst[i] = s;
  }
  h->outputs_gen ^= 1u;
  h->swapped = !h->swapped;
  return DADAM_OK;
}

int dadam_gossip_step(dadam_handle* h, uint32_t slot, const void* const* grads, uint64_t t, uint32_t flags,
                      void* hip_stream) {
  return step_impl(h, slot, grads, t, flags, true, 0, 0, false, hip_stream);
}

int dadam_gossip_step_range(dadam_handle* h, uint32_t slot, const void* const* grads, uint64_t t,
                            uint32_t flags, uint32_t tensor_begin, uint32_t tensor_end, void* hip_stream) {
  return step_impl(h, slot, grads, t, flags, false, tensor_begin, tensor_end, false, hip_stream);
}

int dadam_mix(dadam_handle* h, uint32_t slot, uint32_t flags, void* hip_stream) {
  if (h && (flags & DADAM_FUSE_ACCUM)) return fail(h, DADAM_EINVAL, "dadam_mix takes only the FORCE flags");
  return step_impl(h, slot, nullptr, 1, flags, true, 0, 0, true, hip_stream);
}

int dadam_mix_consensus(dadam_handle* h, uint32_t slot, uint32_t flags, double* consensus_out, void* hip_stream) {
  if (!h) return DADAM_EINVAL;
  if (flags & DADAM_FUSE_ACCUM) return fail(h, DADAM_EINVAL, "dadam_mix_consensus takes only the FORCE flags");
  if (!consensus_out || (reinterpret_cast<uintptr_t>(consensus_out) & 7u))
    return fail(h, DADAM_EINVAL, "consensus_out must be a non-null, 8-byte aligned device pointer");
  return step_impl(h, slot, nullptr, 1, flags, true, 0, 0, true, hip_stream, consensus_out);
}

int dadam_mix_consensus_static(dadam_handle* h, uint32_t slot, uint32_t flags, double* consensus_out, void* hip_stream) {
  if (!h) return DADAM_EINVAL;
  if (flags & DADAM_FUSE_ACCUM) return fail(h, DADAM_EINVAL, "dadam_mix_consensus_static takes only the FORCE flags");
  if (!consensus_out || (reinterpret_cast<uintptr_t>(consensus_out) & 7u))
    return fail(h, DADAM_EINVAL, "consensus_out must be a non-null, 8-byte aligned device pointer");
  if (h->cfg.device != DADAM_DEVICE_NONE) {
    if (!h->d_static_partials) return fail(h, DADAM_ESTATE, "the static scratch array was not resolved on this device");
    if (kConsensusPartials > h->static_capacity)
      return fail(h, DADAM_EINVAL, "the pass needs %u partial sums, the static scratch array holds %u (DADAM_STATIC_SCRATCH_BYTES = %u)",
                  kConsensusPartials, h->static_capacity, DADAM_STATIC_SCRATCH_BYTES);
  }
  return step_impl(h, slot, nullptr, 1, flags, true, 0, 0, true, hip_stream, consensus_out, h->d_static_partials);
}

int dadam_accumulate(dadam_handle* h, const void* const* grads, uint64_t t, void* hip_stream) {
  if (!h) return DADAM_EINVAL;
  int rc = check_bound(h);
  if (rc) return rc;
  if (t == 0) return fail(h, DADAM_EINVAL, "iterations are numbered from 1");
  rc = check_grads(h, grads);
  if (rc) return rc;
  if (h->cfg.accum_s > 1)
    for (uint32_t i = 0; i < h->cfg.n_rows; ++i)
      if (!h->acc[i]) return fail(h, DADAM_ESTATE, "accumulator of row %u is not bound", i);
  rc = check_device(h);
  if (rc) return rc;
  if (h->segs.empty()) return DADAM_OK;
  StepArgs a;
  fill_args(h, nullptr, grads, &a);
  uint32_t w0 = 0, w1 = 0;
  work_range(h, kGridDirect, 0, (uint32_t)h->segs.size() - 1, h->segs.front().lo, h->segs.back().hi, &w0, &w1);
  a.grid = kGridDirect;
  a.work_begin = w0;
  a.clip_lo = h->segs.front().lo;
  a.clip_hi = h->segs.back().hi;
  fill_scalars(h, t, &a.s);
  DeviceGuard guard(h->cfg.device);
  if (guard.err != hipSuccess) return fail(h, DADAM_EHIP, "hipSetDevice: %s", hipGetErrorString(guard.err));
  int e = launch_accumulate((int)h->cfg.grad_dtype, fused_phase(h, t), h->nontemporal, a, w1 - w0, hip_stream, h->vec);
  if (e != (int)hipSuccess)
    return fail(h, DADAM_EHIP, "kernel launch failed: %s", hipGetErrorString((hipError_t)e));
  return DADAM_OK;
}

int dadam_set_lr(dadam_handle* h, float lr) {
  if (!h) return DADAM_EINVAL;
  if (!std::isfinite(lr)) return fail(h, DADAM_EINVAL, "lr is not finite");
  h->lr = lr;
  return DADAM_OK;
}

int dadam_get_plan_info(const dadam_handle* h, dadam_plan_info* out) {
  if (!h || !out) return DADAM_EINVAL;
  out->n_segments = (uint32_t)h->segs.size();
  out->tile_elems = h->tile_elems;
  out->direct_elems = h->direct_elems;
  out->n_tiles_tile = h->n_work_t;
  out->n_tiles_direct = h->n_work_d;
  out->lds_bytes_tile = h->lds_bytes;
  out->tile_mode_possible = h->tile_possible ? 1u : 0u;
  out->lds_limit_bytes = h->lds_limit;
  out->n_xcds = h->n_xcds;
  out->mix_tile_elems = h->mix_tile_elems;
  out->lds_bytes_mix = h->mix_lds_bytes;
  out->n_tiles_mix = h->n_work_m;
  out->tile_waves = (uint32_t)h->shape.waves;
  out->tile_vectors = (uint32_t)h->shape.ut;
  out->mix_waves = (uint32_t)h->mix_shape.waves;
  out->mix_vectors = (uint32_t)h->mix_shape.ut;
  out->streaming = h->nontemporal ? 1u : 0u;
  return DADAM_OK;
}

int dadam_slot_uses_tile_mode(const dadam_handle* h, uint32_t slot) {
  if (!h) return DADAM_EINVAL;
  if (slot >= DADAM_MAX_SLOTS || !h->slots[slot].set) return fail(h, DADAM_ESTATE, "topology slot %u is not set", slot);
  bool tile = false;
  int rc = choose_mode(h, h->slots[slot], 0, &tile);
  if (rc) return rc;
  return tile ? 1 : 0;
}

int dadam_get_row_order(const dadam_handle* h, uint32_t slot, int32_t* order_out) {
  if (!h || !order_out) return DADAM_EINVAL;
  if (slot >= DADAM_MAX_SLOTS || !h->slots[slot].set) return fail(h, DADAM_ESTATE, "topology slot %u is not set", slot);
  const Slot& s = h->slots[slot];
  const uint32_t R = h->cfg.n_rows;
  const bool used = !s.order.empty() && h->n_xcds > 1;
  for (uint32_t i = 0; i < R; ++i) order_out[i] = used ? s.order[i] : (int32_t)i;
  return used ? 1 : 0;
}

int dadam_pack_offsets(const uint64_t* numel, uint32_t n, uint32_t align_elems, uint64_t* offsets, uint64_t* d_out) {
  if (!numel || !offsets || !d_out || align_elems == 0) return DADAM_EINVAL;
  uint64_t cur = 0;
  for (uint32_t k = 0; k < n; ++k) {
    offsets[k] = cur;
    cur += (numel[k] + align_elems - 1) / align_elems * align_elems;
  }
  *d_out = cur;
  return DADAM_OK;
}

int dadam_spread_offsets(const uint64_t* nbytes, uint32_t n, uint64_t arena_bytes, uint64_t* offsets) {
  if (!nbytes || !offsets || n == 0) return DADAM_EINVAL;
  const uint64_t unit = 2ull << 20;
  uint64_t packed = 0;
  for (uint32_t k = 0; k < n; ++k) {
    if (nbytes[k] > (1ull << 46)) return DADAM_EINVAL;
    packed += (nbytes[k] + unit - 1) / unit * unit;
  }
  if (packed > arena_bytes + (((nbytes[n - 1] + unit - 1) / unit * unit) - nbytes[n - 1])) return DADAM_EINVAL;
  const uint64_t slack = arena_bytes > packed ? arena_bytes - packed : 0;
  const uint64_t gap = n > 1 ? slack / (n - 1) / unit * unit : 0;
  uint64_t cur = 0;
  for (uint32_t k = 0; k < n; ++k) {
    offsets[k] = cur;
    cur += (nbytes[k] + unit - 1) / unit * unit + gap;
  }
  return DADAM_OK;
}

int dadam_deal_offsets(const uint64_t* nbytes, uint32_t n, uint64_t lo0, uint64_t hi0, uint64_t lo1, uint64_t hi1,
                       uint32_t every, uint64_t* offsets) {
  if (!nbytes || !offsets || n == 0 || every < 2 || every > 8) return DADAM_EINVAL;
  const uint64_t unit = 2ull << 20;
  const uint64_t lo[2] = {lo0, lo1}, hi[2] = {hi0, hi1};
  for (int r = 0; r < 2; ++r)
    if (lo[r] % unit || hi[r] % unit || lo[r] > hi[r] || hi[r] > (1ull << 50)) return DADAM_EINVAL;
  if (lo0 < hi1 && lo1 < hi0 && lo0 != hi0 && lo1 != hi1) return DADAM_EINVAL;  // the regions overlap
  std::vector<uint64_t> side[2];
  std::vector<uint32_t> number[2];  // which buffers a side holds
  for (uint32_t k = 0; k < n; ++k) {
    if (nbytes[k] > (1ull << 46)) return DADAM_EINVAL;
    const int r = k % every == every - 1 ? 1 : 0;
    side[r].push_back(nbytes[k]);
    number[r].push_back(k);
  }
  for (int r = 0; r < 2; ++r) {
    if (side[r].empty()) continue;
    std::vector<uint64_t> off(side[r].size());
    const int rc = dadam_spread_offsets(side[r].data(), (uint32_t)side[r].size(), hi[r] - lo[r], off.data());
    if (rc != DADAM_OK) return rc;
    // Stagger the buffers inside their gaps by a fixed pseudo-random number of 2 MiB steps, so that their
    // bases do not form an arithmetic progression: for some distances (660 MiB, 884 MiB between 476 MiB
    // buffers) a progression costs 3-4 % of bandwidth, staggered bases never did.  A buffer moves forward
    // by less than the gap behind it; the last one stays where it is.
    for (size_t j = 0; j + 1 < off.size(); ++j) {
      const uint64_t end = off[j] + (side[r][j] + unit - 1) / unit * unit;
      const uint64_t slots = off[j + 1] > end ? (off[j + 1] - end) / unit : 0;
      uint64_t z = ((uint64_t)j + 1) * 0x9E3779B97F4A7C15ull;  // a fixed 64-bit mix of the buffer's number
      z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
      z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
      z ^= z >> 31;
      if (slots > 1) off[j] += z % slots * unit;
    }
    for (size_t j = 0; j < off.size(); ++j) offsets[number[r][j]] = lo[r] + off[j];
  }
  return DADAM_OK;
}

int dadam_place_offsets(const uint64_t* nbytes, uint32_t n, uint64_t arena_bytes, uint64_t device_total_bytes,
                        uint64_t* offsets, uint64_t* regions_out, uint32_t* advice_out) {
  if (!nbytes || !offsets || n == 0) return DADAM_EINVAL;
  const uint64_t unit = 2ull << 20, gib = 1ull << 30;
  std::vector<uint64_t> side[2];
  uint64_t need[2] = {0, 0};
  for (uint32_t k = 0; k < n; ++k) {
    if (nbytes[k] > (1ull << 46)) return DADAM_EINVAL;
    side[k & 1].push_back(nbytes[k]);
    need[k & 1] += (nbytes[k] + unit - 1) / unit * unit;
  }
  if (arena_bytes > (1ull << 50) || device_total_bytes > (1ull << 50)) return DADAM_EINVAL;
  const uint64_t third = (device_total_bytes + 3 * gib / 2) / (3 * gib) * gib;  // a third, to the nearest GiB
  const uint64_t margin = 2 * gib;
  // Region 0 ends `margin` below the boundary between the first two thirds, region 1 starts `margin`
  // above it and ends no later than `margin` below the next boundary (or where the arena ends).
  const uint64_t top = arena_bytes < 2 * third - margin ? arena_bytes : 2 * third - margin;
  uint32_t advice = 0;
  uint64_t lo[2] = {0, 0}, width[2] = {0, 0};
  if (n < 2 || third <= 2 * margin) {
    advice = 0;  // nothing to deal over two sides
  } else if (arena_bytes + 16 * gib < device_total_bytes) {
    advice = DADAM_PLACE_ARENA_ELSEWHERE;
  } else if (need[0] > third - margin || third + margin + need[1] > top) {
    advice = DADAM_PLACE_TOO_LARGE;
  } else {
    for (int r = 0; r < 2; ++r) {
      uint64_t want = (need[r] + need[r] / 5 + unit - 1) / unit * unit;  // 20 % of room for the stagger
      if (want < 64 * gib) want = 64 * gib;
      const uint64_t room = r == 0 ? third - margin : top - (third + margin);
      width[r] = (want < room ? want : room) / unit * unit;  // >= need[r] by the tests above
      lo[r] = r == 0 ? third - margin - width[r] : third + margin;
    }
    advice = DADAM_PLACE_TWO_REGIONS;
  }
  if (advice_out) *advice_out = advice;
  if (advice == DADAM_PLACE_TWO_REGIONS) {
    const int rc = dadam_deal_offsets(nbytes, n, lo[0], lo[0] + width[0], lo[1], lo[1] + width[1], 2, offsets);
    if (rc != DADAM_OK) return rc;
    if (regions_out) {
      regions_out[0] = lo[0]; regions_out[1] = lo[0] + width[0];
      regions_out[2] = lo[1]; regions_out[3] = lo[1] + width[1];
    }
    return DADAM_OK;
  }
  if (regions_out) {
    regions_out[0] = 0; regions_out[1] = arena_bytes;
    regions_out[2] = 0; regions_out[3] = 0;
  }
  return dadam_spread_offsets(nbytes, n, arena_bytes, offsets);
}

const char* dadam_last_error(const dadam_handle* h) { return h ? h->err.c_str() : g_init_error.c_str(); }

void dadam_destroy(dadam_handle* h) {
  if (!h) return;
  if (h->cfg.device != DADAM_DEVICE_NONE) {
    DeviceGuard guard(h->cfg.device);
    for (Slot& s : h->slots) free_slot(s);
    if (h->d_segs) (void)hipFree(h->d_segs);
    if (h->d_partials) (void)hipFree(h->d_partials);
    if (h->d_tables) (void)hipFree(h->d_tables);
  }
  delete h;
}

}  // extern "C"
