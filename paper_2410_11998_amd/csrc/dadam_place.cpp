// Placement of a caller's device buffers inside ONE large allocation ("arena"), by measurement.
//
// On an MI355X a streaming step sustains 0.62-0.66 of peak HBM bandwidth when the arrays it streams together lie
// inside one third (96 GiB) of the card's physical memory and 0.78-0.79 when half of them lie in one third and
// half in another.  Physical addresses are not visible and a large allocation is pieced together from whatever
// is free, so where the thirds begin inside an arena has to be found out: the library's own mixing pass over
// sixteen 64 MiB sources and sixteen outputs runs at 0.78-0.80 of peak when half of its buffers sit in one third
// and half in another and at 0.61-0.73 when all sit in one, repeatably, and timing it over pairs of 1 GiB chunks
// tells which chunks share a third.
//
// This file holds the bookkeeping around such timings (host only, testable with a model of the memory in place
// of the GPU) and the probe that produces them.  Nothing of the method is computed here; the probe calls the
// public entry points of the library like any other client.
#include "dadam.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

namespace {

constexpr uint64_t kUnit = 2ull << 20;
constexpr uint64_t kGiB = 1ull << 30;
constexpr uint32_t kProbeRows = 16;
constexpr uint64_t kProbeElems = 16ull << 20;        // 64 MiB of float32
constexpr uint64_t kProbeBuffer = kProbeElems * 4;
static_assert(2 * (kProbeRows / 2) * kProbeBuffer == DADAM_PROBE_CHUNK_BYTES, "a chunk holds 8 sources and 8 outputs");

uint64_t round_up(uint64_t n) { return (n + kUnit - 1) / kUnit * kUnit; }

// Which chunks run slowly together with the reference chunk (same third)?  false if the rate callback failed.
bool same_third_as(size_t ref, const std::vector<uint64_t>& offs, dadam_pair_rate_fn rate, void* ctx,
                   std::vector<char>* same) {
  std::vector<double> r(offs.size(), -1.0);
  double best = 0.0;
  for (size_t k = 0; k < offs.size(); ++k) {
    if (k == ref) continue;
    r[k] = rate(offs[ref], offs[k], ctx);
    if (!(r[k] >= 0.0)) return false;
    best = std::max(best, r[k]);
  }
  same->assign(offs.size(), 1);
  if (best < 0.75) return true;  // no pairing reaches the two-thirds level: everything shares the reference's third
  for (size_t k = 0; k < offs.size(); ++k)
    if (k != ref) (*same)[k] = r[k] < 0.95 * best ? 1 : 0;
  return true;
}

// The library's mixing pass over 32 buffers of 64 MiB anywhere in the arena, timed with HIP events.
struct Probe {
  char* arena = nullptr;
  uint64_t span = 0;  // bytes of the arena the probe may touch
  dadam_handle* h = nullptr;
  char* state = nullptr;  // 32 x 64 MiB of moment buffers the handle wants bound (the pass does not touch them)
  hipEvent_t e0 = nullptr, e1 = nullptr;
  uint32_t launches = 0;
  int status = DADAM_OK;

  int open(void* arena_base, uint64_t arena_span, int32_t device) {
    arena = static_cast<char*>(arena_base);
    span = arena_span;
    if (hipMalloc((void**)&state, 2 * kProbeRows * kProbeBuffer) != hipSuccess) {
      (void)hipGetLastError();
      state = nullptr;
      return 1;  // no room: the caller falls back to the rule
    }
    dadam_tensor_desc whole = {0, kProbeElems, 0.0f, 0};
    dadam_config cfg;
    memset(&cfg, 0, sizeof(cfg));
    cfg.abi_version = DADAM_ABI_VERSION;
    cfg.n_rows = cfg.n_cols = kProbeRows;
    cfg.d = kProbeElems;
    cfg.n_tensors = 1;
    cfg.tensors = &whole;
    cfg.lr = 1e-3f; cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.eps = 1e-8f;
    cfg.accum_s = 1;
    cfg.beta_vhat = -1.0f;
    cfg.device = device;
    if (dadam_init(&cfg, &h) != DADAM_OK) return DADAM_EHIP;
    // a ring: every source is read by three rows, so the pass stages them once (tile mode), 16 reads + 16 writes
    std::vector<int32_t> rp(kProbeRows + 1), col;
    std::vector<float> w;
    for (uint32_t i = 0; i < kProbeRows; ++i) {
      rp[i] = (int32_t)col.size();
      for (int o : {-1, 0, 1}) { col.push_back((int32_t)((i + kProbeRows + o) % kProbeRows)); w.push_back(1.0f / 3.0f); }
    }
    rp[kProbeRows] = (int32_t)col.size();
    if (dadam_set_topology(h, 0, rp.data(), col.data(), w.data(), nullptr) != DADAM_OK) return DADAM_EHIP;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return DADAM_EHIP;
    return DADAM_OK;
  }

  // Fraction of the HBM peak the pass sustains with its sources at offsets[0..16) and its outputs at [16..32).
  double rate_of_layout(const uint64_t* offsets, int reps = 6) {
    const void* xs[kProbeRows]; void* xd[kProbeRows]; float* m[kProbeRows]; float* v[kProbeRows];
    for (uint32_t k = 0; k < 2 * kProbeRows; ++k)
      if (offsets[k] % 16 != 0 || offsets[k] > span || span - offsets[k] < kProbeBuffer) { status = DADAM_EINVAL; return -1.0; }
    for (uint32_t k = 0; k < kProbeRows; ++k) {
      xs[k] = arena + offsets[k];
      xd[k] = arena + offsets[kProbeRows + k];
      m[k] = reinterpret_cast<float*>(state + k * kProbeBuffer);
      v[k] = reinterpret_cast<float*>(state + (kProbeRows + k) * kProbeBuffer);
    }
    dadam_buffers b = {xs, xd, m, v, nullptr};
    if (dadam_bind(h, &b) != DADAM_OK) { status = DADAM_EHIP; return -1.0; }
    for (int k = 0; k < 2; ++k)
      if (dadam_mix(h, 0, 0, nullptr) != DADAM_OK) { status = DADAM_EHIP; return -1.0; }
    if (hipEventRecord(e0, nullptr) != hipSuccess) { status = DADAM_EHIP; return -1.0; }
    for (int k = 0; k < reps; ++k)
      if (dadam_mix(h, 0, 0, nullptr) != DADAM_OK) { status = DADAM_EHIP; return -1.0; }
    float ms = 0.0f;
    if (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.0f)) { status = DADAM_EHIP; return -1.0; }
    launches += 2 + reps;
    const double seconds = ms / reps / 1e3;
    return 2.0 * kProbeRows * kProbeBuffer / seconds / 8.0e12;
  }

  // Half of the pass's buffers in the chunk at off_a, half in the chunk at off_b.
  double rate(uint64_t off_a, uint64_t off_b) {
    uint64_t o[2 * kProbeRows];
    const uint32_t half = kProbeRows / 2;
    for (uint32_t k = 0; k < half; ++k) {
      o[k] = off_a + k * kProbeBuffer;
      o[half + k] = off_b + k * kProbeBuffer;
      o[kProbeRows + k] = off_a + (half + k) * kProbeBuffer;
      o[kProbeRows + half + k] = off_b + (half + k) * kProbeBuffer;
    }
    return rate_of_layout(o);
  }

  void close() {
    (void)hipDeviceSynchronize();
    if (h) dadam_destroy(h);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (state) (void)hipFree(state);
    h = nullptr; e0 = e1 = nullptr; state = nullptr;
  }
};

double probe_rate(uint64_t a, uint64_t b, void* ctx) { return static_cast<Probe*>(ctx)->rate(a, b); }

}  // namespace

extern "C" {

int dadam_find_stretches(uint64_t arena_bytes, dadam_pair_rate_fn rate, void* ctx, dadam_stretch* out,
                         uint32_t* n_out) {
  if (!rate || !out || !n_out) return DADAM_EINVAL;
  *n_out = 0;
  if (arena_bytes > (1ull << 50)) return DADAM_EINVAL;
  std::vector<uint64_t> offs;
  for (uint64_t o = 0; o + DADAM_PROBE_CHUNK_BYTES <= arena_bytes; o += DADAM_PROBE_STEP_BYTES) offs.push_back(o);
  if (offs.size() < 3) return DADAM_OK;
  for (int attempt = 0; attempt < 2; ++attempt) {
    std::vector<int> third(offs.size(), -1);
    std::vector<char> same;
    if (!same_third_as(0, offs, rate, ctx, &same)) return DADAM_EHIP;
    std::vector<size_t> rest;
    for (size_t k = 0; k < offs.size(); ++k) { if (same[k]) third[k] = 0; else rest.push_back(k); }
    if (!rest.empty()) {
      // the second reference is not the first chunk of the rest: that one may lie across a boundary
      if (!same_third_as(rest[std::min<size_t>(2, rest.size() - 1)], offs, rate, ctx, &same)) return DADAM_EHIP;
      for (size_t k : rest) third[k] = same[k] ? 1 : 2;
    }
    for (size_t k = 1; k + 1 < offs.size(); ++k)  // one chunk at odds with two neighbours that agree: an outlier
      if (third[k - 1] == third[k + 1] && third[k] != third[k - 1]) third[k] = third[k - 1];
    std::vector<dadam_stretch> runs;
    for (size_t k = 0; k < offs.size();) {
      size_t j = k;
      while (j + 1 < offs.size() && third[j + 1] == third[k]) ++j;
      // a run covers its first chunk's start to its last chunk's end
      runs.push_back({(uint32_t)third[k], 0u, offs[k], offs[j] + DADAM_PROBE_CHUNK_BYTES});
      k = j + 1;
    }
    if (runs.size() <= DADAM_MAX_STRETCHES) {
      for (size_t k = 0; k < runs.size(); ++k) out[k] = runs[k];
      *n_out = (uint32_t)runs.size();
      return DADAM_OK;
    }
  }
  return DADAM_OK;  // more stretches than a card has thirds to piece an allocation from: noise, nothing is believed
}

int dadam_regions_from_stretches(const dadam_stretch* runs, uint32_t n_runs, const uint64_t* nbytes, uint32_t n,
                                 uint64_t* regions_out, uint32_t* every_out) {
  if ((!runs && n_runs) || !nbytes || n == 0 || !regions_out || !every_out) return DADAM_EINVAL;
  uint64_t total = 0;
  for (uint32_t k = 0; k < n; ++k) {
    if (nbytes[k] > (1ull << 46)) return DADAM_EINVAL;
    total += round_up(nbytes[k]);
  }
  for (uint32_t every : {2u, 3u, 4u, 6u, 8u}) {
    uint64_t minor = 0;
    for (uint32_t k = every - 1; k < n; k += every) minor += round_up(nbytes[k]);
    const uint64_t major = total - minor;
    const dadam_stretch *ba = nullptr, *bb = nullptr;
    uint64_t best = 0;
    for (uint32_t i = 0; i < n_runs; ++i)      // a holds the larger share
      for (uint32_t j = 0; j < n_runs; ++j) {
        const dadam_stretch &a = runs[i], &b = runs[j];
        if (a.hi < a.lo || b.hi < b.lo) return DADAM_EINVAL;
        if (a.third == b.third || a.hi - a.lo < major || b.hi - b.lo < minor) continue;
        const uint64_t size = std::min(a.hi - a.lo, 96 * kGiB) + std::min(b.hi - b.lo, 96 * kGiB);
        if (!ba || size > best) { best = size; ba = &a; bb = &b; }
      }
    if (!ba) continue;
    // a region is cut down to max(64 GiB, 1.2 x what it holds), at the end of its stretch nearest the other one
    const uint64_t wa = std::min(ba->hi - ba->lo, std::max(64 * kGiB, round_up(major + major / 5)));
    const uint64_t wb = std::min(bb->hi - bb->lo, std::max(64 * kGiB, round_up(minor + minor / 5)));
    if (ba->lo < bb->lo) {
      regions_out[0] = ba->hi - wa; regions_out[1] = ba->hi;
      regions_out[2] = bb->lo;      regions_out[3] = bb->lo + wb;
    } else {
      regions_out[0] = ba->lo;      regions_out[1] = ba->lo + wa;
      regions_out[2] = bb->hi - wb; regions_out[3] = bb->hi;
    }
    *every_out = every;
    return 1;
  }
  return 0;
}

int dadam_place_by_timing(void* arena, uint64_t arena_bytes, int32_t device, const uint64_t* nbytes, uint32_t n,
                          uint64_t device_total_bytes, uint64_t* offsets, dadam_placement* report) {
  if (!arena || !nbytes || !offsets || !report || n == 0 || device < 0) return DADAM_EINVAL;
  if (reinterpret_cast<uintptr_t>(arena) % kUnit != 0) return DADAM_EALIGN;
  memset(report, 0, sizeof(*report));
  int prev = -1;
  if (hipGetDevice(&prev) != hipSuccess || (prev != device && hipSetDevice(device) != hipSuccess)) return DADAM_EHIP;
  const uint64_t span = arena_bytes / kUnit * kUnit;
  int rc = DADAM_OK;
  bool placed = false;
  if (n >= 2 && span >= 2 * DADAM_PROBE_STEP_BYTES + DADAM_PROBE_CHUNK_BYTES) {
    Probe probe;
    const int opened = probe.open(arena, span, device);
    if (opened == 1) {
      report->note = DADAM_NOTE_NO_PROBE;
    } else if (opened != DADAM_OK) {
      rc = DADAM_EHIP;
    } else {
      rc = dadam_find_stretches(span, probe_rate, &probe, report->stretches, &report->n_stretches);
      uint32_t every = 0;
      uint64_t reg[4];
      if (rc == DADAM_OK && report->n_stretches == 0) report->note = DADAM_NOTE_NO_PICTURE;
      if (rc == DADAM_OK && report->n_stretches > 0) {
        const int found = dadam_regions_from_stretches(report->stretches, report->n_stretches, nbytes, n, reg, &every);
        if (found < 0) rc = found;
        else if (found == 0) report->note = DADAM_NOTE_NO_ROOM;
        else {
          // believed only if one more pass across the two regions' far ends runs at the two-thirds level and
          // a pass inside each region does not
          const bool first_lower = reg[0] < reg[2];
          uint64_t lo[2] = {reg[0], reg[2]}, last[2];
          for (int r = 0; r < 2; ++r) {
            const uint64_t hi = reg[2 * r + 1];
            last[r] = hi >= lo[r] + DADAM_PROBE_CHUNK_BYTES ? (hi - DADAM_PROBE_CHUNK_BYTES) / kUnit * kUnit : lo[r];
          }
          const double across = probe.rate(first_lower ? lo[0] : last[0], first_lower ? last[1] : lo[1]);
          double inside[2] = {0.0, 0.0};
          bool confirmed = across >= 0.75;
          for (int r = 0; r < 2 && across >= 0.0; ++r)
            if (last[r] >= lo[r] + DADAM_PROBE_CHUNK_BYTES) {
              inside[r] = probe.rate(lo[r], last[r]);
              if (inside[r] >= 0.95 * across) confirmed = false;
            }
          if (probe.status != DADAM_OK) rc = probe.status;
          report->rate_across = (float)across;
          report->rate_inside[0] = (float)inside[0];
          report->rate_inside[1] = (float)inside[1];
          if (rc == DADAM_OK && !confirmed) report->note = DADAM_NOTE_NOT_CONFIRMED;
          if (rc == DADAM_OK && confirmed) {
            rc = dadam_deal_offsets(nbytes, n, reg[0], reg[1], reg[2], reg[3], every, offsets);
            if (rc == DADAM_OK) {
              placed = true;
              report->policy = DADAM_POLICY_TIMED_REGIONS;
              report->advice = DADAM_PLACE_TWO_REGIONS;
              report->every = every;
              for (int k = 0; k < 4; ++k) report->regions[k] = reg[k];
            }
          }
        }
      }
      report->probe_launches = probe.launches;
    }
    probe.close();
  } else {
    report->note = DADAM_NOTE_NO_PROBE;
  }
  if (rc == DADAM_OK && !placed) {
    rc = dadam_place_offsets(nbytes, n, arena_bytes, device_total_bytes, offsets, report->regions, &report->advice);
    report->policy = report->advice == DADAM_PLACE_TWO_REGIONS ? DADAM_POLICY_RULE_REGIONS : DADAM_POLICY_EQUAL_DISTANCES;
  }
  if (prev != device) (void)hipSetDevice(prev);
  return rc;
}

}  // extern "C"
