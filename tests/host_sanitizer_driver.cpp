// Host-side fuzz driver for the C ABI, meant to be built with AddressSanitizer and
// UndefinedBehaviorSanitizer (tests/test_host_abi.py does that).  The kernel launchers are replaced by
// stubs, so only host logic runs: validation, the tile planner, neighbour-list checks, aliasing rules,
// the layout helpers.  Random, partly malformed inputs; every call must return a status, never crash.
#include "dadam.h"
#include "dadam_internal.h"
#include <cstdio>
#include <algorithm>
#include <utility>
#include <vector>
#include <cmath>
#include <random>
namespace dadam {
int launch_tile(int, int, Phase, TileShape, const StepArgs&, uint32_t, uint32_t, void*) { return 0; }
int launch_direct(int, int, Phase, bool, bool, const StepArgs&, uint32_t, void*) { return 0; }
int launch_accumulate(int, Phase, bool, const StepArgs&, uint32_t, void*, int) { return 0; }
int launch_consensus_zero(double*, void*) { return 0; }
int launch_consensus_sum(const double*, double*, void*) { return 0; }
int static_partials(double** out, uint32_t* capacity) { *out = nullptr; *capacity = kConsensusPartials; return 0; }
int vec_elems(int xdt) { return xdt == DADAM_BF16 ? 8 : 4; }
int direct_unroll() { return 2; }
bool tile_shape_supported(TileShape s) { return (s.waves == 4 || s.waves == 8) && (s.ut == 1 || s.ut == 2); }
}
int main() {
  std::mt19937_64 rng(1);
  int n_ok = 0, n_err = 0;
  for (int iter = 0; iter < 3000; ++iter) {
    uint32_t R = 1 + rng() % (iter % 4 == 0 ? DADAM_MAX_ROWS : 64), C = 1 + rng() % (iter % 4 == 0 ? DADAM_MAX_ROWS : 64);
    uint32_t nt = 1 + rng() % 40;
    std::vector<dadam_tensor_desc> ts(nt);
    uint64_t cur = 0;
    for (auto& t : ts) {
      cur += (rng() % 3 == 0) ? rng() % 17 : 0;
      t.offset_elems = cur; t.numel = rng() % 5000; t.weight_decay = (rng() % 4 == 0 && R <= C) ? 0.01f : 0.f; t.flags = 0;
      cur += t.numel;
    }
    dadam_config cfg{};
    cfg.abi_version = DADAM_ABI_VERSION; cfg.n_rows = R; cfg.n_cols = C; cfg.d = cur + rng() % 9 + 1; cfg.n_tensors = nt; cfg.tensors = ts.data();
    cfg.param_dtype = rng() % 2; cfg.grad_dtype = rng() % 2; cfg.lr = 1e-3f; cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.eps = 1e-8f;
    cfg.accum_s = 1 + rng() % 4; cfg.beta_vhat = -1.f; cfg.device = DADAM_DEVICE_NONE;
    dadam_handle* h = nullptr;
    int rc = dadam_init(&cfg, &h);
    if (rc != 0) { ++n_err; continue; }
    // random topology, sometimes broken
    std::vector<int32_t> rp(R + 1, 0), col; std::vector<float> w;
    for (uint32_t i = 0; i < R; ++i) {
      uint32_t deg = 1 + rng() % C;
      std::vector<int32_t> perm(C); for (uint32_t c = 0; c < C; ++c) perm[c] = c;
      for (uint32_t c = 0; c < deg; ++c) std::swap(perm[c], perm[c + rng() % (C - c)]);
      for (uint32_t c = 0; c < deg; ++c) { col.push_back(perm[c]); w.push_back(1.0f / deg); }
      rp[i + 1] = (int32_t)col.size();
    }
    if (rng() % 5 == 0 && !col.empty()) col[rng() % col.size()] = (int32_t)(rng() % 200) - 50;
    if (rng() % 7 == 0 && !w.empty()) w[rng() % w.size()] = -1.f;
    uint32_t warn = 0;
    rc = dadam_set_topology(h, rng() % 18, rp.data(), col.data(), w.data(), &warn);
    rc == 0 ? ++n_ok : ++n_err;
    // bind with fake addresses
    size_t stride = cfg.d * 4 + 4096;
    std::vector<const void*> xs(C); std::vector<void*> xd(R); std::vector<float*> m(R), v(R), b(R);
    uintptr_t base = 1 << 20; size_t k = 0;
    for (auto& p : xs) p = (const void*)(base + stride * k++);
    bool inplace = rng() % 3 == 0 && R <= C;
    for (uint32_t i = 0; i < R; ++i) xd[i] = inplace ? const_cast<void*>(xs[i]) : (void*)(base + stride * k++);
    for (auto& p : m) p = (float*)(base + stride * k++);
    for (auto& p : v) p = (float*)(base + stride * k++);
    for (auto& p : b) p = (float*)(base + stride * k++);
    if (rng() % 6 == 0) m[rng() % R] = (float*)xs[rng() % C];
    dadam_buffers bufs{xs.data(), xd.data(), m.data(), v.data(), b.data()};
    rc = dadam_bind(h, &bufs);
    rc == 0 ? ++n_ok : ++n_err;
    dadam_plan_info info; dadam_get_plan_info(h, &info);
    for (uint32_t s = 0; s < DADAM_MAX_SLOTS; ++s) (void)dadam_slot_uses_tile_mode(h, s);
    (void)dadam_swap_x(h);
    std::vector<const void*> g(R); for (auto& p : g) p = (const void*)(base + stride * k++);
    (void)dadam_gossip_step(h, 0, g.data(), 1 + rng() % 9, DADAM_FUSE_ACCUM, nullptr);
    (void)dadam_gossip_step_range(h, 0, g.data(), 3, DADAM_FUSE_ACCUM, rng() % (nt + 2), rng() % (nt + 2), nullptr);
    (void)dadam_accumulate(h, g.data(), 2, nullptr);
    (void)dadam_mix(h, 0, 0, nullptr);
    (void)dadam_last_error(h);
    dadam_destroy(h);
  }
  std::vector<uint64_t> nb = {5, 1u << 21, 77, 3u << 20}; std::vector<uint64_t> off(4);
  (void)dadam_spread_offsets(nb.data(), 4, 1ull << 30, off.data());
  // placement advice on random buffer lists: whatever it answers, buffers stay inside the arena,
  // start at multiples of 2 MiB and do not overlap
  for (int it = 0; it < 300; ++it) {
    const uint32_t n = 1 + rng() % 130;
    std::vector<uint64_t> sz(n), o(n);
    for (auto& x : sz) x = (rng() % 5 == 0) ? (uint64_t)(rng() % 4096) << 20 : 1 + rng() % (3u << 20);
    const uint64_t total = (uint64_t)(16 + rng() % 400) << 30;
    const uint64_t arena = (rng() % 3 == 0) ? total - ((uint64_t)(rng() % 12) << 30) : (uint64_t)(1 + rng() % 300) << 30;
    uint64_t reg[4];
    uint32_t advice = 99;
    if (dadam_place_offsets(sz.data(), n, arena, total, o.data(), (rng() & 1) ? reg : nullptr, (rng() & 1) ? &advice : nullptr) != DADAM_OK) { ++n_err; continue; }
    ++n_ok;
    if (advice != 99 && advice != 0 && advice != DADAM_PLACE_TWO_REGIONS && advice != DADAM_PLACE_ARENA_ELSEWHERE && advice != DADAM_PLACE_TOO_LARGE) { printf("unknown advice\n"); return 1; }
    std::vector<std::pair<uint64_t, uint64_t>> iv;
    for (uint32_t k = 0; k < n; ++k) {
      if (o[k] % (2u << 20) != 0 || o[k] + sz[k] > arena + (2u << 20)) { printf("placement out of the arena\n"); return 1; }
      iv.push_back({o[k], o[k] + sz[k]});
    }
    std::sort(iv.begin(), iv.end());
    for (size_t k = 1; k < iv.size(); ++k)
      if (iv[k].first < iv[k - 1].second) { printf("placement overlaps\n"); return 1; }
  }
  // dealing over two random regions (valid or not): accepted answers stay inside their region
  for (int it = 0; it < 300; ++it) {
    const uint32_t n = 1 + rng() % 90;
    std::vector<uint64_t> sz(n), o(n);
    for (auto& x : sz) x = 1 + rng() % (600u << 20);
    uint64_t b[4];
    for (auto& x : b) x = ((uint64_t)(rng() % 140000) << 21) + ((rng() % 50 == 0) ? 4096 : 0);
    if (rng() % 2) std::sort(b, b + 4);
    const uint32_t every = 1 + rng() % 9;
    if (dadam_deal_offsets(sz.data(), n, b[0], b[1], b[2], b[3], every, o.data()) != DADAM_OK) { ++n_err; continue; }
    ++n_ok;
    for (uint32_t k = 0; k < n; ++k) {
      const int r = k % every == every - 1;
      if (o[k] < b[2 * r] || o[k] + sz[k] > b[2 * r + 1]) { printf("dealt out of its region\n"); return 1; }
    }
  }
  // stretches from random pair timings (a model with thirds at a random base, noise, sometimes garbage), then
  // regions from them: accepted regions lie inside stretches of different thirds and hold their shares
  for (int it = 0; it < 200; ++it) {
    struct Model { uint64_t base; int garbage; std::mt19937_64* rng; } m{(uint64_t)(rng() % 250) << 30, (int)(rng() % 6 == 0), &rng};
    auto rate = [](uint64_t a, uint64_t b, void* ctx) -> double {
      Model* mm = static_cast<Model*>(ctx);
      if (mm->garbage) return ((*mm->rng)() % 100) / 100.0;
      const uint64_t third = 96ull << 30;
      const double r = ((a + mm->base) / third) % 3 != ((b + mm->base) / third) % 3 ? 0.79 : 0.66;
      return r * (1.0 + 0.01 * ((int)((*mm->rng)() % 200) - 100) / 100.0);
    };
    const uint64_t span = (uint64_t)(rng() % 280) << 30;
    dadam_stretch st[DADAM_MAX_STRETCHES];
    uint32_t n_st = 99;
    if (dadam_find_stretches(span, rate, &m, st, &n_st) != DADAM_OK || n_st > DADAM_MAX_STRETCHES) { printf("find_stretches failed\n"); return 1; }
    for (uint32_t k = 0; k < n_st; ++k)
      if (st[k].lo >= st[k].hi || st[k].hi > span || st[k].third > 2 || (k && st[k].lo < st[k - 1].hi)) { printf("bad stretch\n"); return 1; }
    const uint32_t n = 1 + rng() % 120;
    std::vector<uint64_t> sz(n), o(n);
    for (auto& x : sz) x = 1 + rng() % (900u << 20);
    uint64_t reg[4]; uint32_t every = 0;
    const int found = dadam_regions_from_stretches(st, n_st, sz.data(), n, reg, &every);
    if (found < 0) { printf("regions_from_stretches failed\n"); return 1; }
    if (found == 1) {
      ++n_ok;
      if (dadam_deal_offsets(sz.data(), n, reg[0], reg[1], reg[2], reg[3], every, o.data()) != DADAM_OK) { printf("regions do not hold their shares\n"); return 1; }
      int owner[2] = {-1, -1};
      for (int r = 0; r < 2; ++r)
        for (uint32_t k = 0; k < n_st; ++k)
          if (reg[2 * r] >= st[k].lo && reg[2 * r + 1] <= st[k].hi) owner[r] = (int)st[k].third;
      if (owner[0] < 0 || owner[1] < 0 || owner[0] == owner[1]) { printf("regions not inside stretches of different thirds\n"); return 1; }
    } else {
      ++n_err;
    }
  }
  printf("sanitizer driver finished: %d ok, %d rejected\n", n_ok, n_err);
  return 0;
}
