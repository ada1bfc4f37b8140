// CPU emulation of the vector access helpers of dadam_kernels.hip.  The test that builds this file cuts
// the helpers' text out of the kernel source verbatim (helpers.inc) and compiles it for the host with
// the address and undefined-behaviour sanitizers: for every element type pair, both kernels' lane
// layouts, full and clipped tiles, every element of the clipped tile must be loaded once and stored
// once, and nothing outside it may be touched (buffers are exactly as long as the data).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#define __device__
#define __forceinline__ inline
static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
constexpr int kWave = 64;
constexpr int kDirectThreads = 256;
constexpr int kHalfWave = 4 * kWave;
constexpr int kHalfGroup = 4 * kDirectThreads;
namespace emu {
#include "helpers.inc"
}
using namespace emu;

static int fails = 0;
template <typename T> float decode(const void* base, uint64_t e) { return load_elem<T>(base, e); }

// one "vector unit" group of NL lanes, UT vectors: tile = NL * VEC * UT elements starting at tbase
template <typename XT, typename ST, int NL, int H, int UT>
void run_case(uint64_t d, uint64_t tbase, uint64_t lo, uint64_t hi, bool full) {
  constexpr int VEC = XT::vec;
  const uint64_t TILE = (uint64_t)NL * VEC * UT;
  // exact-size heap buffers so that the address sanitizer sees any access outside [0, d)
  std::vector<uint8_t>* xs = new std::vector<uint8_t>(d * XT::bytes);
  std::vector<uint8_t>* st = new std::vector<uint8_t>(d * ST::bytes);
  std::vector<uint8_t>* xo = new std::vector<uint8_t>(d * XT::bytes, 0xEE);
  std::vector<uint8_t>* so = new std::vector<uint8_t>(d * ST::bytes, 0xEE);
  for (uint64_t i = 0; i < d; ++i) { store_elem<XT>(xs->data(), i, (float)(i % 251) + 1.0f); store_elem<ST>(st->data(), i, (float)(i % 241) + 2.0f); }
  std::vector<int> seen(d, 0);
  for (int lane = 0; lane < NL; ++lane) {
    for (int u = 0; u < UT; ++u) {
      const uint64_t e = tbase + (uint64_t)u * (NL * VEC) + 4u * (uint32_t)lane;
      float xv[VEC], sv[VEC], raw_out[VEC];
      if (full) {
        load_vals<XT, VEC, H, false, true>(xs->data(), e, lo, hi, xv);
        load_vals<ST, VEC, H, false, true>(st->data(), e, lo, hi, sv);
        unpack_raw<XT>(load_raw<XT, H, false, true>(xs->data(), e, lo, hi), raw_out);
        store_vals<XT, VEC, H, false, true>(xo->data(), e, lo, hi, xv);
        store_vals<ST, VEC, H, false, true>(so->data(), e, lo, hi, sv);
      } else {
        load_vals<XT, VEC, H, true, true>(xs->data(), e, lo, hi, xv);
        load_vals<ST, VEC, H, true, true>(st->data(), e, lo, hi, sv);
        unpack_raw<XT>(load_raw<XT, H, true, true>(xs->data(), e, lo, hi), raw_out);
        store_vals<XT, VEC, H, true, true>(xo->data(), e, lo, hi, xv);
        store_vals<ST, VEC, H, true, true>(so->data(), e, lo, hi, sv);
      }
      for (int j = 0; j < VEC; ++j) if (memcmp(&xv[j], &raw_out[j], 4) != 0) { ++fails; }
      for (int h = 0; h < VEC / 4; ++h) for (int j = 0; j < 4; ++j) { uint64_t ej = e + (uint64_t)h * H + j; if (ej < d && ej >= lo && ej < hi) seen[ej]++; }
    }
  }
  const uint64_t t_lo = tbase > lo ? tbase : lo, t_hi = tbase + TILE < hi ? tbase + TILE : hi;
  for (uint64_t i = 0; i < d; ++i) {
    const bool inside = i >= t_lo && i < t_hi;
    const bool x_same = memcmp(xo->data() + i * XT::bytes, xs->data() + i * XT::bytes, XT::bytes) == 0;
    const bool s_same = memcmp(so->data() + i * ST::bytes, st->data() + i * ST::bytes, ST::bytes) == 0;
    bool x_untouched = true, s_untouched = true;
    for (int b = 0; b < XT::bytes; ++b) x_untouched = x_untouched && (*xo)[i * XT::bytes + b] == 0xEE;
    for (int b = 0; b < ST::bytes; ++b) s_untouched = s_untouched && (*so)[i * ST::bytes + b] == 0xEE;
    if (inside && (!x_same || !s_same || seen[i] != 1)) { if (fails < 10) printf("element %llu inside not copied once (seen %d)\n", (unsigned long long)i, seen[i]); ++fails; }
    if (!inside && (!x_untouched || !s_untouched)) { if (fails < 10) printf("element %llu outside was written\n", (unsigned long long)i); ++fails; }
  }
  delete xs; delete st; delete xo; delete so;
}

template <typename XT, typename ST, int NL, int H, int UT>
void sweep(const char* name) {
  constexpr int VEC = XT::vec;
  const uint64_t TILE = (uint64_t)NL * VEC * UT;
  const uint64_t d = 3 * TILE + 40;
  int before = fails;
  // full tiles
  for (uint64_t t = 0; t < 3; ++t) run_case<XT, ST, NL, H, UT>(d, t * TILE, 0, d, true);
  // clipped tiles: ranges with ragged ends, also ranges inside one tile and the tail tile beyond d
  const uint64_t los[] = {0, 1, 3, 4, 5, TILE - 1, TILE + 7, 2 * TILE - 3};
  const uint64_t his[] = {1, 2, 6, TILE - 5, TILE + 1, 2 * TILE + 9, 3 * TILE + 1, d};
  for (uint64_t lo : los) for (uint64_t hi : his) if (lo < hi)
    for (uint64_t t = 0; t < 4; ++t) run_case<XT, ST, NL, H, UT>(d, t * TILE, lo, hi, false);
  printf("%-44s %s\n", name, fails == before ? "ok" : "FAILED"); fflush(stdout);
}

// The maps from workgroup id to work item: every item exactly once, whatever the sizes.
static void work_orders() {
  int bad = 0;
  for (uint32_t X : {1u, 4u, 8u})
    for (uint32_t n : {1u, 7u, 8u, 9u, 63u, 64u, 257u, 1000u, 4099u})
      for (uint32_t B : {0u, 1u, 3u, 32u, 100u, 5000u}) {
        std::vector<int> seen(n, 0);
        for (uint32_t b = 0; b < n; ++b) {
          const uint32_t t = die_block_order(b, n, X, B);
          if (t >= n) { ++bad; continue; }
          ++seen[t];
        }
        for (uint32_t t = 0; t < n; ++t) bad += seen[t] != 1;
      }
  for (uint32_t X : {2u, 8u})
    for (uint32_t R : {1u, 3u, 8u, 12u, 64u, 100u, 160u})
      for (uint32_t T : {1u, 5u}) {
        const uint32_t G = (R + X - 1) / X;
        std::vector<int> seen(T * R, 0);
        for (uint32_t b = 0; b < T * X * G; ++b) {
          uint32_t tile = 0, pos = 0;
          const bool active = die_group_order(b, R, X, G, tile, pos);
          if (tile >= T || pos >= R) { ++bad; continue; }
          if (active) ++seen[tile * R + pos];
          // a die's rows are a contiguous group of the order
          if (active && (pos < (b % X) * R / X || pos >= (b % X + 1) * R / X)) ++bad;
        }
        for (int c : seen) bad += c != 1;
      }
  printf("work orders %s\n", bad ? "FAIL" : "ok");
  fails += bad;
}

int main() {
  work_orders();
  sweep<TF32, TF32, kWave, kHalfWave, 1>("tile  x f32  state f32  UT1");
  sweep<TF32, TF32, kWave, kHalfWave, 2>("tile  x f32  state f32  UT2");
  sweep<TF32, TBF16, kWave, kHalfWave, 1>("tile  x f32  grad bf16 UT1");
  sweep<TBF16, TF32, kWave, kHalfWave, 1>("tile  x bf16 state f32  UT1");
  sweep<TBF16, TF32, kWave, kHalfWave, 2>("tile  x bf16 state f32  UT2");
  sweep<TBF16, TBF16, kWave, kHalfWave, 2>("tile  x bf16 grad bf16 UT2");
  sweep<TF32, TF32, kDirectThreads, kHalfGroup, 2>("direct x f32  state f32");
  sweep<TF32, TBF16, kDirectThreads, kHalfGroup, 2>("direct x f32  grad bf16");
  sweep<TBF16, TF32, kDirectThreads, kHalfGroup, 2>("direct x bf16 state f32");
  sweep<TBF16, TBF16, kDirectThreads, kHalfGroup, 2>("direct x bf16 grad bf16");
  printf("fails %d\n", fails);
  return fails != 0;
}
