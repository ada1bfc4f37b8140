// Streaming ceilings of an MI355X's memory system for the traffic shapes of the decentralized Adam
// step: what plain kernels that do nothing but move bytes reach, so that the step's fraction of the
// 8 TB/s peak can be judged against what the memory system gives to such traffic at all.
//
// A stand-alone measurement program (not part of libdadam, shares no code with it).  It makes one
// large allocation (physically contiguous in a fresh process) and places its arrays at chosen
// offsets inside it, which also shows how the sustained rate depends on where the arrays sit in
// physical memory.  Every placement is checked against the allocation on the host before a launch;
// every kernel is a plain grid with one tile per workgroup.
//
//   stream_probe            all cases
//   stream_probe quick      one placement per traffic shape
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef float f4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                         \
  do {                                                                                \
    hipError_t e_ = (x);                                                              \
    if (e_ != hipSuccess) {                                                           \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);           \
      exit(1);                                                                        \
    }                                                                                 \
  } while (0)

constexpr double kPeak = 8.0e12;

// Where array k of a family starts: arrays 2j and 2j + 1 form pair j; pairs are `pair` bytes apart,
// the odd member of a pair `odd` bytes above the even one.  (pair = 2 * odd: equal distances;
// odd = the distance between two regions: arrays dealt alternately over the two.)
struct Place {
  size_t pair, odd;
};
__host__ __device__ inline size_t place(Place p, int k) { return (size_t)(k >> 1) * p.pair + (size_t)(k & 1) * p.odd; }
constexpr size_t kGiB = (size_t)1 << 30;
constexpr size_t kMiB = (size_t)1 << 20;

// n_read streams are read, their sum is written to n_write streams (n_write may be 0: the sum is
// then stored only if it equals a value it never has).  Stream k starts at base + place(p, k); one
// workgroup moves one 4 KiB tile of every stream.
__global__ __launch_bounds__(256) void k_streams(char* base, Place p, int n_read, int n_write, float never) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int k = 0; k < n_read; ++k)
    acc += __builtin_nontemporal_load(reinterpret_cast<const f4*>(base + place(p, k)) + e);
  for (int k = 0; k < n_write; ++k)
    __builtin_nontemporal_store(acc, reinterpret_cast<f4*>(base + place(p, n_read + k)) + e);
  if (n_write == 0 && acc.x == never) reinterpret_cast<f4*>(base)[e] = acc;
}

// The traffic of one fused step for R = 16 rows that share their sources (degree 5): per 1 KiB
// tile, 16 source slices staged in LDS, then per row g, m, v, b read and x, b written (FOLD: m and
// v written too).  96 arrays: [0,16) sources, [16,32) g, [32,48) outputs, [48,96) m, v, b per row.
constexpr int kRows = 16;
constexpr int kStepArrays = 6 * kRows;
// BLOCKED: the three state arrays of a row are one array of 3 KiB blocks (m, v, b of a tile side by
// side) instead of three arrays - 64 streams instead of 96 (arrays 48 + 3 i hold row i's blocks and
// are three times as long; arrays 48 + 3 i + 1, + 2 are unused).
template <bool FOLD, bool BLOCKED = false>
__global__ __launch_bounds__(256) void k_step_shape(char* base, Place p) {
  const size_t t = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __shared__ f4 lds[kRows * 64];
  for (int c = wave; c < kRows; c += 4)
    lds[c * 64 + lane] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(base + place(p, c)) + t * 64 + lane);
  __syncthreads();
  for (int i = wave; i < kRows; i += 4) {
    const f4* gp = reinterpret_cast<const f4*>(base + place(p, kRows + i)) + t * 64 + lane;
    f4 *mp, *vp, *bp;
    if (BLOCKED) {
      f4* blk = reinterpret_cast<f4*>(base + place(p, 3 * kRows + 3 * i)) + t * 192;
      mp = blk + lane; vp = blk + 64 + lane; bp = blk + 128 + lane;
    } else {
      mp = reinterpret_cast<f4*>(base + place(p, 3 * kRows + 3 * i + 0)) + t * 64 + lane;
      vp = reinterpret_cast<f4*>(base + place(p, 3 * kRows + 3 * i + 1)) + t * 64 + lane;
      bp = reinterpret_cast<f4*>(base + place(p, 3 * kRows + 3 * i + 2)) + t * 64 + lane;
    }
    f4 g = *gp, m = *mp, v = *vp, b = *bp;
    f4 x = lds[i * 64 + lane] + lds[((i + 1) % kRows) * 64 + lane] + lds[((i + 2) % kRows) * 64 + lane] +
           lds[((i + 4) % kRows) * 64 + lane] + lds[((i + 8) % kRows) * 64 + lane];
    x += g * m + v;
    b += g;
    __builtin_nontemporal_store(x, reinterpret_cast<f4*>(base + place(p, 2 * kRows + i)) + t * 64 + lane);
    __builtin_nontemporal_store(b, bp);
    if (FOLD) {
      __builtin_nontemporal_store(m + b, mp);
      __builtin_nontemporal_store(v + b, vp);
    }
  }
}

struct Arena {
  char* p = nullptr;
  size_t bytes = 0;
};

// Does a family of n arrays of len bytes, array k at offset off + place(p, k), lie inside the arena
// without two arrays overlapping?
bool fits(const Arena& a, size_t off, Place p, int n, size_t len) {
  if (n < 1 || n > 128 || off % 16 || p.pair % 16 || p.odd % 16 || off > a.bytes) return false;
  size_t start[128];
  for (int k = 0; k < n; ++k) {
    start[k] = place(p, k);
    if (start[k] > a.bytes - off || len > a.bytes - off - start[k]) return false;
  }
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < i; ++j) {
      const size_t lo = start[i] < start[j] ? start[i] : start[j];
      const size_t hi = start[i] < start[j] ? start[j] : start[i];
      if (hi - lo < len) return false;
    }
  return true;
}

template <typename Launch>
double time_ms(Launch launch) {
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  launch();
  CK(hipGetLastError());
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a));
  for (int r = 0; r < 4; ++r) launch();
  CK(hipEventRecord(b));
  CK(hipEventSynchronize(b));
  CK(hipGetLastError());
  float ms = 0.f;
  CK(hipEventElapsedTime(&ms, a, b));
  CK(hipEventDestroy(a));
  CK(hipEventDestroy(b));
  return ms / 4.0;
}

void report(const char* shape, const char* where, double bytes, double ms) {
  printf("%-34s %-34s %8.3f ms %6.2f TB/s  %.3f of peak\n", shape, where, ms, bytes / ms / 1e9, bytes / (ms * 1e-3) / kPeak);
  fflush(stdout);
}

void run_streams(const Arena& a, const char* shape, const char* where, size_t off, Place p, int n_read,
                 int n_write, size_t len) {
  if (len % 4096 != 0 || len / 4096 > 0x7fffffffull || !fits(a, off, p, n_read + n_write, len)) {
    printf("%-34s %-34s skipped (does not fit the allocation)\n", shape, where);
    return;
  }
  const unsigned grid = (unsigned)(len / 4096);
  char* base = a.p + off;
  const double ms = time_ms([&] { hipLaunchKernelGGL(k_streams, dim3(grid), dim3(256), 0, 0, base, p, n_read, n_write, 12345.678f); });
  report(shape, where, (double)len * (n_read + n_write), ms);
}

template <bool FOLD>
void run_step(const Arena& a, const char* where, size_t off, Place p, size_t len) {
  const char* shape = FOLD ? "step shape, fold (80 r + 64 w)" : "step shape, plain (80 r + 32 w)";
  if (len % 1024 != 0 || len / 1024 > 0x7fffffffull || !fits(a, off, p, kStepArrays, len)) {
    printf("%-34s %-34s skipped (does not fit the allocation)\n", shape, where);
    return;
  }
  const unsigned grid = (unsigned)(len / 1024);
  char* base = a.p + off;
  const double ms = time_ms([&] { hipLaunchKernelGGL((k_step_shape<FOLD>), dim3(grid), dim3(256), 0, 0, base, p); });
  report(shape, where, (double)len * kRows * (FOLD ? 9 : 7), ms);
}

// The blocked form of the step shape: every array slot must be able to hold 3 * len bytes.
template <bool FOLD>
void run_step_blocked(const Arena& a, const char* where, size_t off, Place p, size_t len) {
  const char* shape = FOLD ? "step shape, fold, blocked state" : "step shape, plain, blocked state";
  if (len % 1024 != 0 || len / 1024 > 0x7fffffffull || !fits(a, off, p, kStepArrays, 3 * len)) {
    printf("%-34s %-34s skipped (does not fit the allocation)\n", shape, where);
    return;
  }
  const unsigned grid = (unsigned)(len / 1024);
  char* base = a.p + off;
  const double ms = time_ms([&] { hipLaunchKernelGGL((k_step_shape<FOLD, true>), dim3(grid), dim3(256), 0, 0, base, p); });
  report(shape, where, (double)len * kRows * (FOLD ? 9 : 7), ms);
}

// n arrays at equal distances over span bytes (2 MiB granularity)
Place even(size_t span, int n) {
  const size_t stride = span / (size_t)n / (2 * kMiB) * (2 * kMiB);
  return Place{2 * stride, stride};
}
Place packed(size_t len) { return Place{2 * len, len}; }
// n arrays dealt alternately over two regions of `width` bytes whose starts are `apart` bytes apart
Place dealt(size_t width, size_t apart, int n) {
  const size_t stride = width / (size_t)((n + 1) / 2) / (2 * kMiB) * (2 * kMiB);
  return Place{stride, apart};
}

int main(int argc, char** argv) {
  const bool quick = argc > 1 && strcmp(argv[1], "quick") == 0;
  size_t free_b = 0, total_b = 0;
  CK(hipMemGetInfo(&free_b, &total_b));
  Arena a;
  a.bytes = 270 * kGiB;
  if (free_b < a.bytes + 8 * kGiB) a.bytes = free_b > 16 * kGiB ? (free_b - 8 * kGiB) / kGiB * kGiB : 0;
  if (a.bytes < 64 * kGiB) {
    printf("not enough free device memory (%zu GiB) for the probe\n", free_b / kGiB);
    return 1;
  }
  CK(hipMalloc((void**)&a.p, a.bytes));
  CK(hipMemset(a.p, 0, a.bytes));
  CK(hipDeviceSynchronize());
  printf("stream_probe: one allocation of %zu GiB (device total %zu GiB); fractions are of %.1f TB/s\n", a.bytes / kGiB,
         total_b / kGiB, kPeak / 1e12);
  printf("%-34s %-34s\n", "traffic shape", "placement of the arrays");

  const size_t len = 475 * kMiB;           // one array of the step shape (GPT-2-small sized, float32)
  const size_t big = 16 * kGiB;            // one long stream
  const size_t whole = a.bytes;
  // "two thirds": regions [30, 94) and [98, 162) GiB, arrays dealt alternately
  const size_t t_off = 30 * kGiB, t_width = 64 * kGiB, t_apart = 68 * kGiB;
  const char* two = "dealt over [30,94) + [98,162) GiB";

  // pure reads
  run_streams(a, "1 read stream of 16 GiB", "at 0 (inside the first third)", 0, packed(big), 1, 0, big);
  run_streams(a, "1 read stream of 16 GiB", "at 88 GiB (across a boundary)", 88 * kGiB, packed(big), 1, 0, big);
  run_streams(a, "96 read streams of 475 MiB", "packed at 0", 0, packed(len), 96, 0, len);
  run_streams(a, "96 read streams of 475 MiB", "equal distances, everything", 0, even(whole, 96), 96, 0, len);
  run_streams(a, "96 read streams of 475 MiB", two, t_off, dealt(t_width, t_apart, 96), 96, 0, len);
  // copies
  run_streams(a, "copy, 1 r + 1 w of 16 GiB", "packed at 0", 0, packed(big), 1, 1, big);
  run_streams(a, "copy, 1 r + 1 w of 16 GiB", "at 40 and 128 GiB", 40 * kGiB, Place{0, 88 * kGiB}, 1, 1, big);
  run_streams(a, "5 r + 2 w of 4 GiB", "packed at 0", 0, packed(4 * kGiB), 5, 2, 4 * kGiB);
  run_streams(a, "5 r + 2 w of 4 GiB", "equal distances, everything", 0, even(whole, 7), 5, 2, 4 * kGiB);
  run_streams(a, "5 r + 2 w of 4 GiB", two, t_off, dealt(t_width, t_apart, 7), 5, 2, 4 * kGiB);
  run_streams(a, "16 r + 16 w of 475 MiB", "packed at 0", 0, packed(len), 16, 16, len);
  run_streams(a, "16 r + 16 w of 475 MiB", "equal distances, everything", 0, even(whole, 32), 16, 16, len);
  run_streams(a, "16 r + 16 w of 475 MiB", two, t_off, dealt(t_width, t_apart, 32), 16, 16, len);
  // the step's own shape
  run_step<false>(a, "packed at 0", 0, packed(len), len);
  run_step<false>(a, "equal distances, everything", 0, even(whole, kStepArrays), len);
  run_step<false>(a, two, t_off, dealt(t_width, t_apart, kStepArrays), len);
  run_step<true>(a, "packed at 0", 0, packed(len), len);
  run_step<true>(a, "equal distances, everything", 0, even(whole, kStepArrays), len);
  run_step<true>(a, two, t_off, dealt(t_width, t_apart, kStepArrays), len);
  // the same with the optimizer state of a row in one blocked array (regions wide enough for 3 * len per slot)
  run_step<false>(a, "dealt over [6,94) + [98,186) GiB", 6 * kGiB, dealt(88 * kGiB, 92 * kGiB, kStepArrays), len);
  run_step_blocked<false>(a, "dealt over [6,94) + [98,186) GiB", 6 * kGiB, dealt(88 * kGiB, 92 * kGiB, kStepArrays), len);
  run_step_blocked<true>(a, "dealt over [6,94) + [98,186) GiB", 6 * kGiB, dealt(88 * kGiB, 92 * kGiB, kStepArrays), len);
  if (!quick) {
    // where in physical memory: packed (44.5 GiB) at several offsets, equal distances over several windows
    run_step<false>(a, "packed at 96 GiB", 96 * kGiB, packed(len), len);
    run_step<false>(a, "packed at 192 GiB", 192 * kGiB, packed(len), len);
    run_step<false>(a, "equal distances, [0, 96) GiB", 0, even(96 * kGiB, kStepArrays), len);
    run_step<false>(a, "equal distances, [96, 192) GiB", 96 * kGiB, even(96 * kGiB, kStepArrays), len);
    run_step<false>(a, "equal distances, [64, 128) GiB", 64 * kGiB, even(64 * kGiB, kStepArrays), len);
    run_step<false>(a, "equal distances, [0, 192) GiB", 0, even(192 * kGiB, kStepArrays), len);
  }
  CK(hipFree(a.p));
  return 0;
}
