// gfx950 kernels of the decentralized (accumulated) Adam step (device code, included by every kernel
// translation unit; the launchers are in dadam_kernels.hip).
//
//
// The work is streaming and elementwise over the packed parameter vector; neighbour mixing couples
// replicas, never elements.  Three kernels:
//
//   k_tile    one workgroup owns a tile of elements for ALL rows: every source buffer's slice of the
//             tile is read from HBM once and parked in LDS, then the wavefronts of the group deal the
//             rows among themselves and update each from LDS.  Lane l of every wavefront works on
//             the same elements for all rows, so LDS is a per-lane indexable store - no lane ever
//             reads what another lane wrote, one barrier separates staging from use.  All sources
//             of the tile are read before anything is written, so updating in place is legal.
//   k_direct  one workgroup updates one tile of one row and streams the row's sources from global
//             memory (a node's own parameters plus receive buffers: no source is shared by two rows).
//   k_acc     accumulate / fold only (Algorithm 3 lines 9-13).
//
// Every access of a full tile is a 128-bit (float32) or 64-bit (bfloat16) load or store per lane,
// laid out so that each instruction of a wavefront covers one contiguous run of memory; lanes at
// the ragged edge of a segment fall back to element accesses.  Neighbour lists are read once per
// row as one coalesced load (one entry per lane) and handed out with readlane, so the inner loop
// has no dependent scalar memory traffic - which also means that no lane may leave a wavefront
// before the last readlane (see direct_body).
#ifndef DADAM_DEVICE_H_
#define DADAM_DEVICE_H_

#include <hip/hip_runtime.h>

#include <type_traits>

#include "dadam_internal.h"

namespace dadam {
namespace {


// distance (in elements) between the two groups of four that an 8-element lane vector consists of
constexpr int kHalfWave = 4 * kWave;             // tile kernel: the lanes of a wavefront work side by side
constexpr int kHalfGroup = 4 * kDirectThreads;   // direct and accumulate kernels: the whole workgroup does

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

// Which work item a workgroup takes.  Consecutive workgroup ids are dispatched to the device's X dies in turn.
//
// Tile mode: the n work items are cut into blocks of B and the blocks go to the dies in turn, so that each die
// (and its L2) walks runs of B consecutive tiles while all dies stay in the same neighbourhood of every array.
// B == 0: one contiguous X-th of the items per die.  A bijection of [0, X * (n / X)); the part of a die's
// share that does not fill a block is taken contiguously, and the last n mod X workgroups keep their item.
__device__ __forceinline__ uint32_t die_block_order(uint32_t b, uint32_t n, uint32_t X, uint32_t B) {
  const uint32_t chunk = n / X;
  if (b >= chunk * X) return b;
  const uint32_t x = b % X, j = b / X;
  if (B == 0) return x * chunk + j;
  const uint32_t whole = chunk / B * B;  // die x's first `whole` workgroups take their blocks
  return j < whole ? ((j / B) * X + x) * B + j % B : whole * X + x * (chunk - whole) + (j - whole);
}

// Direct mode with a sharing order of the R rows: die x takes positions [x R / X, (x + 1) R / X) of the order,
// tile after tile; every die gets G = ceil(R / X) workgroups per tile, and where R / X is not whole the last
// workgroup of some dies has no row (returns false).  Over b in [0, T X G) every (tile < T, position < R)
// comes up exactly once.
__device__ __forceinline__ bool die_group_order(uint32_t b, uint32_t R, uint32_t X, uint32_t G, uint32_t& tile,
                                                uint32_t& position) {
  const uint32_t x = b % X, j = b / X;
  tile = j / G;
  const uint32_t q = j - tile * G;
  const uint32_t first = x * R / X, count = (x + 1) * R / X - first;
  position = q < count ? first + q : 0;
  return q < count;
}

// Element types, with the elements per lane and vector of a handle whose parameters have that type:
// float32 4 (one 128-bit access); bfloat16 8, held as two groups of four (two 64-bit accesses of x and
// g, two 128-bit accesses of each float32 state vector; see load_vals for where the groups lie).
struct TF32 {
  static constexpr int bytes = 4;
  static constexpr int vec = 4;
};
struct TBF16 {
  static constexpr int bytes = 2;
  static constexpr int vec = 8;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// float32 -> bfloat16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  return (f != f) ? ((u >> 16) | 0x40u) : r;
}

template <typename T>
__device__ __forceinline__ float load_elem(const void* base, uint64_t e) {
  if constexpr (T::bytes == 4) {
    return reinterpret_cast<const float*>(base)[e];
  } else {
    return bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(base)[e]);
  }
}

template <typename T>
__device__ __forceinline__ void store_elem(void* base, uint64_t e, float v) {
  if constexpr (T::bytes == 4) {
    reinterpret_cast<float*>(base)[e] = v;
  } else {
    reinterpret_cast<uint16_t*>(base)[e] = (uint16_t)f32_to_bf16_bits(v);
  }
}

// The VEC elements of one lane and vector, of type T, widened to float.  VEC = 4: elements
// [e, e + 4).  VEC = 8: two groups of four, [e, e + 4) and [e + H, e + H + 4), where H is four times
// the number of lanes that work side by side (a wavefront in the tile kernel, a workgroup in the
// others): every access instruction of the group then covers one contiguous run of memory, 16
// bytes per lane for float32 and 8 for bfloat16, and every 128-byte line it touches is touched
// whole.  (Giving a lane 8 consecutive elements instead makes each float32 state access two
// instructions that each touch half of every line: measured 5-13 % slower once stores are involved.)
// e is a multiple of 4, so every group is 16-byte (float32) or 8-byte (bfloat16) aligned.
// MASKED groups that are not wholly inside [lo, hi) touch only the elements that are; the others
// read as zero.
// Streaming accesses: every global datum of a step is touched exactly once, so full-group
// accesses may carry the non-temporal hint (NT) and leave the caches to nobody in particular.
// Which classes of access carry the hint when a handle streams (all eight combinations measured:
// the hints on the stream loads and on the stores carry the gain, the one on source loads is neutral):
constexpr bool kNtSource = true;  // parameter (source) loads
constexpr bool kNtStream = true;  // gradient / moment / accumulator loads
constexpr bool kNtStore = true;   // all stores

template <bool NT, typename V>
__device__ __forceinline__ V vload(const V* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, typename V>
__device__ __forceinline__ void vstore(V* p, V v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

template <typename T, int VEC, int H, bool MASKED, bool NT>
__device__ __forceinline__ void load_vals(const void* base, uint64_t e, uint64_t lo, uint64_t hi,
                                          float (&out)[VEC]) {
  static_assert(VEC == 4 || (VEC == 8 && H >= 4), "a lane holds one or two groups of four elements");
#pragma unroll
  for (int h = 0; h < VEC / 4; ++h) {
    const uint64_t eh = e + (uint64_t)h * H;
    if (!MASKED || (eh >= lo && eh + 4 <= hi)) {
      if constexpr (T::bytes == 4) {
        f4 v = vload<NT && kNtStream>(reinterpret_cast<const f4*>(reinterpret_cast<const float*>(base) + eh));
        out[4 * h + 0] = v.x; out[4 * h + 1] = v.y; out[4 * h + 2] = v.z; out[4 * h + 3] = v.w;
      } else {
        u2 v = vload<NT && kNtStream>(reinterpret_cast<const u2*>(reinterpret_cast<const uint16_t*>(base) + eh));
        out[4 * h + 0] = __uint_as_float(v.x << 16); out[4 * h + 1] = __uint_as_float(v.x & 0xFFFF0000u);
        out[4 * h + 2] = __uint_as_float(v.y << 16); out[4 * h + 3] = __uint_as_float(v.y & 0xFFFF0000u);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t ej = eh + j;
        out[4 * h + j] = (ej >= lo && ej < hi) ? load_elem<T>(base, ej) : 0.0f;
      }
    }
  }
}

template <typename T, int VEC, int H, bool MASKED, bool NT>
__device__ __forceinline__ void store_vals(void* base, uint64_t e, uint64_t lo, uint64_t hi,
                                           const float (&in)[VEC]) {
  static_assert(VEC == 4 || (VEC == 8 && H >= 4), "a lane holds one or two groups of four elements");
#pragma unroll
  for (int h = 0; h < VEC / 4; ++h) {
    const uint64_t eh = e + (uint64_t)h * H;
    if (!MASKED || (eh >= lo && eh + 4 <= hi)) {
      if constexpr (T::bytes == 4) {
        f4 v;
        v.x = in[4 * h + 0]; v.y = in[4 * h + 1]; v.z = in[4 * h + 2]; v.w = in[4 * h + 3];
        vstore<NT && kNtStore>(reinterpret_cast<f4*>(reinterpret_cast<float*>(base) + eh), v);
      } else {
        u2 v;
        v.x = f32_to_bf16_bits(in[4 * h + 0]) | (f32_to_bf16_bits(in[4 * h + 1]) << 16);
        v.y = f32_to_bf16_bits(in[4 * h + 2]) | (f32_to_bf16_bits(in[4 * h + 3]) << 16);
        vstore<NT && kNtStore>(reinterpret_cast<u2*>(reinterpret_cast<uint16_t*>(base) + eh), v);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t ej = eh + j;
        if (ej >= lo && ej < hi) store_elem<T>(base, ej, in[4 * h + j]);
      }
    }
  }
}

// The stores of a row's UT vectors.  With one vector per lane there must be no loop around the store: a loop
// that runs once has a loop-invariant address, the compiler's loop-invariant code motion then "promotes" the
// location to a register and re-creates the store behind the loop - without the non-temporal hint (seen with
// the bfloat16 one-vector tile kernels: 1.2 % slower on the ring of 8; the compile test counts the hints).
template <typename T, int VEC, int H, bool MASKED, bool NT, int UT>
__device__ __forceinline__ void store_vectors(void* base, const uint64_t (&e)[UT], uint64_t lo, uint64_t hi,
                                              const float (&in)[UT][VEC]) {
  if constexpr (UT == 1) {
    store_vals<T, VEC, H, MASKED, NT>(base, e[0], lo, hi, in[0]);
  } else {
#pragma unroll
    for (int u = 0; u < UT; ++u) store_vals<T, VEC, H, MASKED, NT>(base, e[u], lo, hi, in[u]);
  }
}

// The 16 raw bytes of a lane's parameter vector (4 float32, or 2 x 4 bfloat16 in the two groups
// described above), as they are parked in LDS.
template <typename XT, int H, bool MASKED, bool NT>
__device__ __forceinline__ u4 load_raw(const void* base, uint64_t e, uint64_t lo, uint64_t hi) {
  if constexpr (XT::bytes == 4) {
    if (!MASKED || (e >= lo && e + 4 <= hi))
      return vload<NT && kNtSource>(reinterpret_cast<const u4*>(reinterpret_cast<const float*>(base) + e));
    u4 r = {0u, 0u, 0u, 0u};
    const uint32_t* p = reinterpret_cast<const uint32_t*>(base);
    if (e + 0 >= lo && e + 0 < hi) r.x = p[e + 0];
    if (e + 1 >= lo && e + 1 < hi) r.y = p[e + 1];
    if (e + 2 >= lo && e + 2 < hi) r.z = p[e + 2];
    if (e + 3 >= lo && e + 3 < hi) r.w = p[e + 3];
    return r;
  } else {
    static_assert(XT::bytes == 4 || H >= 4, "bfloat16 vectors come in two groups");
    const uint16_t* p = reinterpret_cast<const uint16_t*>(base);
    u2 half[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint64_t eh = e + (uint64_t)h * H;
      if (!MASKED || (eh >= lo && eh + 4 <= hi)) {
        half[h] = vload<NT && kNtSource>(reinterpret_cast<const u2*>(p + eh));
      } else {
        uint32_t q[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) q[j] = (eh + j >= lo && eh + j < hi) ? (uint32_t)p[eh + j] : 0u;
        half[h].x = q[0] | (q[1] << 16);
        half[h].y = q[2] | (q[3] << 16);
      }
    }
    u4 r = {half[0].x, half[0].y, half[1].x, half[1].y};
    return r;
  }
}

template <typename XT>
__device__ __forceinline__ void unpack_raw(u4 r, float (&out)[XT::vec]) {
  if constexpr (XT::bytes == 4) {
    out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y);
    out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
  } else {
    out[0] = __uint_as_float(r.x << 16); out[1] = __uint_as_float(r.x & 0xFFFF0000u);
    out[2] = __uint_as_float(r.y << 16); out[3] = __uint_as_float(r.y & 0xFFFF0000u);
    out[4] = __uint_as_float(r.z << 16); out[5] = __uint_as_float(r.z & 0xFFFF0000u);
    out[6] = __uint_as_float(r.w << 16); out[7] = __uint_as_float(r.w & 0xFFFF0000u);
  }
}

// ---------------------------------------------------------------------------------------------
// Algorithm 3, lines 6-13, for one element.  mix is the finished neighbour sum of line 8.
// Returns x^(t); updates mh, vh, b in registers according to the phase.
// ---------------------------------------------------------------------------------------------
// decay = lambda * x_own (0 where there is no weight decay): the AdamW-style part of the direction.
template <int PHASE>
__device__ __forceinline__ float element_step(const Scalars& s, float mix, float g, float& mh,
                                              float& vh, float& b, float decay) {
  if constexpr (PHASE == kMixOnly || PHASE == kMixConsensus) return mix;
  // lines 6-7: temporary moments from the persistent ones and the fresh gradient
  float m = fmaf(s.beta1, mh, s.omb1 * g);
  float v = fmaf(s.beta2, vh, s.omb2 * (g * g));
  // line 8: bias correction with exponent t_hat, epsilon outside the root
  float denom = sqrtf(v * s.inv_c2) + s.eps;
  float u = (m * s.inv_c1) / denom + decay;
  float x = fmaf(-s.lr, u, mix);
  // line 9
  if constexpr (PHASE == kPlain || PHASE == kFold) b = fmaf(g, s.inv_s, b);
  if constexpr (PHASE == kLoopStart || PHASE == kAlg1) b = g * s.inv_s;
  // lines 10-13
  if constexpr (PHASE == kFold || PHASE == kAlg1) {
    mh = fmaf(s.beta1, mh, s.omb1 * b);
    vh = fmaf(s.betav, vh, s.ombv * (b * b));
    b = 0.0f;
  }
  return x;
}

template <int PHASE>
struct Needs {
  static constexpr bool mixing_only = PHASE == kMixOnly || PHASE == kMixConsensus;
  static constexpr bool grad = !mixing_only;
  static constexpr bool moments_in = !mixing_only;
  static constexpr bool acc_in = PHASE == kPlain || PHASE == kFold;
  static constexpr bool acc_out = PHASE == kPlain || PHASE == kLoopStart || PHASE == kFold;
  static constexpr bool moments_out = PHASE == kFold || PHASE == kAlg1;
};

// Which segment does work item `work` belong to, and which tile of the launch's grid is it?
// (Fields are read one by one through the pointer: copying the struct would put it in scratch.)
__device__ __forceinline__ void locate(const StepArgs& a, uint32_t work, uint64_t& tile_index,
                                       uint64_t& lo, uint64_t& hi, float& weight_decay) {
  const uint32_t grid = a.grid;
  const Segment* seg = a.seg;
  uint32_t s = 0;
  if (a.n_seg > 1) {
    uint32_t l = 0, r = a.n_seg;
    while (r - l > 1) {
      uint32_t mid = (l + r) >> 1;
      if (seg[mid].work0[grid] <= work) l = mid; else r = mid;
    }
    s = l;
  }
  tile_index = seg[s].first_tile[grid] + (work - seg[s].work0[grid]);
  const uint64_t slo = seg[s].lo, shi = seg[s].hi;
  lo = slo > a.clip_lo ? slo : a.clip_lo;
  hi = shi < a.clip_hi ? shi : a.clip_hi;
  weight_decay = seg[s].weight_decay;
}

// Pointers of the bound buffers.  EXT = false: from the argument block (at most kInlineRows rows and
// sources).  EXT = true: from the device-resident tables of a larger handle.  EXT is a parameter of the
// kernels themselves and the launcher picks: the small case is exactly the code it was before large handles
// existed, registers included (choosing per pointer inside the kernel cost 2.5 % with 64 rows, and a choice
// between two reads of the same type even forced the whole argument block into scratch; one branch around
// two bodies in one kernel gave the small case the large one's register count: bfloat16 plain phase 63 -> 71
// vector registers, 8 -> 7 wavefronts per SIMD, 1.2 % slower on the ring of 8).  The tables hold addresses as
// integers; the cast names global memory, or every access through the pointer would become a flat one
// (slower, and counted with the LDS operations the row loop waits for).
enum TableOf : int { kSrc = 0, kDst = 1, kMHat = 2, kVHat = 3, kAcc = 4 };  // order of BoundTables' members
static_assert(sizeof(BoundTables) == 5 * kMaxRows * sizeof(uint64_t), "BoundTables is five arrays of addresses");
template <typename P>
__device__ __forceinline__ P table_entry(const BoundTables* ext, TableOf which, int index) {
  const uint64_t v = reinterpret_cast<const uint64_t*>(ext)[which * kMaxRows + index];
  typedef typename std::remove_pointer<P>::type __attribute__((address_space(1))) * Global;
  return (P)(Global)v;
}
template <bool EXT>
__device__ __forceinline__ const void* src_of(const StepArgs& a, int c) {
  if constexpr (EXT) return table_entry<const void*>(a.ext, kSrc, c);
  else return a.x_src[c];
}
template <bool EXT>
__device__ __forceinline__ void* dst_of(const StepArgs& a, int i) {
  if constexpr (EXT) return table_entry<void*>(a.ext, kDst, i);
  else return a.x_dst[i];
}
template <bool EXT>
__device__ __forceinline__ float* m_hat_of(const StepArgs& a, int i) {
  if constexpr (EXT) return table_entry<float*>(a.ext, kMHat, i);
  else return a.m_hat[i];
}
template <bool EXT>
__device__ __forceinline__ float* v_hat_of(const StepArgs& a, int i) {
  if constexpr (EXT) return table_entry<float*>(a.ext, kVHat, i);
  else return a.v_hat[i];
}
template <bool EXT>
__device__ __forceinline__ float* acc_of(const StepArgs& a, int i) {
  if constexpr (EXT) return table_entry<float*>(a.ext, kAcc, i);
  else return a.acc[i];
}

// Up to 64 entries of row i's neighbour list, one per lane (a row with more entries is walked in chunks
// of 64), the row's length and where its list starts, as wave-uniform values.
struct RowList {
  int32_t col_v;
  float w_v;
  int deg;  // entries of the whole row
  int k0;   // index of the row's first entry in col / w
};

// Entries [k0 + first, k0 + first + 64) of a row of `deg` entries, one per lane.
__device__ __forceinline__ void load_list_chunk(const StepArgs& a, RowList& r, int first, int lane) {
  const int left = r.deg - first;  // >= 1
  const int idx = r.k0 + first + (lane < left ? lane : 0);
  r.col_v = a.col[idx];
  r.w_v = a.w[idx];
}

__device__ __forceinline__ RowList load_row_list(const StepArgs& a, int row, int lane) {
  // row_ptr entries are read by every lane from the same address (one broadcast transaction)
  int k0 = __builtin_amdgcn_readfirstlane(a.row_ptr[row]);
  int k1 = __builtin_amdgcn_readfirstlane(a.row_ptr[row + 1]);
  RowList r;
  r.deg = k1 - k0;  // host guarantees 1 <= deg <= n_cols
  r.k0 = k0;
  load_list_chunk(a, r, 0, lane);
  return r;
}

// All of row_ptr in registers (lane l of pair j holds row_ptr[64 j + l] and row_ptr[64 j + l + 1]; one
// pair covers 64 rows, three the 160 rows a large handle may have), so that a wavefront that walks
// several rows finds each row's bounds with two lane reads instead of a load it would have to wait for
// behind its own earlier stores.
template <bool EXT>
struct RowPtrs {
  static constexpr int pairs = EXT ? (kMaxRows + kWave - 1) / kWave : 1;
  int32_t lo[pairs], hi[pairs];
};

template <bool EXT>
__device__ __forceinline__ RowPtrs<EXT> load_row_ptrs(const StepArgs& a, int lane) {
  RowPtrs<EXT> p;
#pragma unroll
  for (int j = 0; j < RowPtrs<EXT>::pairs; ++j) {
    const int r = j * kWave + lane < (int)a.n_rows ? j * kWave + lane : 0;
    p.lo[j] = a.row_ptr[r];
    p.hi[j] = a.row_ptr[r + 1];
  }
  return p;
}

// First chunk of row `row`'s list (row is wave-uniform).
template <bool EXT>
__device__ __forceinline__ RowList load_row_list(const StepArgs& a, const RowPtrs<EXT>& p, int row, int lane) {
  int k0 = 0, k1 = 0;
  if constexpr (!EXT) {
    k0 = __builtin_amdgcn_readlane(p.lo[0], row);
    k1 = __builtin_amdgcn_readlane(p.hi[0], row);
  } else {
#pragma unroll
    for (int j = 0; j < RowPtrs<EXT>::pairs; ++j)
      if (row >= j * kWave && row < (j + 1) * kWave) {  // wave-uniform: one of the pairs
        k0 = __builtin_amdgcn_readlane(p.lo[j], row - j * kWave);
        k1 = __builtin_amdgcn_readlane(p.hi[j], row - j * kWave);
      }
  }
  RowList r;
  r.deg = k1 - k0;  // host guarantees 1 <= deg <= n_cols
  r.k0 = k0;
  load_list_chunk(a, r, 0, lane);
  return r;
}

// Entry k (0 <= k < 64) of the chunk the list currently holds.
__device__ __forceinline__ int list_col(const RowList& r, int k) {
  return __builtin_amdgcn_readlane(r.col_v, k);
}
__device__ __forceinline__ float list_w(const RowList& r, int k) {
  return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(r.w_v), k));
}

// ---------------------------------------------------------------------------------------------
// tile mode
// ---------------------------------------------------------------------------------------------
// The stream inputs of one row of a tile: gradient, moments, accumulator (whatever the phase needs).
template <typename GT, int PHASE, int VEC, int UT, bool MASKED, bool NT, bool EXT>
__device__ __forceinline__ void load_row_inputs(const StepArgs& a, int i, const uint64_t (&e)[UT], uint64_t lo,
                                                uint64_t hi, float (&g)[UT][VEC], float (&mh)[UT][VEC],
                                                float (&vh)[UT][VEC], float (&b)[UT][VEC]) {
  if constexpr (Needs<PHASE>::grad) {
    const void* gp = a.grad[i];
#pragma unroll
    for (int u = 0; u < UT; ++u) load_vals<GT, VEC, kHalfWave, MASKED, NT>(gp, e[u], lo, hi, g[u]);
  }
  if constexpr (Needs<PHASE>::moments_in) {
    const float* mp = m_hat_of<EXT>(a, i);
    const float* vp = v_hat_of<EXT>(a, i);
#pragma unroll
    for (int u = 0; u < UT; ++u) load_vals<TF32, VEC, kHalfWave, MASKED, NT>(mp, e[u], lo, hi, mh[u]);
#pragma unroll
    for (int u = 0; u < UT; ++u) load_vals<TF32, VEC, kHalfWave, MASKED, NT>(vp, e[u], lo, hi, vh[u]);
  }
  if constexpr (Needs<PHASE>::acc_in) {
    const float* bp = acc_of<EXT>(a, i);
#pragma unroll
    for (int u = 0; u < UT; ++u) load_vals<TF32, VEC, kHalfWave, MASKED, NT>(bp, e[u], lo, hi, b[u]);
  }
}

// Mixing from LDS, the update of Algorithm 3 and the stores of one row of a tile.
template <typename XT, int PHASE, int VEC, int UT, bool MASKED, bool NT, bool EXT>
__device__ __forceinline__ void finish_row(const StepArgs& a, const u4* lds, int i, RowList rl,
                                           const uint64_t (&e)[UT], uint64_t lo, uint64_t hi, float wd, int lane,
                                           float (&g)[UT][VEC], float (&mh)[UT][VEC], float (&vh)[UT][VEC],
                                           float (&b)[UT][VEC]) {
  // neighbour sum in the order the row lists its entries: first a product, then fused
  // multiply-adds
  float mix[UT][VEC];
  {
    const int c0 = list_col(rl, 0);
    const float w0 = list_w(rl, 0);
#pragma unroll
    for (int u = 0; u < UT; ++u) {
      float xs[VEC];
      unpack_raw<XT>(lds[(c0 * UT + u) * kWave + lane], xs);
#pragma unroll
      for (int j = 0; j < VEC; ++j) mix[u][j] = w0 * xs[j];
    }
  }
  for (int k = 1, first = 0; k < rl.deg; ++k) {
    if constexpr (EXT) {
      if (k - first == kWave) {  // a row of more than 64 entries: the next 64 of them
        first = k;
        load_list_chunk(a, rl, first, lane);
      }
    }
    const int c = list_col(rl, k - first);
    const float wk = list_w(rl, k - first);
#pragma unroll
    for (int u = 0; u < UT; ++u) {
      float xs[VEC];
      unpack_raw<XT>(lds[(c * UT + u) * kWave + lane], xs);
#pragma unroll
      for (int j = 0; j < VEC; ++j) mix[u][j] = fmaf(wk, xs[j], mix[u][j]);
    }
  }

  // decoupled weight decay acts on the row's own previous parameters: source buffer i
  float decay[UT][VEC];
#pragma unroll
  for (int u = 0; u < UT; ++u)
#pragma unroll
    for (int j = 0; j < VEC; ++j) decay[u][j] = 0.0f;
  if (!Needs<PHASE>::mixing_only && wd != 0.0f) {
#pragma unroll
    for (int u = 0; u < UT; ++u) {
      float xs[VEC];
      unpack_raw<XT>(lds[(i * UT + u) * kWave + lane], xs);
#pragma unroll
      for (int j = 0; j < VEC; ++j) decay[u][j] = wd * xs[j];
    }
  }

  float xo[UT][VEC];
#pragma unroll
  for (int u = 0; u < UT; ++u)
#pragma unroll
    for (int j = 0; j < VEC; ++j)
      xo[u][j] = element_step<PHASE>(a.s, mix[u][j], g[u][j], mh[u][j], vh[u][j], b[u][j], decay[u][j]);

  store_vectors<XT, VEC, kHalfWave, MASKED, NT>(dst_of<EXT>(a, i), e, lo, hi, xo);
  if constexpr (Needs<PHASE>::acc_out) store_vectors<TF32, VEC, kHalfWave, MASKED, NT>(acc_of<EXT>(a, i), e, lo, hi, b);
  if constexpr (Needs<PHASE>::moments_out) {
    store_vectors<TF32, VEC, kHalfWave, MASKED, NT>(m_hat_of<EXT>(a, i), e, lo, hi, mh);
    store_vectors<TF32, VEC, kHalfWave, MASKED, NT>(v_hat_of<EXT>(a, i), e, lo, hi, vh);
  }
}

template <typename XT, typename GT, int PHASE, int W, int UT, bool MASKED, bool NT, bool EXT>
__device__ __forceinline__ void tile_body(const StepArgs& a, u4* lds, uint64_t tbase, uint64_t lo,
                                          uint64_t hi, float wd, uint32_t tile_id, int lane, int wave) {
  constexpr int VEC = XT::vec;
  uint64_t e[UT];
#pragma unroll
  for (int u = 0; u < UT; ++u) e[u] = tbase + (uint64_t)u * (kWave * VEC) + 4u * (uint32_t)lane;

  const int n_rows = (int)a.n_rows;
  const RowPtrs<EXT> rp = load_row_ptrs<EXT>(a, lane);

  // stage every source buffer's slice of the tile: HBM -> registers -> LDS, once.  With more than
  // two sources per wavefront, a wavefront issues the loads of up to KB of them before it parks
  // the first, so that their latencies overlap (+3 % with 64 sources); with one or two, taking
  // them in turn is faster (3 % in the bfloat16 ring of 8), so both forms are here.
  const int n_cols = (int)a.n_cols;
  if (n_cols > 2 * W) {
    constexpr int KB = 8 / UT;
    for (int c0 = wave; c0 < n_cols; c0 += KB * W) {
      u4 r[KB][UT];
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const int c = c0 + k * W;
        if (c < n_cols) {
          const void* src = src_of<EXT>(a, c);
#pragma unroll
          for (int u = 0; u < UT; ++u) r[k][u] = load_raw<XT, kHalfWave, MASKED, NT>(src, e[u], lo, hi);
        }
      }
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const int c = c0 + k * W;
        if (c < n_cols) {
#pragma unroll
          for (int u = 0; u < UT; ++u) lds[(c * UT + u) * kWave + lane] = r[k][u];
        }
      }
    }
  } else {
    for (int c = wave; c < n_cols; c += W) {
      const void* src = src_of<EXT>(a, c);
      u4 r[UT];
#pragma unroll
      for (int u = 0; u < UT; ++u) r[u] = load_raw<XT, kHalfWave, MASKED, NT>(src, e[u], lo, hi);
#pragma unroll
      for (int u = 0; u < UT; ++u) lds[(c * UT + u) * kWave + lane] = r[u];
    }
  }
  // the first row's neighbour list travels while the group meets at the barrier
  RowList rl_next = load_row_list(a, rp, wave < n_rows ? wave : 0, lane);
  __syncthreads();

  if constexpr (PHASE == kMixConsensus) {
    // Consensus error of the sources, sum_c (x_c - mean)^2 per element, as a by-product: the whole
    // tile is in LDS anyway.  One pass on values shifted by source 0, y_c = x_c - x_0, so that
    // sum y^2 - (sum y)^2 / C does not cancel.  The work is dealt evenly: each wavefront takes
    // PER of the tile's 16-byte slots, and its G = 64 / PER lane groups take every G-th source;
    // the groups' sums of y meet through lane exchanges before they are squared.
    // Elements outside the segment were staged as zeros in every source and add nothing.
    constexpr int PER = UT * kWave / W;
    constexpr int G = kWave / PER;
    static_assert(PER >= 1 && PER * W == UT * kWave && G * PER == kWave, "tile does not divide");
    const int q = wave * PER + (lane % PER);
    const int grp = lane / PER;
    float ref[VEC], s1[VEC], s2[VEC];
    unpack_raw<XT>(lds[q], ref);
#pragma unroll
    for (int j = 0; j < VEC; ++j) { s1[j] = 0.0f; s2[j] = 0.0f; }
    for (int c = 1 + grp; c < n_cols; c += G) {
      float xs[VEC];
      unpack_raw<XT>(lds[c * (UT * kWave) + q], xs);
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const float y = xs[j] - ref[j];
        s1[j] += y;
        s2[j] = fmaf(y, y, s2[j]);
      }
    }
#pragma unroll
    for (int off = PER; off < kWave; off <<= 1)
#pragma unroll
      for (int j = 0; j < VEC; ++j) s1[j] += __shfl_xor(s1[j], off);
    const float inv_c = grp == 0 ? 1.0f / (float)n_cols : 0.0f;
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc += s2[j] - s1[j] * s1[j] * inv_c;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0)
      atomicAdd(a.partials + ((tile_id * (uint32_t)W + (uint32_t)wave) % kConsensusPartials), (double)acc);
  }

  // Each row's list is fetched one row ahead, so that no row waits for a load issued behind the
  // previous row's stores (memory operations of a wavefront retire in order).
  // (Issuing the next row's gradient and state loads early as well was measured and changes
  // nothing: with 8-32 wavefronts per CU in flight the memory system, not latency, is the limit.)
  for (int i = wave; i < n_rows; i += W) {
    const RowList rl = rl_next;
    rl_next = load_row_list(a, rp, i + W < n_rows ? i + W : i, lane);
    float g[UT][VEC], mh[UT][VEC], vh[UT][VEC], b[UT][VEC];
    load_row_inputs<GT, PHASE, VEC, UT, MASKED, NT, EXT>(a, i, e, lo, hi, g, mh, vh, b);
    finish_row<XT, PHASE, VEC, UT, MASKED, NT, EXT>(a, lds, i, rl, e, lo, hi, wd, lane, g, mh, vh, b);
  }
}

template <typename XT, typename GT, int PHASE, int W, int UT, bool NT, bool EXT>
__global__ __launch_bounds__(kWave* W) void k_tile(const StepArgs a) {
  constexpr int VEC = XT::vec;
  constexpr uint64_t TILE = (uint64_t)kWave * VEC * UT;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_bytes[];
  u4* lds = reinterpret_cast<u4*>(lds_bytes);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  // Consecutive workgroup ids are dispatched to the device's X dies (XCDs, 8 on an MI355X) in turn.
  // Left alone, every die would touch every X-th tile of every array.  Instead the tiles are cut into blocks
  // of B = 32 and the blocks go to the dies in turn, so that each die (and its L2) reads and writes runs of
  // 32 consecutive tiles while all dies stay in the same neighbourhood of every array.  Measured on the
  // placed layout, against tile-by-tile round robin: one contiguous X-th of the tiles per die +2.5 %; blocks
  // of 32 tiles another +0.4 % (float32, 16 replicas) to +1.5 % (bfloat16 ring of 8); blocks of 16 ... 1024
  // all lie within 0.5 % of that, powers of two ahead of their neighbours.
  const uint32_t b = die_block_order(blockIdx.x, gridDim.x, a.n_xcd, a.xcd_block);
  uint64_t tile_index, lo, hi;
  float wd;
  locate(a, a.work_begin + b, tile_index, lo, hi, wd);
  const uint64_t tbase = tile_index * TILE;
  const bool full = tbase >= lo && tbase + TILE <= hi;
  if (full) tile_body<XT, GT, PHASE, W, UT, false, NT, EXT>(a, lds, tbase, lo, hi, wd, b, lane, wave);
  else tile_body<XT, GT, PHASE, W, UT, true, NT, EXT>(a, lds, tbase, lo, hi, wd, b, lane, wave);
}

// ---------------------------------------------------------------------------------------------
// direct mode
// ---------------------------------------------------------------------------------------------
constexpr int kUD = 2;  // 16-byte parameter vectors per thread (1 and 4 measured slower)

// Neighbour sum with all loads of DEG sources issued before the first use.  DEG == 0: any degree.
template <typename XT, int DEG, bool MASKED, bool NT, bool EXT>  // NT: hint on the source loads
__device__ __forceinline__ void mix_direct(const StepArgs& a, RowList rl, int lane,
                                           const uint64_t (&e)[kUD], uint64_t lo, uint64_t hi,
                                           float (&mix)[kUD][XT::vec]) {
  constexpr int VEC = XT::vec;
  if constexpr (DEG > 0) {
    u4 r[DEG][kUD];
    float wk[DEG];
#pragma unroll
    for (int k = 0; k < DEG; ++k) {
      const void* src = src_of<EXT>(a, list_col(rl, k));
      wk[k] = list_w(rl, k);
#pragma unroll
      for (int u = 0; u < kUD; ++u) r[k][u] = load_raw<XT, kHalfGroup, MASKED, NT>(src, e[u], lo, hi);
    }
#pragma unroll
    for (int k = 0; k < DEG; ++k)
#pragma unroll
      for (int u = 0; u < kUD; ++u) {
        float xs[VEC];
        unpack_raw<XT>(r[k][u], xs);
#pragma unroll
        for (int j = 0; j < VEC; ++j) mix[u][j] = (k == 0) ? wk[0] * xs[j] : fmaf(wk[k], xs[j], mix[u][j]);
      }
  } else {
    {
      const void* src = src_of<EXT>(a, list_col(rl, 0));
      const float w0 = list_w(rl, 0);
#pragma unroll
      for (int u = 0; u < kUD; ++u) {
        float xs[VEC];
        unpack_raw<XT>(load_raw<XT, kHalfGroup, MASKED, NT>(src, e[u], lo, hi), xs);
#pragma unroll
        for (int j = 0; j < VEC; ++j) mix[u][j] = w0 * xs[j];
      }
    }
    for (int k = 1, first = 0; k < rl.deg; ++k) {
      if constexpr (EXT) {
        if (k - first == kWave) {  // a row of more than 64 entries: the next 64 of them
          first = k;
          load_list_chunk(a, rl, first, lane);
        }
      }
      const void* src = src_of<EXT>(a, list_col(rl, k - first));
      const float wk = list_w(rl, k - first);
#pragma unroll
      for (int u = 0; u < kUD; ++u) {
        float xs[VEC];
        unpack_raw<XT>(load_raw<XT, kHalfGroup, MASKED, NT>(src, e[u], lo, hi), xs);
#pragma unroll
        for (int j = 0; j < VEC; ++j) mix[u][j] = fmaf(wk, xs[j], mix[u][j]);
      }
    }
  }
}

// HINT: 0 no streaming hints, 1 on every vector access, 2 on all but the loads of sources (rows share
// sources: the second reader must find them in the cache, while gradients, state and all stores still stream).
template <typename XT, typename GT, int PHASE, bool MASKED, int HINT, bool EXT>
__device__ __forceinline__ void direct_body(const StepArgs& a, int row, uint64_t tbase, uint64_t lo,
                                            uint64_t hi, float wd, int lane) {
  constexpr bool NT = HINT != 0, NTSRC = HINT == 1;
  constexpr int VEC = XT::vec;
  uint64_t e[kUD];
#pragma unroll
  for (int u = 0; u < kUD; ++u) e[u] = tbase + (uint64_t)u * (kDirectThreads * VEC) + 4u * threadIdx.x;
  // The neighbour list sits one entry per lane and is handed out with readlane, which must find a
  // loaded value in whichever lane it asks.  So no lane may leave before the last readlane: a
  // thread of a clipped tile whose vectors all lie outside the range runs through the body with
  // every access masked off instead of returning early.  (With an early return the compiler is
  // free to sink the list's load below it, into the lanes that stay - and a row whose leading
  // lanes lie before the segment then reads its neighbours' indices from lanes that never loaded.)
  RowList rl = load_row_list(a, row, lane);
  float g[kUD][VEC], mh[kUD][VEC], vh[kUD][VEC], b[kUD][VEC];
  if constexpr (Needs<PHASE>::grad) {
    const void* gp = a.grad[row];
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<GT, VEC, kHalfGroup, MASKED, NT>(gp, e[u], lo, hi, g[u]);
  }
  if constexpr (Needs<PHASE>::moments_in) {
    const float* mp = m_hat_of<EXT>(a, row);
    const float* vp = v_hat_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<TF32, VEC, kHalfGroup, MASKED, NT>(mp, e[u], lo, hi, mh[u]);
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<TF32, VEC, kHalfGroup, MASKED, NT>(vp, e[u], lo, hi, vh[u]);
  }
  if constexpr (Needs<PHASE>::acc_in) {
    const float* bp = acc_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<TF32, VEC, kHalfGroup, MASKED, NT>(bp, e[u], lo, hi, b[u]);
  }
  float mix[kUD][VEC];
  switch (rl.deg) {
    case 1: mix_direct<XT, 1, MASKED, NTSRC, EXT>(a, rl, lane, e, lo, hi, mix); break;
    case 2: mix_direct<XT, 2, MASKED, NTSRC, EXT>(a, rl, lane, e, lo, hi, mix); break;
    case 3: mix_direct<XT, 3, MASKED, NTSRC, EXT>(a, rl, lane, e, lo, hi, mix); break;
    case 4: mix_direct<XT, 4, MASKED, NTSRC, EXT>(a, rl, lane, e, lo, hi, mix); break;
    case 5: mix_direct<XT, 5, MASKED, NTSRC, EXT>(a, rl, lane, e, lo, hi, mix); break;
    default: mix_direct<XT, 0, MASKED, NTSRC, EXT>(a, rl, lane, e, lo, hi, mix); break;
  }
  // decoupled weight decay acts on the row's own previous parameters: source buffer `row` (the
  // load repeats one the mixing sum has just made, so it is served by the cache)
  float decay[kUD][VEC];
#pragma unroll
  for (int u = 0; u < kUD; ++u)
#pragma unroll
    for (int j = 0; j < VEC; ++j) decay[u][j] = 0.0f;
  if (!Needs<PHASE>::mixing_only && wd != 0.0f) {
    const void* own = src_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) {
      float xs[VEC];
      unpack_raw<XT>(load_raw<XT, kHalfGroup, MASKED, false>(own, e[u], lo, hi), xs);
#pragma unroll
      for (int j = 0; j < VEC; ++j) decay[u][j] = wd * xs[j];
    }
  }
  float xo[kUD][VEC];
#pragma unroll
  for (int u = 0; u < kUD; ++u)
#pragma unroll
    for (int j = 0; j < VEC; ++j)
      xo[u][j] = element_step<PHASE>(a.s, mix[u][j], g[u][j], mh[u][j], vh[u][j], b[u][j], decay[u][j]);
  void* xd = dst_of<EXT>(a, row);
#pragma unroll
  for (int u = 0; u < kUD; ++u) store_vals<XT, VEC, kHalfGroup, MASKED, NT>(xd, e[u], lo, hi, xo[u]);
  if constexpr (Needs<PHASE>::acc_out) {
    float* bp = acc_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) store_vals<TF32, VEC, kHalfGroup, MASKED, NT>(bp, e[u], lo, hi, b[u]);
  }
  if constexpr (Needs<PHASE>::moments_out) {
    float* mp = m_hat_of<EXT>(a, row);
    float* vp = v_hat_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) store_vals<TF32, VEC, kHalfGroup, MASKED, NT>(mp, e[u], lo, hi, mh[u]);
#pragma unroll
    for (int u = 0; u < kUD; ++u) store_vals<TF32, VEC, kHalfGroup, MASKED, NT>(vp, e[u], lo, hi, vh[u]);
  }
}

// Work items are numbered tile-major, row-minor, so that workgroups running at the same time work
// on the same elements of different rows.
template <typename XT, typename GT, int PHASE, int HINT, bool EXT>
__global__ __launch_bounds__(kDirectThreads) void k_direct(const StepArgs a) {
  constexpr int VEC = XT::vec;
  constexpr uint64_t TILE = (uint64_t)kDirectThreads * VEC * kUD;
  const int lane = threadIdx.x & (kWave - 1);
  const uint32_t n_rows = a.n_rows;
  uint32_t t;
  int row;
  bool active = true;
  if (a.row_order != nullptr) {
    // Rows share sources.  Consecutive workgroup ids go to the device's X dies in turn; die x takes the
    // rows at positions [x R / X, (x + 1) R / X) of the sharing order (R = n_rows), tile after tile: the
    // rows that read a source run on one die at about the same time, and the second reader finds the
    // source in that die's L2.  Every die gets G = ceil(R / X) workgroups per tile; where R / X is not whole,
    // the last workgroup of some dies has no row and does nothing (the whole workgroup, so no lane leaves
    // a wavefront early).
    uint32_t position;
    active = die_group_order(blockIdx.x, n_rows, a.n_xcd, a.order_group, t, position);
    row = __builtin_amdgcn_readfirstlane(a.row_order[position]);
  } else {
    // Nothing is shared: workgroups in launch order.  (Tile mode's orders were measured here too: one contiguous
    // X-th of the tiles per die costs 1 % on one row with three sources and 4 % bucket by bucket, blocks of 2 to
    // 256 workgroups per die 0.1-1.3 %.)
    t = blockIdx.x / n_rows;
    row = (int)(blockIdx.x - t * n_rows);
  }
  uint64_t tile_index, lo, hi;
  float wd;
  locate(a, a.work_begin + t, tile_index, lo, hi, wd);
  const uint64_t tbase = tile_index * TILE;
  const bool full = tbase >= lo && tbase + TILE <= hi;
  if (active) {  // uniform over the workgroup
    if (full) direct_body<XT, GT, PHASE, false, HINT, EXT>(a, row, tbase, lo, hi, wd, lane);
    else direct_body<XT, GT, PHASE, true, HINT, EXT>(a, row, tbase, lo, hi, wd, lane);
  }
}

// ---------------------------------------------------------------------------------------------
// accumulate / fold only (Algorithm 3 lines 9-13).  Walks the direct kernel's tile grid, so a lane
// vector has as many elements as a parameter vector of the handle (4 or 8).
// ---------------------------------------------------------------------------------------------
template <int PHASE>
__device__ __forceinline__ void acc_step(const Scalars& s, float g, float& mh, float& vh, float& b) {
  if constexpr (PHASE == kPlain || PHASE == kFold) b = fmaf(g, s.inv_s, b);
  if constexpr (PHASE == kLoopStart || PHASE == kAlg1) b = g * s.inv_s;
  if constexpr (PHASE == kFold || PHASE == kAlg1) {
    mh = fmaf(s.beta1, mh, s.omb1 * b);
    vh = fmaf(s.betav, vh, s.ombv * (b * b));
    b = 0.0f;
  }
}

template <typename GT, int VEC, int PHASE, bool MASKED, bool NT, bool EXT>
__device__ __forceinline__ void acc_body(const StepArgs& a, int row, uint64_t tbase, uint64_t lo,
                                         uint64_t hi) {
  uint64_t e[kUD];
#pragma unroll
  for (int u = 0; u < kUD; ++u) e[u] = tbase + (uint64_t)u * (kDirectThreads * VEC) + 4u * threadIdx.x;
  float g[kUD][VEC], mh[kUD][VEC], vh[kUD][VEC], b[kUD][VEC];
  const void* gp = a.grad[row];
#pragma unroll
  for (int u = 0; u < kUD; ++u) load_vals<GT, VEC, kHalfGroup, MASKED, NT>(gp, e[u], lo, hi, g[u]);
  if constexpr (Needs<PHASE>::moments_out) {
    const float* mp = m_hat_of<EXT>(a, row);
    const float* vp = v_hat_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<TF32, VEC, kHalfGroup, MASKED, NT>(mp, e[u], lo, hi, mh[u]);
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<TF32, VEC, kHalfGroup, MASKED, NT>(vp, e[u], lo, hi, vh[u]);
  }
  if constexpr (Needs<PHASE>::acc_in) {
    const float* bp = acc_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) load_vals<TF32, VEC, kHalfGroup, MASKED, NT>(bp, e[u], lo, hi, b[u]);
  }
#pragma unroll
  for (int u = 0; u < kUD; ++u)
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc_step<PHASE>(a.s, g[u][j], mh[u][j], vh[u][j], b[u][j]);
  if constexpr (Needs<PHASE>::acc_out) {
    float* bp = acc_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) store_vals<TF32, VEC, kHalfGroup, MASKED, NT>(bp, e[u], lo, hi, b[u]);
  }
  if constexpr (Needs<PHASE>::moments_out) {
    float* mp = m_hat_of<EXT>(a, row);
    float* vp = v_hat_of<EXT>(a, row);
#pragma unroll
    for (int u = 0; u < kUD; ++u) store_vals<TF32, VEC, kHalfGroup, MASKED, NT>(mp, e[u], lo, hi, mh[u]);
#pragma unroll
    for (int u = 0; u < kUD; ++u) store_vals<TF32, VEC, kHalfGroup, MASKED, NT>(vp, e[u], lo, hi, vh[u]);
  }
}

// VEC is the element count of a direct-mode parameter vector of this handle, so that the
// accumulate kernel walks the same tile grid as the direct kernel.
template <typename GT, int VEC, int PHASE, bool NT, bool EXT>
__global__ __launch_bounds__(kDirectThreads) void k_acc(const StepArgs a) {
  constexpr uint64_t TILE = (uint64_t)kDirectThreads * VEC * kUD;
  const uint32_t n_rows = a.n_rows;
  const uint32_t t = blockIdx.x / n_rows;
  const int row = (int)(blockIdx.x - t * n_rows);
  uint64_t tile_index, lo, hi;
  float wd_unused;
  locate(a, a.work_begin + t, tile_index, lo, hi, wd_unused);
  const uint64_t tbase = tile_index * TILE;
  const bool full = tbase >= lo && tbase + TILE <= hi;
  if (full) acc_body<GT, VEC, PHASE, false, NT, EXT>(a, row, tbase, lo, hi);
  else acc_body<GT, VEC, PHASE, true, NT, EXT>(a, row, tbase, lo, hi);
}

// ---------------------------------------------------------------------------------------------
// dispatch tables
// ---------------------------------------------------------------------------------------------

template <typename XT, typename GT, int W, int UT, bool NT, bool EXT>
KernelFn tile_kernel_for_phase(int phase) {
  switch (phase) {
    case kMixOnly: return k_tile<XT, GT, kMixOnly, W, UT, NT, EXT>;
    case kMixConsensus: return k_tile<XT, GT, kMixConsensus, W, UT, NT, EXT>;
    case kUpdateOnly: return k_tile<XT, GT, kUpdateOnly, W, UT, NT, EXT>;
    case kPlain: return k_tile<XT, GT, kPlain, W, UT, NT, EXT>;
    case kLoopStart: return k_tile<XT, GT, kLoopStart, W, UT, NT, EXT>;
    case kFold: return k_tile<XT, GT, kFold, W, UT, NT, EXT>;
    case kAlg1: return k_tile<XT, GT, kAlg1, W, UT, NT, EXT>;
  }
  return nullptr;
}

template <typename XT, typename GT, bool NT, bool EXT>
KernelFn tile_kernel_for_shape_nt(int phase, TileShape s) {
  if (s.waves == 4 && s.ut == 1) return tile_kernel_for_phase<XT, GT, 4, 1, NT, EXT>(phase);
  if (s.waves == 4 && s.ut == 2) return tile_kernel_for_phase<XT, GT, 4, 2, NT, EXT>(phase);
  if (s.waves == 8 && s.ut == 1) return tile_kernel_for_phase<XT, GT, 8, 1, NT, EXT>(phase);
  if (s.waves == 8 && s.ut == 2) return tile_kernel_for_phase<XT, GT, 8, 2, NT, EXT>(phase);
#ifdef DADAM_TUNING  // further shapes for measurements, same-type pairs only to bound the build time
  if constexpr (XT::bytes == GT::bytes) {
    if (s.waves == 16 && s.ut == 1) return tile_kernel_for_phase<XT, GT, 16, 1, NT, EXT>(phase);
    if (s.waves == 16 && s.ut == 2) return tile_kernel_for_phase<XT, GT, 16, 2, NT, EXT>(phase);
    if (s.waves == 4 && s.ut == 4) return tile_kernel_for_phase<XT, GT, 4, 4, NT, EXT>(phase);
    if (s.waves == 8 && s.ut == 4) return tile_kernel_for_phase<XT, GT, 8, 4, NT, EXT>(phase);
  }
#endif
  return nullptr;
}
template <typename XT, typename GT, int HINT, bool EXT>
KernelFn direct_kernel_for_phase(int phase) {
  switch (phase) {
    case kMixOnly: return k_direct<XT, GT, kMixOnly, HINT, EXT>;
    case kUpdateOnly: return k_direct<XT, GT, kUpdateOnly, HINT, EXT>;
    case kPlain: return k_direct<XT, GT, kPlain, HINT, EXT>;
    case kLoopStart: return k_direct<XT, GT, kLoopStart, HINT, EXT>;
    case kFold: return k_direct<XT, GT, kFold, HINT, EXT>;
    case kAlg1: return k_direct<XT, GT, kAlg1, HINT, EXT>;
  }
  return nullptr;
}

}  // namespace
}  // namespace dadam

#endif  // DADAM_DEVICE_H_
