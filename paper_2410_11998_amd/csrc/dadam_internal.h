// Internal interface between the host side of libdadam (validation, planning, launch set-up) and
// the gfx950 kernels.  Nothing in here is part of the public C ABI (see include/dadam.h).
#ifndef DADAM_INTERNAL_H_
#define DADAM_INTERNAL_H_

#include <stdint.h>

#include "dadam.h"

namespace dadam {

constexpr int kMaxRows = DADAM_MAX_ROWS;  // rows / source buffers a handle may have
constexpr int kInlineRows = 64;           // up to this many, every pointer table travels in the kernel arguments
constexpr int kWave = 64;            // gfx950 wavefront
constexpr int kDirectThreads = 256;  // workgroup of the direct and accumulate kernels

// A maximal run of contiguous tensors with the same hyper-parameters: elements [lo, hi) of every buffer.  Work items are tiles of a
// fixed grid anchored at element 0, so that vector accesses are 16-byte aligned whenever the
// buffers are; a tile that sticks out of [lo, hi) is clipped element by element.
struct Segment {
  uint64_t lo, hi;
  uint64_t first_tile[3];  // per Grid: index of the first tile of that grid that intersects the segment
  uint32_t work0[3];       // per Grid: number of work items (tiles; per row in direct mode) in earlier segments
  float weight_decay;      // decoupled weight decay of the tensors in this segment
};

// Which of the three tile grids a launch walks: the fused step's tiles, the direct/accumulate
// kernels' tiles, or the wider tiles of the mixing-only launch.
enum Grid : uint32_t { kGridTile = 0, kGridDirect = 1, kGridMix = 2 };

// Scalars of one iteration, computed on the host in double and rounded once.
struct Scalars {
  float beta1, omb1;     // beta1, 1 - beta1
  float beta2, omb2;     // beta2, 1 - beta2
  float betav, ombv;     // decay of v_hat in the fold and its complement
  float inv_c1, inv_c2;  // 1 / (1 - beta1^t_hat), 1 / (1 - beta2^t_hat)
  float eps, lr, inv_s;
};

// What a step does with the optimizer state (Algorithm 3, lines 6-13).
enum Phase : int {
  kMixOnly = 0,     // x_dst = W x_src
  kUpdateOnly = 1,  // lines 6-8 only
  kPlain = 2,       // lines 6-9, inside a loop
  kLoopStart = 3,   // lines 6-9, first iteration of a loop: b is known to be zero and not read
  kFold = 4,        // lines 6-13, last iteration of a loop (s > 1)
  kAlg1 = 5,        // s == 1: Algorithm 1, moments updated every iteration, no accumulator
  kMixConsensus = 6,  // x_dst = W x_src and, on the side, sum_c ||x_src[c] - mean||^2 (tile mode only)
  kNumPhases = 7
};

constexpr uint32_t kConsensusPartials = 1024;  // partial sums the tiles scatter their contributions over
static_assert(kConsensusPartials * sizeof(double) == DADAM_STATIC_SCRATCH_BYTES, "the header states the static scratch size");

// Pointer tables of the bound buffers of a handle with more than kInlineRows rows or sources: they do not
// fit the 4 KB kernel-argument segment and live in device memory, one immutable copy per binding and
// exchange state (see dadam_bind).
// Addresses are held as 64-bit integers on purpose: see the kernels' table helpers.
struct BoundTables {
  uint64_t x_src[kMaxRows];
  uint64_t x_dst[kMaxRows];
  uint64_t m_hat[kMaxRows];
  uint64_t v_hat[kMaxRows];
  uint64_t acc[kMaxRows];
};

// Kernel argument block (passed by value; 3.9 KB of the 4 KB kernarg segment).  The tables of the bound
// buffers are used when `ext` is null (at most kInlineRows rows and sources); otherwise `ext` holds them.
// The gradient pointers change from call to call and always travel here.
struct StepArgs {
  const void* x_src[kInlineRows];
  void* x_dst[kInlineRows];
  float* m_hat[kInlineRows];
  float* v_hat[kInlineRows];
  float* acc[kInlineRows];
  const void* grad[kMaxRows];
  const BoundTables* ext;
  const int32_t* row_ptr;  // device CSR of the slot
  const int32_t* col;
  const float* w;
  // Direct kernels: the rows in an order in which neighbours share sources (device; null: rows as numbered).
  // The device's dies take contiguous groups of this order, so that the rows which read a source run on the
  // die whose L2 already holds it.
  const int32_t* row_order;
  uint32_t order_group;  // with row_order: rows per die, ceil(n_rows / n_xcd); the launch has n_xcd * order_group
                         // workgroups per tile, of which those beyond a die's share of the rows have nothing to do
  const Segment* seg;  // device
  uint32_t n_seg;
  uint32_t n_rows, n_cols;
  uint32_t grid;        // Grid: which tile numbering work items refer to
  uint32_t work_begin;  // first work item (in tiles) of this launch
  uint32_t n_xcd;       // dies that consecutive workgroup ids are dealt over (tile order)
  uint32_t xcd_block;   // tile mode: tiles per block; blocks go to the dies in turn (0: one contiguous share each)
  uint64_t clip_lo, clip_hi;  // element range of this launch (whole layout or a tensor range)
  double* partials;           // kConsensusPartials doubles (device), used by kMixConsensus only
  Scalars s;
};

static_assert(sizeof(StepArgs) <= 4096, "the argument block of a launch holds 4 KB");

constexpr uint32_t kDieBlockTiles = 32;  // measured, see k_tile

typedef void (*KernelFn)(const StepArgs);

struct TileShape {
  int waves;  // wavefronts per workgroup (rows are dealt round-robin to them)
  int ut;     // 16-byte vectors per lane and row
  bool nontemporal;  // streaming hint on every full-vector global access
};

// Launchers.  All of them enqueue on `stream` and return the hipError_t of the launch as int.
// xdt / gdt are DADAM_F32 | DADAM_BF16.  n_work is the number of tiles in this launch.
int launch_tile(int xdt, int gdt, Phase phase, TileShape shape, const StepArgs& a, uint32_t n_work,
                uint32_t lds_bytes, void* stream);
// shared: rows share sources; a streaming launch then keeps the hint off the source loads.
int launch_direct(int xdt, int gdt, Phase phase, bool nontemporal, bool shared, const StepArgs& a,
                  uint32_t n_work_tiles, void* stream);
// vec = elements per direct-mode parameter vector of the handle (fixes the tile grid).
int launch_accumulate(int gdt, Phase phase, bool nontemporal, const StepArgs& a, uint32_t n_work_tiles,
                      void* stream, int vec);

// Consensus error: clear the partial sums / add them up in a fixed order into *out (device).
int launch_consensus_zero(double* partials, void* stream);
int launch_consensus_sum(const double* partials, double* out, void* stream);

// The partial-sum array that lives in the library's device image (no allocation): its address on the
// current device and its capacity in doubles.  Returns a hipError_t as int.
int static_partials(double** out, uint32_t* capacity);

// Geometry the host planner needs.
int vec_elems(int xdt);              // elements per 16-byte parameter vector: 4 (f32) or 8 (bf16)
int direct_unroll();                 // vectors per thread in the direct and accumulate kernels
bool tile_shape_supported(TileShape s);

}  // namespace dadam

#endif  // DADAM_INTERNAL_H_
