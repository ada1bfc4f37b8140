/*
 * dadam - the per-iteration decentralized Adam step on one MI355X (gfx950).
 *
 * One call of dadam_gossip_step performs, for every updated replica ("row") i and every
 * element e of the packed parameter vector, iteration t of the paper's Algorithm 3
 * (appendix "Decentralized accumulated Adam"; Algorithm 1 of section 4 is its case s = 1):
 *
 *     t_hat = ceil(t / s)                                                   line 4
 *     m     = beta1 * m_hat_i[e] + (1 - beta1) * g_i[e]                      line 6
 *     v     = beta2 * v_hat_i[e] + (1 - beta2) * g_i[e]^2                    line 7
 *     x_dst_i[e] = sum_k w[k] * x_src[col[k]][e]                             line 8, mixing term
 *                  - lr * (m / (1 - beta1^t_hat)) / (sqrt(v / (1 - beta2^t_hat)) + eps)       (eq. (2), section 2)
 *     b_i[e] += g_i[e] / s                                                   line 9
 *     if t mod s == 0:  m_hat_i[e] = beta1 * m_hat_i[e] + (1 - beta1) * b_i[e]               lines 10-13
 *                       v_hat_i[e] = beta_vhat * v_hat_i[e] + (1 - beta_vhat) * b_i[e]^2
 *                       b_i[e] = 0
 *
 * A tensor with weight_decay lambda > 0 uses the AdamW-style variant the appendix mentions without
 * writing it out; the reading taken is decoupled decay of the replica's OWN previous parameters
 * inside the search direction (which, as the paper stresses, depends on the worker's own quantities
 * only):   x_dst_i[e] = mixing term - lr * (direction + lambda * x_src[i][e]),  at every iteration.
 * Source buffer i must then be row i's own previous parameters (n_rows <= n_cols).
 *
 * k runs over row i of a CSR neighbour list (row_ptr, col, w); the replica itself is an ordinary
 * entry of its row.  Every row reads the previous iterate x^(t-1) (the sources), never a value
 * written by the same call.  m and v are temporaries and are not stored.
 *
 * General rules of this interface
 *   - All entry points are extern "C", take plain pointers and sizes, return an int status
 *     (0 = DADAM_OK, negative = error) and never throw or abort.  The text of the last error of a
 *     handle is available from dadam_last_error().
 *   - "host" / "device" says where a pointer must point.  Large buffers (parameters, gradients,
 *     moments, accumulator) are DEVICE memory owned by the caller; the library never allocates,
 *     frees or copies them and never synchronises a stream.  The library owns only small metadata
 *     (segment table, CSR slots) on host and device.  (One set-up call is the exception and says so:
 *     dadam_place_by_timing overwrites the empty arena it is given, holds 2 GiB of its own while it runs
 *     and returns when its measurements are done.)
 *   - Launching entry points enqueue work on the given HIP stream (a hipStream_t passed as
 *     void*; NULL = the default stream) and return at once.  The caller keeps every buffer alive
 *     and unmodified until that work has finished.
 *   - All validation happens on the host before anything is launched; a failed call launches
 *     nothing.
 *   - At most DADAM_MAX_ROWS rows and DADAM_MAX_ROWS source buffers per handle (tile mode needs 1 KB of
 *     LDS per source buffer: 160 KB for 160).  Up to 64 of each, every launch carries its own copy of the
 *     pointer tables.  Beyond that the tables of the bound buffers live in device memory, one immutable
 *     copy per dadam_bind; the library keeps the last DADAM_BINDINGS_KEPT of them, so work launched under
 *     a binding must have finished before that many further dadam_bind calls are made, and dadam_bind
 *     then copies to the device (it may wait for work in flight; not for use under stream capture).
 *   - A handle is not thread-safe: calls on one handle must come from one thread at a time.  Launches
 *     on different streams may be in flight together (every launch carries its own copy of the pointer
 *     tables and scalars), except dadam_mix_consensus, whose calls share scratch memory of the handle.
 */
#ifndef DADAM_H_
#define DADAM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DADAM_ABI_VERSION 2u
#define DADAM_MAX_ROWS 160u
#define DADAM_MAX_SLOTS 16u
#define DADAM_BINDINGS_KEPT 8u
#define DADAM_DEVICE_NONE (-1) /* host-only handle: validation and planning work, launches fail */

/* element types of parameters and gradients; m_hat, v_hat and b are always float32 */
#define DADAM_F32 0u
#define DADAM_BF16 1u

/* status codes */
#define DADAM_OK 0
#define DADAM_EINVAL (-1) /* null pointer, zero size, bad enum, value out of range            */
#define DADAM_EALIGN (-2) /* a device buffer is not 16-byte aligned                            */
#define DADAM_ETOPO (-3)  /* malformed neighbour list                                          */
#define DADAM_EALIAS (-4) /* buffers overlap in a way that would let a row read a new value     */
#define DADAM_ESTATE (-5) /* call order: no buffers bound, slot not set, host-only handle, ...  */
#define DADAM_EHIP (-6)   /* a HIP runtime call failed                                         */

/* flags of dadam_gossip_step.  Without a FORCE flag the library chooses: tile mode when some source is read
 * by two or more rows and the tile fits in LDS (also when an in-place row needs it), direct mode otherwise -
 * and also, where measured faster, for rows of at most two sources on more than 16 sources and for rows of at
 * most eight sources when a CU would hold only one workgroup of the tile (see dadam_get_row_order).
 * dadam_slot_uses_tile_mode reports the choice. */
#define DADAM_FUSE_ACCUM 1u   /* also do lines 9-13 (accumulate and fold) in the same pass         */
#define DADAM_FORCE_DIRECT 2u /* every row streams its sources from global memory                  */
#define DADAM_FORCE_TILE 4u   /* stage each source tile once in LDS and update all rows from it    */

/* flags reported by dadam_set_topology through *warn */
#define DADAM_WARN_NOT_COLUMN_STOCHASTIC 1u /* square W whose columns do not sum to 1             */

typedef struct dadam_handle dadam_handle; /* opaque, owned by the library */

/* One tensor of the packed layout: elements [offset_elems, offset_elems + numel) of every
 * per-replica buffer.  Tensors must be listed in increasing offset order and must not overlap;
 * elements between tensors (padding) are never read or written.  weight_decay >= 0 is the decoupled
 * weight decay of this tensor (0 = plain Adam; e.g. 3e-5 on all but the normalisation parameters in
 * the paper's ResNet-50 recipe).  flags is reserved and must be 0. */
typedef struct {
  uint64_t offset_elems;
  uint64_t numel;
  float weight_decay;
  uint32_t flags;
} dadam_tensor_desc;

typedef struct {
  uint32_t abi_version; /* DADAM_ABI_VERSION */
  uint32_t n_rows;      /* R: replicas updated by a step                                          */
  uint32_t n_cols;      /* number of source buffers holding x^(t-1) (R for a full simulation;     */
                        /* own parameters + neighbours' receive buffers for one node's share)     */
  uint64_t d;           /* elements per buffer (packed length, padding included)                  */
  uint32_t n_tensors;
  const dadam_tensor_desc* tensors; /* host, copied */
  uint32_t param_dtype;             /* DADAM_F32 | DADAM_BF16: type of x_src and x_dst            */
  uint32_t grad_dtype;              /* DADAM_F32 | DADAM_BF16: type of the gradients              */
  float lr, beta1, beta2, eps;      /* Algorithm 1 / 3 hyper-parameters                           */
  uint32_t accum_s;                 /* s >= 1, iterations per accumulation loop; 1 = Algorithm 1  */
  float beta_vhat; /* decay of v_hat in the fold (line 12).  The listing prints beta_1 there; that is
                      taken as a misprint and the default, selected by a negative value or NaN, is
                      beta2.  Any value in [0, 1) selects it explicitly. */
  int32_t device;  /* HIP device ordinal, or DADAM_DEVICE_NONE */
  uint32_t lds_limit_bytes; /* LDS one workgroup may use.  0: what the device reports (a host-only handle
                               assumes 65536).  A non-zero value plans for that much instead (e.g. to keep
                               room for other kernels' LDS); on a device handle it must not exceed what the
                               device reports. */
  uint32_t n_xcds;          /* accelerator complex dies (each with its own L2) that consecutive workgroup
                               ids are dealt over.  0: what the device reports (host-only handle: 8). */
} dadam_config;

/* Arrays (host) of DEVICE pointers, caller-owned; the arrays themselves are copied.
 * Every buffer holds cfg.d elements and is 16-byte aligned.
 * x_dst[i] may be the very same buffer as one x_src[c] (update in place); any other overlap
 * between two different buffers is rejected with DADAM_EALIAS.  In-place update is legal when the
 * step runs in tile mode, or when source c is read by row i only. */
typedef struct {
  const void* const* x_src; /* [n_cols] x^(t-1) */
  void* const* x_dst;       /* [n_rows] x^(t)   */
  float* const* m_hat;      /* [n_rows] */
  float* const* v_hat;      /* [n_rows] */
  float* const* acc;        /* [n_rows] the accumulator b; may be NULL when accum_s == 1 */
} dadam_buffers;

/* What the planner decided, for tests and tuning. */
typedef struct {
  uint32_t n_segments;      /* maximal runs of contiguous tensors                               */
  uint32_t tile_elems;      /* elements of one tile in tile mode                                */
  uint32_t direct_elems;    /* elements of one work item in direct mode                         */
  uint64_t n_tiles_tile;    /* work items (workgroups) of a full step in tile mode              */
  uint64_t n_tiles_direct;  /* tiles per row in direct mode (work items = this * n_rows)        */
  uint32_t lds_bytes_tile;  /* LDS per workgroup in tile mode                                   */
  uint32_t tile_mode_possible; /* 1 if the source tile fits in LDS                              */
  uint32_t lds_limit_bytes; /* LDS per workgroup the plan was made for                          */
  uint32_t n_xcds;          /* dies the tile order is laid out for                              */
  uint32_t mix_tile_elems;  /* elements of one tile of the mixing-only launch (tile mode)       */
  uint32_t lds_bytes_mix;   /* LDS per workgroup of the mixing-only launch                      */
  uint64_t n_tiles_mix;     /* work items of a mixing-only launch in tile mode                  */
  uint32_t tile_waves, tile_vectors; /* shape of the fused step's tile kernel: wavefronts per workgroup,
                                        16-byte vectors per lane and row                          */
  uint32_t mix_waves, mix_vectors;   /* the same for the mixing-only launch                       */
  uint32_t streaming;       /* 1 if accesses carry the non-temporal hint (large working sets)   */
} dadam_plan_info;

/* Create a handle.  Validates the configuration, builds the segment table from the tensor list
 * and (unless device == DADAM_DEVICE_NONE) uploads it.  *out is set only on success.
 * Errors: DADAM_EINVAL (null, n_rows/n_cols 0 or above DADAM_MAX_ROWS, d == 0, s == 0, dtype,
 * tensors unordered / overlapping / beyond d / negative weight decay / non-zero flags / weight decay with
 * n_rows > n_cols, hyper-parameters out of
 * range: lr finite, 0 <= beta < 1, eps >= 0), DADAM_EHIP. */
int dadam_init(const dadam_config* cfg, dadam_handle** out);

/* Register rows of the mixing matrix W (section 2, eq. (2); Assumption 3 lists the properties the
 * analysis wants) in slot `slot` (< DADAM_MAX_SLOTS); time-varying topologies use one slot per
 * distinct matrix.  row_ptr[n_rows + 1], col_idx[nnz], w[nnz] are HOST arrays and are copied.
 * Checked: row_ptr[0] == 0, non-decreasing, every row non-empty; 0 <= col < n_cols; no column
 * twice in a row; w finite and > 0; |sum of a row - 1| <= 1e-5.  Else DADAM_ETOPO.
 * If n_rows == n_cols and some column sum is off by more than 1e-5, the call still succeeds and
 * sets DADAM_WARN_NOT_COLUMN_STOCHASTIC in *warn (warn may be NULL).
 * A slot may be overwritten only while no launched work still uses it. */
int dadam_set_topology(dadam_handle* h, uint32_t slot, const int32_t* row_ptr,
                       const int32_t* col_idx, const float* w, uint32_t* warn);

/* Bind the device buffers.  May be called again at any time (e.g. to exchange x_src and x_dst);
 * work already launched keeps the pointers it was launched with.
 * Errors: DADAM_EINVAL (null), DADAM_EALIGN, DADAM_EALIAS. */
int dadam_bind(dadam_handle* h, const dadam_buffers* bufs);

/* Exchange the roles of x_src and x_dst (needs n_rows == n_cols): what a ping-pong caller does
 * between two iterations. */
int dadam_swap_x(dadam_handle* h);

/* Iteration t (1-based) of Algorithm 3 as written at the top of this file, using the neighbour
 * list in `slot` and grads[n_rows] (HOST array of DEVICE pointers, each cfg.d elements of
 * grad_dtype, 16-byte aligned, not overlapping any output).  With DADAM_FUSE_ACCUM lines 4-13 are
 * done in one pass; without it only lines 4-8 (x_dst) and the caller follows with
 * dadam_accumulate(grads, t) - never both for one t.  On the first iteration of a loop
 * ((t-1) mod s == 0) the accumulator is taken to be zero and is not read.
 * Errors: DADAM_ESTATE (nothing bound, slot empty, host-only handle), DADAM_EINVAL (t == 0, null,
 * both FORCE flags), DADAM_EALIGN, DADAM_EALIAS (in-place rows that the chosen mode cannot do, or
 * DADAM_FORCE_TILE when the source tile does not fit in LDS -> DADAM_EINVAL), DADAM_EHIP. */
int dadam_gossip_step(dadam_handle* h, uint32_t slot, const void* const* grads, uint64_t t,
                      uint32_t flags, void* hip_stream);

/* The same restricted to tensors [tensor_begin, tensor_end) of the layout (a "bucket" in the
 * sense of section 2.1, where parameters are updated and communicated bucket by bucket).
 * Disjoint ranges of one iteration touch disjoint elements, also where two ranges meet inside one
 * tile and when parameters are updated in place, so they may run on different streams at the same
 * time (issued from one host thread); a range of iteration t + 1 must be ordered after the same
 * range of iteration t.  An empty range is a successful no-op. */
int dadam_gossip_step_range(dadam_handle* h, uint32_t slot, const void* const* grads, uint64_t t,
                            uint32_t flags, uint32_t tensor_begin, uint32_t tensor_end,
                            void* hip_stream);

/* Lines 9-13 of Algorithm 3 alone: b += g / s and, when t mod s == 0, the fold into m_hat and
 * v_hat followed by b = 0. */
int dadam_accumulate(dadam_handle* h, const void* const* grads, uint64_t t, void* hip_stream);

/* x_dst = W x_src: eq. (2) with a zero search direction (pure gossip averaging).  flags: 0 or one
 * of DADAM_FORCE_DIRECT / DADAM_FORCE_TILE. */
int dadam_mix(dadam_handle* h, uint32_t slot, uint32_t flags, void* hip_stream);

/* dadam_mix plus, at no extra HBM traffic, the consensus error of the SOURCES,
 *     *consensus_out = sum over source buffers c and elements e of (x_src[c][e] - mean_c x_src[.][e])^2,
 * the squared distance of the replicas from their average whose decay per gossip round the paper
 * plots to compare topologies (section "Important aspects ...", heterogeneous communication; the
 * consensus lemma bounds the same quantity).  consensus_out is a DEVICE pointer to one double,
 * written by work enqueued on the stream; per-element arithmetic is float32, the sum double.
 * Available in tile mode only (the sources of a tile are then on chip together); DADAM_ESTATE
 * otherwise.  Calls on one handle must not overlap in time: they share the handle's partial sums. */
int dadam_mix_consensus(dadam_handle* h, uint32_t slot, uint32_t flags, double* consensus_out,
                        void* hip_stream);

/* dadam_mix_consensus for callers that cannot allocate device memory or tolerate a library that does:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results; the partial sums of the consensus error live in an array of DADAM_STATIC_SCRATCH_BYTES
 * bytes inside the library's own device image (every GPU holds its copy from the moment the library is
 * loaded until the process ends) instead of the handle's allocated buffer.  The call itself allocates and
 * frees nothing and clears the array with a kernel before use (it keeps the previous call's contents).
 * ALL handles and calls on one GPU share that one array: two such calls must not overlap in time on a
 * GPU, whatever their streams or handles.  A pass that needed more partial sums than the array holds
 * would be refused with DADAM_EINVAL (today every pass needs exactly DADAM_STATIC_SCRATCH_BYTES / 8).
 * Other errors as dadam_mix_consensus. */
#define DADAM_STATIC_SCRATCH_BYTES 8192u
int dadam_mix_consensus_static(dadam_handle* h, uint32_t slot, uint32_t flags, double* consensus_out,
                               void* hip_stream);

/* Change the step size used by later calls (learning-rate schedules). */
int dadam_set_lr(dadam_handle* h, float lr);

/* Planner facts for this handle. */
int dadam_get_plan_info(const dadam_handle* h, dadam_plan_info* out);

/* 1 if a step with this slot would run in tile mode when no FORCE flag is given, 0 for direct
 * mode, negative status on error. */
int dadam_slot_uses_tile_mode(const dadam_handle* h, uint32_t slot);

/* The order in which direct mode takes the rows of this slot (order_out: n_rows entries, a permutation of
 * 0 .. n_rows-1).  When rows share sources (and the device has more than one die), rows that
 * share sources are neighbours in this order and each die works on one contiguous group of it, so that a
 * source two rows read comes from memory once and from that die's L2 the second time (one-peer graph on 64
 * replicas, mixing only: 0.54-0.61 of peak with rows as numbered when the two readers sit on different dies,
 * 0.76 when they share one).  The order changes nothing in what is computed.  Returns 1 if such an order is
 * in use, 0 if rows are taken as numbered (order_out is then the identity), negative status on error. */
int dadam_get_row_order(const dadam_handle* h, uint32_t slot, int32_t* order_out);

/* Offsets of a packed layout: tensor k starts at the next multiple of align_elems elements after
 * tensor k-1 ends.  numel[n] in, offsets[n] out (both host); returns the packed length through
 * *d_out. */
int dadam_pack_offsets(const uint64_t* numel, uint32_t n, uint32_t align_elems, uint64_t* offsets,
                       uint64_t* d_out);

/* Layout advice for HBM, part 1: equal distances.  Places n buffers of nbytes[k] bytes in a range of
 * arena_bytes bytes, in the given order, each at a multiple of 2 MiB, with equal gaps between
 * consecutive buffers so that the first starts at 0 and the last ends near the end of the range.
 * nbytes[n] in, offsets[n] out (host).
 * Errors: DADAM_EINVAL if a pointer is null, n == 0, or the buffers do not fit. */
int dadam_spread_offsets(const uint64_t* nbytes, uint32_t n, uint64_t arena_bytes, uint64_t* offsets);

/* Layout advice for HBM, part 2: where to put the buffers.  Measured on MI355X: the same step over
 * the same bytes sustains 0.62-0.66 of peak bandwidth when the buffers it streams together all lie
 * inside one third (96 GiB) of the device's physical memory - which is where a fresh process's
 * allocations land - and 0.78-0.79 when every group of buffers that is streamed together lies half
 * in one third and half in another.  Nobody outside the driver sees physical addresses, and where the
 * driver puts one allocation relative to another is not predictable (measured: an arena pushed into
 * place by an allocation made before it, or placed by the amount of memory in use, lands elsewhere and
 * runs at 0.64-0.72).  What does hold is that ONE allocation of nearly the whole device (within 16 GiB of
 * device_total_bytes) covers the physical memory in order, so that offsets inside it are physical
 * positions to within what it leaves out.  For such an arena this helper deals the buffers alternately
 * over two regions, one ending 2 GiB below and one starting 2 GiB above the boundary between the first
 * two thirds: buffers 0, 2, 4, ... below, 1, 3, 5, ... above, spread over each region (64 GiB wide, wider
 * when the buffers need it) and staggered inside their gaps by a fixed pseudo-random number of 2 MiB
 * steps, so that the bases do not form an arithmetic progression (for some distances between bases that
 * costs 3-4 %).  Any run of consecutive buffers - all sources, all outputs, one kind of state - is then
 * split evenly.  nbytes[n] in, offsets[n] out (host), every offset a multiple of 2 MiB.  regions_out (may
 * be null) receives lo0, hi0, lo1, hi1 of the two regions, or 0, arena_bytes, 0, 0 for the fall-back.
 * *advice_out (may be null) says what was done:
 *   DADAM_PLACE_TWO_REGIONS     the rule above was applied;
 *   DADAM_PLACE_ARENA_ELSEWHERE the arena does not cover the device: offsets in it say nothing about
 *                               physical positions, and the buffers are placed at equal distances over
 *                               the whole arena instead (0.70-0.77 measured for arenas of 230-275 GiB,
 *                               the packed level if the arena happens to lie inside one third);
 *   DADAM_PLACE_TOO_LARGE       half of the buffers do not fit below the boundary or the other half
 *                               between it and the next one: equal distances over the whole arena.
 * The caller hands `arena + offsets[k]` to dadam_bind and may use the space between the buffers for
 * anything else.
 * Errors: DADAM_EINVAL if a pointer is null, n == 0, or the buffers do not fit the arena at all. */
#define DADAM_PLACE_TWO_REGIONS 1u
#define DADAM_PLACE_ARENA_ELSEWHERE 2u
#define DADAM_PLACE_TOO_LARGE 4u
int dadam_place_offsets(const uint64_t* nbytes, uint32_t n, uint64_t arena_bytes, uint64_t device_total_bytes,
                        uint64_t* offsets, uint64_t* regions_out, uint32_t* advice_out);

/* Layout advice for HBM, part 3: the dealing itself, for a caller that knows two
 * regions [lo0, hi0) and [lo1, hi1) of one arena to lie in different thirds of the physical memory - e.g.
 * because it has timed a streaming probe over pairs of chunks of its arena, which tells same third from
 * different third reliably (paper_2410_11998_amd/arena.py does that).  dadam_deal_offsets places every
 * `every`-th buffer (numbers every-1, 2*every-1, ...) in the second region and the others in the first, spread
 * over each region and staggered as described under dadam_place_offsets.  every = 2 deals alternately (the
 * layout measured at 0.79 of peak); every = 4 puts a quarter of the buffers in the second region, for a second
 * region with little room (a 16-source mixing pass dealt 3:1 still ran at 0.79).  2 <= every <= 8.  Region
 * bounds are multiples of 2 MiB and the regions do not overlap.
 * Errors: DADAM_EINVAL (null, n == 0, every out of range, bounds unaligned or overlapping, a side's buffers do
 * not fit). */
int dadam_deal_offsets(const uint64_t* nbytes, uint32_t n, uint64_t lo0, uint64_t hi0, uint64_t lo1, uint64_t hi1,
                       uint32_t every, uint64_t* offsets);

/* Layout advice for HBM, part 4: finding the thirds by measurement.
 *
 * Where the thirds of the physical memory begin inside a caller's allocation cannot be computed (a large
 * allocation is pieced together from whatever is free: made first, its bytes [0, 96 GiB) lie in one third; made
 * after 100 GiB of other allocations, the second boundary was seen at 160 GiB), but it can be measured: the
 * library's mixing pass over sixteen 64 MiB sources and sixteen outputs runs at 0.78-0.80 of peak when half of
 * its buffers sit in one third and half in another, and at 0.61-0.73 when all sit in one.
 *
 * dadam_find_stretches: the bookkeeping.  `rate(off_a, off_b, ctx)` is the fraction of peak a streaming pass
 * sustains with half of its buffers in the DADAM_PROBE_CHUNK_BYTES at arena offset off_a and half in those at
 * off_b (negative: failure, reported as DADAM_EHIP).  One chunk every DADAM_PROBE_STEP_BYTES is compared with a
 * reference chunk; those that run fast with it (>= 0.95 of the fastest pairing, which must itself reach 0.75)
 * lie in another third; a second reference among them tells the other two thirds apart.  out receives at most
 * DADAM_MAX_STRETCHES stretches [lo, hi) with the id (0, 1, 2) of their third, in address order; the same third
 * may come back later in the arena.  More stretches than that is noise: the timing is repeated once, then
 * *n_out = 0.  An arena too small for three chunks also gives *n_out = 0.  Host only.
 *
 * dadam_regions_from_stretches: the two regions (regions_out[4] = lo0, hi0, lo1, hi1) to deal the buffers
 * over with dadam_deal_offsets and its `every`: alternately (every = 2) over the two stretches of different
 * thirds with the most room if half of the buffers fit each, otherwise every 3rd, 4th, 6th or 8th buffer in
 * the smaller stretch (160 / 200 GiB allocated before the arena: 0.75 / 0.73 of peak against 0.60 / 0.64 at
 * equal distances).  Returns 1 if found, 0 if no two stretches of different thirds hold the buffers.
 *
 * dadam_place_by_timing: the whole procedure on a device.  `arena` is DEVICE memory (2 MiB aligned,
 * arena_bytes long, contents are overwritten: call it before anything is stored there).  The library times
 * its own pass over the arena (about half a second, some hundreds of short launches on the null stream, 2 GiB
 * of temporary device memory), finds the stretches, chooses the regions, confirms them with one more pass
 * across the two regions and one inside each, and deals the buffers; if that yields nothing it falls back to
 * dadam_place_offsets (device_total_bytes is passed on).  offsets[n] and *report say what was done.  Synchronous.
 * Errors: DADAM_EINVAL, DADAM_EALIGN, DADAM_EHIP. */
#define DADAM_PROBE_CHUNK_BYTES 1073741824ull
#define DADAM_PROBE_STEP_BYTES 4294967296ull
#define DADAM_MAX_STRETCHES 6u
#define DADAM_POLICY_TIMED_REGIONS 1u  /* two regions found by timing, dealt with report.every             */
#define DADAM_POLICY_RULE_REGIONS 2u   /* dadam_place_offsets' two regions (arena covers the device)        */
#define DADAM_POLICY_EQUAL_DISTANCES 3u
#define DADAM_NOTE_NO_PROBE 1u         /* arena too small for the probe, one buffer only, or no 2 GiB to spare */
#define DADAM_NOTE_NO_PICTURE 2u       /* the timings gave no consistent picture of the thirds              */
#define DADAM_NOTE_NO_ROOM 3u          /* no two stretches of different thirds hold the buffers             */
#define DADAM_NOTE_NOT_CONFIRMED 4u    /* the confirming passes disagreed with the stretches                */
typedef double (*dadam_pair_rate_fn)(uint64_t off_a, uint64_t off_b, void* ctx);
typedef struct {
  uint32_t third;    /* 0, 1, 2: stretches with the same id share a third */
  uint32_t reserved; /* 0 */
  uint64_t lo, hi;   /* arena offsets */
} dadam_stretch;
typedef struct {
  uint32_t policy;         /* DADAM_POLICY_* */
  uint32_t advice;         /* DADAM_PLACE_* as dadam_place_offsets reports it */
  uint32_t every;          /* DADAM_POLICY_TIMED_REGIONS: every `every`-th buffer lies in the second region */
  uint32_t note;           /* 0, or why the timing was not used: DADAM_NOTE_* */
  uint32_t n_stretches;
  uint32_t probe_launches; /* mixing passes the probe launched */
  dadam_stretch stretches[DADAM_MAX_STRETCHES];
  uint64_t regions[4];     /* lo0, hi0, lo1, hi1 (lo1 = hi1 = 0: one region) */
  float rate_across;       /* fraction of peak of the confirming pass across the regions, 0 if none ran */
  float rate_inside[2];    /* ... and inside each region */
  uint32_t reserved;
} dadam_placement;
int dadam_find_stretches(uint64_t arena_bytes, dadam_pair_rate_fn rate, void* ctx, dadam_stretch* out,
                         uint32_t* n_out);
int dadam_regions_from_stretches(const dadam_stretch* stretches, uint32_t n_stretches, const uint64_t* nbytes,
                                 uint32_t n, uint64_t* regions_out, uint32_t* every_out);
int dadam_place_by_timing(void* arena, uint64_t arena_bytes, int32_t device, const uint64_t* nbytes, uint32_t n,
                          uint64_t device_total_bytes, uint64_t* offsets, dadam_placement* report);

/* Text of the last error recorded on this handle ("" if none).  With h == NULL: the text of the
 * last dadam_init failure of the calling thread.  The pointer stays valid until the next call on
 * the same handle (thread). */
const char* dadam_last_error(const dadam_handle* h);

/* Free the handle and its metadata.  The caller makes sure launched work has finished. */
void dadam_destroy(dadam_handle* h);

#ifdef __cplusplus
}
#endif
#endif /* DADAM_H_ */
