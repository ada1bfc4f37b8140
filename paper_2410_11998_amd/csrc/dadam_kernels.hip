// Launchers of the gfx950 kernels, the accumulate-only and consensus kernels, and the scratch array of the
// entry point that does not allocate.  The tile and direct kernels are compiled in parts
// (dadam_kernels_part.hip, once per pair of element types and streaming hint) from dadam_device.h.
#include <hip/hip_runtime.h>

#include <map>
#include <mutex>
#include <utility>

#include "dadam_device.h"

// Scratch memory of the entry point that may not allocate (dadam_mix_consensus_static): the partial sums
// of the consensus error, in the library's own image instead of a hipMalloc'ed buffer.  Every GPU the
// library runs on holds its own copy at its own address; host code never uses this name as an
// address, only what hipGetSymbolAddress returned for the current device (static_partials below).
// The compiler makes a static device variable visible to the runtime only once it has seen host code
// refer to it, at the end of the translation unit: nothing may force it out earlier (no `used`
// attribute), or the symbol stays local to the code object and the look-up by name aborts.
static __device__ __align__(256) double scratch[dadam::kConsensusPartials];

namespace dadam {

// what the parts define
#define DADAM_PART(name)                                       \
  KernelFn tile_kernel_##name(int phase, TileShape s);         \
  KernelFn direct_kernel_##name(int phase, bool shared);       \
  KernelFn tile_kernel_##name##_ext(int phase, TileShape s);   \
  KernelFn direct_kernel_##name##_ext(int phase, bool shared)
DADAM_PART(f32_f32_nt);
DADAM_PART(f32_f32);
DADAM_PART(bf16_bf16_nt);
DADAM_PART(bf16_bf16);
DADAM_PART(bf16_f32_nt);
DADAM_PART(bf16_f32);
DADAM_PART(f32_bf16_nt);
DADAM_PART(f32_bf16);
#undef DADAM_PART

namespace {

// ---------------------------------------------------------------------------------------------
// consensus error: partial sums are cleared by a kernel (not a memset, so that the sequence can be
// captured in a graph) and added up by one workgroup in a fixed order
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_consensus_zero(double* partials) {
  for (uint32_t i = threadIdx.x; i < kConsensusPartials; i += 256) partials[i] = 0.0;
}

__global__ __launch_bounds__(256) void k_consensus_sum(const double* partials, double* out) {
  __shared__ double red[256];
  double s = 0.0;
  for (uint32_t i = threadIdx.x; i < kConsensusPartials; i += 256) s += partials[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = red[0] < 0.0 ? 0.0 : red[0];
}

// ---------------------------------------------------------------------------------------------
// dispatch tables
// ---------------------------------------------------------------------------------------------
template <typename GT, int VEC, bool NT, bool EXT>
KernelFn acc_kernel_for_phase(int phase) {
  switch (phase) {
    case kPlain: return k_acc<GT, VEC, kPlain, NT, EXT>;
    case kLoopStart: return k_acc<GT, VEC, kLoopStart, NT, EXT>;
    case kFold: return k_acc<GT, VEC, kFold, NT, EXT>;
    case kAlg1: return k_acc<GT, VEC, kAlg1, NT, EXT>;
  }
  return nullptr;
}

// A kernel may use more than 64 KB of dynamic LDS only after its limit has been raised; that is done
// once per (device, kernel), up to the largest size asked for so far.
int raise_lds_limit(KernelFn fn, uint32_t lds) {
  static std::mutex mu;
  static std::map<std::pair<int, const void*>, uint32_t> raised;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  std::lock_guard<std::mutex> lock(mu);
  uint32_t& have = raised[{dev, reinterpret_cast<const void*>(fn)}];
  if (have >= lds) return (int)hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e == hipSuccess) have = lds;
  return (int)e;
}

int launch(KernelFn fn, uint32_t grid, uint32_t block, uint32_t lds, const StepArgs& a, void* stream) {
  if (fn == nullptr) return (int)hipErrorInvalidDeviceFunction;
  if (grid == 0) return (int)hipSuccess;
  if (lds > 65536u) {
    const int e = raise_lds_limit(fn, lds);
    if (e != (int)hipSuccess) return e;
  }
  hipLaunchKernelGGL(fn, dim3(grid), dim3(block), lds, reinterpret_cast<hipStream_t>(stream), a);
  return (int)hipGetLastError();
}

static_assert(sizeof(StepArgs) <= 4096, "kernel argument block must fit the kernarg segment");

}  // namespace

// Address and capacity (in doubles) of `scratch` on the CURRENT device, resolved once per device.
int static_partials(double** out, uint32_t* capacity) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static double* addr[kMaxDevices] = {};
  *out = nullptr;
  *capacity = (uint32_t)(sizeof(scratch) / sizeof(double));
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    addr[dev] = static_cast<double*>(p);
  }
  *out = addr[dev];
  return (int)hipSuccess;
}

int launch_consensus_zero(double* partials, void* stream) {
  hipLaunchKernelGGL(k_consensus_zero, dim3(1), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), partials);
  return (int)hipGetLastError();
}

int launch_consensus_sum(const double* partials, double* out, void* stream) {
  hipLaunchKernelGGL(k_consensus_sum, dim3(1), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), partials, out);
  return (int)hipGetLastError();
}

int vec_elems(int xdt) { return xdt == DADAM_BF16 ? TBF16::vec : TF32::vec; }
int direct_unroll() { return kUD; }
bool tile_shape_supported(TileShape s) {
#ifdef DADAM_TUNING
  if ((s.waves == 16 && (s.ut == 1 || s.ut == 2)) || ((s.waves == 4 || s.waves == 8) && s.ut == 4)) return true;
#endif
  return (s.waves == 4 || s.waves == 8) && (s.ut == 1 || s.ut == 2);
}

int launch_tile(int xdt, int gdt, Phase phase, TileShape shape, const StepArgs& a, uint32_t n_work,
                uint32_t lds_bytes, void* stream) {
  // A handle with more than 64 rows or sources keeps its pointer tables in device memory and runs kernels
  // compiled for that (kernels of their own, so that the small handles' register budget is not theirs).
  KernelFn fn = nullptr;
  const bool nt = shape.nontemporal, ext = a.ext != nullptr;
#define DADAM_PICK(name) (ext ? (nt ? tile_kernel_##name##_nt_ext(phase, shape) : tile_kernel_##name##_ext(phase, shape)) \
                              : (nt ? tile_kernel_##name##_nt(phase, shape) : tile_kernel_##name(phase, shape)))
  if (xdt == DADAM_F32 && gdt == DADAM_F32) fn = DADAM_PICK(f32_f32);
  if (xdt == DADAM_BF16 && gdt == DADAM_BF16) fn = DADAM_PICK(bf16_bf16);
  if (xdt == DADAM_BF16 && gdt == DADAM_F32) fn = DADAM_PICK(bf16_f32);
  if (xdt == DADAM_F32 && gdt == DADAM_BF16) fn = DADAM_PICK(f32_bf16);
#undef DADAM_PICK
  return launch(fn, n_work, (uint32_t)(kWave * shape.waves), lds_bytes, a, stream);
}

int launch_direct(int xdt, int gdt, Phase phase, bool nt, bool shared, const StepArgs& a, uint32_t n_work_tiles,
                  void* stream) {
  KernelFn fn = nullptr;
  const bool ext = a.ext != nullptr;
#define DADAM_PICK(name) (ext ? (nt ? direct_kernel_##name##_nt_ext(phase, shared) : direct_kernel_##name##_ext(phase, shared)) \
                              : (nt ? direct_kernel_##name##_nt(phase, shared) : direct_kernel_##name(phase, shared)))
  if (xdt == DADAM_F32 && gdt == DADAM_F32) fn = DADAM_PICK(f32_f32);
  if (xdt == DADAM_BF16 && gdt == DADAM_BF16) fn = DADAM_PICK(bf16_bf16);
  if (xdt == DADAM_BF16 && gdt == DADAM_F32) fn = DADAM_PICK(bf16_f32);
  if (xdt == DADAM_F32 && gdt == DADAM_BF16) fn = DADAM_PICK(f32_bf16);
#undef DADAM_PICK
  // with a sharing order every die gets the same number of workgroups per tile (see k_direct)
  const uint32_t per_tile = a.row_order != nullptr ? a.n_xcd * a.order_group : a.n_rows;
  return launch(fn, n_work_tiles * per_tile, kDirectThreads, 0, a, stream);
}

int launch_accumulate(int gdt, Phase phase, bool nt, const StepArgs& a, uint32_t n_work_tiles, void* stream,
                      int vec) {
  KernelFn fn = nullptr;
  const bool ext = a.ext != nullptr;
#define DADAM_PICK(GT, VEC)                                                                                      \
  (ext ? (nt ? acc_kernel_for_phase<GT, VEC, true, true>(phase) : acc_kernel_for_phase<GT, VEC, false, true>(phase)) \
       : (nt ? acc_kernel_for_phase<GT, VEC, true, false>(phase) : acc_kernel_for_phase<GT, VEC, false, false>(phase)))
  if (gdt == DADAM_F32 && vec == 4) fn = DADAM_PICK(TF32, 4);
  if (gdt == DADAM_F32 && vec == 8) fn = DADAM_PICK(TF32, 8);
  if (gdt == DADAM_BF16 && vec == 4) fn = DADAM_PICK(TBF16, 4);
  if (gdt == DADAM_BF16 && vec == 8) fn = DADAM_PICK(TBF16, 8);
#undef DADAM_PICK
  // with a sharing order every die gets the same number of workgroups per tile (see k_direct)
  const uint32_t per_tile = a.row_order != nullptr ? a.n_xcd * a.order_group : a.n_rows;
  return launch(fn, n_work_tiles * per_tile, kDirectThreads, 0, a, stream);
}

}  // namespace dadam
