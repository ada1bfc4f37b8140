// One part of the tile and direct kernels: a pair of element types (parameters, gradients) with or
// without the streaming hint, chosen by the build (paper_2410_11998_amd/build.py compiles this file once
// per part, in parallel; together the parts hold every instantiation the launchers can ask for).
//   -DDADAM_PART_XT=TF32|TBF16 -DDADAM_PART_GT=TF32|TBF16 -DDADAM_PART_NT=true|false -DDADAM_PART_EXT=true|false
//   -DDADAM_PART_NAME=<suffix>
#include "dadam_device.h"

#if !defined(DADAM_PART_XT) || !defined(DADAM_PART_GT) || !defined(DADAM_PART_NT) || !defined(DADAM_PART_EXT) || \
    !defined(DADAM_PART_NAME)
#error "compile with -DDADAM_PART_XT, -DDADAM_PART_GT, -DDADAM_PART_NT, -DDADAM_PART_EXT and -DDADAM_PART_NAME"
#endif
#define DADAM_JOIN2(a, b) a##b
#define DADAM_JOIN(a, b) DADAM_JOIN2(a, b)

namespace dadam {

KernelFn DADAM_JOIN(tile_kernel_, DADAM_PART_NAME)(int phase, TileShape s) {
  return tile_kernel_for_shape_nt<DADAM_PART_XT, DADAM_PART_GT, DADAM_PART_NT, DADAM_PART_EXT>(phase, s);
}

// shared: rows share sources (a streaming part then keeps the hint off the source loads)
KernelFn DADAM_JOIN(direct_kernel_, DADAM_PART_NAME)(int phase, bool shared) {
  if (!DADAM_PART_NT) return direct_kernel_for_phase<DADAM_PART_XT, DADAM_PART_GT, 0, DADAM_PART_EXT>(phase);
  return shared ? direct_kernel_for_phase<DADAM_PART_XT, DADAM_PART_GT, DADAM_PART_NT ? 2 : 0, DADAM_PART_EXT>(phase)
                : direct_kernel_for_phase<DADAM_PART_XT, DADAM_PART_GT, DADAM_PART_NT ? 1 : 0, DADAM_PART_EXT>(phase);
}

}  // namespace dadam
