// Tiny-matrix StridedBatchedGemm path (placeholder until the kernel lands: nothing is supported,
// so the selector never routes here).
#include "sb_internal.h"

bool sb_tiny_supports(sb_dtype, const SbArgs &) { return false; }
bool sb_tiny_preferred(sb_dtype, const SbArgs &) { return false; }
hipError_t sb_launch_tiny(sb_dtype, const SbArgs &, hipStream_t) { return hipErrorNotSupported; }
