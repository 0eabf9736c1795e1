// MFMA-tiled StridedBatchedGemm path (placeholder until the kernel lands: nothing is supported,
// so the selector never routes here).
#include "sb_internal.h"

bool sb_mfma_supports(sb_dtype, const SbArgs &) { return false; }
bool sb_mfma_preferred(sb_dtype, const SbArgs &) { return false; }
hipError_t sb_launch_mfma(sb_dtype, const SbArgs &, hipStream_t) { return hipErrorNotSupported; }
