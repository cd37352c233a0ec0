// Workspace layout shared by ctx.hip (sizing) and the kernels that use it.
#pragma once
#include <stddef.h>
#include <stdint.h>

// moe_permute: one wave ranks PERMUTE_CHUNK consecutive (token, slot) pairs; the
// workspace holds one per-expert histogram per chunk (int32 [chunks, E]).
#define PERMUTE_CHUNK 1024

static inline int64_t moe_permute_chunks(int64_t pairs) { return (pairs + PERMUTE_CHUNK - 1) / PERMUTE_CHUNK; }
static inline size_t moe_permute_ws_bytes(int64_t pairs, int E) {
    return (size_t)(moe_permute_chunks(pairs) > 0 ? moe_permute_chunks(pairs) : 1) * (size_t)E * sizeof(int32_t);
}

// moe_grouped_gemm_wgrad: slices of fp32 partial tiles (each the size of one expert's weight gradient) the workspace
// provides for the split of the contraction under a skewed load.
#define MOE_WS_SPLIT_SLICES 8
