// Blockwise FP8 quantisation (Sec. 5.3.2).
#include "common.h"

extern "C" moe_status moe_fp8_quantize(moe_ctx* ctx, void* stream, const void* X, moe_qblock block,
                                       int groups, int64_t rows, int cols, const int32_t* rows_dev,
                                       void* q, float* scale) {
    if (!ctx) return MOE_ERR_ARG;
    MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_fp8_quantize: not built yet");
}
