// Internal definitions shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "moe_hip.h"

struct moe_ctx {
    int device;
    void* ws;          // device workspace
    size_t ws_bytes;
    int* dev_err;      // device error word (first 256 bytes of ws are reserved for it)
    int num_cu;
    char err[512];
};

#define MOE_WS_RESERVED 256  // bytes at the head of the workspace: error word at 0, ...
#define MOE_WS_ZEROS 128     // ... and 128 bytes that stay zero for the whole life of the context

#define MOE_FAIL(ctx, code, ...)                                   \
    do {                                                           \
        if (ctx) snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__); \
        return (code);                                             \
    } while (0)

#define MOE_HIP_CHECK(ctx, expr)                                                        \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) MOE_FAIL(ctx, MOE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define MOE_LAUNCH_CHECK(ctx, name)                                                     \
    do {                                                                                \
        hipError_t e_ = hipGetLastError();                                              \
        if (e_ != hipSuccess) MOE_FAIL(ctx, MOE_ERR_HIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

static inline size_t moe_dtype_size(moe_dtype dt) { return dt == MOE_F32 ? 4 : (dt == MOE_BF16 ? 2 : 1); }
static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// --- device helpers --------------------------------------------------------
typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two fp32 -> packed bf16 pair, round to nearest even (hardware conversion on gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2_t v;
    v[0] = (bf16_t)lo;
    v[1] = (bf16_t)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// blockwise fp8 (Sec. 5.3.2): scale of a block from its amax, and four fp32 -> four E4M3 codes packed in a dword
// (fp32 division, clamp to +-448, hardware round-to-nearest-even conversion).  Shared by the quantiser kernels and
// the GEMM epilogues that quantise their own output, so both produce the same bits.
__device__ __forceinline__ float block_scale(float amax) { return amax > 0.0f ? amax / 448.0f : 1.0f; }
__device__ __forceinline__ uint32_t cvt4_e4m3(float a, float b, float c, float d, float scale) {
    a = __builtin_fminf(__builtin_fmaxf(a / scale, -448.0f), 448.0f);
    b = __builtin_fminf(__builtin_fmaxf(b / scale, -448.0f), 448.0f);
    c = __builtin_fminf(__builtin_fmaxf(c / scale, -448.0f), 448.0f);
    d = __builtin_fminf(__builtin_fmaxf(d / scale, -448.0f), 448.0f);
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (uint32_t)w;
}

// all-fp32 grouped GEMMs (gemm_f32.hip), reached from the public entry points with dt = MOE_F32
moe_status moe_gg_f32_fwd(moe_ctx* ctx, hipStream_t s, const void* A, const void* B, const int32_t* offsets, int E, int N,
                          int K, int64_t Rcap, int swiglu, const float* row_prob, void* C, void* C_act);
moe_status moe_gg_f32_dgrad(moe_ctx* ctx, hipStream_t s, const void* dC, const void* B, const int32_t* offsets, int E, int N,
                            int K, int64_t Rcap, const void* Z_saved, const float* row_prob, void* dA);
moe_status moe_gg_f32_wgrad(moe_ctx* ctx, hipStream_t s, const void* A, const void* dC, const int32_t* offsets, int E, int N,
                            int K, int64_t Rcap, int accumulate, void* dB);

// message buffer (512 bytes, one per host thread) of the calls that take no context; moe_last_error(NULL) returns it
char* moe_ctxless_error();

// shared by the fill launches of several files
void moe_launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t s);
