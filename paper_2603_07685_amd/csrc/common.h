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
// x / scale without a division per element.  The quantisers are bound by vector arithmetic when every element pays the
// dozen instructions of a correctly rounded fp32 division, so the division is done once per block, r = 1 / scale, and
// an element costs a product and two fused multiply-adds: q0 = x r, q = fma(fma(-q0, scale, x), r, q0).  With r the
// correctly rounded reciprocal, q0 is a faithful quotient, the inner fma is the exact residual x - q0 scale, and the
// corrected q is the correctly rounded quotient (Markstein's division theorem), i.e. bit for bit what x / scale gives,
// as long as nothing under- or overflows on the way.  That holds for scales in [2^-40, 2^120] (block maxima from about
// 2^-31 up to the top of the bf16 range): r is normal; the residual of an element of magnitude 2^-77 or more is exact
// and a normal number whenever it matters (a residual below 2^-126 means q0 was already the correctly rounded
// quotient, so it would not matter even if denormals were flushed); a smaller element has a quotient below 2^-37, and
// whatever fp32 value comes out near that converts to the code 0 like the exact one (E4M3's smallest step is 2^-9).
// A wave in which any lane holds a scale outside the range takes the plain division for that piece (quant_fast_ok +
// a ballot: a uniform branch).
__device__ __forceinline__ bool quant_fast_ok(float scale) { return scale >= 0x1p-40f && scale <= 0x1p120f; }
__device__ __forceinline__ bool quant_fast_all(bool ok) { return __builtin_amdgcn_ballot_w64(!ok) == 0; }
__device__ __forceinline__ float quant_div(float x, float scale, float rcp) {
    const float q0 = x * rcp;
    // (the sign is x's: the scale is positive, and for x = -0 the sum of the two zeros would come out positive)
    return __builtin_copysignf(__builtin_fmaf(__builtin_fmaf(-q0, scale, x), rcp, q0), x);
}
__device__ __forceinline__ uint32_t cvt4_e4m3(float a, float b, float c, float d, float scale) {
    const float rcp = 1.0f / scale;
    if (quant_fast_all(quant_fast_ok(scale))) {
        a = quant_div(a, scale, rcp);
        b = quant_div(b, scale, rcp);
        c = quant_div(c, scale, rcp);
        d = quant_div(d, scale, rcp);
    } else {
        a = a / scale;
        b = b / scale;
        c = c / scale;
        d = d / scale;
    }
    a = __builtin_fminf(__builtin_fmaxf(a, -448.0f), 448.0f);
    b = __builtin_fminf(__builtin_fmaxf(b, -448.0f), 448.0f);
    c = __builtin_fminf(__builtin_fmaxf(c, -448.0f), 448.0f);
    d = __builtin_fminf(__builtin_fmaxf(d, -448.0f), 448.0f);
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (uint32_t)w;
}

// MXFP8 (Sec. 5.3.3): the E8M0 exponent of a block from its largest magnitude, e = ceil(log2(amax / 448)) taken from
// the bits of amax (clamped to +-127, 0 for an all-zero block), and the E4M3 codes of x * 2^-e (exact scaling, RNE).
// One copy for every kernel that quantises (stand-alone quantisers and GEMM epilogues): identical bits everywhere.
__device__ __forceinline__ int mx_exponent(float amax) {
    if (!(amax > 0.0f)) return 0;
    const uint32_t b = __float_as_uint(amax);
    int e = (int)((b >> 23) & 0xFF) - 127 - 8 + ((b & 0x7FFFFFu) > 0x600000u ? 1 : 0);
    if (((b >> 23) & 0xFF) == 0) e = -127;  // subnormal maximum: far below the clamp
    return e < -127 ? -127 : (e > 127 ? 127 : e);
}
// Four bf16 values (two packed pairs) -> four E4M3 codes of x / 2^e, with the hardware's scaled conversion
// (v_cvt_scalef32_pk_fp8_bf16 divides by the power of two in the scale operand's exponent field, round to nearest
// even); one exponent for all four, or one per element (two conversions per pair, one byte kept of each).
typedef short s16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float mx_scale_f32(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }  // 2^e
__device__ __forceinline__ uint32_t mx_cvt4_bf16(uint32_t w01, uint32_t w23, float scale) {
    s16x2_t o = {0, 0};
    o = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(o, __builtin_bit_cast(bf16x2_t, w01), scale, false);
    o = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(o, __builtin_bit_cast(bf16x2_t, w23), scale, true);
    return __builtin_bit_cast(uint32_t, o);
}
__device__ __forceinline__ uint32_t mx_cvt4_bf16_each(uint32_t w01, uint32_t w23, float s0, float s1, float s2, float s3) {
    s16x2_t ev = {0, 0}, od = {0, 0};
    ev = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(ev, __builtin_bit_cast(bf16x2_t, w01), s0, false);
    ev = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(ev, __builtin_bit_cast(bf16x2_t, w23), s2, true);
    od = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(od, __builtin_bit_cast(bf16x2_t, w01), s1, false);
    od = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(od, __builtin_bit_cast(bf16x2_t, w23), s3, true);
    return (__builtin_bit_cast(uint32_t, ev) & 0x00FF00FFu) | (__builtin_bit_cast(uint32_t, od) & 0xFF00FF00u);
}
// largest magnitude of the eight bf16 values of a 16-byte piece, as fp32 (the bits of |x| order like unsigned integers)
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_absmax_bits(uint32_t m, uint32_t w) {   // both halves at once
    const u16x2_t a = __builtin_bit_cast(u16x2_t, m), b = __builtin_bit_cast(u16x2_t, w & 0x7FFF7FFFu);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
}
__device__ __forceinline__ float bf16_absmax_finish(uint32_t m) {
    const uint32_t hi = m >> 16, lo = m & 0xFFFFu;
    return __uint_as_float((hi > lo ? hi : lo) << 16);
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
