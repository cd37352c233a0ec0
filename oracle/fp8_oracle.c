/*
 * CPU oracle for the blockwise FP8 recipe.  TEST INFRASTRUCTURE ONLY; shares
 * nothing with the HIP library.
 *
 * Sec. 5.3.2 ("Blockwise FP8"): E4M3 for every tensor, activations and gradients
 * scaled per 1x128 tile, weights per 128x128 block, FP32 accumulation.  The
 * paper does not give the code format's limits, the scale format or the rounding
 * rule; the readings taken here:
 *   - the 8-bit format is the OCP E4M3 "fn" variant gfx950 implements: bias 7,
 *     subnormals, no infinities, S.1111.111 is NaN, largest finite value 448;
 *   - scale = amax / 448 as an fp32 number (amax == 0 -> scale 1);
 *   - code = nearest representable value to clamp(x / scale, +-448), the division
 *     and the rounding decision both in fp32, ties to the even mantissa;
 *   - a 1x128 tile runs along the contraction dimension of the GEMM that reads
 *     the tensor: along the row for forward/dgrad operands, down the token
 *     dimension (128 consecutive rows of one expert's padded range) for the wgrad
 *     operands (Sec. 5.4.1: the wgrad contraction is the token dimension and is
 *     zero-padded; Sec. 5.4.2/5.4.3: a block never spans two experts).
 * The rounding is done by brute force against the table of all 127 positive
 * finite values, which is itself built from the format definition.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* value of an E4M3fn code (NaN codes decode to NAN) */
float orc_e4m3_decode(uint8_t c) {
    int sign = c >> 7, ex = (c >> 3) & 0xF, man = c & 7;
    float v;
    if (ex == 0xF && man == 7) return NAN;
    if (ex == 0) v = ldexpf((float)man / 8.0f, -6);          /* subnormal: 0.mmm * 2^-6 */
    else v = ldexpf(1.0f + (float)man / 8.0f, ex - 7);        /* normal:    1.mmm * 2^(e-7) */
    return sign ? -v : v;
}

/* nearest code to x (saturating at +-448, ties to even code, NaN -> 0x7F) */
uint8_t orc_e4m3_encode(float x) {
    if (isnan(x)) return 0x7F;
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    float a = fabsf(x);
    if (a > 448.0f) a = 448.0f;
    int best = 0;
    float bestd = a; /* distance to code 0 (value 0) */
    for (int c = 1; c <= 0x7E; ++c) {
        float d = fabsf(orc_e4m3_decode((uint8_t)c) - a); /* exact: both operands have few bits */
        if (d < bestd || (d == bestd && (c & 1) == 0)) { best = c; bestd = d; }
    }
    return (uint8_t)(sign | best);
}

static float block_scale(float amax) { return amax > 0.0f ? amax / 448.0f : 1.0f; }

static uint8_t quant_one(float x, float scale) {
    float y = x / scale; /* fp32 division */
    if (y > 448.0f) y = 448.0f;
    if (y < -448.0f) y = -448.0f;
    return orc_e4m3_encode(y);
}

/* 1x128 tiles along each row: X[rows,K] -> q[rows,K], scale[rows,K/128]. K % 128 == 0. */
int orc_fp8_quant_1x128(const float* X, int64_t rows, int K, uint8_t* q, float* scale) {
    if (K % 128) return -1;
    int nb = K / 128;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int b = 0; b < nb; ++b) {
            const float* x = X + r * K + b * 128;
            float amax = 0.0f;
            for (int i = 0; i < 128; ++i) amax = fmaxf(amax, fabsf(x[i]));
            float s = block_scale(amax);
            scale[r * nb + b] = s;
            for (int i = 0; i < 128; ++i) q[r * K + b * 128 + i] = quant_one(x[i], s);
        }
    return 0;
}

/* 128x1 tiles down the rows: X[R,N] -> q[R,N], scale[R/128,N]. R % 128 == 0. */
int orc_fp8_quant_128x1(const float* X, int64_t R, int N, uint8_t* q, float* scale) {
    if (R % 128) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < R / 128; ++b)
        for (int n = 0; n < N; ++n) {
            float amax = 0.0f;
            for (int i = 0; i < 128; ++i) amax = fmaxf(amax, fabsf(X[(b * 128 + i) * N + n]));
            float s = block_scale(amax);
            scale[b * N + n] = s;
            for (int i = 0; i < 128; ++i) q[(b * 128 + i) * N + n] = quant_one(X[(b * 128 + i) * N + n], s);
        }
    return 0;
}

/* 128x128 blocks: W[G,N,K] (G matrices) -> q, scale[G,N/128,K/128]. */
int orc_fp8_quant_128x128(const float* W, int G, int N, int K, uint8_t* q, float* scale) {
    if (N % 128 || K % 128) return -1;
    int nbn = N / 128, nbk = K / 128;
#pragma omp parallel for collapse(2) schedule(static)
    for (int g = 0; g < G; ++g)
        for (int bn = 0; bn < nbn; ++bn)
            for (int bk = 0; bk < nbk; ++bk) {
                const float* w = W + (int64_t)g * N * K;
                float amax = 0.0f;
                for (int i = 0; i < 128; ++i)
                    for (int j = 0; j < 128; ++j)
                        amax = fmaxf(amax, fabsf(w[(int64_t)(bn * 128 + i) * K + bk * 128 + j]));
                float s = block_scale(amax);
                scale[((int64_t)g * nbn + bn) * nbk + bk] = s;
                for (int i = 0; i < 128; ++i)
                    for (int j = 0; j < 128; ++j) {
                        int64_t o = (int64_t)g * N * K + (int64_t)(bn * 128 + i) * K + bk * 128 + j;
                        q[o] = quant_one(w[(int64_t)(bn * 128 + i) * K + bk * 128 + j], s);
                    }
            }
    return 0;
}

/* dequantise: value = decode(code) * scale of the block the element lies in.
 * mode 0: 1x128 (scale[rows,K/128]); 1: 128x1 (scale[rows/128,K]); 2: 128x128 per
 * matrix of a [G,rows,K] stack (scale[G,rows/128,K/128]); out is double. */
int orc_fp8_dequant(const uint8_t* q, const float* scale, int mode, int G, int64_t rows, int K, double* out) {
    for (int g = 0; g < G; ++g)
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < rows; ++r)
            for (int c = 0; c < K; ++c) {
                int64_t o = ((int64_t)g * rows + r) * K + c;
                float s;
                if (mode == 0) s = scale[r * (K / 128) + c / 128];
                else if (mode == 1) s = scale[(r / 128) * K + c];
                else s = scale[((int64_t)g * (rows / 128) + r / 128) * (K / 128) + c / 128];
                out[o] = (double)orc_e4m3_decode(q[o]) * (double)s;
            }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* MXFP8 (Sec. 5.3.3): E4M3 elements, 1x32 blocks, E8M0 (power-of-two) scales */
/* ------------------------------------------------------------------------ */
/*
 * The paper fixes the block (1x32 along the contraction dimension of the consuming GEMM,
 * hence a row-wise and a column-wise quantised copy), the element format and the scale
 * format, not how the scale is chosen.  Reading taken here: the scale is the smallest
 * power of two that brings the block's largest magnitude inside the E4M3 range,
 *     e = ceil(log2(amax / 448)),  scale = 2^e,  E8M0 byte = e + 127  (clamped to 0..254),
 * so no element saturates; an all-zero block gets scale 1 (byte 127).  Elements are
 * code = nearest E4M3 value to x / 2^e (exact division), ties to even.
 * The exponent is computed exactly from the binary representation: amax = m * 2^x with
 * m in [0.5, 1) and 448 = 0.875 * 2^9 give e = x - 9 if m <= 0.875, else x - 8.
 */
static int mx_exponent(float amax) {
    if (!(amax > 0.0f)) return 0;
    int x;
    float m = frexpf(amax, &x);
    int e = (m <= 0.875f) ? x - 9 : x - 8;
    if (e < -127) e = -127;
    if (e > 127) e = 127;
    return e;
}
uint8_t orc_e8m0_from_amax(float amax) { return (uint8_t)(mx_exponent(amax) + 127); }
double orc_e8m0_decode(uint8_t b) { return ldexp(1.0, (int)b - 127); }

/* row-wise: X[rows,K] -> q[rows,K], e8[rows,K/32]; blocks of 32 along each row.  K % 32 == 0. */
int orc_mx_quant_1x32(const float* X, int64_t rows, int K, uint8_t* q, uint8_t* e8) {
    if (K % 32) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int b = 0; b < K / 32; ++b) {
            const float* x = X + r * K + b * 32;
            float amax = 0.0f;
            for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(x[i]));
            int e = mx_exponent(amax);
            e8[r * (K / 32) + b] = (uint8_t)(e + 127);
            for (int i = 0; i < 32; ++i) q[r * K + b * 32 + i] = orc_e4m3_encode(ldexpf(x[i], -e));
        }
    return 0;
}

/* column-wise, for a weight stack W[G,N,K] read with N as the contraction dimension (dgrad):
 * blocks of 32 consecutive n for a fixed k; q[G,N,K] keeps W's layout, e8[G,K,N/32] is laid out
 * so that the scales of one output column k are contiguous.  N % 32 == 0. */
int orc_mx_quant_32x1(const float* W, int G, int N, int K, uint8_t* q, uint8_t* e8) {
    if (N % 32) return -1;
    for (int g = 0; g < G; ++g)
        for (int k = 0; k < K; ++k)
            for (int b = 0; b < N / 32; ++b) {
                float amax = 0.0f;
                for (int i = 0; i < 32; ++i)
                    amax = fmaxf(amax, fabsf(W[((int64_t)g * N + b * 32 + i) * K + k]));
                int e = mx_exponent(amax);
                e8[((int64_t)g * K + k) * (N / 32) + b] = (uint8_t)(e + 127);
                for (int i = 0; i < 32; ++i) {
                    int64_t at = ((int64_t)g * N + b * 32 + i) * K + k;
                    q[at] = orc_e4m3_encode(ldexpf(W[at], -e));
                }
            }
    return 0;
}

/* dequantise to double.  mode 0: row-wise (G = 1, e8[rows,K/32]); mode 1: column-wise stack
 * (rows = N, e8[G,K,N/32]). */
int orc_mx_dequant(const uint8_t* q, const uint8_t* e8, int mode, int G, int64_t rows, int K, double* out) {
    for (int g = 0; g < G; ++g)
        for (int64_t r = 0; r < rows; ++r)
            for (int k = 0; k < K; ++k) {
                int64_t at = ((int64_t)g * rows + r) * K + k;
                uint8_t b = mode == 0 ? e8[r * (K / 32) + k / 32] : e8[((int64_t)g * K + k) * (rows / 32) + r / 32];
                out[at] = (double)orc_e4m3_decode(q[at]) * orc_e8m0_decode(b);
            }
    return 0;
}
