// Blockwise FP8 quantisation (Sec. 5.3.2): E4M3 codes + fp32 block scales, grouped over all experts
// in one launch with the live row count read from the device (Sec. 5.4.2).
//
//   scale = amax(block) / 448   (1 for an all-zero block)
//   code  = nearest E4M3 to clamp(x / scale, +-448): fp32 division, hardware round-to-nearest-even
//           conversion (v_cvt_pk_fp8_f32; gfx950 implements the OCP "fn" format: no inf, max 448)
// All three kernels are bandwidth-bound: 2 bytes read + 1 byte written per element.
//   1x128   : 16 lanes own one block (8 elements per lane), amax by butterfly over those 16 lanes.
//   128x1   : a wave owns a 128-row x 512-column panel, 8 columns per lane; first pass keeps the running
//             column amax in registers, second pass re-reads the panel (from L2) and converts.
//   128x128 : a 256-thread workgroup owns one block, 64 elements per thread held in registers.
#include "common.h"

__device__ __forceinline__ float amax8(u32x4_t v) {
    float m = fabsf(bf16_lo(v.x));
    m = fmaxf(m, fabsf(bf16_hi(v.x)));
    m = fmaxf(m, fmaxf(fabsf(bf16_lo(v.y)), fabsf(bf16_hi(v.y))));
    m = fmaxf(m, fmaxf(fabsf(bf16_lo(v.z)), fabsf(bf16_hi(v.z))));
    m = fmaxf(m, fmaxf(fabsf(bf16_lo(v.w)), fabsf(bf16_hi(v.w))));
    return m;
}

__device__ __forceinline__ u32x2_t cvt8_e4m3(u32x4_t v, float scale) {
    u32x2_t o;
    o.x = cvt4_e4m3(bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y), scale);
    o.y = cvt4_e4m3(bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w), scale);
    return o;
}

// ---- 1x128 ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void quant_1x128_kernel(const u32x4_t* __restrict__ X, int64_t rows, int cols,
                                                          const int32_t* __restrict__ rows_dev,
                                                          u32x2_t* __restrict__ q, float* __restrict__ scale) {
    const int64_t live = rows_dev ? min((int64_t)*rows_dev, rows) : rows;
    const int bpr = cols / 128;                       // blocks per row
    const int64_t nblocks = live * bpr;
    const int sub = threadIdx.x & 15;                 // lane inside its 16-lane block group
    int64_t b = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 4;
    const int64_t stride = ((int64_t)gridDim.x * blockDim.x) >> 4;
    for (; b < nblocks; b += stride) {                // uniform inside a 16-lane group
        const int64_t vec = b * 16 + sub;             // 16-byte vector index (row-major, 16 per block)
        const u32x4_t v = X[vec];
        float m = amax8(v);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        const float s = block_scale(m);
        q[vec] = cvt8_e4m3(v, s);
        if (sub == 0) scale[b] = s;
    }
}

// ---- 128x1 ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void quant_128x1_kernel(const u32x4_t* __restrict__ X, int64_t rows, int cols,
                                                          const int32_t* __restrict__ rows_dev,
                                                          u32x2_t* __restrict__ q, float* __restrict__ scale) {
    const int64_t live = rows_dev ? min((int64_t)*rows_dev, rows) : rows;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int vpr = cols / 8;                          // 16-byte vectors per row
    const int panels_c = (vpr + 63) / 64;              // 512-column panels per row block
    const int64_t npanels = (live / 128) * panels_c;
    for (int64_t p = (int64_t)blockIdx.x * 4 + wave; p < npanels; p += (int64_t)gridDim.x * 4) {
        const int64_t rb = p / panels_c;
        const int vc = (int)(p % panels_c) * 64 + lane;
        if (vc >= vpr) continue;
        const u32x4_t* src = X + rb * 128 * vpr + vc;
        float m[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int r = 0; r < 128; ++r) {
            const u32x4_t v = src[(int64_t)r * vpr];
            m[0] = fmaxf(m[0], fabsf(bf16_lo(v.x))); m[1] = fmaxf(m[1], fabsf(bf16_hi(v.x)));
            m[2] = fmaxf(m[2], fabsf(bf16_lo(v.y))); m[3] = fmaxf(m[3], fabsf(bf16_hi(v.y)));
            m[4] = fmaxf(m[4], fabsf(bf16_lo(v.z))); m[5] = fmaxf(m[5], fabsf(bf16_hi(v.z)));
            m[6] = fmaxf(m[6], fabsf(bf16_lo(v.w))); m[7] = fmaxf(m[7], fabsf(bf16_hi(v.w)));
        }
        float s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) s[i] = block_scale(m[i]);
        f32x4_t* sd = (f32x4_t*)(scale + rb * cols + (int64_t)vc * 8);
        sd[0] = f32x4_t{s[0], s[1], s[2], s[3]};
        sd[1] = f32x4_t{s[4], s[5], s[6], s[7]};
        u32x2_t* dst = q + rb * 128 * vpr + vc;
        float rc[8];   // (one division per column block, then a product and two fmas per element: see quant_div)
        bool fast = true;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            rc[i] = 1.0f / s[i];
            fast &= quant_fast_ok(s[i]);
        }
        fast = quant_fast_all(fast);
        for (int r = 0; r < 128; ++r) {
            const u32x4_t v = src[(int64_t)r * vpr];
            float x[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                          bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
            if (fast) {
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] = quant_div(x[i], s[i], rc[i]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] = x[i] / s[i];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = __builtin_fminf(__builtin_fmaxf(x[i], -448.0f), 448.0f);
            int w0 = 0, w1 = 0;
            w0 = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w0, false);
            w0 = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w0, true);
            w1 = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], w1, false);
            w1 = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], w1, true);
            dst[(int64_t)r * vpr] = u32x2_t{(uint32_t)w0, (uint32_t)w1};
        }
    }
}

// ---- 128x128 -------------------------------------------------------------------------------
// grid = groups * (rows/128) * (cols/128) workgroups of 256 threads
__global__ __launch_bounds__(256) void quant_128x128_kernel(const u32x4_t* __restrict__ W, int rows, int cols,
                                                            u32x2_t* __restrict__ q, float* __restrict__ scale) {
    __shared__ float part[4];
    const int nbr = rows / 128, nbc = cols / 128;
    const int b = blockIdx.x;
    const int g = b / (nbr * nbc), rb = (b / nbc) % nbr, cb = b % nbc;
    const int vpr = cols / 8;
    const int tr = threadIdx.x >> 4, tc = threadIdx.x & 15;   // 16 rows x 16 vectors per pass
    const int64_t base = ((int64_t)g * rows + rb * 128) * vpr + cb * 16 + tc;
    u32x4_t v[8];
    float m = 0.f;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        v[it] = W[base + (int64_t)(it * 16 + tr) * vpr];
        m = fmaxf(m, amax8(v[it]));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    const float s = block_scale(m);
    if (threadIdx.x == 0) scale[b] = s;
#pragma unroll
    for (int it = 0; it < 8; ++it) q[base + (int64_t)(it * 16 + tr) * vpr] = cvt8_e4m3(v[it], s);
}

static moe_status fp8_rowcol_launch(moe_ctx* ctx, hipStream_t s, const char* who, const void* X, int64_t rows, int cols,
                                    const int32_t* rows_dev, void* q_row, float* s_row, void* q_col, float* s_col,
                                    const int32_t* src_of, int k, const float* pair_scale, int groups);

extern "C" moe_status moe_fp8_quantize(moe_ctx* ctx, void* stream, const void* X, moe_qblock block,
                                       int groups, int64_t rows, int cols, const int32_t* rows_dev,
                                       void* q, float* scale) {
    if (!ctx) return MOE_ERR_ARG;
    if (!X || !q || !scale) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize: NULL pointer");
    if (rows < 0 || cols < 1 || groups < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize: bad sizes");
    if (cols % 8) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize: cols must be a multiple of 8");
    hipStream_t s = (hipStream_t)stream;
    const int cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
    if (rows == 0) return MOE_OK;
    switch (block) {
        case MOE_Q_1x128: {
            if (cols % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(1x128): cols %% 128 != 0");
            if (groups != 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(1x128): groups must be 1");
            const int64_t nb = rows * (cols / 128);
            int64_t grid = ceil_div64(nb * 16, 256);
            if (grid > (int64_t)cu * 32) grid = (int64_t)cu * 32;
            hipLaunchKernelGGL(quant_1x128_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                               rows_dev, (u32x2_t*)q, scale);
            break;
        }
        case MOE_Q_128x1: {
            if (rows % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(128x1): rows %% 128 != 0");
            if (groups != 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(128x1): groups must be 1");
            if (cols % 128 == 0) {  // the tiled kernel below: the same bits at about twice the rate
                moe_status st = fp8_rowcol_launch(ctx, s, "moe_fp8_quantize(128x1)", X, rows, cols, rows_dev, nullptr, nullptr, q, scale,
                                                  nullptr, 1, nullptr, 1);
                if (st != MOE_OK) return st;
                break;
            }
            const int64_t npanels = (rows / 128) * ceil_div64(cols / 8, 64);
            int64_t grid = ceil_div64(npanels, 4);
            if (grid > (int64_t)cu * 16) grid = (int64_t)cu * 16;
            hipLaunchKernelGGL(quant_128x1_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                               rows_dev, (u32x2_t*)q, scale);
            break;
        }
        case MOE_Q_128x128: {
            if (rows % 128 || cols % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(128x128): rows, cols %% 128 != 0");
            if (rows_dev) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(128x128): rows_dev is not used for weights");
            const int64_t nb = (int64_t)groups * (rows / 128) * (cols / 128);
            if (nb > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize(128x128): too many blocks");
            hipLaunchKernelGGL(quant_128x128_kernel, dim3((unsigned)nb), dim3(256), 0, s, (const u32x4_t*)X, (int)rows, cols,
                               (u32x2_t*)q, scale);
            break;
        }
        default:
            MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize: bad block kind");
    }
    MOE_LAUNCH_CHECK(ctx, "moe_fp8_quantize");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// Blockwise recipe, row- and column-wise copies in one pass (Sec. 5.3.3: a tensor that two GEMMs read with different
// contraction dimensions is quantised once per direction; Sec. 5.4.2: one grouped launch; Sec. 5.4.1: padding and
// the permutation fused in).  A 256-thread workgroup owns a tile of 128 rows x 128 columns: exactly one 1x128 block
// of each of its rows and one 128x1 block of each of its columns.  Wave w owns rows 32 w .. 32 w + 31; a lane reads
// eight 16-byte pieces: piece i is row 32 w + 4 i + lane / 16, columns 8 (lane % 16) .. + 7.
//   row-wise : the block is the 16 lanes of one piece (four butterfly steps);
//   col-wise : the block is the same element of the lane's 8 pieces, of the 4 lanes 16 apart and of the 4 waves
//              (maxima meet in LDS).
// Either copy may be switched off (q_row or q_col NULL).  GATHER: row r of the input is pair_scale[s] * X[s / k, :]
// rounded to bf16 (no scale, no rounding when pair_scale is NULL) with s = src_of[r], zero where s < 0.
// Scales and codes are formed exactly as in the single-direction kernels above (amax / 448, fp32 division,
// hardware conversion), so both copies are bit-identical to theirs.
// ---------------------------------------------------------------------------
// floor(s / k) for a map entry 0 <= s < 2^31 as one widening multiplication (division by an invariant integer,
// rounded-up constant): with l = ceil(log2 k) and m = ceil(2^(31 + l) / k) <= 2^32 - 1, (s * m) >> (31 + l) == s / k
// for every such s, and the product stays below 2^63.
struct gather_div_t { uint32_t m; int sh; };
static inline gather_div_t gather_div(int k) {
    int l = 0;
    while ((1 << l) < k) ++l;
    return gather_div_t{(uint32_t)(((1ull << (31 + l)) + (uint64_t)k - 1) / (uint64_t)k), 31 + l};
}

__device__ __forceinline__ uint32_t scale2_bf16_bw(uint32_t w, float sc) { return pack_bf16(sc * bf16_lo(w), sc * bf16_hi(w)); }

template <bool GATHER>
__global__ __launch_bounds__(256) void fp8_quant_rowcol_kernel(const u32x4_t* __restrict__ X, int64_t rows, int cols,
                                                               const int32_t* __restrict__ rows_dev,
                                                               const int32_t* __restrict__ src_of, uint32_t k_magic, int k_shift,
                                                               const float* __restrict__ pair_scale, int groups,
                                                               u32x2_t* __restrict__ q_row, float* __restrict__ s_row,
                                                               u32x2_t* __restrict__ q_col, float* __restrict__ s_col) {
    __shared__ float cmax[4][128];
    const int64_t live = rows_dev ? min((int64_t)*rows_dev, rows) : rows;
    const int ctiles = cols / 128;
    int64_t rt = blockIdx.x / ctiles;
    const int ct = blockIdx.x % ctiles;
    if (GATHER && groups > 1) {  // row tiles expert-interleaved: the k copies of a token are read close together in time
        const int64_t S = (rows / 128 + groups - 1) / groups;
        rt = (rt % groups) * S + rt / groups;
    }
    const int64_t row0 = rt * 128;
    if (row0 >= live || row0 >= rows) return;  // uniform over the workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int vpr = cols / 8;
    const int64_t v0 = (row0 + wave * 32 + (lane >> 4)) * vpr + ct * 16 + (lane & 15);
    u32x4_t x[8];
    if (GATHER) {
        // Three passes, so that the eight map entries, then the eight rows, then the eight weights are each in
        // flight together (one pass per piece would chain sixteen memory latencies per lane), and no branch: a lane
        // whose row is padding reads 16 aligned bytes of this tile's 512 bytes of map entries instead, which always
        // exist, and drops them.
        const void* const spare = (const void*)(((uintptr_t)(src_of + row0) + 15) & ~(uintptr_t)15);
        int32_t sidx[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) sidx[i] = src_of[row0 + wave * 32 + 4 * i + (lane >> 4)];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t tok = (int64_t)(((uint64_t)(uint32_t)sidx[i] * k_magic) >> k_shift);  // sidx / k (gather_div)
            uint64_t live_at = (uint64_t)(X + (tok * vpr + ct * 16 + (lane & 15)));
            asm volatile("" : "+v"(live_at));  // (formed for every lane: a select then, not a branch around the multiplications)
            x[i] = *(const u32x4_t*)(sidx[i] >= 0 ? live_at : (uint64_t)spare);
        }
        if (pair_scale) {
            float psc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) psc[i] = *(sidx[i] >= 0 ? pair_scale + sidx[i] : (const float*)spare);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                x[i] = u32x4_t{scale2_bf16_bw(x[i].x, psc[i]), scale2_bf16_bw(x[i].y, psc[i]), scale2_bf16_bw(x[i].z, psc[i]),
                               scale2_bf16_bw(x[i].w, psc[i])};
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (sidx[i] < 0) x[i] = u32x4_t{0, 0, 0, 0};
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = X[v0 + (int64_t)i * 4 * vpr];
    }
    if (q_col) {  // (first: the other waves' maxima are on their way while this wave converts its rows)
        float m[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) m[c] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            m[0] = fmaxf(m[0], fabsf(bf16_lo(x[i].x))); m[1] = fmaxf(m[1], fabsf(bf16_hi(x[i].x)));
            m[2] = fmaxf(m[2], fabsf(bf16_lo(x[i].y))); m[3] = fmaxf(m[3], fabsf(bf16_hi(x[i].y)));
            m[4] = fmaxf(m[4], fabsf(bf16_lo(x[i].z))); m[5] = fmaxf(m[5], fabsf(bf16_hi(x[i].z)));
            m[6] = fmaxf(m[6], fabsf(bf16_lo(x[i].w))); m[7] = fmaxf(m[7], fabsf(bf16_hi(x[i].w)));
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            m[c] = fmaxf(m[c], __shfl_xor(m[c], 16));
            m[c] = fmaxf(m[c], __shfl_xor(m[c], 32));
            if (lane < 16) cmax[wave][8 * lane + c] = m[c];
        }
    }
    if (q_row) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float m = amax8(x[i]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
            const float sc = block_scale(m);
            q_row[v0 + (int64_t)i * 4 * vpr] = cvt8_e4m3(x[i], sc);
            if ((lane & 15) == 0) s_row[(row0 + wave * 32 + 4 * i + (lane >> 4)) * ctiles + ct] = sc;
        }
    }
    if (q_col) {
        __syncthreads();
        float sc[8], rc[8];
        bool fast = true;
        const int cb = 8 * (lane & 15);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            sc[c] = block_scale(fmaxf(fmaxf(cmax[0][cb + c], cmax[1][cb + c]), fmaxf(cmax[2][cb + c], cmax[3][cb + c])));
            rc[c] = 1.0f / sc[c];
            fast &= quant_fast_ok(sc[c]);
        }
        fast = quant_fast_all(fast);   // (see quant_div: one division per column block instead of one per element)
        if (wave == 0 && lane < 16) {
            f32x4_t* sd = (f32x4_t*)(s_col + rt * cols + ct * 128 + cb);
            sd[0] = f32x4_t{sc[0], sc[1], sc[2], sc[3]};
            sd[1] = f32x4_t{sc[4], sc[5], sc[6], sc[7]};
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float v[8] = {bf16_lo(x[i].x), bf16_hi(x[i].x), bf16_lo(x[i].y), bf16_hi(x[i].y),
                          bf16_lo(x[i].z), bf16_hi(x[i].z), bf16_lo(x[i].w), bf16_hi(x[i].w)};
            if (fast) {
#pragma unroll
                for (int c = 0; c < 8; ++c) v[c] = quant_div(v[c], sc[c], rc[c]);
            } else {
#pragma unroll
                for (int c = 0; c < 8; ++c) v[c] = v[c] / sc[c];
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) v[c] = __builtin_fminf(__builtin_fmaxf(v[c], -448.0f), 448.0f);
            int w0 = 0, w1 = 0;
            w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], w0, false);
            w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], w0, true);
            w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], w1, false);
            w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], w1, true);
            q_col[v0 + (int64_t)i * 4 * vpr] = u32x2_t{(uint32_t)w0, (uint32_t)w1};
        }
    }
}

static moe_status fp8_rowcol_launch(moe_ctx* ctx, hipStream_t s, const char* who, const void* X, int64_t rows, int cols,
                                    const int32_t* rows_dev, void* q_row, float* s_row, void* q_col, float* s_col,
                                    const int32_t* src_of, int k, const float* pair_scale, int groups) {
    if (rows % 128 || cols % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: rows and cols must be multiples of 128", who);
    if ((q_row == nullptr) != (s_row == nullptr) || (q_col == nullptr) != (s_col == nullptr) || (!q_row && !q_col))
        MOE_FAIL(ctx, MOE_ERR_ARG, "%s: codes and scales of a copy go together, and at least one copy is needed", who);
    if (groups < 1) groups = 1;
    const int64_t tiles_r = src_of ? (rows / 128 + groups - 1) / groups * groups : rows / 128;
    const int64_t nblk = tiles_r * (cols / 128);
    if (nblk > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: too many tiles", who);
    if (src_of)
        hipLaunchKernelGGL(fp8_quant_rowcol_kernel<true>, dim3((unsigned)nblk), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                           rows_dev, src_of, gather_div(k).m, gather_div(k).sh, pair_scale, groups, (u32x2_t*)q_row, s_row,
                           (u32x2_t*)q_col, s_col);
    else
        hipLaunchKernelGGL(fp8_quant_rowcol_kernel<false>, dim3((unsigned)nblk), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                           rows_dev, nullptr, 0, 0, nullptr, 1, (u32x2_t*)q_row, s_row, (u32x2_t*)q_col, s_col);
    return MOE_OK;
}

extern "C" moe_status moe_fp8_quantize_rowcol(moe_ctx* ctx, void* stream, const void* X, int64_t rows, int cols,
                                              const int32_t* rows_dev, void* q_row, float* scale_row,
                                              void* q_col, float* scale_col) {
    if (!ctx) return MOE_ERR_ARG;
    if (!X) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize_rowcol: NULL pointer");
    if (rows < 0 || cols < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize_rowcol: bad sizes");
    if (rows == 0) return MOE_OK;
    moe_status st = fp8_rowcol_launch(ctx, (hipStream_t)stream, "moe_fp8_quantize_rowcol", X, rows, cols, rows_dev, q_row,
                                      scale_row, q_col, scale_col, nullptr, 1, nullptr, 1);
    if (st != MOE_OK) return st;
    MOE_LAUNCH_CHECK(ctx, "moe_fp8_quantize_rowcol");
    return MOE_OK;
}

extern "C" moe_status moe_fp8_quantize_rowcol_gather(moe_ctx* ctx, void* stream, const void* X, const int32_t* src_of, int k,
                                                     const float* pair_scale, int groups, int64_t rows, int cols,
                                                     const int32_t* rows_dev, void* q_row, float* scale_row,
                                                     void* q_col, float* scale_col) {
    if (!ctx) return MOE_ERR_ARG;
    if (!X || !src_of) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize_rowcol_gather: NULL pointer");
    if (rows < 0 || cols < 1 || k < 1 || k > 32 || groups < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_fp8_quantize_rowcol_gather: bad sizes");
    if (rows == 0) return MOE_OK;
    moe_status st = fp8_rowcol_launch(ctx, (hipStream_t)stream, "moe_fp8_quantize_rowcol_gather", X, rows, cols, rows_dev,
                                      q_row, scale_row, q_col, scale_col, src_of, k, pair_scale, groups);
    if (st != MOE_OK) return st;
    MOE_LAUNCH_CHECK(ctx, "moe_fp8_quantize_rowcol_gather");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// MXFP8 (Sec. 5.3.3): E4M3 elements in 1x32 blocks with E8M0 (power-of-two) scales.
//   e = ceil(log2(amax / 448)) from the bits of amax = 1.f * 2^(E-127): e = E - 127 - 8 (+1 if 1.f > 1.75),
//   clamped to +-127; an all-zero block gets e = 0.  code = nearest E4M3 to x * 2^-e (exact scaling).
//   1x32 : 4 lanes own one block (8 elements each); a wave reads 1 KB and writes 512 B contiguous.
//   32x1 : blocks of 32 consecutive rows of a column, for a tensor read with its row index as the contraction
//          (weights in the data gradient, both operands of the weight gradient); made alone or together with
//          the 1x32 copy in one pass over the input (mx_quant_rowcol_kernel).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mx_quant_1x32_kernel(const u32x4_t* __restrict__ X, int64_t rows, int cols,
                                                            const int32_t* __restrict__ rows_dev,
                                                            u32x2_t* __restrict__ q, uint8_t* __restrict__ e8) {
    const int64_t live = rows_dev ? min((int64_t)*rows_dev, rows) : rows;
    const int64_t nvec = live * (cols / 8);            // 16-byte vectors; 4 per block, blocks never straddle rows
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; v < ((nvec + 3) & ~(int64_t)3); v += stride) {  // whole 4-lane groups stay together
        const bool in = v < nvec;
        const u32x4_t x = in ? X[v] : u32x4_t{0, 0, 0, 0};
        float m = amax8(x);
        m = fmaxf(m, __shfl_xor(m, 1));
        m = fmaxf(m, __shfl_xor(m, 2));
        const int e = mx_exponent(m);
        if (in) {
            u32x2_t o;
            o.x = mx_cvt4_bf16(x.x, x.y, mx_scale_f32(e));
            o.y = mx_cvt4_bf16(x.z, x.w, mx_scale_f32(e));
            q[v] = o;
            if ((v & 3) == 0) e8[v >> 2] = (uint8_t)(e + 127);
        }
    }
}

// Row- and column-wise copies in one pass (either may be switched off).  A 256-thread workgroup owns a tile of
// 128 rows x 128 columns; wave w owns its rows 32 w .. 32 w + 31, i.e. one 32-row block of every column.  A lane
// reads eight 16-byte pieces: piece i is row 4 i + lane / 16, columns 8 (lane % 16) .. + 7.
//   row-wise  : a 1x32 block is 4 adjacent lanes of one piece (two butterfly steps);
//   col-wise  : a 32x1 block is the same element of the lane's 8 pieces and of the 4 lanes 16 apart.
// The column scales of the four waves meet in LDS and leave as one dword per column:
// e8_col[(row / 128) * cols + col] holds the four 32-row blocks of rows 128 (row / 128) .. + 127, the unit in
// which the GEMMs walk a contraction over rows.
// GATHER: the input is not stored in row order: row r of it is pair_scale[s] * X[s / k, :] rounded to bf16
// (no scale, no rounding when pair_scale is NULL) with s = src_of[r], and zero where s < 0 -- the permuted
// tokens (Sec. 4.3.3) or the combine's backward, quantised without ever being written out in bf16.
__device__ __forceinline__ uint32_t scale2_bf16(uint32_t w, float sc) { return pack_bf16(sc * bf16_lo(w), sc * bf16_hi(w)); }

template <bool GATHER>
__global__ __launch_bounds__(256) void mx_quant_rowcol_kernel(const u32x4_t* __restrict__ X, int64_t rows, int cols,
                                                              const int32_t* __restrict__ rows_dev,
                                                              const int32_t* __restrict__ src_of, uint32_t k_magic, int k_shift,
                                                              const float* __restrict__ pair_scale, int groups,
                                                              u32x2_t* __restrict__ q_row, uint32_t* __restrict__ e8_row,
                                                              u32x2_t* __restrict__ q_col, uint32_t* __restrict__ e8_col) {
    __shared__ uint8_t sc[4][128];
    const int64_t live = rows_dev ? min((int64_t)*rows_dev, rows) : rows;
    const int ctiles = cols / 128;
    int64_t rt = blockIdx.x / ctiles;
    const int ct = blockIdx.x % ctiles;
    if (GATHER && groups > 1) {
        // Visit the row tiles expert-interleaved: with `groups` experts of roughly equal extent, consecutive
        // workgroups take the same relative position in different experts, which (stable order inside an expert)
        // is roughly the same window of source tokens, so the k copies of a token are read while it is cached.
        // Only the order changes: rt -> (rt % groups) * S + rt / groups is one-to-one onto [0, groups * S).
        const int64_t S = (rows / 128 + groups - 1) / groups;
        rt = (rt % groups) * S + rt / groups;
    }
    const int64_t row0 = rt * 128;
    if (row0 >= live || row0 >= rows) return;  // uniform over the workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int vpr = cols / 8;                                       // 16-byte pieces per row
    const int64_t v0 = (row0 + wave * 32 + (lane >> 4)) * vpr + ct * 16 + (lane & 15);
    u32x4_t x[8];
    if (GATHER) {
        // Three passes, so that the eight map entries, then the eight rows, then the eight weights are each in
        // flight together (one pass per piece would chain sixteen memory latencies per lane), and no branch: a lane
        // whose row is padding reads 16 aligned bytes of this tile's 512 bytes of map entries instead, which always
        // exist, and drops them.
        const void* const spare = (const void*)(((uintptr_t)(src_of + row0) + 15) & ~(uintptr_t)15);
        int32_t sidx[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) sidx[i] = src_of[row0 + wave * 32 + 4 * i + (lane >> 4)];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t tok = (int64_t)(((uint64_t)(uint32_t)sidx[i] * k_magic) >> k_shift);  // sidx / k (gather_div)
            uint64_t live_at = (uint64_t)(X + (tok * vpr + ct * 16 + (lane & 15)));
            asm volatile("" : "+v"(live_at));  // (formed for every lane: a select then, not a branch around the multiplications)
            x[i] = *(const u32x4_t*)(sidx[i] >= 0 ? live_at : (uint64_t)spare);
        }
        if (pair_scale) {
            float psc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) psc[i] = *(sidx[i] >= 0 ? pair_scale + sidx[i] : (const float*)spare);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                x[i] = u32x4_t{scale2_bf16(x[i].x, psc[i]), scale2_bf16(x[i].y, psc[i]), scale2_bf16(x[i].z, psc[i]),
                               scale2_bf16(x[i].w, psc[i])};
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (sidx[i] < 0) x[i] = u32x4_t{0, 0, 0, 0};
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = X[v0 + (int64_t)i * 4 * vpr];
    }
    if (q_row) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float m = amax8(x[i]);
            m = fmaxf(m, __shfl_xor(m, 1));
            m = fmaxf(m, __shfl_xor(m, 2));
            const int e = mx_exponent(m);
            u32x2_t o;
            o.x = mx_cvt4_bf16(x[i].x, x[i].y, mx_scale_f32(e));
            o.y = mx_cvt4_bf16(x[i].z, x[i].w, mx_scale_f32(e));
            q_row[v0 + (int64_t)i * 4 * vpr] = o;
            // the row's four block bytes of this tile, gathered into the first of its 16 lanes
            const int b = e + 127, base = lane & 48;
            const uint32_t w = (uint32_t)__shfl(b, base) | ((uint32_t)__shfl(b, base + 4) << 8) |
                               ((uint32_t)__shfl(b, base + 8) << 16) | ((uint32_t)__shfl(b, base + 12) << 24);
            if ((lane & 15) == 0) e8_row[((row0 + wave * 32 + 4 * i + (lane >> 4)) * (cols / 32) + ct * 4) >> 2] = w;
        }
    }
    if (q_col) {
        float m[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) m[c] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            m[0] = fmaxf(m[0], fabsf(bf16_lo(x[i].x))); m[1] = fmaxf(m[1], fabsf(bf16_hi(x[i].x)));
            m[2] = fmaxf(m[2], fabsf(bf16_lo(x[i].y))); m[3] = fmaxf(m[3], fabsf(bf16_hi(x[i].y)));
            m[4] = fmaxf(m[4], fabsf(bf16_lo(x[i].z))); m[5] = fmaxf(m[5], fabsf(bf16_hi(x[i].z)));
            m[6] = fmaxf(m[6], fabsf(bf16_lo(x[i].w))); m[7] = fmaxf(m[7], fabsf(bf16_hi(x[i].w)));
        }
        int e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            m[c] = fmaxf(m[c], __shfl_xor(m[c], 16));
            m[c] = fmaxf(m[c], __shfl_xor(m[c], 32));
            e[c] = mx_exponent(m[c]);
            if (lane < 16) sc[wave][8 * lane + c] = (uint8_t)(e[c] + 127);
        }
        float sf[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) sf[c] = mx_scale_f32(e[c]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const u32x2_t o = {mx_cvt4_bf16_each(x[i].x, x[i].y, sf[0], sf[1], sf[2], sf[3]),
                               mx_cvt4_bf16_each(x[i].z, x[i].w, sf[4], sf[5], sf[6], sf[7])};
            q_col[v0 + (int64_t)i * 4 * vpr] = o;
        }
        __syncthreads();
        if (threadIdx.x < 128) {
            const int c = threadIdx.x;
            e8_col[rt * cols + ct * 128 + c] = (uint32_t)sc[0][c] | ((uint32_t)sc[1][c] << 8) | ((uint32_t)sc[2][c] << 16) |
                                               ((uint32_t)sc[3][c] << 24);
        }
    }
}

static moe_status mx_rowcol_launch(moe_ctx* ctx, hipStream_t s, const char* who, const void* X, int64_t rows, int cols,
                                   const int32_t* rows_dev, void* q_row, uint8_t* e8_row, void* q_col, uint8_t* e8_col,
                                   const int32_t* src_of = nullptr, int k = 1, const float* pair_scale = nullptr,
                                   int groups = 1) {
    if (rows % 128 || cols % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: rows and cols must be multiples of 128", who);
    if (groups < 1) groups = 1;
    const int64_t tiles_r = src_of ? (rows / 128 + groups - 1) / groups * groups : rows / 128;
    const int64_t nblk = tiles_r * (cols / 128);
    if (nblk > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: too many tiles", who);
    if (src_of)
        hipLaunchKernelGGL(mx_quant_rowcol_kernel<true>, dim3((unsigned)nblk), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                           rows_dev, src_of, gather_div(k).m, gather_div(k).sh, pair_scale, groups, (u32x2_t*)q_row, (uint32_t*)e8_row, (u32x2_t*)q_col,
                           (uint32_t*)e8_col);
    else
        hipLaunchKernelGGL(mx_quant_rowcol_kernel<false>, dim3((unsigned)nblk), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                           rows_dev, nullptr, 0, 0, nullptr, 1, (u32x2_t*)q_row, (uint32_t*)e8_row, (u32x2_t*)q_col,
                           (uint32_t*)e8_col);
    return MOE_OK;
}

extern "C" moe_status moe_mx_quantize(moe_ctx* ctx, void* stream, const void* X, moe_mxblock block,
                                      int groups, int64_t rows, int cols, const int32_t* rows_dev,
                                      void* q, uint8_t* e8m0) {
    if (!ctx) return MOE_ERR_ARG;
    if (!X || !q || !e8m0) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize: NULL pointer");
    if (rows < 0 || cols < 1 || groups < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize: bad sizes");
    hipStream_t s = (hipStream_t)stream;
    const int cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
    if (rows == 0) return MOE_OK;
    switch (block) {
        case MOE_MX_1x32: {
            if (cols % 32) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize(1x32): cols %% 32 != 0");
            if (groups != 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize(1x32): groups must be 1 (fold them into rows)");
            int64_t grid = ceil_div64(rows * (cols / 8), 256);
            if (grid > (int64_t)cu * 32) grid = (int64_t)cu * 32;
            hipLaunchKernelGGL(mx_quant_1x32_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const u32x4_t*)X, rows, cols,
                               rows_dev, (u32x2_t*)q, e8m0);
            break;
        }
        case MOE_MX_32x1: {
            if (rows % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize(32x1): rows %% 128 != 0");
            if (groups != 1 && rows_dev) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize(32x1): rows_dev needs groups == 1");
            moe_status st = mx_rowcol_launch(ctx, s, "moe_mx_quantize(32x1)", X, (int64_t)groups * rows, cols, rows_dev, nullptr,
                                             nullptr, q, e8m0);
            if (st != MOE_OK) return st;
            break;
        }
        default:
            MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize: bad block kind");
    }
    MOE_LAUNCH_CHECK(ctx, "moe_mx_quantize");
    return MOE_OK;
}

extern "C" moe_status moe_mx_quantize_rowcol(moe_ctx* ctx, void* stream, const void* X, int64_t rows, int cols,
                                             const int32_t* rows_dev, void* q_row, uint8_t* e8m0_row,
                                             void* q_col, uint8_t* e8m0_col) {
    if (!ctx) return MOE_ERR_ARG;
    if (!X || !q_row || !e8m0_row || !q_col || !e8m0_col) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize_rowcol: NULL pointer");
    if (rows < 0 || cols < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize_rowcol: bad sizes");
    if (rows == 0) return MOE_OK;
    moe_status st = mx_rowcol_launch(ctx, (hipStream_t)stream, "moe_mx_quantize_rowcol", X, rows, cols, rows_dev, q_row,
                                     e8m0_row, q_col, e8m0_col);
    if (st != MOE_OK) return st;
    MOE_LAUNCH_CHECK(ctx, "moe_mx_quantize_rowcol");
    return MOE_OK;
}

extern "C" moe_status moe_mx_quantize_rowcol_gather(moe_ctx* ctx, void* stream, const void* X, const int32_t* src_of, int k,
                                                    const float* pair_scale, int groups, int64_t rows, int cols,
                                                    const int32_t* rows_dev, void* q_row, uint8_t* e8m0_row,
                                                    void* q_col, uint8_t* e8m0_col) {
    if (!ctx) return MOE_ERR_ARG;
    if (!X || !src_of || !q_row || !e8m0_row || !q_col || !e8m0_col)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize_rowcol_gather: NULL pointer");
    if (rows < 0 || cols < 1 || k < 1 || k > 32 || groups < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_mx_quantize_rowcol_gather: bad sizes");
    if (rows == 0) return MOE_OK;
    moe_status st = mx_rowcol_launch(ctx, (hipStream_t)stream, "moe_mx_quantize_rowcol_gather", X, rows, cols, rows_dev, q_row,
                                     e8m0_row, q_col, e8m0_col, src_of, k, pair_scale, groups);
    if (st != MOE_OK) return st;
    MOE_LAUNCH_CHECK(ctx, "moe_mx_quantize_rowcol_gather");
    return MOE_OK;
}
