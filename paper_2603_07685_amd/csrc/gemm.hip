// Grouped GEMM for the expert MLP (Sec. 2.1.4, 4.3.2), device-initiated (Sec. 4.3.7):
// one persistent launch, every expert's extent is read from `offsets` on the device.
//
// Tiling (bf16): a workgroup of 8 wavefronts owns a 256x256 output tile and walks the
// contraction dimension in steps of 64.  Both operand tiles (256x64 bf16 = 32 KB each)
// are brought in by direct global->LDS loads (16 B per lane) into two LDS stages, so
// the loads of step i+1 are in flight while the MFMAs of step i run.  A tile row is
// 128 B in LDS; its eight 16-byte slots are XOR-swizzled with the row number so the
// ds_read_b128 operand fetches of the 32x32x16 MFMA spread over all banks.  Waves
// are arranged 2 (rows) x 4 (columns); a wave's two 32-column sub-tiles are 128
// columns apart so that, with the SwiGLU epilogue, they are the gate and up columns
// of the same output features and the activation is applied on the fp32 accumulators.
#include "common.h"

#define GG_BM 256
#define GG_BN 256
#define GG_BK 64
#define GG_THREADS 512
#define GG_MAX_E 1024
#define GG_STAGE_BYTES (GG_BM * GG_BK * 2)  // one operand tile: 32 KB

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void gbl_void_t;

__device__ __forceinline__ void dma16(const void* g, void* lds_wave_base) {
    // each lane moves 16 bytes: LDS destination = wave-uniform base + lane * 16
    __builtin_amdgcn_global_load_lds((gbl_void_t*)g, (lds_void_t*)lds_wave_base, 16, 0, 0);
}

// s_waitcnt vmcnt(0) only (gfx9 encoding: expcnt and lgkmcnt fields left at their maxima)
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

struct gg_tile {
    int e, m0, m_end, tn;
};

// Tile id -> (expert, first row, row end, column tile).  tile_start[] is the
// exclusive prefix of per-expert tile counts.  Inside an expert the tiles are
// ordered in bands of GG_BAND row-tiles, column-major inside a band, so that
// workgroups running at the same time share operand panels in L2.
#define GG_BAND 8
__device__ __forceinline__ gg_tile gg_locate(int tid, int& e_hint, const int* tile_start, const int* offs, int E,
                                             int tiles_n) {
    int e = e_hint;
    while (e + 1 < E && tid >= tile_start[e + 1]) ++e;
    e_hint = e;
    const int u = tid - tile_start[e];
    const int rows = offs[e + 1] - offs[e];
    const int tiles_m = (rows + GG_BM - 1) / GG_BM;
    const int band_sz = GG_BAND * tiles_n;
    const int band = u / band_sz;
    const int in_band = u - band * band_sz;
    const int band_rows = min(GG_BAND, tiles_m - band * GG_BAND);
    const int tm = band * GG_BAND + in_band % band_rows;
    const int tn = in_band / band_rows;
    gg_tile t;
    t.e = e;
    t.m0 = offs[e] + tm * GG_BM;
    t.m_end = offs[e + 1];
    t.tn = tn;
    return t;
}

// EPI: 0 = store C (bf16), 1 = SwiGLU: store Z (optional) and act = silu(gate)*up.
template <int EPI>
__global__ __launch_bounds__(GG_THREADS, 1) void gg_nt_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const int32_t* __restrict__ offsets, int E, int N,
    int K, int64_t Rcap, bf16_t* __restrict__ C, bf16_t* __restrict__ Cact, int* __restrict__ dev_err) {
    __shared__ __attribute__((aligned(1024))) char ldsA0[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsA1[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsB0[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsB1[GG_STAGE_BYTES];
    __shared__ int offs[GG_MAX_E + 1];
    __shared__ int tile_start[GG_MAX_E + 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 2;  // 0..1 : 128-row half
    const int wn = wave & 3;   // 0..3 : 32-column strip inside each 128-column half

    // ---- tile schedule, computed by every workgroup from the device-resident offsets ----
    const int f_half = N >> 1;
    const int tiles_n = EPI ? (f_half + 127) / 128 : (N + GG_BN - 1) / GG_BN;
    for (int e = tid; e <= E; e += GG_THREADS) offs[e] = offsets[e];
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            tile_start[e] = run;
            int rows = offs[e + 1] - offs[e];
            run += rows > 0 ? ((rows + GG_BM - 1) / GG_BM) * tiles_n : 0;
        }
        tile_start[E] = run;
        if (offs[E] > Rcap || offs[0] < 0) {  // inconsistent offsets: refuse to touch memory
            tile_start[E] = 0;
            if (blockIdx.x == 0) atomicExch(dev_err, 1);
        }
    }
    __syncthreads();
    const int total_tiles = tile_start[E];

    // workgroups land on the 8 XCDs round-robin; give each XCD a contiguous run of tiles
    const int G = gridDim.x;
    const int per_xcd = G >> 3;
    const int q = (G & 7) ? (int)blockIdx.x : ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);

    // ---- per-lane constants ----
    const int ld_row = lane >> 3;                    // row inside an 8-row DMA chunk
    const int ld_chunk = (lane & 7) ^ ld_row;        // global 16-byte chunk this lane fetches (swizzle)
    const int fr_row = lane & 31;                    // row inside a 32-row MFMA operand block
    const int fr_khalf = lane >> 5;                  // which 8-element half of the 16-wide k step
    const int fr_swz = lane & 7;

    int e_hint = 0;
    for (int t = q; t < total_tiles; t += G) {
        const gg_tile tl = gg_locate(t, e_hint, tile_start, offs, E, tiles_n);
        const int nA = EPI ? tl.tn * 128 : tl.tn * GG_BN;               // first column of sub-tile 0
        const int nB = EPI ? f_half + tl.tn * 128 : tl.tn * GG_BN + 128;  // first column of sub-tile 1

        // global source pointers of this lane's four DMA chunks per operand
        const char* ag[4];
        const char* bg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = wave * 32 + i * 8 + ld_row;  // tile row 0..255
            int64_t ar = (int64_t)tl.m0 + p;
            ar = ar < Rcap ? ar : Rcap - 1;
            ag[i] = (const char*)A + (ar * K + ld_chunk * 8) * 2;
            int bn = (p < 128 ? nA : nB - 128) + p;
            bn = bn < N ? bn : N - 1;
            bg[i] = (const char*)B + (((int64_t)tl.e * N + bn) * K + ld_chunk * 8) * 2;
        }

        f32x16_t acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;

        const int KT = K / GG_BK;
        // stage 0 <- k-tile 0
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma16(ag[i], ldsA0 + (wave * 32 + i * 8) * 128);
            dma16(bg[i], ldsB0 + (wave * 32 + i * 8) * 128);
        }
        wait_vm0();
        __syncthreads();

        const int a_rd = (wm * 128 + fr_row) * 128;
        const int b_rd = (wn * 32 + fr_row) * 128;

        auto compute = [&](const char* sa, const char* sb) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int slot = ((kk * 2 + fr_khalf) ^ fr_swz) * 16;
                bf16x8_t af[4], bfr[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) af[i] = *(const bf16x8_t*)(sa + a_rd + i * 32 * 128 + slot);
#pragma unroll
                for (int j = 0; j < 2; ++j) bfr[j] = *(const bf16x8_t*)(sb + b_rd + j * 128 * 128 + slot);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            }
        };

        for (int kt = 0; kt < KT; kt += 2) {
            // stage 1 <- k-tile kt+1 while stage 0 is consumed
            if (kt + 1 < KT) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    dma16(ag[i] + (kt + 1) * 128, ldsA1 + (wave * 32 + i * 8) * 128);
                    dma16(bg[i] + (kt + 1) * 128, ldsB1 + (wave * 32 + i * 8) * 128);
                }
            }
            compute(ldsA0, ldsB0);
            wait_vm0();
            __syncthreads();
            if (kt + 1 < KT) {
                if (kt + 2 < KT) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        dma16(ag[i] + (kt + 2) * 128, ldsA0 + (wave * 32 + i * 8) * 128);
                        dma16(bg[i] + (kt + 2) * 128, ldsB0 + (wave * 32 + i * 8) * 128);
                    }
                }
                compute(ldsA1, ldsB1);
                wait_vm0();
                __syncthreads();
            }
        }

        // ---- epilogue: accumulators -> bf16 -> global (lane owns one column, 16 rows per block) ----
        const int col0 = nA + wn * 32 + fr_row;  // column of sub-tile 0
        const int col1 = nB + wn * 32 + fr_row;  // column of sub-tile 1
        const int lim0 = EPI ? f_half : N;       // sub-tile 0 columns must stay below this
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int r = tl.m0 + wm * 128 + i * 32 + (x >> 2) * 8 + fr_khalf * 4 + (x & 3);
                if (r < tl.m_end) {
                    const float v0 = acc[i][0][x], v1 = acc[i][1][x];
                    if (EPI) {
                        if (col0 < lim0) {
                            if (C) {
                                C[(int64_t)r * N + col0] = (bf16_t)v0;
                                C[(int64_t)r * N + col1] = (bf16_t)v1;
                            }
                            Cact[(int64_t)r * f_half + col0] = (bf16_t)(silu_f(v0) * v1);
                        }
                    } else {
                        if (col0 < lim0) C[(int64_t)r * N + col0] = (bf16_t)v0;
                        if (col1 < N) C[(int64_t)r * N + col1] = (bf16_t)v1;
                    }
                }
            }
        }
        __syncthreads();  // stage 0 is refilled by the next tile's prologue
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static moe_status gg_check_common(moe_ctx* ctx, const char* who, const void* a, const void* b, const int32_t* offsets,
                                  int E, int N, int K, int64_t Rcap, moe_dtype dt) {
    if (!a || !b || !offsets) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: NULL pointer", who);
    if (E < 1 || E > GG_MAX_E || N < 1 || K < 1 || Rcap < 1 || Rcap > 0x7fffffffLL)
        MOE_FAIL(ctx, MOE_ERR_ARG, "%s: need 1<=E<=%d, N,K>=1, 1<=Rcap<2^31", who, GG_MAX_E);
    if (dt == MOE_F32) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: fp32 operands are not supported", who);
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_fwd(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                           const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                           moe_dtype dt, moe_epilogue epi,
                                           const float* a_scale, const float* b_scale,
                                           void* C, void* C_act) {
    if (!ctx) return MOE_ERR_ARG;
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_fwd", A, B, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    if (epi == MOE_EPI_SWIGLU) {
        if (!C_act) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: SWIGLU needs C_act");
        if (N % 2) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: SWIGLU needs even N");
    } else if (epi == MOE_EPI_NONE) {
        if (!C) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: C is NULL");
    } else {
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: bad epilogue");
    }
    if (dt == MOE_FP8_E4M3) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd: fp8 path not built yet");
    (void)a_scale;
    (void)b_scale;
    if (K % GG_BK) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd: K=%d must be a multiple of %d", K, GG_BK);
    hipStream_t s = (hipStream_t)stream;
    const int grid = ctx->num_cu > 0 ? ctx->num_cu : 256;
    if (epi == MOE_EPI_SWIGLU)
        hipLaunchKernelGGL(gg_nt_kernel<1>, dim3(grid), dim3(GG_THREADS), 0, s, (const bf16_t*)A, (const bf16_t*)B, offsets,
                           E, N, K, Rcap, (bf16_t*)C, (bf16_t*)C_act, ctx->dev_err);
    else
        hipLaunchKernelGGL(gg_nt_kernel<0>, dim3(grid), dim3(GG_THREADS), 0, s, (const bf16_t*)A, (const bf16_t*)B, offsets,
                           E, N, K, Rcap, (bf16_t*)C, (bf16_t*)C_act, ctx->dev_err);
    MOE_LAUNCH_CHECK(ctx, "gg_nt_kernel");
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_dgrad(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                             const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                             moe_dtype dt, const void* Z_saved,
                                             const float* dc_scale, const float* b_scale, void* dA) {
    if (!ctx) return MOE_ERR_ARG;
    MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad: not built yet");
}

extern "C" moe_status moe_grouped_gemm_wgrad(moe_ctx* ctx, void* stream, const void* A, const void* dC,
                                             const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                             moe_dtype dt, const float* a_scale, const float* dc_scale,
                                             int accumulate, moe_dtype out_dt, void* dB) {
    if (!ctx) return MOE_ERR_ARG;
    MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wgrad: not built yet");
}
