// Grouped GEMM for the expert MLP (Sec. 2.1.4, 4.3.2), device-initiated (Sec. 4.3.7):
// one persistent launch per call, every expert's extent is read from `offsets` on the
// device; forward, data-gradient and weight-gradient (Sec. 4.2.3 "W/D split") are three
// instantiations of one kernel.
//
// The kernel computes OUT[i,j] = sum_c P[i,c] * Q[j,c] on a 256x256 output tile per
// workgroup (8 wavefronts, 2 x 4), walking the contraction index c in steps of 64:
//     forward : P = activations [rows,K]   Q = W_e [N,K]        OUT = C[rows,N]
//     dgrad   : P = dC [rows,N]            Q = W_e as [K,N]^T   OUT = dA[rows,K]
//     wgrad   : P = dC as [N,rows]^T       Q = A as [K,rows]^T  OUT = dW_e[N,K]
// Operand tiles (32 KB each) are fetched by direct global->LDS loads, 16 B per lane,
// into two LDS stages, so step s+1 streams in while the MFMAs of step s run.
// An operand whose contraction index is contiguous in memory ("k-major", tile
// [256][64]) is read for the 32x32x16 bf16 MFMA with ds_read_b128; one whose
// contraction index is the memory row ("c-major", tile [64][256]: the weight in dgrad,
// both operands in wgrad) is read with the transposing ds_read_b64_tr_b16, so no
// transposed copy of weights or activations is ever made.  Both tile layouts XOR-swizzle
// their 16-byte slots so the operand reads spread over the LDS banks; the swizzle is
// applied on the global side of the DMA (each lane picks which 16 bytes it fetches).
// A wave's two 32-column sub-tiles are 128 columns apart: with the SwiGLU epilogue they
// are the gate and up columns of the same features, so the activation (forward) and its
// derivative (fc2 dgrad) are applied to the fp32 accumulators in registers.
#include "common.h"

#define GG_BM 256
#define GG_BN 256
#define GG_BK 64
#define GG_THREADS 512
#define GG_MAX_E 1024
#define GG_STAGE_BYTES (GG_BM * GG_BK * 2)  // one operand tile: 32 KB
#define GG_BAND 8                           // row-tiles per band of the tile order

enum { GG_FWD = 0, GG_DGRAD = 1, GG_WGRAD = 2 };
enum { GG_EPI_STORE = 0, GG_EPI_SWIGLU = 1, GG_EPI_SWIGLU_BWD = 2 };

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void gbl_void_t;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

__device__ __forceinline__ void dma16(const void* g, void* lds_wave_base) {
    // each lane moves 16 bytes: LDS destination = wave-uniform base + lane * 16
    __builtin_amdgcn_global_load_lds((gbl_void_t*)g, (lds_void_t*)lds_wave_base, 16, 0, 0);
}

// s_waitcnt vmcnt(0) only (gfx9 encoding: expcnt and lgkmcnt fields left at their maxima)
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ float sigmoid_f(float g) { return 1.0f / (1.0f + __expf(-g)); }

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the address of
// 4 consecutive 16-bit elements (row i/4, columns 4*(i%4)..+3 of a 4x16 block) and
// receives column i of that block (rows 0..3).  Two of them give the 8 contraction
// values per lane that the 32x32x16 MFMA operand needs.
__device__ __forceinline__ bf16x8_t lds_read_tr8(const char* p_lo, const char* p_hi) {
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p_lo);
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p_hi);
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
}

struct gg_args {
    const bf16_t* P;      // fwd: A, dgrad: dC, wgrad: dC
    const bf16_t* Q;      // fwd/dgrad: W [E,N,K], wgrad: A
    const int32_t* offsets;
    int E, N, K;
    int64_t Rcap;
    void* out;            // fwd: C (may be NULL with SWIGLU), dgrad: dA or dZ, wgrad: dW
    bf16_t* out_act;      // fwd SWIGLU: activation output
    const bf16_t* Zsaved; // dgrad SWIGLU_BWD: saved pre-activation [rows, 2K]
    const char* zeros;    // >= 16 zero bytes (feeds the wgrad contraction tail)
    int* dev_err;
    int accumulate;       // wgrad: out += result
};

// MODE: GG_FWD / GG_DGRAD / GG_WGRAD.  EPI: see enum.  OUT_F32: fp32 output (wgrad only).
template <int MODE, int EPI, bool OUT_F32>
__global__ __launch_bounds__(GG_THREADS, 1) void gg_kernel(const gg_args a) {
    __shared__ __attribute__((aligned(1024))) char ldsP0[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsP1[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsQ0[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsQ1[GG_STAGE_BYTES];
    __shared__ int offs[GG_MAX_E + 1];
    __shared__ int tile_start[GG_MAX_E + 1];

    constexpr bool P_CMAJ = (MODE == GG_WGRAD);
    constexpr bool Q_CMAJ = (MODE != GG_FWD);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 2;  // 0..1 : 128-row half of the tile
    const int wn = wave & 3;   // 0..3 : 32-column strip inside each 128-column half
    const int E = a.E, N = a.N, K = a.K;

    // Output geometry.  J = extent of j (output columns).
    //   fwd:   J = N (with SWIGLU the column tiles pair gate/up: N/2 features in tiles of 128)
    //   dgrad: J = K;  wgrad: i runs over N, J = K.
    const int J = (MODE == GG_FWD) ? N : K;
    const int half_cols = (EPI == GG_EPI_SWIGLU) ? (N >> 1) : 0;
    const int tiles_j = (EPI == GG_EPI_SWIGLU) ? (half_cols + 127) / 128 : (J + GG_BN - 1) / GG_BN;
    const int tiles_i_w = (N + GG_BM - 1) / GG_BM;  // wgrad only

    // ---- tile schedule, computed by every workgroup from the device-resident offsets ----
    for (int e = tid; e <= E; e += GG_THREADS) offs[e] = a.offsets[e];
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        bool bad = offs[0] < 0 || offs[E] > a.Rcap;
        for (int e = 0; e < E; ++e) {
            tile_start[e] = run;
            const int rows = offs[e + 1] - offs[e];
            bad |= rows < 0;
            if (MODE == GG_WGRAD) run += tiles_i_w * tiles_j;
            else run += rows > 0 ? ((rows + GG_BM - 1) / GG_BM) * tiles_j : 0;
        }
        tile_start[E] = run;
        if (bad) {  // inconsistent offsets: touch no tensor memory, raise the error word
            tile_start[E] = 0;
            if (blockIdx.x == 0) atomicExch(a.dev_err, 1);
        }
    }
    __syncthreads();
    const int total_tiles = tile_start[E];

    // workgroups land on the 8 XCDs round-robin; give each XCD a contiguous run of tiles
    const int G = gridDim.x;
    const int q = (G & 7) ? (int)blockIdx.x : ((int)blockIdx.x & 7) * (G >> 3) + ((int)blockIdx.x >> 3);

    // ---- per-lane constants: DMA side ----
    // k-major tile: a 1 KB DMA chunk = 8 rows x 128 B; lane -> (row l/8, slot l%8), slot ^= row%8
    const int km_row = lane >> 3;
    const int km_gslot = (lane & 7) ^ km_row;
    // c-major tile: a 1 KB chunk = 2 rows x 512 B; lane -> (row l/32, slot l%32), slot ^= 4*(row%4)
    const int cm_row = lane >> 5;
    // ---- per-lane constants: fragment side ----
    const int fr_row = lane & 31;
    const int fr_khalf = lane >> 5;
    const int fr_swz = lane & 7;
    const int tr_i = lane & 15;
    const int tr_blk = lane >> 4;
    // c-major read: row = kk*16 + 8*(blk>>1) + 4*hh + (i>>2); slot = (colblock/8 ^ 4*(i>>2)) + 2*(blk&1) + ((i&3)>>1)
    const int tr_rowoff = (8 * (tr_blk >> 1) + (tr_i >> 2)) * 512;
    const int tr_low = 2 * (tr_blk & 1) + ((tr_i & 3) >> 1);
    const int tr_xor = 4 * (tr_i >> 2);
    const int tr_byte = (tr_i & 1) * 8;

    int p_rd[4], q_rd[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (P_CMAJ) p_rd[i] = tr_rowoff + ((((wm * 128 + i * 32) >> 3) ^ tr_xor) + tr_low) * 16 + tr_byte;
        else p_rd[i] = (wm * 128 + i * 32 + fr_row) * 128;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (Q_CMAJ) q_rd[j] = tr_rowoff + ((((j * 128 + wn * 32) >> 3) ^ tr_xor) + tr_low) * 16 + tr_byte;
        else q_rd[j] = (j * 128 + wn * 32 + fr_row) * 128;
    }

    int e_hint = 0;
    for (int t = q; t < total_tiles; t += G) {
        // ---- locate the tile ----
        int e = e_hint;
        while (e + 1 < E && t >= tile_start[e + 1]) ++e;
        e_hint = e;
        const int u = t - tile_start[e];
        const int row_lo = offs[e], row_hi = offs[e + 1];
        int ti, tj;
        {
            const int tiles_i = (MODE == GG_WGRAD) ? tiles_i_w : (row_hi - row_lo + GG_BM - 1) / GG_BM;
            const int band_sz = GG_BAND * tiles_j;
            const int band = u / band_sz;
            const int in_band = u - band * band_sz;
            const int band_rows = min(GG_BAND, tiles_i - band * GG_BAND);
            ti = band * GG_BAND + in_band % band_rows;
            tj = in_band / band_rows;
        }
        // output row/column origin of the two 128-column halves
        const int i0 = (MODE == GG_WGRAD) ? ti * GG_BM : row_lo + ti * GG_BM;
        const int i_end = (MODE == GG_WGRAD) ? N : row_hi;
        const int j0 = (EPI == GG_EPI_SWIGLU) ? tj * 128 : tj * GG_BN;
        const int j1 = (EPI == GG_EPI_SWIGLU) ? half_cols + tj * 128 : tj * GG_BN + 128;
        // contraction range
        const int c_lo = (MODE == GG_WGRAD) ? row_lo : 0;
        const int c_hi = (MODE == GG_WGRAD) ? row_hi : (MODE == GG_FWD ? K : N);
        const int KT = (c_hi - c_lo + GG_BK - 1) / GG_BK;

        // ---- DMA source pointers (4 chunks per operand per lane) ----
        const char* pg[4];
        const char* qg[4];
        int64_t p_step, q_step;  // byte advance per contraction step
        if (P_CMAJ) {
            // P = dC [rows, N]: contraction row c, columns i0..i0+255
            p_step = (int64_t)GG_BK * N * 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (wave * 4 + i) * 2 + cm_row;
                const int slot = (lane & 31) ^ (4 * (row & 3));
                int col = i0 + slot * 8;
                col = col <= N - 8 ? col : N - 8;
                pg[i] = (const char*)a.P + ((int64_t)(c_lo + row) * N + col) * 2;
            }
        } else {
            const int ldp = (MODE == GG_FWD) ? K : N;
            p_step = GG_BK * 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int64_t r = (int64_t)i0 + wave * 32 + i * 8 + km_row;
                r = r < a.Rcap ? r : a.Rcap - 1;
                pg[i] = (const char*)a.P + (r * ldp + km_gslot * 8) * 2;
            }
        }
        if (Q_CMAJ) {
            // dgrad: Q = W_e [N,K]: contraction row n, columns (k) j0.. ; wgrad: Q = A [rows,K]
            q_step = (int64_t)GG_BK * K * 2;
            const char* qbase = (MODE == GG_DGRAD) ? (const char*)a.Q + (int64_t)e * N * K * 2 : (const char*)a.Q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (wave * 4 + i) * 2 + cm_row;
                const int slot = (lane & 31) ^ (4 * (row & 3));
                int col = (slot < 16 ? j0 : j1 - 128) + slot * 8;
                col = col <= K - 8 ? col : K - 8;
                qg[i] = qbase + ((int64_t)(c_lo + row) * K + col) * 2;
            }
        } else {
            q_step = GG_BK * 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int p = wave * 32 + i * 8 + km_row;
                int n = (p < 128 ? j0 : j1 - 128) + p;
                n = n < N ? n : N - 1;
                qg[i] = (const char*)a.Q + (((int64_t)e * N + n) * K + km_gslot * 8) * 2;
            }
        }

        auto issue = [&](int kt, char* sp, char* sq) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const char* ps = pg[i] + kt * p_step;
                const char* qs = qg[i] + kt * q_step;
                if (MODE == GG_WGRAD) {  // contraction tail of the expert: feed zeros
                    const int row = c_lo + kt * GG_BK + (wave * 4 + i) * 2 + cm_row;
                    ps = row < c_hi ? ps : a.zeros;
                    qs = row < c_hi ? qs : a.zeros;
                }
                dma16(ps, sp + (wave * 4 + i) * 1024);
                dma16(qs, sq + (wave * 4 + i) * 1024);
            }
        };

        f32x16_t acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;

        auto compute = [&](const char* sp, const char* sq) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int km_slot = ((kk * 2 + fr_khalf) ^ fr_swz) * 16;
                bf16x8_t pf[4], qf[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (P_CMAJ) pf[i] = lds_read_tr8(sp + p_rd[i] + kk * 8192, sp + p_rd[i] + kk * 8192 + 2048);
                    else pf[i] = *(const bf16x8_t*)(sp + p_rd[i] + km_slot);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (Q_CMAJ) qf[j] = lds_read_tr8(sq + q_rd[j] + kk * 8192, sq + q_rd[j] + kk * 8192 + 2048);
                    else qf[j] = *(const bf16x8_t*)(sq + q_rd[j] + km_slot);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[i], qf[j], acc[i][j], 0, 0, 0);
            }
        };

        if (KT > 0) {
            issue(0, ldsP0, ldsQ0);
            wait_vm0();
            __syncthreads();
            for (int kt = 0; kt < KT; kt += 2) {
                if (kt + 1 < KT) issue(kt + 1, ldsP1, ldsQ1);
                compute(ldsP0, ldsQ0);
                wait_vm0();
                __syncthreads();
                if (kt + 1 < KT) {
                    if (kt + 2 < KT) issue(kt + 2, ldsP0, ldsQ0);
                    compute(ldsP1, ldsQ1);
                    wait_vm0();
                    __syncthreads();
                }
            }
        }

        // ---- epilogue: a lane owns one column of each sub-tile and 16 rows per 32x32 block ----
        const int col0 = j0 + wn * 32 + fr_row;
        const int col1 = j1 + wn * 32 + fr_row;
        const int lim0 = (EPI == GG_EPI_SWIGLU) ? half_cols : J;
        const bool ok0 = col0 < lim0;
        const bool ok1 = (EPI == GG_EPI_SWIGLU) ? ok0 : col1 < J;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int r = i0 + wm * 128 + i * 32 + (x >> 2) * 8 + fr_khalf * 4 + (x & 3);
                if (r >= i_end) continue;
                const float v0 = acc[i][0][x], v1 = acc[i][1][x];
                if (EPI == GG_EPI_SWIGLU) {
                    if (ok0) {
                        bf16_t* C = (bf16_t*)a.out;
                        if (C) {
                            C[(int64_t)r * N + col0] = (bf16_t)v0;
                            C[(int64_t)r * N + col1] = (bf16_t)v1;
                        }
                        a.out_act[(int64_t)r * half_cols + col0] = (bf16_t)(v0 * sigmoid_f(v0) * v1);
                    }
                } else if (EPI == GG_EPI_SWIGLU_BWD) {
                    // dZ[r, c] = dA * up * s (1 + g (1 - s)),  dZ[r, K + c] = dA * g * s,  s = sigmoid(g)
                    bf16_t* dZ = (bf16_t*)a.out;
                    const int64_t zr = (int64_t)r * 2 * K;
                    if (ok0) {
                        const float g = (float)a.Zsaved[zr + col0], up = (float)a.Zsaved[zr + K + col0];
                        const float s = sigmoid_f(g);
                        dZ[zr + col0] = (bf16_t)(v0 * up * s * (1.0f + g * (1.0f - s)));
                        dZ[zr + K + col0] = (bf16_t)(v0 * g * s);
                    }
                    if (ok1) {
                        const float g = (float)a.Zsaved[zr + col1], up = (float)a.Zsaved[zr + K + col1];
                        const float s = sigmoid_f(g);
                        dZ[zr + col1] = (bf16_t)(v1 * up * s * (1.0f + g * (1.0f - s)));
                        dZ[zr + K + col1] = (bf16_t)(v1 * g * s);
                    }
                } else {
                    const int64_t base = (MODE == GG_WGRAD) ? ((int64_t)e * N + r) * K : (int64_t)r * J;
                    if (OUT_F32) {
                        float* o = (float*)a.out;
                        if (ok0) o[base + col0] = a.accumulate ? o[base + col0] + v0 : v0;
                        if (ok1) o[base + col1] = a.accumulate ? o[base + col1] + v1 : v1;
                    } else {
                        bf16_t* o = (bf16_t*)a.out;
                        if (ok0) o[base + col0] = (bf16_t)(a.accumulate ? (float)o[base + col0] + v0 : v0);
                        if (ok1) o[base + col1] = (bf16_t)(a.accumulate ? (float)o[base + col1] + v1 : v1);
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
static moe_status gg_check_common(moe_ctx* ctx, const char* who, const void* p, const void* q, const int32_t* offsets,
                                  int E, int N, int K, int64_t Rcap, moe_dtype dt) {
    if (!p || !q || !offsets) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: NULL pointer", who);
    if (E < 1 || E > GG_MAX_E || N < 1 || K < 1 || Rcap < 1 || Rcap > 0x7fffffffLL)
        MOE_FAIL(ctx, MOE_ERR_ARG, "%s: need 1<=E<=%d, N,K>=1, 1<=Rcap<2^31", who, GG_MAX_E);
    if (N % 8 || K % 8) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: N and K must be multiples of 8 (16-byte rows)", who);
    if (dt == MOE_F32) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: fp32 operands are not supported", who);
    if (dt == MOE_FP8_E4M3) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: fp8 path not built yet", who);
    if (dt != MOE_BF16) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: bad dtype", who);
    return MOE_OK;
}

static gg_args gg_make(moe_ctx* ctx, const void* P, const void* Q, const int32_t* offsets, int E, int N, int K,
                       int64_t Rcap, void* out) {
    gg_args a;
    memset(&a, 0, sizeof(a));
    a.P = (const bf16_t*)P;
    a.Q = (const bf16_t*)Q;
    a.offsets = offsets;
    a.E = E;
    a.N = N;
    a.K = K;
    a.Rcap = Rcap;
    a.out = out;
    a.zeros = (const char*)ctx->ws + MOE_WS_ZEROS;
    a.dev_err = ctx->dev_err;
    return a;
}

extern "C" moe_status moe_grouped_gemm_fwd(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                           const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                           moe_dtype dt, moe_epilogue epi,
                                           const float* a_scale, const float* b_scale,
                                           void* C, void* C_act) {
    if (!ctx) return MOE_ERR_ARG;
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_fwd", A, B, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    (void)a_scale;
    (void)b_scale;
    if (epi == MOE_EPI_SWIGLU) {
        if (!C_act) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: SWIGLU needs C_act");
        if (N % 16) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: SWIGLU needs N %% 16 == 0");
    } else if (epi == MOE_EPI_NONE) {
        if (!C) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: C is NULL");
    } else {
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: bad epilogue");
    }
    if (K % GG_BK) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd: K=%d must be a multiple of %d", K, GG_BK);
    gg_args a = gg_make(ctx, A, B, offsets, E, N, K, Rcap, C);
    a.out_act = (bf16_t*)C_act;
    hipStream_t s = (hipStream_t)stream;
    const int grid = ctx->num_cu > 0 ? ctx->num_cu : 256;
    if (epi == MOE_EPI_SWIGLU)
        hipLaunchKernelGGL((gg_kernel<GG_FWD, GG_EPI_SWIGLU, false>), dim3(grid), dim3(GG_THREADS), 0, s, a);
    else
        hipLaunchKernelGGL((gg_kernel<GG_FWD, GG_EPI_STORE, false>), dim3(grid), dim3(GG_THREADS), 0, s, a);
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<fwd>");
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_dgrad(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                             const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                             moe_dtype dt, const void* Z_saved,
                                             const float* dc_scale, const float* b_scale, void* dA) {
    if (!ctx) return MOE_ERR_ARG;
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_dgrad", dC, B, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    (void)dc_scale;
    (void)b_scale;
    if (!dA) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad: dA is NULL");
    if (N % GG_BK) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad: N=%d must be a multiple of %d", N, GG_BK);
    gg_args a = gg_make(ctx, dC, B, offsets, E, N, K, Rcap, dA);
    a.Zsaved = (const bf16_t*)Z_saved;
    hipStream_t s = (hipStream_t)stream;
    const int grid = ctx->num_cu > 0 ? ctx->num_cu : 256;
    if (Z_saved)
        hipLaunchKernelGGL((gg_kernel<GG_DGRAD, GG_EPI_SWIGLU_BWD, false>), dim3(grid), dim3(GG_THREADS), 0, s, a);
    else
        hipLaunchKernelGGL((gg_kernel<GG_DGRAD, GG_EPI_STORE, false>), dim3(grid), dim3(GG_THREADS), 0, s, a);
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<dgrad>");
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_wgrad(moe_ctx* ctx, void* stream, const void* A, const void* dC,
                                             const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                             moe_dtype dt, const float* a_scale, const float* dc_scale,
                                             int accumulate, moe_dtype out_dt, void* dB) {
    if (!ctx) return MOE_ERR_ARG;
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_wgrad", dC, A, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    (void)a_scale;
    (void)dc_scale;
    if (!dB) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: dB is NULL");
    if (out_dt != MOE_BF16 && out_dt != MOE_F32) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: out_dt must be bf16 or f32");
    gg_args a = gg_make(ctx, dC, A, offsets, E, N, K, Rcap, dB);
    a.accumulate = accumulate ? 1 : 0;
    hipStream_t s = (hipStream_t)stream;
    const int grid = ctx->num_cu > 0 ? ctx->num_cu : 256;
    if (out_dt == MOE_F32)
        hipLaunchKernelGGL((gg_kernel<GG_WGRAD, GG_EPI_STORE, true>), dim3(grid), dim3(GG_THREADS), 0, s, a);
    else
        hipLaunchKernelGGL((gg_kernel<GG_WGRAD, GG_EPI_STORE, false>), dim3(grid), dim3(GG_THREADS), 0, s, a);
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<wgrad>");
    return MOE_OK;
}
