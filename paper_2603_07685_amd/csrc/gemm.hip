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
#ifndef GG_PINGPONG
#define GG_PINGPONG 1  // 1: ping-pong schedule; 0: plain multi-stage pipeline
#endif
#ifndef GG_SPREAD
#define GG_SPREAD 1  // 1: DMA instructions are interleaved with the MFMAs of the compute phase
#endif
#ifndef GG_PFD
#define GG_PFD 0   // L2 prefetch distance in stages (0 = off)
#endif
#ifndef GG_BK
#define GG_BK 32   // contraction elements per pipeline stage (32 or 64)
#endif
#ifndef GG_NS
#define GG_NS 4    // LDS pipeline stages (2..4); GG_NS * 2 * GG_STAGE_BYTES must fit in 160 KB
#endif
#define GG_THREADS 512
#define GG_MAX_E 1024
#define GG_STAGE_BYTES (GG_BM * GG_BK * 2)  // one operand tile per stage
#define GG_ROWB (GG_BK * 2)                 // bytes of a k-major tile row
#define GG_KM_SLOTS (GG_ROWB / 16)          // 16-byte slots per k-major row
#define GG_KM_ROWS (1024 / GG_ROWB)         // k-major rows per 1 KB DMA chunk
#define GG_CH (GG_BM / GG_KM_ROWS / 8)      // DMA chunks per wave per operand per stage
#define GG_KK (GG_BK / 16)                  // 16-wide MFMA sub-steps per stage
#ifndef GG_BAND
#define GG_BAND 4                           // row-tiles per band of the tile order
#endif
// k-major tile swizzle: 16-byte slot ^= KM_SWZ(row).  256 / GG_ROWB rows share one 256-byte
// bank line; XOR-ing the slot with the row bits above that makes 16 consecutive rows hit 16
// different (position in line, slot) pairs: a conflict-free ds_read_b128 for 16 lanes at a time
// (measured: SQ_LDS_BANK_CONFLICT = 0).
#define GG_KM_SHIFT (GG_BK == 64 ? 1 : 2)
#define KM_SWZ(row) (((row) >> GG_KM_SHIFT) & (GG_KM_SLOTS - 1))

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
// Workgroup barrier without the memory fence __syncthreads() carries: the fence would drain
// every DMA load in flight (vmcnt(0)) and serialise the pipeline.  The wave has already waited
// for its own loads of the stage being published (wait_stage); LDS reads after the barrier are
// ordered by the hardware.  The empty asm statements keep the compiler from moving memory
// operations across the barrier.
__device__ __forceinline__ void stage_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);  // nothing (MFMAs included) is scheduled across
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }       // lgkmcnt(0)
__device__ __forceinline__ void wait_vm0_lgkm0() { __builtin_amdgcn_s_waitcnt(0x0070); }   // vmcnt(0) lgkmcnt(0)

// wait until at most `newer` * GG_CH * 2 of this wave's DMA loads are still in flight
__device__ __forceinline__ void wait_stage(int newer) {
    if (newer <= 0) __builtin_amdgcn_s_waitcnt(0x0F70);
    else if (newer == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * GG_CH));
    else __builtin_amdgcn_s_waitcnt(0x0F70 | (4 * GG_CH));
}

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

// 4 consecutive bf16 <-> 4 floats, one 8-byte access
__device__ __forceinline__ void st4_bf16(bf16_t* p, const float* v) {
    u32x2_t w = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
    *(u32x2_t*)p = w;
}
__device__ __forceinline__ void ld4_bf16(const bf16_t* p, float* v) {
    const u32x2_t w = *(const u32x2_t*)p;
    v[0] = bf16_lo(w.x);
    v[1] = bf16_hi(w.x);
    v[2] = bf16_lo(w.y);
    v[3] = bf16_hi(w.y);
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
static_assert(!(GG_PINGPONG && GG_SPREAD) || (GG_NS >= 3 && GG_BK == 32), "interleaved DMA needs a third stage to land in");
static_assert(GG_NS >= 2 && GG_NS <= 4 && (GG_BK == 32 || GG_BK == 64), "unsupported pipeline shape");
static_assert(2 * (GG_NS - 2) * GG_CH < 16, "wait_stage immediate must fit the 4-bit vmcnt field");
static_assert(2 * GG_NS * GG_STAGE_BYTES <= 144 * 1024, "pipeline stages exceed the LDS budget");

template <int MODE, int EPI, bool OUT_F32>
__global__ __launch_bounds__(GG_THREADS, 1) void gg_kernel(const gg_args a) {
    // one LDS object per stage and operand: distinct objects let the compiler see that the
    // DMA writes of a later stage do not alias the operand reads of the current one
    __shared__ __attribute__((aligned(1024))) char ldsP0[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsP1[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsP2[GG_NS > 2 ? GG_STAGE_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char ldsP3[GG_NS > 3 ? GG_STAGE_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char ldsQ0[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsQ1[GG_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsQ2[GG_NS > 2 ? GG_STAGE_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char ldsQ3[GG_NS > 3 ? GG_STAGE_BYTES : 16];
#if GG_PFD > 0
    __shared__ __attribute__((aligned(256))) char pf_dummy[8 * 256];
#endif
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
    // k-major tile: a 1 KB DMA chunk = 8 rows x 128 B; lane -> (row l/8, slot l%8), slot ^= KM_SWZ(row)
    const int km_row = lane / GG_KM_SLOTS;
    // c-major tile: a 1 KB chunk = 2 rows x 512 B; lane -> (row l/32, slot l%32), slot ^= 4*(row%4)
    const int cm_row = lane >> 5;
    // ---- per-lane constants: fragment side ----
    const int fr_row = lane & 31;
    const int fr_khalf = lane >> 5;
    const int fr_swz = KM_SWZ(lane & 31);
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
        else p_rd[i] = (wm * 128 + i * 32 + fr_row) * GG_ROWB;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (Q_CMAJ) q_rd[j] = tr_rowoff + ((((j * 128 + wn * 32) >> 3) ^ tr_xor) + tr_low) * 16 + tr_byte;
        else q_rd[j] = (j * 128 + wn * 32 + fr_row) * GG_ROWB;
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
        const char* pg[GG_CH];
        const char* qg[GG_CH];
        int64_t p_step, q_step;  // byte advance per contraction step
        if (P_CMAJ) {
            // P = dC [rows, N]: contraction row c, columns i0..i0+255
            p_step = (int64_t)GG_BK * N * 2;
#pragma unroll
            for (int i = 0; i < GG_CH; ++i) {
                const int row = (wave * GG_CH + i) * 2 + cm_row;
                const int slot = (lane & 31) ^ (4 * (row & 3));
                int col = i0 + slot * 8;
                col = col <= N - 8 ? col : N - 8;
                pg[i] = (const char*)a.P + ((int64_t)(c_lo + row) * N + col) * 2;
            }
        } else {
            const int ldp = (MODE == GG_FWD) ? K : N;
            p_step = GG_BK * 2;
#pragma unroll
            for (int i = 0; i < GG_CH; ++i) {
                const int p = (wave * GG_CH + i) * GG_KM_ROWS + km_row;  // tile row 0..255
                int64_t r = (int64_t)i0 + p;
                r = r < a.Rcap ? r : a.Rcap - 1;
                const int km_gslot = (lane & (GG_KM_SLOTS - 1)) ^ KM_SWZ(p);
                pg[i] = (const char*)a.P + (r * ldp + km_gslot * 8) * 2;
            }
        }
        if (Q_CMAJ) {
            // dgrad: Q = W_e [N,K]: contraction row n, columns (k) j0.. ; wgrad: Q = A [rows,K]
            q_step = (int64_t)GG_BK * K * 2;
            const char* qbase = (MODE == GG_DGRAD) ? (const char*)a.Q + (int64_t)e * N * K * 2 : (const char*)a.Q;
#pragma unroll
            for (int i = 0; i < GG_CH; ++i) {
                const int row = (wave * GG_CH + i) * 2 + cm_row;
                const int slot = (lane & 31) ^ (4 * (row & 3));
                int col = (slot < 16 ? j0 : j1 - 128) + slot * 8;
                col = col <= K - 8 ? col : K - 8;
                qg[i] = qbase + ((int64_t)(c_lo + row) * K + col) * 2;
            }
        } else {
            q_step = GG_BK * 2;
#pragma unroll
            for (int i = 0; i < GG_CH; ++i) {
                const int p = (wave * GG_CH + i) * GG_KM_ROWS + km_row;  // tile row 0..255
                int n = (p < 128 ? j0 : j1 - 128) + p;
                n = n < N ? n : N - 1;
                const int km_gslot = (lane & (GG_KM_SLOTS - 1)) ^ KM_SWZ(p);
                qg[i] = (const char*)a.Q + (((int64_t)e * N + n) * K + km_gslot * 8) * 2;
            }
        }

#if GG_PFD > 0
        const char* pf_ptr;
        {
            const int prow = wave * 32 + (lane & 31);  // tile row 0..255 of P (lanes 0-31) or Q (lanes 32-63)
            if (lane < 32) {
                int64_t r = (int64_t)i0 + prow;
                r = r < a.Rcap ? r : a.Rcap - 1;
                pf_ptr = (const char*)a.P + r * K * 2;
            } else {
                int n = (prow < 128 ? j0 : j1 - 128) + prow;
                n = n < N ? n : N - 1;
                pf_ptr = (const char*)a.Q + ((int64_t)e * N + n) * K * 2;
            }
        }
#endif
#ifdef GG_KROT
        const int krot = KT > 0 ? (int)(((unsigned)q * GG_KROT) % (unsigned)KT) : 0;
#endif
        auto issue = [&](int kt, char* sp, char* sq) {
#ifdef GG_DBG_NODMA
            if (kt > 0) return;
#endif
#ifdef GG_KROT
            // contraction steps taken in a rotated order that differs between workgroups, so the
            // workgroups of an XCD do not all ask the same L2 channels for the same k at once
            kt = (kt + krot) % KT;
#endif
#pragma unroll
            for (int i = 0; i < GG_CH; ++i) {
                const char* ps = pg[i] + kt * p_step;
                const char* qs = qg[i] + kt * q_step;
                if (MODE == GG_WGRAD) {  // contraction tail of the expert: feed zeros
                    const int row = c_lo + kt * GG_BK + (wave * GG_CH + i) * 2 + cm_row;
                    ps = row < c_hi ? ps : a.zeros;
                    qs = row < c_hi ? qs : a.zeros;
                }
                dma16(ps, sp + (wave * GG_CH + i) * 1024);
                dma16(qs, sq + (wave * GG_CH + i) * 1024);
            }
#if GG_PFD > 0
            // L2 prefetch: touch one dword of every 128-byte line of the stage GG_PFD steps ahead
            // (into a dummy LDS word), so that the later DMA finds the line already filled in L2
            if (MODE == GG_FWD && kt + GG_PFD < KT && ((kt + GG_PFD) * GG_ROWB) % 128 == 0)
                __builtin_amdgcn_global_load_lds((gbl_void_t*)(pf_ptr + (int64_t)(kt + GG_PFD) * GG_ROWB),
                                                 (lds_void_t*)(pf_dummy + wave * 256), 4, 0, 0);
#endif
        };

        // one of the 2 * GG_CH DMA instructions of a stage (idx: operand = idx & 1, chunk = idx >> 1)
        auto issue_one = [&](int kt, char* sp, char* sq, int idx) {
            const int i = idx >> 1;
            const char* src = (idx & 1) ? qg[i] + kt * q_step : pg[i] + kt * p_step;
            if (MODE == GG_WGRAD) {
                const int row = c_lo + kt * GG_BK + (wave * GG_CH + i) * 2 + cm_row;
                src = row < c_hi ? src : a.zeros;
            }
            dma16(src, ((idx & 1) ? sq : sp) + (wave * GG_CH + i) * 1024);
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
            for (int kk = 0; kk < GG_KK; ++kk) {
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
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[j], pf[i], acc[i][j], 0, 0, 0);
            }
        };

#if GG_PINGPONG
        // Ping-pong schedule.  The two waves that share a SIMD (wave w and w+4) run one phase apart:
        // while one issues the 16 MFMAs of a phase with all operands already in registers, the other
        // fetches its next operands from LDS (and issues the DMA of a later stage); they swap at a
        // workgroup barrier.  The matrix pipe always has a wave with a full queue of independent MFMAs.
        //   per phase h:   A_h: LDS -> registers      barrier      B_h: 16 MFMAs      barrier
        //   group 1 (waves 4-7) takes one extra barrier up front, group 0 one at the end.
        // A phase covers 32 contraction elements: a whole stage when BK = 32 (GG_NS stages, up to
        // GG_NS-1 stages of DMA in flight to cover the L2-miss latency), half a stage when BK = 64.
        // The DMA that refills a buffer is issued at the start of the A phase that follows the last A
        // phase reading it in the other group (one barrier later), and each wave waits for its own
        // loads of the next stage at the end of the A phase before that stage's first read.
        {
            char* const SP[4] = {ldsP0, ldsP1, ldsP2, ldsP3};
            char* const SQ[4] = {ldsQ0, ldsQ1, ldsQ2, ldsQ3};
            bf16x8_t pf[2][4], qf[2][2];
            auto fetch = [&](const char* sp, const char* sq, int half) {
#ifdef GG_DBG_NOMMA
                return;
#endif
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    const int kk = half * 2 + k2;
                    const int km_slot = ((kk * 2 + fr_khalf) ^ fr_swz) * 16;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (P_CMAJ) pf[k2][i] = lds_read_tr8(sp + p_rd[i] + kk * 8192, sp + p_rd[i] + kk * 8192 + 2048);
                        else pf[k2][i] = *(const bf16x8_t*)(sp + p_rd[i] + km_slot);
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (Q_CMAJ) qf[k2][j] = lds_read_tr8(sq + q_rd[j] + kk * 8192, sq + q_rd[j] + kk * 8192 + 2048);
                        else qf[k2][j] = *(const bf16x8_t*)(sq + q_rd[j] + km_slot);
                    }
                }
            };
            // 16 MFMAs; with GG_SPREAD the DMA instructions idx0 .. idx0+3 of stage `kt_dma` are slipped
            // in after every fourth MFMA so the memory requests are spread over the phase
            auto mma = [&](bool do_dma, int kt_dma, char* dp, char* dq, int idx0) {
#ifdef GG_DBG_NOMMA
                return;
#endif
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[k2][j], pf[k2][i], acc[i][j], 0, 0, 0);
#if GG_SPREAD
                        if ((i & 1) == 1) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (do_dma) issue_one(kt_dma, dp, dq, idx0 + k2 * 2 + (i >> 1));
                            __builtin_amdgcn_sched_barrier(0);
                        }
#endif
                    }
            };
            if (KT > 0) {
#pragma unroll
                for (int s = 0; s < GG_NS - 1; ++s)
                    if (s < KT) issue(s, SP[s], SQ[s]);
                wait_stage(min(GG_NS - 2, KT - 1));
                stage_barrier();
                if (wm == 1) stage_barrier();  // group 1 starts one phase later
                for (int kt = 0; kt < KT; kt += GG_NS) {
#pragma unroll
                    for (int s = 0; s < GG_NS; ++s) {
                        const int j = kt + s;
                        if (j < KT) {  // uniform
                            const bool more = j + GG_NS - 1 < KT;
                            char* const dp = SP[(s + GG_NS - 1) % GG_NS];
                            char* const dq = SQ[(s + GG_NS - 1) % GG_NS];
#if !GG_SPREAD
                            if (more) issue(j + GG_NS - 1, dp, dq);
#endif
#if GG_BK == 64
                            fetch(SP[s], SQ[s], 0);
                            wait_lgkm0();
                            stage_barrier();
                            mma(more, j + GG_NS - 1, dp, dq, 0);
                            stage_barrier();
                            fetch(SP[s], SQ[s], 1);
#else
                            fetch(SP[s], SQ[s], 0);
#endif
                            wait_lgkm0();
                            if (j + 1 < KT) wait_stage(min(GG_NS - 2 - (GG_SPREAD ? 1 : 0), KT - 2 - j));
                            stage_barrier();
                            mma(more, j + GG_NS - 1, dp, dq, GG_BK == 64 ? 4 : 0);
                            stage_barrier();
                        }
                    }
                }
                if (wm == 0) stage_barrier();  // re-align the two groups
            }
        }
#else
        {
            char* const SP[4] = {ldsP0, ldsP1, ldsP2, ldsP3};
            char* const SQ[4] = {ldsQ0, ldsQ1, ldsQ2, ldsQ3};
            // prologue: stages 0 .. NS-2 in flight
#pragma unroll
            for (int s = 0; s < GG_NS - 1; ++s)
                if (s < KT) issue(s, SP[s], SQ[s]);
            for (int kt = 0; kt < KT; kt += GG_NS) {
#pragma unroll
                for (int s = 0; s < GG_NS; ++s) {
                    const int j = kt + s;
                    if (j < KT) {  // uniform
                        // stage j must have landed; up to NS-2 younger stages may stay in flight
                        wait_stage(min(GG_NS - 2, KT - 1 - j));
                        stage_barrier();  // everyone's stage j is in LDS, everyone is done with stage j-1
                        if (j + GG_NS - 1 < KT)
                            issue(j + GG_NS - 1, SP[(s + GG_NS - 1) % GG_NS], SQ[(s + GG_NS - 1) % GG_NS]);
                        compute(SP[s], SQ[s]);
                    }
                }
            }
        }

#endif

        // ---- epilogue ----
        // The MFMAs were issued as (Q fragment, P fragment), so a lane's 16 accumulators of a 32x32
        // block are one output row (P index = lane % 32) and four groups of 4 consecutive output
        // columns (Q index = 8 g + 4 (lane / 32) + 0..3): every store is 8 contiguous bytes of bf16
        // (16 of fp32) and the SwiGLU partners sit in the same lane.
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = i0 + wm * 128 + i * 32 + fr_row;
            if (r >= i_end) continue;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c0 = j0 + wn * 32 + 8 * g + 4 * fr_khalf;
                const int c1 = j1 + wn * 32 + 8 * g + 4 * fr_khalf;
                float v0[4], v1[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    v0[x] = acc[i][0][4 * g + x];
                    v1[x] = acc[i][1][4 * g + x];
                }
                if (EPI == GG_EPI_SWIGLU) {
                    if (c0 < half_cols) {
                        bf16_t* C = (bf16_t*)a.out;
                        if (C) {
                            st4_bf16(C + (int64_t)r * N + c0, v0);
                            st4_bf16(C + (int64_t)r * N + c1, v1);
                        }
                        float act[4];
#pragma unroll
                        for (int x = 0; x < 4; ++x) act[x] = v0[x] * sigmoid_f(v0[x]) * v1[x];
                        st4_bf16(a.out_act + (int64_t)r * half_cols + c0, act);
                    }
                } else if (EPI == GG_EPI_SWIGLU_BWD) {
                    // dZ[r, c] = dA * up * s (1 + g (1 - s)),  dZ[r, K + c] = dA * g * s,  s = sigmoid(g)
                    bf16_t* dZ = (bf16_t*)a.out;
                    const int64_t zr = (int64_t)r * 2 * K;
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) {
                        const int c = h2 ? c1 : c0;
                        const float* v = h2 ? v1 : v0;
                        if (c < K) {
                            float gt[4], up[4], dg[4], du[4];
                            ld4_bf16(a.Zsaved + zr + c, gt);
                            ld4_bf16(a.Zsaved + zr + K + c, up);
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                const float sg = sigmoid_f(gt[x]);
                                dg[x] = v[x] * up[x] * sg * (1.0f + gt[x] * (1.0f - sg));
                                du[x] = v[x] * gt[x] * sg;
                            }
                            st4_bf16(dZ + zr + c, dg);
                            st4_bf16(dZ + zr + K + c, du);
                        }
                    }
                } else {
                    const int64_t base = (MODE == GG_WGRAD) ? ((int64_t)e * N + r) * K : (int64_t)r * J;
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) {
                        const int c = h2 ? c1 : c0;
                        float* v = h2 ? v1 : v0;
                        if (c < J) {
                            if (OUT_F32) {
                                f32x4_t* o = (f32x4_t*)((float*)a.out + base + c);
                                f32x4_t w = {v[0], v[1], v[2], v[3]};
                                if (a.accumulate) w += *o;
                                *o = w;
                            } else {
                                bf16_t* o = (bf16_t*)a.out + base + c;
                                if (a.accumulate) {
                                    float old[4];
                                    ld4_bf16(o, old);
#pragma unroll
                                    for (int x = 0; x < 4; ++x) v[x] += old[x];
                                }
                                st4_bf16(o, v);
                            }
                        }
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
