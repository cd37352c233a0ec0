// Grouped GEMM for the expert MLP (Sec. 2.1.4, 4.3.2), device-initiated (Sec. 4.3.7): one
// persistent launch per call, every expert's extent is read from `offsets` on the device;
// forward, data-gradient and weight-gradient (Sec. 4.2.3 "W/D split") in bf16 and MXFP8 (Sec. 5.3.3),
// forward and data-gradient also in blockwise fp8 (Sec. 5.3.2), are instantiations of one kernel.
//
// The kernel computes OUT[i,j] = sum_c P[i,c] * Q[j,c] on a 256x256 output tile per workgroup.  Two bodies share
// the schedule, the tile set-up, the LDS layouts and the epilogue (template parameter NW):
//   bf16:        4 wavefronts as 2 x 2, one per SIMD with 512 registers; wave tile 128x128 = 8x8 blocks of the
//                16x16x32 MFMA; operands staged through registers (described at the stage loop)
//   fp8 / MXFP8: 8 wavefronts as 2 x 4; wave tile 128x64 = 4x2 blocks of the 32x32x64 MFMA; operands by DMA, the
//                "ping-pong" schedule below
//     forward : P = activations [rows,K]   Q = W_e [N,K]        OUT = C[rows,N]
//     dgrad   : P = dC [rows,N]            Q = W_e as [K,N]^T   OUT = dA[rows,K]
//     wgrad   : P = dC as [N,rows]^T       Q = A as [K,rows]^T  OUT = dW_e[N,K]
//
// Operand stream.  The contraction is walked in stages of 128 bytes per operand row (64 bf16 or
// 128 fp8 elements): every global request of the DMA is then a whole 128-byte cache line, which
// the L1/L2 path serves at about twice the rate of half-line requests (measured: 20 vs 10 TB/s on
// a GEMM-like sharing pattern).  Each stage's two 32 KB operand tiles go into one of two stage buffers: by direct
// global->LDS loads (eight-wave body; 16 B per lane, issued through inline asm and synchronised by the kernel's
// own waits, see dma16 below) or through registers (four-wave body), with the same chunk -> lane mapping.
//
// LDS layouts.  An operand whose contraction index is contiguous in memory ("k-major", tile
// [256 rows][128 B]) is read with ds_read_b128; one whose contraction index is the memory row
// ("c-major", tile [64 or 128 rows][256 columns]: the weight in dgrad, both operands in wgrad) is
// read with the transposing ds_read_b64_tr_b16 / _b8, so no transposed copy of weights or
// activations is ever made.  The 16-byte slots of every tile are XOR-swizzled with the row so the
// operand reads are free of bank conflicts; the swizzle is applied on the global side of the DMA
// (each lane chooses which 16 bytes it fetches; the LDS side of a DMA is always lane-linear).
//
// Schedule of the eight-wave body ("ping-pong").  A stage is consumed in two halves.  The two waves that share a SIMD
// (wave w and w+4) belong to two groups that run one phase apart: while one issues the MFMAs of a
// half-stage with all operands already in registers, the other fetches its next operands from
// LDS; they swap at fence-free workgroup barriers.  Each group has its own copy of the stage loop.
//   per stage s:  A(s,0) | B(s,0) | A(s,1) | B(s,1)    A: LDS -> registers,  B: MFMAs,  '|' = barrier
//   group 1 (waves 4-7) takes one extra barrier up front, group 0 one at the end; in time:
//     group 0:  A(s,0)*   B(s,0)   A(s,1)   B(s,1)   A(s+1,0)* ...
//     group 1:  B(s-1,1)* A(s,0)   B(s,0)   A(s,1)   B(s,1)*   ...      (* = issues its half of stage s+1; group 1: or at A(s,0))
// Buffer (s+1)%2 was last read in A(s-1,1); group 1 finishes that phase one barrier before group 0
// enters A(s,0), so group 0 refills it at the start of A(s,0) and group 1 either in the same slot, between
// the MFMAs of its B(s-1,1) (weight gradients), or one slot later at the start of its own A(s,0) (forward,
// data gradient: see the stage loop).  Each wave waits for its own loads of stage s+1 before the barrier that
// precedes group 0's A(s+1,0): group 0 at the end of B(s,1), group 1 at the end of A(s,1).
// The first stage of a tile is issued before the epilogue of the tile before it.
//
// MFMAs are issued as (Q fragment, P fragment): a lane's accumulators of a block are one output row and 4
// consecutive columns (16x16 blocks; four such groups in a 32x32 block), and the wave's column blocks come in two
// halves 128 columns apart, i.e. the gate and up columns of the same features when the SwiGLU epilogue is on.  The epilogue stages the fp32 accumulators through LDS and writes whole tile rows; the
// activation (forward) and its derivative (fc2 dgrad) are applied to the fp32 values there.
//
// fp8: operands are E4M3 codes; a half-stage is one v_mfma_scale_f32_32x32x64_f8f6f4 per block with unit
// hardware scales.  The fp32 block scales (1x128 per activation row, 128x128 per weight block) are
// applied in software: a lane's accumulators of one block all share the factor
// s = a_scale[row, kb] * b_scale[block], so the accumulator is kept in units of the current
// factor: at every 128-wide contraction block (= stage) it is multiplied by s_prev / s_new before the raw
// products are added, and by the last factor in the epilogue.  No second set of accumulators.
// The scales of a block reach LDS with the operands of its stage.
#include "common.h"

#define GG_BM 256
#define GG_BN 256
#ifndef GG_BAND
#define GG_BAND 4  // row-tiles per band of the tile order
#endif
#define GG_THREADS 512
#define GG_MAX_E 1024
#define GG_MAX_SPLIT 8          // most slices of partial tiles a weight-gradient call uses (workspace: that many fp32 copies of one expert's dW)
#define GG_MAX_SPLIT_EXPERTS 4  // an expert is split into at least two pieces
#define GG_ROWB 128                     // bytes of a k-major tile row per stage: one cache line
#define GG_STAGE_BYTES (GG_BM * GG_ROWB)  // one operand tile per stage: 32 KB
// k-major swizzle: two 128-byte rows share a 256-byte bank line; slot ^= bits 1..3 of the row makes
// 16 consecutive rows hit 16 different (position in line, slot) pairs (SQ_LDS_BANK_CONFLICT = 0)
#define KM_SWZ(row) (((row) >> 1) & 7)

enum { GG_FWD = 0, GG_DGRAD = 1, GG_WGRAD = 2 };
enum { GG_EPI_STORE = 0, GG_EPI_SWIGLU = 1, GG_EPI_SWIGLU_BWD = 2 };

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void gbl_void_t;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef int i32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) i32x2_t lds_i32x2_t;

static_assert(2 * 2 * GG_STAGE_BYTES <= 144 * 1024, "pipeline stages exceed the LDS budget");

// Global -> LDS DMA: each lane moves 16 (or 4) bytes; LDS destination = M0 + lane * size.
// Written as inline asm on purpose.  With the builtin, the compiler tracks every DMA as a pending LDS
// write and decides on its own, per LDS read, whether to wait for it (s_waitcnt vmcnt); around a
// software pipeline with conditional issue it cannot prove the buffers apart and puts vmcnt(0) in front
// of fragment reads, which drains the pipeline every stage.  The kernel waits explicitly for exactly the
// stage it is about to read (wait_vm0 + barrier), so the compiler needs to see only an opaque memory
// write.  (Waits the compiler adds for its own global loads stay correct: the memory counter completes
// in order, so extra older or younger entries only make such a wait longer.)
// The LDS destination is passed as a wave-uniform register part plus a constant part (buffer + chunk).
// The register part goes through an empty asm first: the sum is then formed at each use (one scalar add)
// instead of sixteen loop-invariant sums each holding a scalar register across the stage loop.
__device__ __forceinline__ uint32_t lds_addr(void* p) { return (uint32_t)(uintptr_t)(lds_void_t*)p; }
__device__ __forceinline__ uint32_t m0_value(uint32_t lds_wave, uint32_t lds_const) {
    asm volatile("" : "+s"(lds_wave));
    return lds_wave + lds_const;
}
// scalar base + 32-bit lane offset (readfirstlane: a no-op for a value the compiler already keeps in
// scalar registers, and the guarantee the "s" constraint needs where it does not)
__device__ __forceinline__ void dma16(const char* base, uint32_t off, uint32_t lds_wave, uint32_t lds_const) {
    const uint64_t b = (uint64_t)base;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    base = (const char*)(((uint64_t)hi << 32) | lo);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(m0_value(lds_wave, lds_const)), "v"(off), "s"(base) : "memory", "m0");
}
// per-lane 64-bit address
__device__ __forceinline__ void dma16(const char* src, uint32_t lds_wave, uint32_t lds_const) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(m0_value(lds_wave, lds_const)), "v"(src) : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void* src, uint32_t lds_wave, uint32_t lds_const) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :: "s"(m0_value(lds_wave, lds_const)), "v"(src) : "memory", "m0");
}

// Workgroup barrier without the memory fence __syncthreads() carries: the fence would drain every
// DMA load in flight (vmcnt(0)) and serialise the pipeline.  The wave has already waited for its own
// loads of the stage being published; LDS reads after the barrier are ordered by the hardware.
// The empty asm statements and sched_barriers keep the compiler from moving anything across.
__device__ __forceinline__ void stage_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }  // lgkmcnt(0)
// s_waitcnt vmcnt(0) only (gfx9 encoding, other counters at their maxima): this wave's DMA loads landed
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// vmcnt(1): everything but the wave's youngest vector-memory operation (the L2 warm-up load, see PF below)
__device__ __forceinline__ void wait_vm1() { __builtin_amdgcn_s_waitcnt(0x0F71); }

// (hardware reciprocal, 1 ulp: an IEEE division is ten instructions per element in an epilogue one wave runs alone)
__device__ __forceinline__ float sigmoid_f(float g) { return __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the address of 4 consecutive
// 16-bit elements (row i/4, columns 4*(i%4)..+3 of a 4x16 block) and receives column i of that block
// (rows 0..3).  Two of them give the 8 contraction values a lane feeds to the 32x32x16 MFMA.
__device__ __forceinline__ bf16x8_t lds_read_tr16x8(const char* p_lo, const char* p_hi) {
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p_lo);
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p_hi);
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
}
// ds_read_b64_tr_b8: lane i of a 16-lane group supplies the address of 8 consecutive bytes (row i/2,
// columns 8*(i%2)..+7 of an 8x16 block) and receives column i (rows 0..7).  Four reads, 8 rows apart,
// give the 32 contraction values a lane feeds to the 32x32x64 fp8 MFMA.
// `second` is the row distance between the lane's first and second group of 16 contraction values.
__device__ __forceinline__ i32x8_t lds_read_tr8x32(const char* p, int second = 16) {
    i32x2_t r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2_t*)p);
    i32x2_t r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2_t*)(p + 8 * 256));
    i32x2_t r2 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2_t*)(p + second * 256));
    i32x2_t r3 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2_t*)(p + (second + 8) * 256));
    i32x8_t v = {r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
    return v;
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
    const void* P;         // fwd: A, dgrad: dC, wgrad: dC   (bf16, or E4M3 codes)
    const void* Q;         // fwd/dgrad: W [E,N,K], wgrad: A
    const float* p_scale;  // fp8: [rows, C/128] for the row-indexed operand (C = contraction length)
    const float* q_scale;  // fp8: [E, N/128, K/128] for the weights
    const int32_t* offsets;
    int E, N, K;
    int64_t Rcap;
    void* out;             // fwd: C (may be NULL with SWIGLU), dgrad: dA or dZ, wgrad: dW
    bf16_t* out_act;       // fwd SWIGLU: activation output
    const bf16_t* Zsaved;  // dgrad SWIGLU_BWD: saved pre-activation [rows, 2K]
    const char* zeros;     // >= 16 zero bytes (feeds the wgrad contraction tail)
    int* dev_err;
    int accumulate;        // wgrad: out += result
    const float* row_prob; // eq. (2): routing weight of each row (fwd SWIGLU: scales the activation;
                           //   dgrad SWIGLU_BWD: scales dZ); NULL = 1
    // blockwise fp8 only: the epilogue also emits the 1x128 codes and scales of its bf16 output (fwd SWIGLU: of the
    // activation [rows, N/2]; dgrad SWIGLU_BWD: of dZ [rows, 2K]), the operand of the next GEMM (Sec. 5.4.2)
    uint8_t* out_q;
    float* out_q_scale;
    // MXFP8: the same tensors as 1x32 codes + E8M0 bytes [rows, cols/32] (out_q, out_q_e8) and, optionally, as the
    // 32x1 copy for the weight gradient (out_qc, scales [rows/128, cols, 4]: one dword = the four 32-row blocks)
    uint8_t* out_q_e8;
    uint8_t* out_qc;
    uint8_t* out_qc_e8;
    int* tile_counter;     // wgrad: zeroed device counter for the dynamic tile order under skewed loads (see the kernel)
    // wgrad, bf16: deterministic split of the contraction for experts far above the mean load (see the kernel)
    int split_cap;         // how many expert-sized slices of fp32 partial tiles `partials` can hold (0: never split)
    float* partials;       // [split_cap][tiles per expert][256 x 256] fp32
    int* split_info;       // [1 + 3 * GG_MAX_SPLIT_EXPERTS]: count, then (expert, pieces, first slice) for the reduce kernel
    float* dprob_part;     // eq. (2), dgrad SWIGLU_BWD: [Rcap, 2 ceil(K/256)] partial <dA, act(Z)> per row, two per column tile
    // Permutation fused into the operand fetch (Sec. 4.3.3; GATH variants): the gathered operand (P or Q) points to
    // the unpermuted tensor [g_T, row length], and row r of the operand is its row g_src_of[r] / g_k, or zeros where
    // g_src_of[r] < 0 (padding, rows behind offsets[E])
    const int32_t* g_src_of;
    uint32_t g_magic;      // ceil(2^31 / g_k): ((2 s + 1) * g_magic) >> 32 == s / g_k for every 0 <= s with s * g_k < 2^30
    int g_k;
    int g_T;
};
// offset of a gathered row that has no source: behind every record count a gathered operand can have (checked on the
// host), and far enough from 2^32 that a column offset added to it cannot wrap
#define GG_NO_ROW 0xF0000000u

// MODE: GG_FWD / GG_DGRAD / GG_WGRAD.  EPI: see enum.  OUT_F32: fp32 output (wgrad only).
// F8: 0 = bf16 operands; 1 = E4M3 codes with fp32 block scales applied in software
// (blockwise recipe, fwd and dgrad only); 2 = E4M3 codes with one E8M0 scale per 32 contraction elements, applied by the matrix
// instruction itself (MXFP8, Sec. 5.3.3).
// NW: waves per workgroup.  8 = two groups of four waves (wave tile 128 x 64) that alternate between fragment reads
// and MFMAs, operands by global -> LDS DMA; 4 = one wave per SIMD with 512 registers (wave tile 128 x 128 as 8 x 8
// blocks of the 16x16x32 MFMA), operands staged through registers one stage ahead, fragment reads pipelined inside
// the wave (bf16 only).
// GATH: 0 = both operands as they lie in memory; 1 / 2 = the rows of P / Q are fetched through the row map from the
// unpermuted tensor (four-wave body only; Q only in the weight gradient, whose two operands are both indexed by
// permuted rows).
template <int MODE, int EPI, bool OUT_F32, int F8, int NW, int GATH = 0>
__global__ __launch_bounds__(NW * 64, 1) __attribute__((amdgpu_waves_per_eu(1, NW == 4 ? 1 : 2))) void gg_kernel(const gg_args a) {
    constexpr bool FP8 = F8 != 0;  // one-byte operands
    constexpr bool MX = F8 == 2;   // hardware block scales
    static_assert(NW == 8 || (NW == 4 && !FP8), "four-wave workgroups are built for bf16 operands only");
    static_assert(GATH == 0 || (NW == 4 && (GATH == 1 || (GATH == 2 && MODE == GG_WGRAD))), "gathered operands: four-wave body; Q only in the weight gradient");
    constexpr int THREADS = NW * 64;
    constexpr int HW = NW / 2;     // waves per 128-row half of the tile
    constexpr int NJ = 16 / NW;    // 32-column blocks per wave: NJ / 2 in each 128-column half
    constexpr int CH = 32 / NW;    // 1 KB chunks per wave per operand per stage
    constexpr int RPW = 64 / NW;   // staged output rows per wave and epilogue pass
#ifndef GG_PF
#define GG_PF 0
#endif
    // L2 warm-up loads (GG_PF bit 0: bf16 variants, bit 1: one-byte variants), off by default: measured at the
    // DeepSeek-V3-style shape they gain 3-17 % per bf16 call on all-zero operands (clock not power-limited) and lose
    // 1.5-4.5 % on N(0, 0.02^2) operands, where the sustained clock is set by power and the extra requests only add
    // to it; the one-byte variants change by -5 .. +3 % per call, no net gain
    constexpr bool PF = NW == 8 && (FP8 ? (GG_PF & 2) != 0 : (GG_PF & 1) != 0);
    // fp8: the block scales of a stage travel with it, behind the P tile: 256 row scales (position
    // 4 * (row % 32) + row / 32 inside each 128-row half, so a lane finds its four rows in one 16-byte
    // read) and, from position 256 on, the two column-block scales (replicated)
    // (blockwise weight gradient: both operands carry one scale per tile row / column and stage, and the rescaling
    // needs the previous stage's too: 256 + 256 current, then 256 + 256 previous)
    constexpr bool BW_WGRAD = F8 == 1 && MODE == GG_WGRAD;
    constexpr int SC_BYTES = FP8 ? (BW_WGRAD ? 4096 : 2048) : 0;
    // One LDS array: [P0 | scales0 | Q0 | P1 | scales1 | Q1 | pad].  Buffer 1 (from P1 on) doubles as the
    // staging area of the epilogue: 64 tile rows x 260 floats.
    constexpr int BUF_BYTES = 2 * GG_STAGE_BYTES + SC_BYTES;
    constexpr int STG_PITCH = 260;                       // floats per staged row: 256 + 4 (bank rotation)
    constexpr int STG_BYTES = 64 * STG_PITCH * 4;
    constexpr int LDS_BYTES = BUF_BYTES + (BUF_BYTES > STG_BYTES ? BUF_BYTES : STG_BYTES) + 256;  // + a dummy word row
    __shared__ __attribute__((aligned(1024))) char lds_buf[LDS_BYTES];
    char* const ldsP0 = lds_buf;
    char* const ldsQ0 = lds_buf + GG_STAGE_BYTES + SC_BYTES;
    char* const ldsP1 = lds_buf + BUF_BYTES;
    char* const ldsQ1 = ldsP1 + GG_STAGE_BYTES + SC_BYTES;
    // MXFP8 quantising epilogues: column maxima of the four waves that share a 32-row block meet here
    constexpr bool MXQ = F8 == 2 && NW == 8 && EPI != GG_EPI_STORE;
    __shared__ __attribute__((aligned(16))) uint32_t qx[MXQ ? 8 * 64 * 4 : 4];
    __shared__ __attribute__((aligned(16))) float qe[MXQ ? 2 * 512 : 4];  // per tile half: the block scale 2^e of every column
    __shared__ int offs[GG_MAX_E + 1];
    __shared__ int tile_start[GG_MAX_E + 1];
    __shared__ int dyn_next;
    // weight gradient with a split contraction: sorted position -> first work item, and (pieces | first slice << 8)
    __shared__ int item_start[(MODE == GG_WGRAD && NW == 4) ? GG_MAX_E + 1 : 1];
    __shared__ int split_of[(MODE == GG_WGRAD && NW == 4) ? GG_MAX_E : 1];
    constexpr bool SPLITK = MODE == GG_WGRAD && NW == 4;

    constexpr bool P_CMAJ = (MODE == GG_WGRAD);
    constexpr bool Q_CMAJ = (MODE != GG_FWD);
    constexpr int ES = FP8 ? 1 : 2;            // operand element size
    constexpr int BKE = GG_ROWB / ES;           // contraction elements per stage: 64 bf16 / 128 fp8
    constexpr int CM_ROWS = 1024 / (256 * ES);  // c-major rows per 1 KB DMA chunk: 2 bf16 / 4 fp8
    constexpr int CM_SLOTS = 256 * ES / 16;     // 16-byte slots per c-major row: 32 bf16 / 16 fp8
    constexpr int EPS = 16 / ES;                // elements per 16-byte slot
    // Gathered operand (GATH).  Row-major (forward, data gradient): the rows of a tile are fixed, eight lane offsets
    // hold their places in the unpermuted tensor for the whole tile.  Contraction-major (weight gradient): every
    // stage brings 64 new rows, 16 per wave; a wave fetches the 16 map entries of a stage three stages ahead (one
    // 4-byte load per lane), turns them into byte offsets, and passes them through a few LDS words of its own to the
    // lanes that need them: chunk c of a lane (rows 2 c + lane / 32) finds the offsets of its eight chunks in two
    // 16-byte reads, a stage before the loads that use them (gfetch / gconv / gput / gread below).  Rows without a
    // source, rows behind the contraction range and stages behind the last get GG_NO_ROW, which the buffer
    // descriptor turns into zeros.
    constexpr bool G_ROW = GATH == 1 && !P_CMAJ;
    constexpr bool G_CM = GATH != 0 && MODE == GG_WGRAD;
    __shared__ __attribute__((aligned(16))) uint32_t gring[G_CM ? 3 * 4 * 16 : 4];  // [slot][wave][row parity][chunk]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps wave-derived values in SGPRs
    const int wm = wave / HW;  // 0..1 : 128-row half of the tile
    const int wn = wave % HW;  // strip of 16 NJ columns inside each 128-column half
    // tile column of the wave's jb-th 32-column block
    auto blk_col = [&](int jb) { return (jb / (NJ / 2)) * 128 + wn * (16 * NJ) + (jb % (NJ / 2)) * 32; };
    const int E = a.E, N = a.N, K = a.K;
    // gathered operand: bytes per row of the unpermuted tensor; this lane's row among the 64 of a stage when it
    // fetches map entries, and where it reads offsets back (contraction-major chunks hold rows 2 i + lane / 32)
    const uint32_t g_rowb = (uint32_t)(((GATH == 2 || MODE == GG_FWD) ? K : N) * ES);
    const int g_row16 = 16 * wave + (lane & 15);
    const uint32_t gl_rd = lds_addr(gring) + wave * 64 + (lane >> 5) * 32;
    const uint32_t gl_wr = lds_addr(gring) + wave * 64 + ((lane & 1) * 8 + ((lane & 15) >> 1)) * 4;
    // map entry -> source row -> its byte offset, in two steps (each holds one quarter-rate multiplication; inside the
    // stage loop they sit behind different MFMAs).  No branches: every lane computes, the select comes last (left alone,
    // the compiler predicates the multiplications and puts a branch between the MFMAs).
    auto g_tok_of = [&](int s) -> uint32_t {
        uint32_t tok = __umulhi(2u * (uint32_t)s + 1u, a.g_magic);   // s / g_k
        asm volatile("" : "+v"(tok));
        return tok;
    };
    auto g_off_at = [&](int s, uint32_t tok, bool live) -> uint32_t {
        uint32_t off = tok * g_rowb;
        asm volatile("" : "+v"(off));
        const bool ok = (s >= 0) & live;
        return ok ? off : GG_NO_ROW;
    };
    auto g_off_of = [&](int s, bool live) -> uint32_t { return g_off_at(s, g_tok_of(s), live); };

    // Output geometry.  J = extent of j (output columns).
    //   fwd:   J = N (with SWIGLU the column tiles pair gate/up: N/2 features in tiles of 128)
    //   dgrad: J = K;  wgrad: i runs over N, J = K.
    const int J = (MODE == GG_FWD) ? N : K;
    const int half_cols = (EPI == GG_EPI_SWIGLU) ? (N >> 1) : 0;
    const int tiles_j = (EPI == GG_EPI_SWIGLU) ? (half_cols + 127) / 128 : (J + GG_BN - 1) / GG_BN;
    const int tiles_i_w = (N + GG_BM - 1) / GG_BM;  // wgrad only

    // ---- tile schedule, computed by every workgroup from the device-resident offsets ----
    for (int e = tid; e <= E; e += THREADS) offs[e] = a.offsets[e];
    __syncthreads();
    // wgrad: every expert has the same number of output tiles but a tile costs its expert's row count, so the
    // experts are walked in descending order of rows (rank sort, ties by index; tile_start[i] = i-th largest
    // expert) and the tile list is dealt to the XCDs in a snake (see tile_of): equal work per workgroup
    // whatever the load skew.  Only the order of the tiles changes, never what a tile computes.
    if (MODE == GG_WGRAD) {
        for (int e = tid; e < E; e += THREADS) {
            const int re = offs[e + 1] - offs[e];
            int rank = 0;
            for (int o = 0; o < E; ++o) {
                const int ro = offs[o + 1] - offs[o];
                rank += (ro > re) || (ro == re && o < e);
            }
            tile_start[rank] = e;
        }
    }
    if (SPLITK) __syncthreads();  // (thread 0 walks the sorted experts below)
    if (tid == 0) {
        int run = 0;
        bool bad = offs[0] < 0 || offs[E] > a.Rcap;
        for (int e = 0; e < E; ++e) {
            if (MODE != GG_WGRAD) tile_start[e] = run;
            const int rows = offs[e + 1] - offs[e];
            bad |= rows < 0;
            // MXFP8 wgrad: a 32-row scale block (and the 128-row stage) must not straddle two experts
            // (the same for the 128-row scale blocks of the blockwise recipe)
            if (FP8 && MODE == GG_WGRAD) bad |= (rows & 127) != 0 || (offs[e] & 127) != 0;
            if (MXQ && a.out_qc) bad |= (rows & 127) != 0 || (offs[e] & 127) != 0;  // 32-row blocks inside one expert
            if (MODE == GG_WGRAD) run += tiles_i_w * tiles_j;
            else run += rows > 0 ? ((rows + GG_BM - 1) / GG_BM) * tiles_j : 0;
        }
        tile_start[E] = run;
        if (SPLITK) {
            // Deterministic split of the contraction (Sec. 4.3.1 names the imbalance it answers).  Under a skewed load
            // one tile of the largest expert can be most of a workgroup's share; such experts are cut into pieces of
            // about the mean expert's row count (whole stages), each piece is a work item of its own that leaves its
            // 256 x 256 result as an fp32 partial tile in the workspace, and a second kernel adds the pieces of a tile
            // in increasing order: the same sums in the same order whatever the timing.  Decided here, from the
            // offsets alone and identically in every workgroup: experts in descending size, pieces = rows / mean
            // rounded up for experts above twice the mean, while the workspace has slices left.
            const int tpe = tiles_i_w * tiles_j;
            const int64_t rows_all = offs[E] - offs[0];
            const int emax = tile_start[0];
            const bool skew = !bad && a.split_cap >= 2 && (int64_t)(offs[emax + 1] - offs[emax]) * E > 2 * rows_all;
            const int mean = (int)((rows_all / E + 127) / 128 * 128);
            int used = 0, nsplit = 0, items = 0;
            for (int i = 0; i < E; ++i) {
                const int ee = tile_start[i];
                const int rows = offs[ee + 1] - offs[ee];
                int pieces = 1;
                if (skew && mean > 0 && rows > 2 * mean && nsplit < GG_MAX_SPLIT_EXPERTS) {
                    pieces = min((rows + mean - 1) / mean, a.split_cap - used);
                    if (pieces < 2) pieces = 1;
                }
                item_start[i] = items;
                split_of[i] = pieces | (used << 8);
                if (pieces > 1) {
                    if (blockIdx.x == 0) {
                        a.split_info[1 + 3 * nsplit] = ee;
                        a.split_info[2 + 3 * nsplit] = pieces;
                        a.split_info[3 + 3 * nsplit] = used;
                    }
                    used += pieces;
                    ++nsplit;
                }
                items += pieces * tpe;
            }
            item_start[E] = items;
            if (blockIdx.x == 0) a.split_info[0] = nsplit;
            tile_start[E] = items;
        }
        if (bad) {  // inconsistent offsets: touch no tensor memory, raise the error word
            tile_start[E] = 0;
            if (blockIdx.x == 0) {
                atomicExch(a.dev_err, 1);
                if (SPLITK) a.split_info[0] = 0;
            }
        }
    }
    __syncthreads();
    // values read back from LDS are the same in every lane: say so, so that everything derived from
    // them (tile origin, operand bases, trip counts) lives in scalar registers
    const int total_tiles = __builtin_amdgcn_readfirstlane(tile_start[E]);

    // workgroups land on the 8 XCDs round-robin; give each XCD a contiguous run of tiles
    const int G = gridDim.x;
    const int q = (G & 7) ? (int)blockIdx.x : ((int)blockIdx.x & 7) * (G >> 3) + ((int)blockIdx.x >> 3);

    // ---- per-lane constants: DMA side ----
    // k-major tile: a 1 KB chunk = 8 rows x 128 B; lane -> (row l/8, slot l%8), slot ^= KM_SWZ(row)
    const int km_row = lane >> 3;
    // c-major tile: a 1 KB chunk = CM_ROWS rows; lane -> (row l / CM_SLOTS, slot l % CM_SLOTS)
    //   bf16: slot ^= 4 * (row % 4) (four waves: and ^= 2 * (row / 16 % 2));  fp8: slot ^= 2 * (row % 8)
    const int cm_row = lane / CM_SLOTS;
    // ---- per-lane constants: fragment side ----
    const int fr_row = lane & 31;
    const int fr_khalf = lane >> 5;
    const int fr_swz = KM_SWZ(lane & 31);
    const int tr_i = lane & 15;
    const int tr_blk = lane >> 4;
    // c-major read of a 32-column operand block at column block cb (a multiple of 32):
    //   bf16 (row pitch 512 B, 64 rows): row = 16 kk + 8 (blk >> 1) + 4 hh + (i >> 2),
    //        slot = (cb / 8 ^ 4 (i >> 2)) + 2 (blk & 1) + ((i & 3) >> 1), byte (i & 1) * 8
    //   fp8  (row pitch 256 B, 128 rows): row = 64 half + 32 (blk >> 1) + 8 g + (i >> 1),
    //        slot = (cb / 16 ^ 2 (i >> 1)) + (blk & 1), byte (i & 1) * 8
    // (MX: the scaled MFMA takes K 0..31 of a 64-step, the first scale block, from bytes 0..15 of both lane
    // halves and K 32..63 from bytes 16..31, so a lane of half h holds K 16 h + 0..15 and 32 + 16 h + 0..15;
    // without block scales the order inside the step does not matter and a lane holds 32 consecutive K)
    const int tr_rowoff = MX    ? (16 * (tr_blk >> 1) + (tr_i >> 1)) * 256
                          : FP8 ? (32 * (tr_blk >> 1) + (tr_i >> 1)) * 256
                                : (8 * (tr_blk >> 1) + (tr_i >> 2)) * 512;
    const int tr_low = FP8 ? (tr_blk & 1) : 2 * (tr_blk & 1) + ((tr_i & 3) >> 1);
    const int tr_xor = FP8 ? 2 * (tr_i >> 1) : 4 * (tr_i >> 2);
    const int tr_byte = (tr_i & 1) * 8;

    // four waves: 16 x 16 blocks.  Row-major: lane -> (row l % 16, 16-byte slot l / 16 of the step's 64 bytes), one
    // slot offset per step (the swizzle depends on l % 16 only).  Contraction-major: lane group l / 16 covers the
    // contraction rows 8 (l / 16) .. + 7 of a step in two transposing reads of 4 rows.
    // Which 8 of the 32 contraction elements of a step a lane group holds is free as long as both operands agree.
    // With a contraction-major operand in play, group g takes the rows 16 (g % 2) + 8 (g / 2) .. + 7: the two groups
    // that the LDS serves in one pass (lanes 0..31, then 32..63) then differ in bit 4 of the row, which the swizzle
    // of these tiles turns into a different 32-byte half of a 64-byte bank segment (without it both groups of a pass
    // read the same banks: SQ_LDS_BANK_CONFLICT was a third of the LDS cycles of the weight gradient).
    // (Data gradient: its row-major operand is read 16 bytes per lane, conflict-free only with group g on the g-th
    // 16 bytes of a step; so there the groups keep rows 8 g .. + 7 and the swizzle uses bit 3 of the row instead.)
    constexpr bool SWZ3 = NW == 4 && MODE == GG_DGRAD;   // which row bit separates the two groups of a pass: 3, else 4
    int p4[8], q4[8], km4[2];
    if (NW == 4) {
        const int l16 = lane & 15, kq = lane >> 4;
        const int kperm = (Q_CMAJ && !SWZ3) ? 2 * (kq & 1) + (kq >> 1) : kq;
        km4[0] = ((kperm) ^ KM_SWZ(l16)) * 16;
        km4[1] = ((4 + kperm) ^ KM_SWZ(l16)) * 16;
        const int cm_off = (8 * kperm + (l16 >> 2)) * 512 + (l16 & 1) * 8;
        const int cm_xor = tr_xor ^ (2 * (kq & 1));   // the separating row bit = kq & 1 in both assignments
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int prow = wm * 128 + 16 * i;                             // tile row of P block i
            const int qrow = (i / 4) * 128 + wn * 64 + (i % 4) * 16;        // tile column of Q block i
            p4[i] = P_CMAJ ? cm_off + (((prow / 8) ^ cm_xor) + ((l16 & 3) >> 1)) * 16 : (prow + l16) * GG_ROWB;
            q4[i] = Q_CMAJ ? cm_off + (((qrow / 8) ^ cm_xor) + ((l16 & 3) >> 1)) * 16 : (qrow + l16) * GG_ROWB;
        }
    }
    int p_rd[4], q_rd[NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (P_CMAJ) p_rd[i] = tr_rowoff + ((((wm * 128 + i * 32) / EPS) ^ tr_xor) + tr_low) * 16 + tr_byte;
        else p_rd[i] = (wm * 128 + i * 32 + fr_row) * GG_ROWB;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (Q_CMAJ) q_rd[j] = tr_rowoff + (((blk_col(j) / EPS) ^ tr_xor) + tr_low) * 16 + tr_byte;
        else q_rd[j] = (blk_col(j) + fr_row) * GG_ROWB;
    }

    // ---- state of the tile being set up / multiplied (assigned by setup_tile) ----
    int e = 0, i0 = 0, i_end = 0, j0 = 0, j1 = 0;  // expert, output row origin and end, column origins of the two halves
    int c_lo = 0, c_hi = 0, KT = 0;                // contraction range and its stage count
    // DMA sources: a wave-uniform 64-bit base per operand (advances with the stage) plus CH 32-bit
    // per-lane offsets; offsets stay below 2^32 because they are tile-relative
    const char* p_base = nullptr;
    const char* q_base = nullptr;
    uint32_t po[CH], qo[CH];
    // four waves: chunk i of a wave sits (i / 2) x a fixed stride behind chunk i % 2 (the swizzle alternates with the
    // parity of the chunk), so two lane offsets and a wave-uniform stride per operand replace 2 x 8 registers; rows are
    // not clamped here, the record count of the buffer descriptor covers the end of the tensor
    uint32_t po2[2] = {0, 0}, qo2[4] = {0, 0, 0, 0};   // (qo2[2..3]: data gradient only, chunks 4..7 of a wave, see SWZ3)
    uint32_t po8[G_ROW ? 8 : 1] = {};   // gathered row-major P: one offset per chunk
    uint32_t gv[G_CM ? 8 : 1] = {};     // gathered contraction-major operand: the row offsets of the chunks about to be loaded
    uint32_t p_cstride = 0, q_cstride = 0;
    // the buffer descriptor of each operand at the stage being loaded (set by the stage's first chunk, see load_one),
    // and what it is made from: bytes per row and the largest whole-row count below 4 GB (contraction-major operands),
    // the byte count of the tile's tensor from its stage-0 base on, clamped (row-major operands; set with the tile),
    // the size of a gathered tensor
    uint32_t d_lo[2] = {0, 0}, d_hi[2] = {0, 0}, d_rec[2] = {0, 0};
    const uint32_t p_rowb = (uint32_t)(((MODE == GG_FWD) ? K : N) * ES), q_rowb = (uint32_t)(K * ES);
    const uint32_t p_rowcap = __builtin_amdgcn_readfirstlane(0xffffffffu / p_rowb);
    const uint32_t q_rowcap = __builtin_amdgcn_readfirstlane(0xffffffffu / q_rowb);
    const uint32_t g_total = (uint32_t)a.g_T * g_rowb;
    uint32_t p_rec0 = 0, q_rec0 = 0;
    int64_t p_step = 0, q_step = 0;  // byte advance per stage
    const float* sc_src = nullptr;   // fp8: this lane's scale for block 0
    int64_t sc_step = 0;             // fp8: element advance per block
    // L2 warm-up (bf16): see PF below
    uint32_t pf_off = 0;
    bool pf_on = false, pf_q = false;
    int KT_pf = 0;
    int e_hint = 0;
    int part_slot = -1, part_tile = 0;  // split contraction: slice and tile of the partial result (-1: the result itself)
    // contraction-major gather: the map entry of this lane's row of stage kt (rows behind the map read 0 and are
    // masked by the range test in gconv), its byte offset, the ring slot it is parked in, and the read-back of the
    // row of chunk c
    auto gfetch = [&](int kt) __attribute__((always_inline)) -> int {
        const __amdgpu_buffer_rsrc_t rs =
            __builtin_amdgcn_make_buffer_rsrc((void*)a.g_src_of, 0, (int)((uint32_t)a.Rcap * 4u), 0x00020000);
        // (the stage's first row through readfirstlane: otherwise the loop counter is strength-reduced into this
        // lane-dependent row number and the stage loop becomes a divergent loop on an exec mask)
        return (int)__builtin_amdgcn_raw_buffer_load_b32(rs, (__builtin_amdgcn_readfirstlane(c_lo + kt * BKE) + g_row16) * 4, 0, 0);
    };
    auto gconv = [&](int kt, int s) __attribute__((always_inline)) -> uint32_t {
        return g_off_of(s, (__builtin_amdgcn_readfirstlane(c_lo + kt * BKE) + g_row16) < c_hi);
    };
    typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
    auto gput = [&](int slot, uint32_t v) __attribute__((always_inline)) {
        *(lds_u32_t*)(uintptr_t)(gl_wr + slot * 256) = v;
    };
    typedef __attribute__((address_space(3))) u32x4_t lds_u32x4_t;
    auto gread = [&](int slot, int half) __attribute__((always_inline)) {  // the offsets of chunks 4 half .. 4 half + 3
        const u32x4_t v = *(const lds_u32x4_t*)(uintptr_t)(gl_rd + slot * 256 + half * 16);
        gv[4 * half] = v[0];
        gv[4 * half + 1] = v[1];
        gv[4 * half + 2] = v[2];
        gv[4 * half + 3] = v[3];
    };
    auto setup_tile = [&](int t) __attribute__((always_inline)) {
        // (four waves: the lane constants of the set-up are formed here from a lane id the compiler cannot see through;
        // computed once at kernel start they would occupy registers through every stage loop, or spill)
        int lane = threadIdx.x & 63;
        if (NW == 4) asm volatile("" : "+v"(lane));
        const int km_row = lane >> 3, cm_row = lane / CM_SLOTS;
        // ---- locate the tile: bands of GG_BAND row-tiles, column-major inside a band ----
        int u;
        int piece = 0, pieces = 1;
        if (SPLITK) {
            // work item -> (sorted position, piece, tile); a workgroup's items come in increasing order
            const int tpe = tiles_i_w * tiles_j;
            int es = e_hint;
            while (es + 1 < E && t >= __builtin_amdgcn_readfirstlane(item_start[es + 1])) ++es;
            e_hint = es;
            e = __builtin_amdgcn_readfirstlane(tile_start[es]);
            const int sp = __builtin_amdgcn_readfirstlane(split_of[es]);
            pieces = sp & 255;
            u = t - __builtin_amdgcn_readfirstlane(item_start[es]);
            piece = __builtin_amdgcn_readfirstlane(u / tpe);
            u -= piece * tpe;
            part_slot = pieces > 1 ? (sp >> 8) + piece : -1;
            part_tile = u;
        } else if (MODE == GG_WGRAD) {
            const int tpe = tiles_i_w * tiles_j;
            const int es = __builtin_amdgcn_readfirstlane(t / tpe);
            e = __builtin_amdgcn_readfirstlane(tile_start[es]);
            u = t - es * tpe;
        } else {
            e = e_hint;
            while (e + 1 < E && t >= __builtin_amdgcn_readfirstlane(tile_start[e + 1])) ++e;
            e_hint = e;
            u = t - __builtin_amdgcn_readfirstlane(tile_start[e]);
        }
        const int row_lo = __builtin_amdgcn_readfirstlane(offs[e]), row_hi = __builtin_amdgcn_readfirstlane(offs[e + 1]);
        int ti, tj;
        {
            const int tiles_i = (MODE == GG_WGRAD) ? tiles_i_w : (row_hi - row_lo + GG_BM - 1) / GG_BM;
            const int band_sz = GG_BAND * tiles_j;
            const int band = u / band_sz;
            const int in_band = u - band * band_sz;
            const int band_rows = min(GG_BAND, tiles_i - band * GG_BAND);
            // (integer divisions run on the vector unit: without the readfirstlanes their uniform results, and the
            // operand bases, record counts and trip count derived from them, live in vector registers, and the stage
            // loop rebuilds every buffer descriptor with 64-bit vector arithmetic between its MFMAs)
            ti = __builtin_amdgcn_readfirstlane(band * GG_BAND + in_band % band_rows);
            tj = __builtin_amdgcn_readfirstlane(in_band / band_rows);
        }
        // output row/column origin of the two 128-column halves
        i0 = (MODE == GG_WGRAD) ? ti * GG_BM : row_lo + ti * GG_BM;
        i_end = (MODE == GG_WGRAD) ? N : row_hi;
        j0 = (EPI == GG_EPI_SWIGLU) ? tj * 128 : tj * GG_BN;
        j1 = (EPI == GG_EPI_SWIGLU) ? half_cols + tj * 128 : tj * GG_BN + 128;
        // contraction range
        c_lo = (MODE == GG_WGRAD) ? row_lo : 0;
        c_hi = (MODE == GG_WGRAD) ? row_hi : (MODE == GG_FWD ? K : N);
        if (SPLITK && pieces > 1) {  // this piece's share of the expert's rows, in whole stages
            const int len = __builtin_amdgcn_readfirstlane(((row_hi - row_lo + pieces - 1) / pieces + BKE - 1) / BKE * BKE);
            c_lo = min(row_lo + piece * len, row_hi);
            c_hi = min(c_lo + len, row_hi);
        }
        c_lo = __builtin_amdgcn_readfirstlane(c_lo);
        c_hi = __builtin_amdgcn_readfirstlane(c_hi);
        KT = __builtin_amdgcn_readfirstlane((c_hi - c_lo + BKE - 1) / BKE);

        // ---- DMA sources: a wave-uniform 64-bit base per operand (advances with the stage) plus
        //      CH 32-bit per-lane offsets; offsets stay below 2^32 because they are tile-relative ----
        if (P_CMAJ) {
            // P = dC [rows, N]: contraction row c, columns i0..i0+255
            p_step = (int64_t)BKE * N * ES;
            p_base = (const char*)a.P + (int64_t)c_lo * N * ES;
            p_cstride = (uint32_t)(2 * CM_ROWS * N * ES);
#pragma unroll
            for (int i = 0; i < (NW == 4 ? 2 : CH); ++i) {
                const int row = (wave * CH + i) * CM_ROWS + cm_row;
                const int slot = (lane & (CM_SLOTS - 1)) ^ (FP8 ? 2 * (row & 7) : 4 * (row & 3) ^ (NW == 4 ? 2 * ((row >> 4) & 1) : 0));
                int col = i0 + slot * EPS;
                col = col <= N - EPS ? col : N - EPS;
                if (NW == 4) po2[i] = (uint32_t)((row * N + col) * ES);
                else po[i] = (uint32_t)((row * N + col) * ES);
                if (GATH == 1) po2[i] = (uint32_t)(col * ES);  // the row comes from the map
            }
            if (GATH == 1) {
                p_step = 0;
                p_base = (const char*)a.P;
            }
        } else if (G_ROW) {
            const int ldp = (MODE == GG_FWD) ? K : N;
            (void)ldp;
            p_step = GG_ROWB;
            p_base = (const char*)a.P;
            int sidx[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t r = (int64_t)i0 + (wave * CH + i) * 8 + km_row;
                sidx[i] = r < a.Rcap ? a.g_src_of[r] : -1;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int p = (wave * CH + i) * 8 + km_row;  // tile row 0..255
                po8[i] = g_off_of(sidx[i], true) + (uint32_t)(((lane & 7) ^ KM_SWZ(p)) * 16);
            }
        } else {
            const int ldp = (MODE == GG_FWD) ? K : N;
            p_step = GG_ROWB;
            p_base = (const char*)a.P + (int64_t)i0 * ldp * ES;
            {   // rows of the activation tensor from the tile's first row up to its capacity
                const int64_t tot = (a.Rcap - i0) * (int64_t)ldp * ES;
                p_rec0 = __builtin_amdgcn_readfirstlane(tot > 0xffffffffLL ? 0xffffffffu : (uint32_t)tot);
            }
            p_cstride = (uint32_t)(16 * ldp * ES);
#pragma unroll
            for (int i = 0; i < (NW == 4 ? 2 : CH); ++i) {
                const int p = (wave * CH + i) * 8 + km_row;  // tile row 0..255
                int64_t r = (int64_t)i0 + p;
                if (NW != 4) r = r < a.Rcap ? r : a.Rcap - 1;   // i0 < Rcap, so r - i0 >= 0
                const int gslot = (lane & 7) ^ KM_SWZ(p);
                if (NW == 4) po2[i] = (uint32_t)((r - i0) * ldp * ES + gslot * 16);
                else po[i] = (uint32_t)((r - i0) * ldp * ES + gslot * 16);
            }
        }
        if (Q_CMAJ) {
            // dgrad: Q = W_e [N,K]: contraction row n, columns (k) j0.. ; wgrad: Q = A [rows,K]
            q_step = (int64_t)BKE * K * ES;
            q_base = (MODE == GG_DGRAD ? (const char*)a.Q + (int64_t)e * N * K * ES : (const char*)a.Q) + (int64_t)c_lo * K * ES;
            q_cstride = (uint32_t)(2 * CM_ROWS * K * ES);
#pragma unroll
            for (int i = 0; i < (NW == 4 ? (SWZ3 ? 4 : 2) : CH); ++i) {
                // (SWZ3: entries 2, 3 are chunks 4, 5 of the wave, whose rows have bit 3 set)
                const int row = (wave * CH + (SWZ3 ? (i & 1) + 4 * (i >> 1) : i)) * CM_ROWS + cm_row;
                const int sep = SWZ3 ? (row >> 3) & 1 : (row >> 4) & 1;
                const int slot = (lane & (CM_SLOTS - 1)) ^ (FP8 ? 2 * (row & 7) : 4 * (row & 3) ^ (NW == 4 ? 2 * sep : 0));
                int col = (slot < CM_SLOTS / 2 ? j0 : j1 - 128) + slot * EPS;
                col = col <= K - EPS ? col : K - EPS;
                if (NW == 4) qo2[i] = (uint32_t)((row * K + col) * ES);
                else qo[i] = (uint32_t)((row * K + col) * ES);
                if (GATH == 2) qo2[i] = (uint32_t)(col * ES);  // the row comes from the map
            }
            if (GATH == 2) {
                q_step = 0;
                q_base = (const char*)a.Q;
            }
        } else {
            q_step = GG_ROWB;
            q_base = (const char*)a.Q + (int64_t)e * N * K * ES;
            {   // the weights of this expert
                const int64_t tot = (int64_t)N * K * ES;
                q_rec0 = __builtin_amdgcn_readfirstlane(tot > 0xffffffffLL ? 0xffffffffu : (uint32_t)tot);
            }
            q_cstride = (uint32_t)(16 * K * ES);
#pragma unroll
            for (int i = 0; i < (NW == 4 ? 2 : CH); ++i) {
                const int p = (wave * CH + i) * 8 + km_row;  // tile row 0..255
                int n = (p < 128 ? j0 : j1 - 128) + p;
                if (NW != 4) n = n < N ? n : N - 1;
                const int gslot = (lane & 7) ^ KM_SWZ(p);
                if (NW == 4) qo2[i] = (uint32_t)(((int64_t)n * K) * ES + gslot * 16);
                else qo[i] = (uint32_t)(((int64_t)n * K) * ES + gslot * 16);
            }
        }

        // ---- L2 warm-up share of this wave (see PF): lanes 8x of DMA chunk (ti & 3) of Q, lanes 8x + 1 of half a
        //      chunk of P; lanes 8x .. 8x + 7 of a chunk fetch from one 128-byte line ----
        if (PF) {
            const int a_in = ti & 3, b_in = tj & 7;
            const uint32_t qsel = a_in == 0 ? qo[0] : a_in == 1 ? qo[1] : a_in == 2 ? qo[2] : qo[3];
            const uint32_t psel = (b_in >> 1) == 0 ? po[0] : (b_in >> 1) == 1 ? po[1] : (b_in >> 1) == 2 ? po[2] : po[3];
            pf_q = (lane & 7) == 0;
            pf_on = pf_q || ((lane & 7) == 1 && (lane >> 5) == (b_in & 1));
            pf_off = pf_q ? qsel : psel;
            KT_pf = (MODE == GG_WGRAD) ? (c_hi - c_lo) / BKE : KT;  // wgrad: only stages that lie wholly inside the expert
        }

        // ---- fp8 block scales: s = p_scale[row, kb] * q_scale[block]; per lane 4 rows x 2 column blocks ----
        // The accumulators are kept in units of the current block's scale: entering block kb they are
        // multiplied by s(kb-1) / s(kb), and by the last s in the epilogue.  The scales of block kb reach
        // LDS with the operands of stage kb (one more 4-byte-per-lane DMA by waves 0..4).
        const int CB = (c_hi - c_lo) / 128;  // contraction blocks = stages
        if (MX) {
            // one dword = the four E8M0 bytes (32-element blocks) of one tile row for this stage of 128 contraction
            // elements.  Waves 0..3 fetch the 256 P rows (position layout as below), waves 4..7 the 256 Q rows:
            // position p' = 64 (wave - 4) + lane holds Q tile row 128 (p' & 1) + (p' >> 1), so a lane finds the rows
            // of its two column blocks in one 8-byte read.
            // 1x32 copies (contraction along the memory row): [row, C/128] dwords, one step per stage;
            // 32x1 copies (contraction along the rows): [c/128, columns] dwords, `columns` per stage.
            if (wave < 4) {
                const int pp = wave * 64 + lane;
                int64_t r = (int64_t)i0 + (pp >> 7) * 128 + (pp & 3) * 32 + ((pp & 127) >> 2);
                if (MODE == GG_WGRAD) {  // P tile row = output row n
                    r = r < N ? r : N - 1;
                    sc_src = a.p_scale + (int64_t)(c_lo >> 7) * N + r;
                    sc_step = N;
                } else {
                    r = r < a.Rcap ? r : a.Rcap - 1;
                    sc_src = a.p_scale + r * CB;
                    sc_step = 1;
                }
            } else {
                const int pp = (wave - 4) * 64 + lane;
                const int rho = 128 * (pp & 1) + (pp >> 1);
                int col = (rho < 128 ? j0 : j1 - 128) + rho;  // output column = weight row (fwd) / weight column (dgrad)
                col = col < J ? col : J - 1;
                if (MODE == GG_FWD) {         // e8m0 [E*N, K/32]
                    sc_src = a.q_scale + ((int64_t)e * N + col) * CB;
                    sc_step = 1;
                } else if (MODE == GG_DGRAD) {  // e8m0 [E*N/128, K, 4]
                    sc_src = a.q_scale + (int64_t)e * (N >> 7) * K + col;
                    sc_step = K;
                } else {                      // e8m0 [Rcap/128, K, 4]
                    sc_src = a.q_scale + (int64_t)(c_lo >> 7) * K + col;
                    sc_step = K;
                }
            }
        } else if (BW_WGRAD) {
            // 128x1 scales of both operands: [c / 128, columns] floats, one row of them per stage.  Waves 0..3 fetch the
            // 256 scales of the tile's rows (= columns n of dC; position layout as in the forward kernel: a lane finds
            // its four rows in one 16-byte read), waves 4..7 the 256 of the tile's columns (= columns k of A), in
            // tile-column order.
            if (wave < 4) {
                const int pp = wave * 64 + lane;
                int64_t r = (int64_t)i0 + (pp >> 7) * 128 + (pp & 3) * 32 + ((pp & 127) >> 2);
                r = r < N ? r : N - 1;
                sc_src = a.p_scale + (int64_t)(c_lo >> 7) * N + r;
                sc_step = N;
            } else {
                const int c = (wave - 4) * 64 + lane;
                int col = (c < 128 ? j0 : j1 - 128) + c;
                col = col < K ? col : K - 1;
                sc_src = a.q_scale + (int64_t)(c_lo >> 7) * K + col;
                sc_step = K;
            }
        } else if (FP8) {
            if (wave < 4) {  // row scales: LDS position p = 64 wave + lane holds tile row ...
                const int pp = wave * 64 + lane;
                int64_t r = (int64_t)i0 + (pp >> 7) * 128 + (pp & 3) * 32 + ((pp & 127) >> 2);
                r = r < a.Rcap ? r : a.Rcap - 1;
                sc_src = a.p_scale + r * CB;
                sc_step = 1;
            } else {         // column-block scales (issued by wave 4 only): even lanes block j0, odd lanes j1
                int col = (lane & 1) ? j1 : j0;
                col = col < J ? col : J - 1;
                if (MODE == GG_FWD) {  // q_scale[e, col/128, kb]
                    sc_src = a.q_scale + ((int64_t)e * (N / 128) + col / 128) * (K / 128);
                    sc_step = 1;
                } else {               // dgrad contracts over N: q_scale[e, kb, col/128]
                    sc_src = a.q_scale + (int64_t)e * (N / 128) * (K / 128) + col / 128;
                    sc_step = K / 128;
                }
            }
        }
        if (G_CM) {  // the row offsets of the first three stages, one slot each (inside the stage loop: slot 0 only)
            const int s0 = gfetch(0), s1 = gfetch(1), s2 = gfetch(2);
            gput(0, gconv(0, s0));
            gput(1, gconv(1, s1));
            gput(2, gconv(2, s2));
        }
    };

        // one of the 2 CH DMA instructions of stage kt (idx: operand = idx & 1, chunk = idx >> 1)
        auto issue_one = [&](int kt, char* sp, char* sq, int idx) {
            const int i = idx >> 1;
            const uint32_t off = (idx & 1) ? qo[i] : po[i];
            const char* base = (idx & 1) ? q_base + kt * q_step : p_base + kt * p_step;  // wave-uniform
            const uint32_t dst_wave = wave * (CH * 1024), dst_const = lds_addr((idx & 1) ? sq : sp) + i * 1024;
            if (MODE == GG_WGRAD && !FP8) {  // contraction tail of the expert: feed zeros (one-byte operands: whole stages only)
                const int row = c_lo + kt * BKE + (wave * CH + i) * CM_ROWS + cm_row;
                uint32_t o = off;
                asm volatile("" : "+v"(o));  // opaque: keeps base + offset from being hoisted as 64-bit lane pointers
                dma16(row < c_hi ? base + o : a.zeros, dst_wave, dst_const);
            } else {
                dma16(base, off, dst_wave, dst_const);
            }
        };

        auto issue_scales = [&](int kb, float* ss) {
            if (BW_WGRAD) {  // this stage's scales and, behind them, the previous stage's (stage 0: its own, ratio 1)
                dma4(sc_src + kb * sc_step, wave * 256, lds_addr(ss));
                dma4(sc_src + (kb > 0 ? kb - 1 : 0) * sc_step, wave * 256, lds_addr(ss) + 2048);
                return;
            }
            if (MX || wave <= 4) {
                const float* src = sc_src + kb * sc_step;
                dma4(src, wave * 256, lds_addr(ss));
            }
        };

    // NW == 4: the operands of one stage in flight, in registers: 2 CH 16-byte loads per lane and stage, the same
    // chunk -> lane mapping as the DMA.  Plain loads and LDS stores: the compiler counts the loads in flight itself
    // and waits, before each store, for exactly the load that feeds it.  A register is stored (stage j + 1) and at
    // once reloaded (stage j + 2), so every load has a full stage to arrive.  (A second register set, two stages
    // ahead, measured 1-3 % slower: it leaves the register allocator no slack.)
    u32x4_t R[NW == 4 ? 2 * CH : 1];
    // Loads go through buffer descriptors (base = the operand at this stage, wave-uniform; 32-bit lane offset): a
    // lane whose offset is not below the record count reads zeros, with no branch and no address arithmetic.
    // Contraction-major operands count the bytes up to the end of the contraction range (the tail rows of an
    // expert, and whole stages past the end, read zeros); row-major operands (rows clamped, always valid) get
    // everything or, for a stage past the end, nothing.
    auto load_one = [&](int kt, int idx) __attribute__((always_inline)) {
        const int i = idx >> 1;
        const bool isq = idx & 1;
        const bool g_cm = G_CM && (isq ? GATH == 2 : GATH == 1);  // this operand's rows come through the ring
        const bool g_row = G_ROW && !isq;                          // ... or from the tile's eight row offsets
        const uint32_t off = g_cm    ? gv[i] + (isq ? qo2[i & 1] : po2[i & 1])
                             : g_row ? po8[i]
                             : (isq && SWZ3) ? qo2[(i & 1) + 2 * (i >> 2)] + (uint32_t)((i >> 1) & 1) * q_cstride
                                             : (isq ? qo2[i & 1] : po2[i & 1]) + (uint32_t)(i >> 1) * (isq ? q_cstride : p_cstride);
        if (i == 0) {
            // The first chunk of an operand in a stage builds the descriptor the other seven share: base = the operand
            // at this stage; record count = the bytes from there to the end of what may be read, in 32-bit scalar
            // arithmetic (counts above 4 GB are clamped: lane offsets are tile-relative and far below that).  The stage
            // number passes through an empty asm so that this arithmetic stays in the MFMA gap of this chunk: hoisted
            // to the top of the loop body, the descriptors of two stages were some fifty scalar and 64-bit vector
            // compare instructions in front of a single MFMA.
            int ks = kt;
            asm volatile("" : "+s"(ks));
            // (wave-uniform; the byte advance per stage fits 32 bits, so the product is one 32 x 32 -> 64 multiplication)
            const char* base = isq ? q_base + (uint64_t)(uint32_t)ks * (uint32_t)q_step : p_base + (uint64_t)(uint32_t)ks * (uint32_t)p_step;
            const bool cmaj = isq ? Q_CMAJ : P_CMAJ;
            uint32_t records;
            if (g_cm) {
                records = g_total;
            } else if (g_row) {
                records = ks >= KT ? 0u : g_total - (uint32_t)ks * GG_ROWB;
            } else if (cmaj) {   // whole rows up to the end of the contraction range
                const uint32_t left = (uint32_t)max(c_hi - c_lo - ks * BKE, 0);
                records = min(left, isq ? q_rowcap : p_rowcap) * (isq ? q_rowb : p_rowb);
            } else {             // row-major: the tensor from this stage's first byte on; nothing behind the last stage
                records = ks >= KT ? 0u : (isq ? q_rec0 : p_rec0) - (uint32_t)ks * GG_ROWB;
            }
            // (readfirstlane: free for values already in scalar registers, and the promise of uniformity the descriptor needs)
            const uint64_t b = (uint64_t)base;
            d_lo[isq] = __builtin_amdgcn_readfirstlane((uint32_t)b);
            d_hi[isq] = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
            d_rec[isq] = __builtin_amdgcn_readfirstlane(records);
        }
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(((uint64_t)d_hi[isq] << 32) | d_lo[isq]), 0, (int)d_rec[isq], 0x00020000);
        R[idx] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0));
    };
    auto store_one = [&](char* sp, char* sq, int idx) __attribute__((always_inline)) {
        asm volatile("" : "+v"(R[idx]));  // (held in ordinary vector registers: the accumulation registers are all taken)
        *(u32x4_t*)(((idx & 1) ? sq : sp) + wave * (CH * 1024) + (idx >> 1) * 1024 + lane * 16) = R[idx];
    };

    // PF: L2 warm-up.  With two stage buffers a stage's DMA can be issued only 3/4 of a stage before it is needed,
    // less than the latency of an L2 miss, and about one line in five misses (first touch by the XCD).  The
    // workgroups that run together on an XCD share each P tile 8 ways and each Q tile 4 ways, so each takes
    // 1/8 and 1/4 of the lines of the stage after next (12 lines per wave) and touches them with one 4-byte
    // load into a dummy LDS word; the load is the wave's youngest vector-memory operation when the wave waits
    // for its DMA (wait_vm1), so it never delays the stage being waited for.
    uint32_t pf_lds = lds_addr(lds_buf + LDS_BYTES - 256);  // dummy words behind everything else
    asm volatile("" : "+s"(pf_lds));                      // (formed here, in uniform code, not where it is used)
    auto prefetch = [&](int kt) {
        if (pf_on) {
            uint64_t src = (uint64_t)(pf_q ? q_base + kt * q_step : p_base + kt * p_step) + pf_off;
            asm volatile("" : "+v"(src));  // a per-lane address in vector registers, whatever the compiler can prove
            const uint32_t m0v = __builtin_amdgcn_readfirstlane(pf_lds);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(m0v), "v"(src) : "memory", "m0");
        }
    };

    char* const SP[2] = {ldsP0, ldsP1};
    char* const SQ[2] = {ldsQ0, ldsQ1};
    float* const SS[2] = {(float*)(ldsP0 + GG_STAGE_BYTES), (float*)(ldsP1 + GG_STAGE_BYTES)};
    // stage 0 of a tile: every wave issues its share.  It is issued before the epilogue of the previous tile,
    // so that the first fetch of a tile overlaps the output phase of the one before
    auto issue_stage0 = [&]() __attribute__((always_inline)) {
        if (NW == 4) {  // into the registers
            if (KT > 0) {
                if (G_CM) {
                    gread(0, 0);
                    gread(0, 1);
                }
#pragma unroll
                for (int x = 0; x < 2 * CH; ++x) load_one(0, x);
            }
            return;
        }
        if (KT > 0) {
#pragma unroll
            for (int x = 0; x < 2 * CH; ++x) issue_one(0, SP[0], SQ[0], x);
            if (FP8) issue_scales(0, SS[0]);
        }
    };

    // n-th tile of this workgroup.  Forward / data gradient: q, q + G, ... (equal-cost tiles).  Weight gradient: the
    // list is in descending cost; chunks of G / 8 consecutive tiles go to the XCDs in a snake (0..7, 7..0, ...),
    // the i-th workgroup of an XCD takes the i-th tile of each of its chunks.
    auto tile_of = [&](int n) -> int {
        if (MODE == GG_WGRAD && !(G & 7)) {
            const int x = (int)blockIdx.x & 7, i = (int)blockIdx.x >> 3;
            return (8 * n + ((n & 1) ? 7 - x : x)) * (G >> 3) + i;
        }
        return q + n * G;
    };
    // Weight gradient under a skewed load (largest expert above twice the mean): a static deal cannot balance when one
    // tile of the largest expert is most of a workgroup's share, so the workgroups then draw tiles from a device
    // counter in the same descending-cost order (longest-processing-time-first list scheduling): whoever finishes
    // early takes the next tile.  Which workgroup computes a tile changes, what the tile computes does not.  The
    // draw for the tile after this one is issued at the top of a tile and collected after its contraction.
    bool dyn = false;
    if (MODE == GG_WGRAD && a.tile_counter != nullptr && total_tiles > 0) {
        const int emax = __builtin_amdgcn_readfirstlane(tile_start[0]);
        const int64_t rows_max = __builtin_amdgcn_readfirstlane(offs[emax + 1]) - __builtin_amdgcn_readfirstlane(offs[emax]);
        const int64_t rows_all = __builtin_amdgcn_readfirstlane(offs[E]) - __builtin_amdgcn_readfirstlane(offs[0]);
        dyn = rows_max * E > 2 * rows_all;
    }
    auto draw = [&]() -> int {  // thread 0 only
        return tid == 0 ? atomicAdd(a.tile_counter, 1) : 0;
    };
    auto publish = [&](int v) -> int {  // thread 0's value to every wave
        if (tid == 0) dyn_next = v;
        wait_lgkm0();
        stage_barrier();
        return __builtin_amdgcn_readfirstlane(dyn_next);
    };
    int t_first = tile_of(0);
    if (dyn) t_first = publish(draw());
    t_first = __builtin_amdgcn_readfirstlane(t_first);
    if (t_first < total_tiles) {
        setup_tile(t_first);
        issue_stage0();
    }
    for (int n_tile = 0, t = t_first; t < total_tiles; ++n_tile) {
        int drawn = 0;
        if (dyn) drawn = draw();
        float ps_cur[4] = {1.f, 1.f, 1.f, 1.f}, qs_cur[NJ];
        f32x16_t acc[4][NJ];  // eight waves: 32 x 32 blocks
        f32x4_t acc4[8][8];   // four waves: 16 x 16 blocks (P block i, Q block j)
        if (NW == 4) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int x = 0; x < 4; ++x) acc4[i][j][x] = 0.f;
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) qs_cur[j] = 1.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;

        {
            // operand fragments of one half-stage: bf16 2 x (4 + 2) x 4 VGPRs, fp8 (4 + 2) x 8 VGPRs
            bf16x8_t pf[2][4], qf[2][NJ];
            i32x8_t pf8[4], qf8[2];

            // MFMAs (and the fp8 rescaling multiplies) have no side effects, so nothing else stops the
            // compiler from sinking them past DMA issues, LDS reads and barriers towards the next use of
            // the accumulators, which keeps two half-stages of fragments alive and undoes the schedule.
            // An empty asm that "modifies" a block of accumulators pins its producer in program order.
            auto pin = [](f32x16_t& v) { asm volatile("" : "+v"(v)::"memory"); };

            auto fetch = [&](const char* sp, const char* sq, int half) {
                if (FP8) {
                    const int sl0 = MX ? 4 * half + fr_khalf : 4 * half + 2 * fr_khalf;  // 16-byte slot of the lane's first 16 K
                    const int sl1 = MX ? sl0 + 2 : sl0 + 1;
                    const int s0 = (sl0 ^ fr_swz) * 16, s1 = (sl1 ^ fr_swz) * 16;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (P_CMAJ) {
                            pf8[i] = lds_read_tr8x32(sp + p_rd[i] + half * 64 * 256, MX ? 32 : 16);
                        } else {
                            const i32x4_t lo = *(const i32x4_t*)(sp + p_rd[i] + s0), hi = *(const i32x4_t*)(sp + p_rd[i] + s1);
                            pf8[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (Q_CMAJ) {
                            qf8[j] = lds_read_tr8x32(sq + q_rd[j] + half * 64 * 256, MX ? 32 : 16);
                        } else {
                            const i32x4_t lo = *(const i32x4_t*)(sq + q_rd[j] + s0), hi = *(const i32x4_t*)(sq + q_rd[j] + s1);
                            qf8[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        }
                    }
                } else {
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2) {
                        const int kk = half * 2 + k2;
                        const int km_slot = ((kk * 2 + fr_khalf) ^ fr_swz) * 16;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if (P_CMAJ) pf[k2][i] = lds_read_tr16x8(sp + p_rd[i] + kk * 8192, sp + p_rd[i] + kk * 8192 + 2048);
                            else pf[k2][i] = *(const bf16x8_t*)(sp + p_rd[i] + km_slot);
                        }
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            if (Q_CMAJ) qf[k2][j] = lds_read_tr16x8(sq + q_rd[j] + kk * 8192, sq + q_rd[j] + kk * 8192 + 2048);
                            else qf[k2][j] = *(const bf16x8_t*)(sq + q_rd[j] + km_slot);
                        }
                    }
                }
            };
            // the MFMAs of one half-stage, with the 2 CH DMA instructions of stage kt_dma slipped in
            int psr[4] = {127, 127, 127, 127}, qsr[2] = {127, 127};  // MX: scale bytes of the current stage
            // blockwise forward / data gradient: s(kb-1) / s(kb) of every block of accumulators for the stage being entered,
            // set in the read phase.  Where the 128 multiplies are done was measured both ways (per-slot timestamps): in
            // the read phase that phase lasts 1030 cycles against the 550 of the MFMA phase it alternates with; in front
            // of each block's first MFMA the read phase drops to 450 and the MFMA phase grows to 950 (vector
            // instructions do not overlap the wave's own MFMAs here).  The second is 2-9 % faster per call except for
            // the fc1 forward with its 56-stage tiles (9 % slower), which keeps the first.
            constexpr bool RESCALE_IN_B = F8 == 1 && !BW_WGRAD && !(MODE == GG_FWD && EPI == GG_EPI_SWIGLU);
            float ratio8[4][2];
            auto mma = [&](bool do_dma, int kt_dma, char* dp, char* dq, int half) {
                if (FP8) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            if (RESCALE_IN_B && half == 0) {
#pragma unroll
                                for (int x = 0; x < 16; ++x) acc[i][j][x] *= ratio8[i][j];
                            }
                            // MX: the lane's 32 contraction elements are one scale block; its E8M0 byte sits in byte 0
                            // (first half-stage) / byte 2 (second) of the pre-shifted scale registers
                            if (!MX) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(qf8[j], pf8[i], acc[i][j], 0, 0, 0, 127, 0, 127);
                            else if (half == 0) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(qf8[j], pf8[i], acc[i][j], 0, 0, 0, qsr[j], 0, psr[i]);
                            else acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(qf8[j], pf8[i], acc[i][j], 0, 0, 2, qsr[j], 2, psr[i]);
                            pin(acc[i][j]);
                            __builtin_amdgcn_sched_barrier(0);
                            if (do_dma) issue_one(kt_dma, dp, dq, i * 2 + j);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                } else {
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
#pragma unroll
                            for (int j = 0; j < 2; ++j)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[k2][j], pf[k2][i], acc[i][j], 0, 0, 0);
                            pin(acc[i][0]);
                            pin(acc[i][1]);
                            __builtin_amdgcn_sched_barrier(0);
                            if (do_dma) issue_one(kt_dma, dp, dq, k2 * 4 + i);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
            };
            // fp8: entering contraction block kb, bring the accumulators to the new block's units
            // (block 0 multiplies zeros by 1 / s_0, which is finite: scales are positive; no special case,
            // so that the compiler does not peel the first stage off the loop)
            f32x4_t pn;
            float qn[2];
            auto read_scales = [&](const float* ss) {
                if (MX) {
                    const i32x4_t pw = *(const i32x4_t*)(ss + wm * 128 + fr_row * 4);
                    const i32x2_t qw = *(const i32x2_t*)(ss + 256 + (wn * 32 + fr_row) * 2);
                    const int sh = 8 * fr_khalf;  // this lane's 32 elements are block khalf (first half) / 2 + khalf (second)
#pragma unroll
                    for (int i = 0; i < 4; ++i) psr[i] = (int)((uint32_t)pw[i] >> sh);
                    qsr[0] = (int)((uint32_t)qw.x >> sh);
                    qsr[1] = (int)((uint32_t)qw.y >> sh);
                    return;
                }
                pn = *(const f32x4_t*)(ss + wm * 128 + fr_row * 4);
                qn[0] = ss[256];
                qn[1] = ss[257];
            };
            auto rescale = [&]() {
                float qs_nxt[2], qr[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    qs_nxt[j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, qn[j])));
                    qr[j] = qs_cur[j] * __builtin_amdgcn_rcpf(qs_nxt[j]);
                    qs_cur[j] = qs_nxt[j];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float pr = ps_cur[i] * __builtin_amdgcn_rcpf(pn[i]);
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        ratio8[i][j] = pr * qr[j];
                        if (!RESCALE_IN_B) {
#pragma unroll
                            for (int x = 0; x < 16; ++x) acc[i][j][x] *= ratio8[i][j];
                        }
                    }
                    if (!RESCALE_IN_B) {
                        pin(acc[i][0]);
                        pin(acc[i][1]);
                    }
                    ps_cur[i] = pn[i];
                }
            };

            // Blockwise weight gradient: the factor of an accumulator is a product, s = sP[n] * sQ[k] (128x1 scales of
            // dC and A for this stage's 128 rows), different for every element of a block, so every element gets its
            // own ratio s(kb-1) / s(kb) = rP[row] * rQ[column]: per lane 4 row ratios and 2 x 16 column ratios, formed
            // from the current and previous scales in LDS, four columns at a time (no scale stays in registers).
            // Two multiplies per accumulator and stage: the plain-ALU price of a scale that changes along the
            // contraction on both operands.
            auto scale_cols = [&](const float* ss, bool ratio, const float (&rp)[4]) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int c = 256 + blk_col(j) + 8 * g + 4 * fr_khalf;
                        const f32x4_t qn4 = *(const f32x4_t*)(ss + c);
                        f32x4_t q4 = qn4;
                        if (ratio) {
                            const f32x4_t qp4 = *(const f32x4_t*)(ss + 512 + c);
#pragma unroll
                            for (int x = 0; x < 4; ++x) q4[x] = qp4[x] * __builtin_amdgcn_rcpf(qn4[x]);
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
#pragma unroll
                            for (int x = 0; x < 4; ++x) acc[i][j][4 * g + x] *= rp[i] * q4[x];
                        }
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pin(acc[i][0]);
                    pin(acc[i][1]);
                }
            };
            auto rescale_w = [&](const float* ss) {
                const f32x4_t pn4 = *(const f32x4_t*)(ss + wm * 128 + fr_row * 4);
                const f32x4_t pp4 = *(const f32x4_t*)(ss + 512 + wm * 128 + fr_row * 4);
                float rp[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) rp[i] = pp4[i] * __builtin_amdgcn_rcpf(pn4[i]);
                scale_cols(ss, true, rp);
            };
            auto final_scale_w = [&](const float* ss) {  // out of the last stage's units
                const f32x4_t pn4 = *(const f32x4_t*)(ss + wm * 128 + fr_row * 4);
                const float rp[4] = {pn4[0], pn4[1], pn4[2], pn4[3]};
                scale_cols(ss, false, rp);
            };

            // The two wave groups (wm = 0 / 1) run the same stages one slot apart: while one group issues
            // MFMAs the other reads fragments.  Each group has its own copy of the loop, so that every wait
            // is unconditional inside it (the compiler's own wait insertion then sees exactly which DMA is
            // outstanding at each LDS read and adds nothing).  Both copies execute the same number of
            // barriers: 2 + 4 KT.
            //   slot:      1        2        3        4        5 ...
            //   group 0:   A(j,0)   B(j,0)   A(j,1)   B(j,1)   A(j+1,0)
            //   group 1:   B(j-1,1) A(j,0)   B(j,0)   A(j,1)   B(j,1)
            // A = fragment reads of a half-stage (+ fp8 rescale), B = its MFMAs.  Stage j+1 goes into the
            // buffer stage j-1 used, whose last reader is group 1's A(j-1,1) in the slot before slot 1:
            // group 0 issues its share of stage j+1 at the start of A(j,0), group 1 during B(j-1,1), both in
            // slot 1, and both wait for their share in slot 4.
            auto half_a = [&](int s, int half) {
                if (FP8 && !BW_WGRAD && half == 0) {
                    read_scales(SS[s]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                fetch(SP[s], SQ[s], half);
                __builtin_amdgcn_sched_barrier(0);
                if (BW_WGRAD && half == 0) rescale_w(SS[s]);
                else if (FP8 && !MX && half == 0) rescale();  // after the fragment reads in program order: overlaps them
                wait_lgkm0();
            };
            if (NW == 4) {
                // One wave per SIMD and 16x16x32 MFMAs (at equal peak rate they draw less power than the 32x32x16
                // shape, and power sets the sustained clock): the wave tile is 8 x 8 blocks of 16 x 16.  A stage
                // (buffer s = j % 2) is two contraction steps of 32; a step runs the P blocks i = 0..7 in turn against
                // the 8 Q fragments of the step, 64 MFMAs of 16 cycles.  Q fragments are double-buffered by step, P
                // fragments go round a ring of four (P block i + 2 is read while block i runs).
                // A wave alone on its SIMD issues in order, so every other instruction is written into the gap behind
                // one MFMA and issues in its shadow; the 64 of a stage (32 fragment reads, 16 LDS stores of stage
                // j + 1, 16 global loads of stage j + 2 into the registers those stores free) are spread over the
                // 128 gaps, so that the LDS and the address unit of the memory pipe see a steady trickle instead of
                // bursts that fill their queues and stall the wave.
                // One barrier per stage, 12 MFMAs before its end: by then the last fragments of buffer s have
                // arrived and stage j + 1 is complete in buffer s ^ 1; behind it the first fragments of stage j + 1
                // are read while the last MFMAs of stage j run.
                if (KT > 0) {
                    bf16x8_t qr[2][8], pr[4];
                    // row-major operands: one LDS address per buffer and step (lane row and swizzled slot folded in), the
                    // block as an immediate offset
                    typedef __attribute__((address_space(3))) bf16x8_t lds_bf16x8_t;
                    uint32_t vbp[2][2], vbq[2][2];
#pragma unroll
                    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            vbp[sb][ks] = lds_addr(SP[sb]) + (wm * 128 + (lane & 15)) * GG_ROWB + km4[ks];
                            vbq[sb][ks] = lds_addr(SQ[sb]) + (wn * 64 + (lane & 15)) * GG_ROWB + km4[ks];
                            asm volatile("" : "+v"(vbp[sb][ks]), "+v"(vbq[sb][ks]));
                        }
                    auto rdP = [&](int sb, int ks, int i, int slot) __attribute__((always_inline)) {
                        const char* sp = SP[sb] + p4[i];
                        if (P_CMAJ) pr[slot] = lds_read_tr16x8(sp + ks * 16384, sp + ks * 16384 + 2048);
                        else pr[slot] = *(const lds_bf16x8_t*)(uintptr_t)(vbp[sb][ks] + i * 16 * GG_ROWB);
                    };
                    auto rdQ = [&](int sb, int ks, int jq, int set) __attribute__((always_inline)) {
                        const char* sq = SQ[sb] + q4[jq];
                        if (Q_CMAJ) qr[set][jq] = lds_read_tr16x8(sq + ks * 16384, sq + ks * 16384 + 2048);
                        else qr[set][jq] = *(const lds_bf16x8_t*)(uintptr_t)(vbq[sb][ks] + ((jq / 4) * 128 + (jq % 4) * 16) * GG_ROWB);
                    };
                    int g_ent = 0;
                    uint32_t g_tok = 0, g_cnv = 0;
                    auto stage4 = [&](int j, int s) __attribute__((always_inline)) {
                        // (nothing here is conditional: behind the last stage the moves and reads go on, unused)
                        static_assert(NW != 4 || CH == 8, "the gap assignment below is for 16 chunks per stage");
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int jq = 0; jq < 8; ++jq) {
                            const int b = 8 * ks + i, M = 8 * b + jq, off = jq;
                            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc4[i][jq]) : "v"(qr[ks][jq]), "v"(pr[b & 3]));
                            __builtin_amdgcn_sched_barrier(0);
                            if (G_CM) {
                                // gathered operand: the map entries of stage j + 3 are requested early in the stage,
                                // become offsets late in it and are stored to the wave's LDS words ahead of the
                                // stage's barrier; the lanes that will load with them in stage j + 1 read them back
                                // behind the barrier and behind the last load of this stage (read ahead of the
                                // barrier they would make its wait for outstanding LDS reads a real one)
                                if (M == 2) g_ent = gfetch(j + 3);
                                if (M == 100) {
                                    // (opaque up to here: the compiler otherwise starts on the entry, and waits for its
                                    // load together with half of the stage's operand loads, forty MFMAs earlier)
                                    asm volatile("" : "+v"(g_ent));
                                    g_tok = g_tok_of(g_ent);
                                }
                                if (M == 104) g_cnv = g_off_at(g_ent, g_tok, (__builtin_amdgcn_readfirstlane(c_lo + (j + 3) * BKE) + g_row16) < c_hi);
                                if (M == 106) gput(0, g_cnv);
                                if (M == 126) gread(0, 0);
                                if (M == 127) gread(0, 1);
                            }
                            int mv = -1;  // move slot: 2 x chunk = store, 2 x chunk + 1 = load
                            if (b < 8) {
                                if (off == 5) mv = 2 * b;
                                if (off == 7) mv = 2 * b + 1;
                            } else if (b <= 13) {
                                if (off == 3) mv = 16 + 3 * (b - 8);
                                if (off == 5) mv = 17 + 3 * (b - 8);
                                if (off == 7) mv = 18 + 3 * (b - 8);
                            }
                            if (off == 1 && i <= 5) rdP(s, ks, i + 2, (b + 2) & 3);       // two blocks ahead
                            else if (ks == 0 && off == 3) rdQ(s, 1, i, 1);                 // the Q fragments of step 1
                            else if (M == 50) rdP(s, 1, 0, 0);                             // P blocks 0, 1 of step 1
                            else if (M == 57) rdP(s, 1, 1, 1);
                            else if (mv >= 0 && mv < 32 && (mv & 1) == 0) store_one(SP[s ^ 1], SQ[s ^ 1], mv >> 1);
                            else if (mv >= 0 && mv < 32) load_one(j + 2, mv >> 1);
                            else if (M == 115) {  // the last fragments of this buffer have arrived, stage j + 1 has landed
                                wait_lgkm0();
                                stage_barrier();
                            } else if (M == 117) rdP(s ^ 1, 0, 0, 0);                      // behind the barrier: the first
                            else if (M == 125) rdP(s ^ 1, 0, 1, 1);                        // fragments of stage j + 1
                            else if (M == 116) rdQ(s ^ 1, 0, 0, 0);
                            else if (M >= 118 && M <= 124) rdQ(s ^ 1, 0, M - 117, 0);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    };
                    // stage 0 from the registers to buffer 0 (it was requested before the previous tile's epilogue),
                    // stage 1 into the freed registers, the first fragments
#pragma unroll
                    for (int x = 0; x < 2 * CH; ++x) store_one(SP[0], SQ[0], x);
                    if (G_CM) {
                        gread(1, 0);
                        gread(1, 1);
                    }
#pragma unroll
                    for (int x = 0; x < 2 * CH; ++x) load_one(1, x);
                    if (G_CM) {  // the offsets the loads of the first stage of the loop (those of stage 2) will use
                        gread(2, 0);
                        gread(2, 1);
                    }
                    wait_lgkm0();
                    stage_barrier();
#pragma unroll
                    for (int jq = 0; jq < 8; ++jq) rdQ(0, 0, jq, 0);
                    rdP(0, 0, 0, 0);
                    rdP(0, 0, 1, 1);
                    asm volatile("s_nop 7" ::: "memory");  // (likewise: the zeroed accumulators, written by ordinary moves)
                    // (always pairs of stages, an odd count padded with a stage of zeros: with an exit between the two
                    // halves, or an odd stage behind the loop, the register allocator no longer keeps the 256
                    // accumulation registers in place and spills hundreds of them)
                    for (int j = 0; j < KT; j += 2) {
                        stage4(j, 0);
                        stage4(j + 1, 1);
                    }
                    wait_lgkm0();     // (the unused reads and stores of the last stage: landed before the buffers are reused)
                    stage_barrier();  // every wave is past its last fragment read
                    // (the MFMAs are inline assembly: the compiler does not know that their results need 18 more cycles
                    // before ordinary instructions may read them)
                    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
                    // (and every later read of an accumulator depends on a statement behind those nops: volatile asm
                    // statements keep their order, so no read can be scheduled ahead of the wait)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int jq = 0; jq < 8; ++jq) asm volatile("" : "+a"(acc4[i][jq]));
                }
            } else if (KT > 0 && wm == 0) {
                wait_vm0();  // stage 0, issued before the previous tile's epilogue
                stage_barrier();
                // Where group 0 issues its share of stage j+1: at the top of A(j,0), in one run (the first moment the buffer
                // is free), or -- blockwise weight gradient -- between the MFMAs of B(j,0), one slot after group 1 has
                // done the same in its B(j-1,1): the memory pipe then sees 32 KB per slot, each run hidden behind a
                // group's MFMAs (7-9 % per call there; the other variants pay for the address registers that must
                // then live beside the fragments with spills inside the loop, or simply do not gain).
                constexpr bool G0_DMA_IN_B = BW_WGRAD;
                auto stage0 = [&](int j, int s) {
                    if (!G0_DMA_IN_B && j + 1 < KT) {
#pragma unroll
                        for (int x = 0; x < 2 * CH; ++x) issue_one(j + 1, SP[s ^ 1], SQ[s ^ 1], x);
                        if (FP8) issue_scales(j + 1, SS[s ^ 1]);
                    }
                    const bool pf = PF && j + 2 < KT_pf;
                    if (pf) prefetch(j + 2);
                    half_a(s, 0);
                    stage_barrier();
                    mma(G0_DMA_IN_B && j + 1 < KT, j + 1, SP[s ^ 1], SQ[s ^ 1], 0);
                    if (G0_DMA_IN_B && FP8 && j + 1 < KT) issue_scales(j + 1, SS[s ^ 1]);
                    stage_barrier();
                    half_a(s, 1);
                    stage_barrier();
                    mma(false, 0, nullptr, nullptr, 1);
                    if (pf) wait_vm1();  // stage j+1 landed (the warm-up load may still be in flight)
                    else wait_vm0();
                    stage_barrier();
                };
                // (an odd stage count leaves through an exit edge, not a skipped block: the compiler then sees
                // that no path re-enters the loop with a DMA into the buffer about to be read still pending)
                for (int j = 0; j < KT; j += 2) {
                    stage0(j, 0);
                    if (j + 1 >= KT) break;
                    stage0(j + 1, 1);
                }
                stage_barrier();  // group 1's last slot
            } else if (KT > 0) {
                wait_vm0();
                stage_barrier();
                // Where group 1 issues its share of a stage.  Weight gradients: between the MFMAs of its B(j,1), in the
                // same slot as group 0 (the first slot the buffer is free).  Forward and data gradient: one slot later, at
                // the start of its A(j+1,0), like group 0 in its own: the memory pipe then takes the two groups' 32 KB in
                // two slots instead of 64 KB in one, where the second group's issue blocked for ~1200 cycles per
                // stage (per-slot timestamps); 1-2 % per call, the weight gradients lose as much and keep the old place.
                constexpr bool DMA_IN_B = MODE == GG_WGRAD;
                if (DMA_IN_B && KT > 1) {  // slot 1: group 0 reads stage 0, both groups issue their share of stage 1
#pragma unroll
                    for (int x = 0; x < 2 * CH; ++x) issue_one(1, SP[1], SQ[1], x);
                    if (FP8) issue_scales(1, SS[1]);
                }
                if (PF && 2 < KT_pf) prefetch(2);
                stage_barrier();  // group 0's first slot
                auto stage1 = [&](int j, int s) {
                    if (!DMA_IN_B && j + 1 < KT) {
#pragma unroll
                        for (int x = 0; x < 2 * CH; ++x) issue_one(j + 1, SP[s ^ 1], SQ[s ^ 1], x);
                        if (FP8) issue_scales(j + 1, SS[s ^ 1]);
                    }
                    half_a(s, 0);
                    stage_barrier();
                    mma(false, 0, nullptr, nullptr, 0);
                    stage_barrier();
                    half_a(s, 1);
                    if (PF && j + 2 < KT_pf) wait_vm1();  // stage j+1 landed (issued before the warm-up load of stage j+2)
                    else wait_vm0();
                    stage_barrier();
                    mma(DMA_IN_B && j + 2 < KT, j + 2, SP[s], SQ[s], 1);
                    if (DMA_IN_B && FP8 && j + 2 < KT) issue_scales(j + 2, SS[s]);
                    if (PF && j + 3 < KT_pf) prefetch(j + 3);
                    stage_barrier();
                };
                for (int j = 0; j < KT; j += 2) {
                    stage1(j, 0);
                    if (j + 1 >= KT) break;
                    stage1(j + 1, 1);
                }
            }
            if (BW_WGRAD) {
                // the accumulators are in units of the last stage's scales, which sit in that stage's buffer until the
                // next tile's first stage is issued: convert now, and let every wave finish before anyone issues
                if (KT > 0) final_scale_w((const float*)(lds_buf + ((KT - 1) & 1) * BUF_BYTES + GG_STAGE_BYTES));
                wait_lgkm0();
                stage_barrier();
            }
        }

        // ---- next tile: set it up and start its first stage, then write this tile out ----
        // (every wave is past its last LDS read here: the stage loop ends with a barrier after the last
        // fragment reads of both groups)
        const int ep_e = e, ep_i0 = i0, ep_i_end = i_end, ep_j0 = j0, ep_j1 = j1;
        const int ep_part = part_slot, ep_ptile = part_tile;
        // (readfirstlane: the choice between a drawn and a dealt tile otherwise counts as lane-dependent, and with it the
        // whole geometry of the next tile: its operand bases and trip count then live in vector registers and the stage
        // loop of the weight gradient rebuilds its buffer descriptors with 64-bit vector arithmetic between MFMAs)
        const int t_next = __builtin_amdgcn_readfirstlane(dyn ? publish(drawn) : tile_of(n_tile + 1));
        // (four-wave SwiGLU backward: the registers that would hold the next tile's first stage carry the saved
        // pre-activations instead, many units ahead; the next tile is set up behind the output phase)
        constexpr bool LATE_SETUP = NW == 4 && EPI != GG_EPI_STORE;
        if (!LATE_SETUP && t_next < total_tiles) {
            setup_tile(t_next);
            issue_stage0();
        }

        // ---- epilogue ----
        // A lane holds, per 32x32 block, one output row (P index = lane % 32) and four groups of 4 consecutive
        // output columns (Q index = 8 g + 4 (lane / 32) + 0..3): written out directly, a store instruction
        // would touch 32 rows x 16 bytes.  Instead the accumulators go through LDS (fp32), one 32-row block
        // of both wave groups (64 tile rows) per pass, and come back one whole tile row per wave and
        // instruction: lane l owns columns 4 l .. 4 l + 3 of the 256, so every global access is 256-512
        // contiguous bytes.  Buffer 1 is free here: the next tile's stage 0 went to buffer 0, its stage 1 is
        // issued after the barrier that follows this epilogue.
        if constexpr (NW == 4) {
            // Four waves: every wave writes out its own 128 x 128 share (two strips of 64 columns, 128 apart in the
            // tile) with no help from the others, so the output phase has no barrier at all.  A lane holds one row and
            // 4 columns of each 16 x 16 block; to leave as whole cache lines the values take a round trip through a
            // private 16 KB of buffer 1, one 16-row x 64-column unit at a time (row pitch 68 floats: the 16 lanes of a
            // store and of a load hit 64 different banks), and come back as 8 consecutive columns per lane: a store
            // instruction is then 8 rows x 128 contiguous bytes (bf16).  The LDS executes a wave's instructions in
            // order, so a unit is read back right behind its stores; three units rotate, the next one is already on
            // its way through the LDS while the current one is converted and stored.  The SwiGLU is applied to the
            // accumulators before the trip (gate and up of a feature sit in the same lane, blocks jq and jq + 4),
            // its derivative behind it, on the saved pre-activations fetched three units ahead.
            // (Buffer 1 is not written by anyone until every wave has passed the first barrier of the next tile.)
            float* const wst = (float*)(ldsP1 + wave * 16384);
            constexpr int UP = 68, UNIT = 16 * UP;
            // (the lane constants of this phase are formed here, from a lane id the compiler cannot see through: hoisted
            // out of the tile loop they would sit in registers for the whole stage loop, which has none to spare)
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int l16 = ln & 15, lq = ln >> 4;           // accumulator layout: row l16, columns 4 lq + 0..3 of a block
            const int rr = ln >> 3, c8 = (ln & 7) * 8;       // row-major layout: rows rr and rr + 8, columns c8 .. c8 + 7
            const int wr_off = l16 * UP + 4 * lq, rd_off = rr * UP + c8;
            const int row0 = ep_i0 + wm * 128;               // first output row of this wave
            const int col_lo = ep_j0 + wn * 64 + c8, col_hi = ep_j1 + wn * 64 + c8;   // this lane's columns in the two strips
            struct unit_t { f32x4_t v[2][2]; };               // [row group][columns 0..3 / 4..7]
            auto put = [&](int slot, const f32x4_t (&v)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) *(f32x4_t*)(wst + slot * UNIT + wr_off + 16 * j) = v[j];
            };
            auto get = [&](int slot) __attribute__((always_inline)) {
                unit_t u;
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    u.v[g][0] = *(const f32x4_t*)(wst + slot * UNIT + rd_off + 8 * g * UP);
                    u.v[g][1] = *(const f32x4_t*)(wst + slot * UNIT + rd_off + 8 * g * UP + 4);
                }
                return u;
            };
            auto pack8 = [](const f32x4_t& a, const f32x4_t& b) {
                const u32x4_t w = {pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]), pack_bf16(b[2], b[3])};
                return w;
            };
            if constexpr (EPI == GG_EPI_SWIGLU) {
                // units of P block i: gate strip, up strip (the saved pre-activations, if wanted), activation
                bf16_t* const C = (bf16_t*)a.out;
                const bool feat_ok = ep_j0 + wn * 64 + c8 < half_cols;   // (N / 2 need not fill the last tile)
                constexpr int NU = 24;
                // (every accumulator is read once, into ordinary registers, when its block comes up: left to the
                // compiler, the two uses of each value, as pre-activation and in the activation, ended in scratch)
                f32x4_t g4[4], u4[4];
                auto make = [&](int u, f32x4_t (&v)[4]) __attribute__((always_inline)) {
                    const int i = u / 3, t = u % 3;
                    if (t == 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            g4[j] = acc4[i][j];
                            u4[j] = acc4[i][4 + j];
                            asm volatile("" : "+v"(g4[j]), "+v"(u4[j]));
                        }
                    }
                    if (t < 2) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = t == 0 ? g4[j] : u4[j];
                    } else {
                        float pr = 1.0f;
                        if (a.row_prob) {
                            const int r = row0 + 16 * i + l16;
                            pr = r < ep_i_end ? a.row_prob[r] : 0.0f;
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                const float gt = g4[j][x], up = u4[j][x];
                                v[j][x] = pr * (gt * sigmoid_f(gt) * up);
                            }
                            __builtin_amdgcn_sched_barrier(0);   // (four values at a time: interleaving all sixteen chains costs 60 registers)
                        }
                    }
                };
                // (addresses: a wave-uniform row base per unit plus one 32-bit lane offset per tensor and strip; whole
                // 64-bit addresses per lane, formed ahead for all units, are what spilled)
                const uint32_t vz_lo = (uint32_t)(rr * N + col_lo) * 2, vz_hi = (uint32_t)(rr * N + col_hi) * 2;
                const uint32_t va = (uint32_t)(rr * half_cols + col_lo) * 2;
                auto emit = [&](int u, const unit_t& o) __attribute__((always_inline)) {
                    const int i = u / 3, t = u % 3;
                    if (t < 2 && !C) return;
                    if (!feat_ok) return;
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const int rb = row0 + 16 * i + 8 * g;   // wave-uniform
                        if (rb + rr >= ep_i_end) continue;
                        const u32x4_t w = pack8(o.v[g][0], o.v[g][1]);
                        if (t == 2) *(u32x4_t*)((char*)a.out_act + (int64_t)rb * half_cols * 2 + va) = w;
                        else *(u32x4_t*)((char*)C + (int64_t)rb * N * 2 + (t == 0 ? vz_lo : vz_hi)) = w;
                    }
                };
                // (one unit at a time here: with the next unit already on its way, as in the other two output phases, the
                // activation's temporaries no longer fit beside the operands in flight for the next tile)
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    f32x4_t v[4];
                    make(u, v);
                    put(u % 3, v);
                    const unit_t cur = get(u % 3);
                    emit(u, cur);
                    __builtin_amdgcn_sched_barrier(0);   // (units in program order: left free, the scheduler starts them all at once and spills)
                }
            } else if constexpr (EPI == GG_EPI_SWIGLU_BWD) {
                // units: (P block i, strip hf).  dZ[r, c] = dA up s (1 + g (1 - s)), dZ[r, K + c] = dA g s, s = sigmoid(g),
                // from the saved [gate | up]; the row's share of dL/dp, <dA, silu(gate) up> over the wave's 128 columns,
                // is one partial sum per row and wave (added in a fixed order: strip 0 then strip 1, lanes by xor 1, 2, 4)
                bf16_t* const dZ = (bf16_t*)a.out;
#ifndef GG_ZD
#define GG_ZD 5
#endif
                constexpr int NU = 16, ZD = GG_ZD;   // saved pre-activations are requested ZD units ahead
                u32x4_t zg[ZD][2], zu[ZD][2];
                // (addresses: a wave-uniform row base per unit plus a 32-bit lane offset per strip)
                const uint32_t vo_lo = (uint32_t)(rr * 2 * K + col_lo) * 2, vo_hi = (uint32_t)(rr * 2 * K + col_hi) * 2;
                auto zload = [&](int u) __attribute__((always_inline)) {
                    const int i = u / 2, hf = u % 2;
                    const int c = hf == 0 ? col_lo : col_hi;
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const int rb = row0 + 16 * i + 8 * g;   // wave-uniform
                        if (rb + rr < ep_i_end && c < K) {
                            const char* zb = (const char*)a.Zsaved + (int64_t)rb * 2 * K * 2 + (hf == 0 ? vo_lo : vo_hi);
                            zg[u % ZD][g] = *(const u32x4_t*)zb;
                            zu[u % ZD][g] = *(const u32x4_t*)(zb + 2 * K);
                        }
                    }
                };
                float dots[2] = {0.f, 0.f};
                auto emit = [&](int u, const unit_t& o) __attribute__((always_inline)) {
                    const int i = u / 2, hf = u % 2;
                    const int c = hf == 0 ? col_lo : col_hi;
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const int r = row0 + 16 * i + rr + 8 * g;
                        float dot = 0.f;
                        if (r < ep_i_end && c < K) {
                            const u32x4_t zgv = zg[u % ZD][g], zuv = zu[u % ZD][g];
                            const float gt[8] = {bf16_lo(zgv.x), bf16_hi(zgv.x), bf16_lo(zgv.y), bf16_hi(zgv.y),
                                                 bf16_lo(zgv.z), bf16_hi(zgv.z), bf16_lo(zgv.w), bf16_hi(zgv.w)};
                            const float up[8] = {bf16_lo(zuv.x), bf16_hi(zuv.x), bf16_lo(zuv.y), bf16_hi(zuv.y),
                                                 bf16_lo(zuv.z), bf16_hi(zuv.z), bf16_lo(zuv.w), bf16_hi(zuv.w)};
                            const float pr = a.row_prob ? a.row_prob[r] : 1.0f;
                            float dg[8], du[8];
#pragma unroll
                            for (int x = 0; x < 8; ++x) {
                                const float da = o.v[g][x >> 2][x & 3];
                                const float sg = sigmoid_f(gt[x]);
                                dg[x] = pr * da * up[x] * sg * (1.0f + gt[x] * (1.0f - sg));
                                du[x] = pr * da * gt[x] * sg;
                                dot += da * (gt[x] * sg * up[x]);
                            }
                            const u32x4_t wg = {pack_bf16(dg[0], dg[1]), pack_bf16(dg[2], dg[3]), pack_bf16(dg[4], dg[5]), pack_bf16(dg[6], dg[7])};
                            const u32x4_t wu = {pack_bf16(du[0], du[1]), pack_bf16(du[2], du[3]), pack_bf16(du[4], du[5]), pack_bf16(du[6], du[7])};
                            char* ob = (char*)dZ + (int64_t)(r - rr) * 2 * K * 2 + (hf == 0 ? vo_lo : vo_hi);
                            *(u32x4_t*)ob = wg;
                            *(u32x4_t*)(ob + 2 * K) = wu;
                        }
                        __builtin_amdgcn_sched_barrier(0);   // (one row group at a time: keeps the temporaries of the derivative at 8 values)
                        if (a.dprob_part) {
                            dot += __shfl_xor(dot, 1);
                            dot += __shfl_xor(dot, 2);
                            dot += __shfl_xor(dot, 4);
                            dots[g] = hf == 0 ? dot : dots[g] + dot;
                            if (hf == 1 && (ln & 7) == 0 && r < ep_i_end)
                                a.dprob_part[(int64_t)r * (2 * tiles_j) + 2 * (ep_j0 / GG_BN) + wn] = dots[g];
                        }
                    }
                };
#pragma unroll
                for (int u = 0; u < ZD; ++u) zload(u);
                f32x4_t v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = acc4[0][j];
                put(0, v);
                unit_t cur = get(0);
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    unit_t nxt;
                    if (u + 1 < NU) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = acc4[(u + 1) / 2][4 * ((u + 1) % 2) + j];
                        put((u + 1) % 3, v);
                        nxt = get((u + 1) % 3);
                    }
                    emit(u, cur);
                    if (u + ZD < NU) zload(u + ZD);
                    if (u + 1 < NU) cur = nxt;
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // plain store (forward fc2, data gradients, weight gradients, the gate's fp32 logits)
                constexpr int NU = 16;
                const int ld = (MODE == GG_WGRAD) ? K : J;
                constexpr int OB = OUT_F32 ? 4 : 2;
                // (addresses: a wave-uniform row base per unit plus a 32-bit lane offset per strip)
                const uint32_t vo_lo = (uint32_t)(rr * ld + col_lo) * OB, vo_hi = (uint32_t)(rr * ld + col_hi) * OB;
                // (a piece of a split contraction: the whole 256 x 256 tile goes to its slice of the workspace in fp32,
                // row pitch 256; the reduce kernel knows which part of it is inside the matrix)
                float* const part = (SPLITK && ep_part >= 0)
                                        ? a.partials + ((int64_t)ep_part * (tiles_i_w * tiles_j) + ep_ptile) * (GG_BM * GG_BN) +
                                              (wm * 128 + rr) * GG_BN + wn * 64 + c8
                                        : nullptr;
                auto emit = [&](int u, const unit_t& o) __attribute__((always_inline)) {
                    const int i = u / 2, hf = u % 2;
                    if (SPLITK && part) {
#pragma unroll
                        for (int g = 0; g < 2; ++g) {
                            f32x4_t* q = (f32x4_t*)(part + (16 * i + 8 * g) * GG_BN + hf * 128);
                            q[0] = o.v[g][0];
                            q[1] = o.v[g][1];
                        }
                        return;
                    }
                    const int c = hf == 0 ? col_lo : col_hi;
                    if (c >= J) return;
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const int rb = row0 + 16 * i + 8 * g;   // wave-uniform
                        if (rb + rr >= ep_i_end) continue;
                        char* const at = (char*)a.out + ((MODE == GG_WGRAD) ? ((int64_t)ep_e * N + rb) : (int64_t)rb) * ld * OB +
                                         (hf == 0 ? vo_lo : vo_hi);
                        f32x4_t lo = o.v[g][0], hi = o.v[g][1];
                        if (OUT_F32) {
                            f32x4_t* q = (f32x4_t*)at;
                            if (a.accumulate) {
                                lo += q[0];
                                hi += q[1];
                            }
                            q[0] = lo;
                            q[1] = hi;
                        } else {
                            u32x4_t* q = (u32x4_t*)at;
                            if (a.accumulate) {
                                const u32x4_t w = *q;
                                lo += f32x4_t{bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y)};
                                hi += f32x4_t{bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
                            }
                            *q = pack8(lo, hi);
                        }
                    }
                };
                f32x4_t v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = acc4[0][j];
                put(0, v);
                unit_t cur = get(0);
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    unit_t nxt;
                    if (u + 1 < NU) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = acc4[(u + 1) / 2][4 * ((u + 1) % 2) + j];
                        put((u + 1) % 3, v);
                        nxt = get((u + 1) % 3);
                    }
                    emit(u, cur);
                    if (u + 1 < NU) cur = nxt;
                    __builtin_amdgcn_sched_barrier(0);   // (units in program order: left free, the scheduler starts them all at once and spills)
                }
            }
        } else {
            float* const stg = (float*)ldsP1;
            const int cl = lane * 4;                                          // column inside the 256-wide tile
            const int c = cl < 128 ? ep_j0 + cl : ep_j1 + cl - 128;           // output column of this lane
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // SwiGLU backward: the saved pre-activations of the first 8 rows this wave writes in this pass are requested
                // before the accumulators go to LDS, so their latency overlaps the staging and its barrier
                // (bf16 in the eight-wave body only: the one-byte variants have no registers to spare for it)
                constexpr bool Z_EARLY = EPI == GG_EPI_SWIGLU_BWD && !FP8;
                constexpr int ZE = 8;
                u32x2_t zg[ZE], zu[ZE];
                if (Z_EARLY) {
#pragma unroll
                    for (int x8 = 0; x8 < ZE; ++x8) {
                        const int rr = wave * RPW + x8;
                        const int r = ep_i0 + (rr >> 5) * 128 + i * 32 + (rr & 31);
                        if (r < ep_i_end && c < K) {
                            const int64_t zr = (int64_t)r * 2 * K;
                            zg[x8] = *(const u32x2_t*)(a.Zsaved + zr + c);
                            zu[x8] = *(const u32x2_t*)(a.Zsaved + zr + K + c);
                        }
                    }
                }
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int h2 = 0; h2 < NJ; ++h2) {
                        f32x4_t v;
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            v[x] = acc[i][h2][4 * g + x];
                            if (FP8 && !MX && !BW_WGRAD) v[x] *= ps_cur[i] * qs_cur[h2];
                        }
                        *(f32x4_t*)(stg + (wm * 32 + fr_row) * STG_PITCH + blk_col(h2) + 8 * g + 4 * fr_khalf) = v;
                    }
                wait_lgkm0();
                stage_barrier();
                float cmx[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // MXFP8 column copy: column maxima of this wave's rows
                auto out_row = [&](int x8, bool early, bool have, f32x4_t vin) {
                    const int rr = wave * RPW + x8;                           // staged row 0..63
                    const int r = ep_i0 + (rr >> 5) * 128 + i * 32 + (rr & 31);
                    if (r >= ep_i_end) return;                                // wave-uniform
                    const f32x4_t v = have ? vin : *(const f32x4_t*)(stg + rr * STG_PITCH + cl);
                    if (EPI == GG_EPI_SWIGLU) {
                        bf16_t* C = (bf16_t*)a.out;                           // [gate | up] pre-activations
                        if (C && ep_j0 + (cl & 127) < half_cols) {
                            const float t4[4] = {v[0], v[1], v[2], v[3]};
                            st4_bf16(C + (int64_t)r * N + c, t4);
                        }
                    } else if (EPI == GG_EPI_SWIGLU_BWD) {
                        // dZ[r, c] = dA * up * s (1 + g (1 - s)),  dZ[r, K + c] = dA * g * s,  s = sigmoid(g)
                        float dot = 0.f;
                        if (c < K) {
                            bf16_t* dZ = (bf16_t*)a.out;
                            const int64_t zr = (int64_t)r * 2 * K;
                            u32x2_t zgv, zuv;  // (not through the arrays when the row loop is rolled: no runtime index)
                            if (Z_EARLY && early) {
                                zgv = zg[x8 < ZE ? x8 : 0];
                                zuv = zu[x8 < ZE ? x8 : 0];
                            } else {
                                zgv = *(const u32x2_t*)(a.Zsaved + zr + c);
                                zuv = *(const u32x2_t*)(a.Zsaved + zr + K + c);
                            }
                            const float gt[4] = {bf16_lo(zgv.x), bf16_hi(zgv.x), bf16_lo(zgv.y), bf16_hi(zgv.y)};
                            const float up[4] = {bf16_lo(zuv.x), bf16_hi(zuv.x), bf16_lo(zuv.y), bf16_hi(zuv.y)};
                            float dg[4], du[4];
                            const float pr = a.row_prob ? a.row_prob[r] : 1.0f;
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                const float sg = sigmoid_f(gt[x]);
                                dg[x] = pr * v[x] * up[x] * sg * (1.0f + gt[x] * (1.0f - sg));
                                du[x] = pr * v[x] * gt[x] * sg;
                                dot += v[x] * (gt[x] * sg * up[x]);  // <dA, silu(gate) * up>: the row's share of dL/dp
                            }
                            st4_bf16(dZ + zr + c, dg);
                            st4_bf16(dZ + zr + K + c, du);
                            if (F8 == 1 && a.out_q) {
                                // the 32 lanes of a half-wave hold one 1x128 block of the gate part and one of the up
                                // part of this row (K % 128 == 0: a half is inside K or outside as a whole); quantise
                                // the values as they were just stored (bf16), as the stand-alone quantiser would
                                const uint32_t g01 = pack_bf16(dg[0], dg[1]), g23 = pack_bf16(dg[2], dg[3]);
                                const uint32_t u01 = pack_bf16(du[0], du[1]), u23 = pack_bf16(du[2], du[3]);
                                float mg = fmaxf(fmaxf(fabsf(bf16_lo(g01)), fabsf(bf16_hi(g01))), fmaxf(fabsf(bf16_lo(g23)), fabsf(bf16_hi(g23))));
                                float mu = fmaxf(fmaxf(fabsf(bf16_lo(u01)), fabsf(bf16_hi(u01))), fmaxf(fabsf(bf16_lo(u23)), fabsf(bf16_hi(u23))));
#pragma unroll
                                for (int o = 16; o > 0; o >>= 1) {
                                    mg = fmaxf(mg, __shfl_xor(mg, o));
                                    mu = fmaxf(mu, __shfl_xor(mu, o));
                                }
                                const float sgs = block_scale(mg), sus = block_scale(mu);
                                uint32_t* q = (uint32_t*)(a.out_q + zr);
                                q[c >> 2] = cvt4_e4m3(bf16_lo(g01), bf16_hi(g01), bf16_lo(g23), bf16_hi(g23), sgs);
                                q[(K + c) >> 2] = cvt4_e4m3(bf16_lo(u01), bf16_hi(u01), bf16_lo(u23), bf16_hi(u23), sus);
                                if ((lane & 31) == 0) {
                                    float* sc = a.out_q_scale + (int64_t)r * (2 * K / 128);
                                    sc[c >> 7] = sgs;
                                    sc[(K + c) >> 7] = sus;
                                }
                            }
                            if (MXQ && a.out_q) {
                                // MXFP8 copies of dZ: the values as stored (bf16) replace the row's consumed staging
                                // words -- gate part at byte 8 * lane, up part 512 bytes further, i.e. the row in column
                                // order -- and are quantised 16 columns per lane once the whole pass is there (below)
                                const uint32_t g01 = pack_bf16(dg[0], dg[1]), g23 = pack_bf16(dg[2], dg[3]);
                                const uint32_t u01 = pack_bf16(du[0], du[1]), u23 = pack_bf16(du[2], du[3]);
                                uint32_t* srow = (uint32_t*)(stg + rr * STG_PITCH);
                                *(u32x2_t*)(srow + 2 * lane) = u32x2_t{g01, g23};
                                *(u32x2_t*)(srow + 128 + 2 * lane) = u32x2_t{u01, u23};
                                if (a.out_qc) {
                                    cmx[0] = fmaxf(cmx[0], fabsf(bf16_lo(g01))); cmx[1] = fmaxf(cmx[1], fabsf(bf16_hi(g01)));
                                    cmx[2] = fmaxf(cmx[2], fabsf(bf16_lo(g23))); cmx[3] = fmaxf(cmx[3], fabsf(bf16_hi(g23)));
                                    cmx[4] = fmaxf(cmx[4], fabsf(bf16_lo(u01))); cmx[5] = fmaxf(cmx[5], fabsf(bf16_hi(u01)));
                                    cmx[6] = fmaxf(cmx[6], fabsf(bf16_lo(u23))); cmx[7] = fmaxf(cmx[7], fabsf(bf16_hi(u23)));
                                }
                            }
                        }
                        if (a.dprob_part) {  // a half-wave holds 128 of the 256 columns of this row and tile: two partial sums
#pragma unroll
                            for (int o = 16; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
                            if ((lane & 31) == 0) a.dprob_part[(int64_t)r * (2 * tiles_j) + 2 * (ep_j0 / GG_BN) + (lane >> 5)] = dot;
                        }
                    } else if (c < J) {
                        const int64_t base = (MODE == GG_WGRAD) ? ((int64_t)ep_e * N + r) * K : (int64_t)r * J;
                        if (OUT_F32) {
                            f32x4_t* o = (f32x4_t*)((float*)a.out + base + c);
                            f32x4_t w = v;
                            if (a.accumulate) w += *o;
                            *o = w;
                        } else {
                            bf16_t* o = (bf16_t*)a.out + base + c;
                            float t4[4] = {v[0], v[1], v[2], v[3]};
                            if (a.accumulate) {
                                float old[4];
                                ld4_bf16(o, old);
#pragma unroll
                                for (int x = 0; x < 4; ++x) t4[x] += old[x];
                            }
                            st4_bf16(o, t4);
                        }
                    }
                };
                // (the pass loop must unroll completely: the accumulators are indexed by it.  The compiler gives up on
                // that above a size limit, so the row loops of the one-byte SwiGLU variants stay rolled; their plain-store
                // variants are small enough for the batches of 8 rows: 0-2 % per call)
                const f32x4_t none = {0.f, 0.f, 0.f, 0.f};
                if (FP8 && EPI != GG_EPI_STORE) {
#pragma unroll 1
                    for (int x8 = 0; x8 < RPW; ++x8) out_row(x8, false, false, none);
                } else {
                    // rows in batches of 8: all the staged values first (unconditional LDS reads, nothing between them),
                    // then the rows; read inside the rows, every LDS latency would be taken in turn
#pragma unroll
                    for (int x0 = 0; x0 < RPW; x0 += 8) {
                        f32x4_t vb[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) vb[u] = *(const f32x4_t*)(stg + (wave * RPW + x0 + u) * STG_PITCH + cl);
                        // plain store of 8 whole rows (the common case): no test or branch per row, one address chain
                        const int rr0 = wave * RPW + x0;
                        const int r0 = ep_i0 + (rr0 >> 5) * 128 + i * 32 + (rr0 & 31);  // the 8 rows are consecutive
                        if (EPI == GG_EPI_STORE && !a.accumulate && r0 + 8 <= ep_i_end) {
                            if (c < J) {
                                const int64_t ld = (MODE == GG_WGRAD) ? K : J;
                                const int64_t base = (MODE == GG_WGRAD) ? ((int64_t)ep_e * N + r0) * K : (int64_t)r0 * J;
                                if (OUT_F32) {
                                    float* o = (float*)a.out + base + c;
#pragma unroll
                                    for (int u = 0; u < 8; ++u) *(f32x4_t*)(o + u * ld) = vb[u];
                                } else {
                                    bf16_t* o = (bf16_t*)a.out + base + c;
#pragma unroll
                                    for (int u = 0; u < 8; ++u) {
                                        const float t4[4] = {vb[u][0], vb[u][1], vb[u][2], vb[u][3]};
                                        st4_bf16(o + u * ld, t4);
                                    }
                                }
                            }
                        } else {
#pragma unroll
                            for (int u = 0; u < 8; ++u) out_row(x0 + u, Z_EARLY && x0 == 0, true, vb[u]);
                        }
                    }
                }
                if (EPI == GG_EPI_SWIGLU) {
                    // activation: a lane pairs gate and up of 4 features; two tile rows per instruction
                    const int fl = (lane & 31) * 4;
#pragma unroll(FP8 ? 1 : 4)
                    for (int x4 = 0; x4 < RPW / 2; ++x4) {
                        const int rr = wave * RPW + 2 * x4 + (lane >> 5);
                        const int r = ep_i0 + (rr >> 5) * 128 + i * 32 + (rr & 31);
                        if (r < ep_i_end && ep_j0 + fl < half_cols) {  // uniform over a half-wave when N % 256 == 0 (fp8)
                            const f32x4_t gt = *(const f32x4_t*)(stg + rr * STG_PITCH + fl);
                            const f32x4_t up = *(const f32x4_t*)(stg + rr * STG_PITCH + 128 + fl);
                            float act[4];
                            const float pr = a.row_prob ? a.row_prob[r] : 1.0f;
#pragma unroll
                            for (int x = 0; x < 4; ++x) act[x] = pr * (gt[x] * sigmoid_f(gt[x]) * up[x]);
                            st4_bf16(a.out_act + (int64_t)r * half_cols + ep_j0 + fl, act);
                            if (F8 == 1 && a.out_q) {
                                // the half-wave holds the row's 128 activations of this tile = one 1x128 block of fc2's
                                // input: quantise the values as stored (bf16), as the stand-alone quantiser would
                                const uint32_t a01 = pack_bf16(act[0], act[1]), a23 = pack_bf16(act[2], act[3]);
                                float m = fmaxf(fmaxf(fabsf(bf16_lo(a01)), fabsf(bf16_hi(a01))), fmaxf(fabsf(bf16_lo(a23)), fabsf(bf16_hi(a23))));
#pragma unroll
                                for (int o = 16; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
                                const float sa = block_scale(m);
                                ((uint32_t*)(a.out_q + (int64_t)r * half_cols))[(ep_j0 + fl) >> 2] =
                                    cvt4_e4m3(bf16_lo(a01), bf16_hi(a01), bf16_lo(a23), bf16_hi(a23), sa);
                                if ((lane & 31) == 0) a.out_q_scale[(int64_t)r * (half_cols / 128) + ep_j0 / 128] = sa;
                            }
                            if (MXQ && a.out_q) {
                                // MXFP8 copies of A: the values as stored (bf16) go over the row's consumed gate words, in
                                // feature order, and are quantised 16 features per lane once the pass is complete (below)
                                const uint32_t a01 = pack_bf16(act[0], act[1]), a23 = pack_bf16(act[2], act[3]);
                                *(u32x2_t*)((uint32_t*)(stg + rr * STG_PITCH) + 2 * (lane & 31)) = u32x2_t{a01, a23};
                                if (a.out_qc) {
                                    cmx[0] = fmaxf(cmx[0], fabsf(bf16_lo(a01))); cmx[1] = fmaxf(cmx[1], fabsf(bf16_hi(a01)));
                                    cmx[2] = fmaxf(cmx[2], fabsf(bf16_lo(a23))); cmx[3] = fmaxf(cmx[3], fabsf(bf16_hi(a23)));
                                }
                            }
                        }
                    }
                }
                // MXFP8 quantising epilogue (Sec. 5.4.2), second half.  The pass's rows of this wave (eight) now lie in
                // the staging area as bf16 in column order.  A lane takes 16 consecutive columns of one row (16 codes =
                // one 16-byte store): the 1x32 copy needs the maximum of two neighbouring lanes; for the 32x1 copy the
                // 32 rows of a block are this pass's rows of one tile half, eight per wave, so the four waves of the
                // half first exchange their column maxima through LDS and each keeps the exponents of its columns as a
                // byte table of its own.
                if (MXQ && a.out_q) {
                    const bool colq = a.out_qc != nullptr;                     // uniform over the grid
                    const int hb = wave & 4;                                   // first wave of this wave's tile half
                    const int r_blk = ep_i0 + (wave >> 2) * 128 + i * 32;      // first row of the 32-row block
                    constexpr int HALVES = EPI == GG_EPI_SWIGLU ? 1 : 2;       // column parts per row (A: one; dZ: gate, up)
                    const int width = HALVES == 1 ? half_cols : 2 * K;         // row length of the quantised tensor
                    if (colq) {
                        if (EPI == GG_EPI_SWIGLU) {
#pragma unroll
                            for (int x = 0; x < 4; ++x) cmx[x] = fmaxf(cmx[x], __shfl_xor(cmx[x], 32));  // the two rows of a lane pair
                            if (lane < 32) *(f32x4_t*)(qx + (wave * 64 + lane) * 4) = f32x4_t{cmx[0], cmx[1], cmx[2], cmx[3]};
                        } else {
                            // (maxima of bf16 values are bf16 values: packed without loss)
                            *(u32x4_t*)(qx + (wave * 64 + lane) * 4) = u32x4_t{pack_bf16(cmx[0], cmx[1]), pack_bf16(cmx[2], cmx[3]),
                                                                                pack_bf16(cmx[4], cmx[5]), pack_bf16(cmx[6], cmx[7])};
                        }
                        wait_lgkm0();
                        stage_barrier();
                        int ex[8];
                        if (EPI == GG_EPI_SWIGLU) {
                            f32x4_t m = *(const f32x4_t*)(qx + (hb * 64 + (lane & 31)) * 4);
#pragma unroll
                            for (int w2 = 1; w2 < 4; ++w2) {
                                const f32x4_t o = *(const f32x4_t*)(qx + ((hb + w2) * 64 + (lane & 31)) * 4);
#pragma unroll
                                for (int x = 0; x < 4; ++x) m[x] = fmaxf(m[x], o[x]);
                            }
#pragma unroll
                            for (int x = 0; x < 4; ++x) ex[x] = mx_exponent(m[x]);
                        } else {
                            u32x4_t pm = *(const u32x4_t*)(qx + (hb * 64 + lane) * 4);
                            float m[8] = {bf16_lo(pm.x), bf16_hi(pm.x), bf16_lo(pm.y), bf16_hi(pm.y),
                                          bf16_lo(pm.z), bf16_hi(pm.z), bf16_lo(pm.w), bf16_hi(pm.w)};
#pragma unroll
                            for (int w2 = 1; w2 < 4; ++w2) {
                                const u32x4_t o = *(const u32x4_t*)(qx + ((hb + w2) * 64 + lane) * 4);
                                const float of[8] = {bf16_lo(o.x), bf16_hi(o.x), bf16_lo(o.y), bf16_hi(o.y),
                                                     bf16_lo(o.z), bf16_hi(o.z), bf16_lo(o.w), bf16_hi(o.w)};
#pragma unroll
                                for (int x = 0; x < 8; ++x) m[x] = fmaxf(m[x], of[x]);
                            }
#pragma unroll
                            for (int x = 0; x < 8; ++x) ex[x] = mx_exponent(m[x]);
                        }
                        // the half's table of column scales 2^e (part p of the row at 256 p; its four waves write the same
                        // values and each reads behind its own writes), and, from the first wave of each half, the E8M0
                        // bytes: byte i of the dword of (128-row group, column)
                        float* qh = qe + (wave >> 2) * 512;
#pragma unroll
                        for (int p2 = 0; p2 < HALVES; ++p2) {
                            const int* e4 = ex + 4 * p2;
                            const f32x4_t w = {mx_scale_f32(e4[0]), mx_scale_f32(e4[1]), mx_scale_f32(e4[2]), mx_scale_f32(e4[3])};
                            if (HALVES == 2 || lane < 32) *(f32x4_t*)(qh + 256 * p2 + 4 * (HALVES == 2 ? lane : (lane & 31))) = w;
                        }
                        if ((wave & 3) == 0 && r_blk < ep_i_end) {
                            if (EPI == GG_EPI_SWIGLU) {
                                if (lane < 32) {
                                    uint8_t* sc = a.out_qc_e8 + ((int64_t)(r_blk >> 7) * width + ep_j0 + lane * 4) * 4 + i;
#pragma unroll
                                    for (int x = 0; x < 4; ++x) sc[4 * x] = (uint8_t)(ex[x] + 127);
                                }
                            } else if (c < K) {
                                uint8_t* sc = a.out_qc_e8 + ((int64_t)(r_blk >> 7) * width + c) * 4 + i;
#pragma unroll
                                for (int x = 0; x < 4; ++x) {
                                    sc[4 * x] = (uint8_t)(ex[x] + 127);
                                    sc[4 * (K + x)] = (uint8_t)(ex[4 + x] + 127);
                                }
                            }
                        }
                    }
                    const int row = lane >> 3, rr = wave * RPW + row;             // RPW = 8 rows per wave and pass
                    const int r = r_blk + (rr & 31);
#pragma unroll
                    for (int t2 = 0; t2 < 2 * HALVES; ++t2) {
                        const int p2 = t2 >> 1;                                    // part of the row (dZ: gate / up)
                        const int sc16 = ((lane & 7) + 8 * (t2 & 1)) * 16;         // first of the lane's 16 columns in the tile
                        if (HALVES == 1 && t2 == 1) break;                         // (A: 128 columns per tile row, one task)
                        const int colt = HALVES == 1 ? ep_j0 + sc16 : (sc16 < 128 ? ep_j0 + sc16 : ep_j1 + sc16 - 128);
                        if (r >= ep_i_end || colt >= (HALVES == 1 ? half_cols : K)) continue;
                        const u32x4_t* sp = (const u32x4_t*)((const uint32_t*)(stg + rr * STG_PITCH) + 128 * p2 + sc16 / 2);
                        const u32x4_t v0 = sp[0], v1 = sp[1];
                        uint32_t mb = 0;
                        mb = bf16_absmax_bits(mb, v0.x); mb = bf16_absmax_bits(mb, v0.y); mb = bf16_absmax_bits(mb, v0.z);
                        mb = bf16_absmax_bits(mb, v0.w); mb = bf16_absmax_bits(mb, v1.x); mb = bf16_absmax_bits(mb, v1.y);
                        mb = bf16_absmax_bits(mb, v1.z); mb = bf16_absmax_bits(mb, v1.w);
                        float m = bf16_absmax_finish(mb);
                        m = fmaxf(m, __shfl_xor(m, 1));                            // a 1x32 block = two neighbouring lanes
                        const int er = mx_exponent(m);
                        const float sr = mx_scale_f32(er);
                        const int64_t at = (int64_t)r * width + (int64_t)p2 * K + colt;
                        *(u32x4_t*)(a.out_q + at) = u32x4_t{mx_cvt4_bf16(v0.x, v0.y, sr), mx_cvt4_bf16(v0.z, v0.w, sr),
                                                            mx_cvt4_bf16(v1.x, v1.y, sr), mx_cvt4_bf16(v1.z, v1.w, sr)};
                        if ((lane & 1) == 0) a.out_q_e8[at >> 5] = (uint8_t)(er + 127);
                        if (colq) {
                            const f32x4_t* sp4 = (const f32x4_t*)(qe + (wave >> 2) * 512 + 256 * p2 + sc16);
                            const f32x4_t s0 = sp4[0], s1 = sp4[1], s2 = sp4[2], s3 = sp4[3];
                            *(u32x4_t*)(a.out_qc + at) = u32x4_t{mx_cvt4_bf16_each(v0.x, v0.y, s0[0], s0[1], s0[2], s0[3]),
                                                                 mx_cvt4_bf16_each(v0.z, v0.w, s1[0], s1[1], s1[2], s1[3]),
                                                                 mx_cvt4_bf16_each(v1.x, v1.y, s2[0], s2[1], s2[2], s2[3]),
                                                                 mx_cvt4_bf16_each(v1.z, v1.w, s3[0], s3[1], s3[2], s3[3])};
                        }
                    }
                }
                wait_lgkm0();
                stage_barrier();  // the staging rows are rewritten by the next pass (or the next tile's stage 1)
            }
        }
        if (LATE_SETUP && t_next < total_tiles) {
            setup_tile(t_next);
            issue_stage0();
        }
        t = t_next;
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
    if (dt == MOE_F32) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: fp32 operands are not supported", who);
    if (dt != MOE_BF16 && dt != MOE_FP8_E4M3 && dt != MOE_MXFP8_E4M3) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: bad dtype", who);
    if (dt != MOE_BF16 && (N % 128 || K % 128))
        MOE_FAIL(ctx, MOE_ERR_ARG, "%s: fp8 needs N and K to be multiples of 128 (block scales)", who);
    if (N % 8 || K % 8) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: N and K must be multiples of 8 (16-byte rows)", who);
    // (the kernels advance their operands by 128 rows of N or K elements per stage in 32-bit arithmetic, and address
    // one expert's weights with 32-bit offsets)
    if (N > (1 << 24) || K > (1 << 24) || (int64_t)N * K * 2 > 0xffffffffLL)
        MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: N, K up to 2^24 and N*K up to 2^31 elements per expert", who);
    return MOE_OK;
}

static gg_args gg_make(moe_ctx* ctx, const void* P, const void* Q, const int32_t* offsets, int E, int N, int K,
                       int64_t Rcap, void* out) {
    gg_args a;
    memset(&a, 0, sizeof(a));
    a.P = P;
    a.Q = Q;
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

#define MOE_WS_TILE_COUNTER 48  // byte offset of the wgrad tile counter in the reserved head of the workspace
#define MOE_WS_SPLIT_INFO 64    // ... of the list of split experts (1 + 3 * GG_MAX_SPLIT_EXPERTS ints)

// Second step of a weight gradient with a split contraction: dW tile = sum of its pieces' partial tiles, piece 0
// first, then the ordinary output step (type, accumulate, matrix edges).  grid = (tiles per expert,
// GG_MAX_SPLIT_EXPERTS); the list of split experts was written by the first kernel.
template <bool OUT_F32>
__global__ __launch_bounds__(256) void gg_split_reduce_kernel(const float* __restrict__ partials, const int* __restrict__ info,
                                                              int N, int K, int accumulate, void* __restrict__ out) {
    const int j = blockIdx.y;
    if (j >= info[0]) return;
    const int e = info[1 + 3 * j], pieces = info[2 + 3 * j], slice0 = info[3 + 3 * j];
    const int tiles_j = (K + GG_BN - 1) / GG_BN, tiles_i = (N + GG_BM - 1) / GG_BM, tpe = tiles_i * tiles_j;
    const int u = blockIdx.x;
    // the tile order of the first kernel: bands of GG_BAND row tiles, column-major inside a band
    const int band_sz = GG_BAND * tiles_j, band = u / band_sz, in_band = u - band * band_sz;
    const int band_rows = min(GG_BAND, tiles_i - band * GG_BAND);
    const int ti = band * GG_BAND + in_band % band_rows, tj = in_band / band_rows;
    const int c = (threadIdx.x & 63) * 4, r0 = threadIdx.x >> 6;
    const int col = tj * GG_BN + c;
    if (col >= K) return;
    for (int r = r0; r < GG_BM; r += 4) {
        const int row = ti * GG_BM + r;
        if (row >= N) break;
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < pieces; ++p)
            v += *(const f32x4_t*)(partials + ((int64_t)(slice0 + p) * tpe + u) * (GG_BM * GG_BN) + r * GG_BN + c);
        const int64_t at = ((int64_t)e * N + row) * K + col;
        if (OUT_F32) {
            f32x4_t* o = (f32x4_t*)((float*)out + at);
            if (accumulate) v += *o;
            *o = v;
        } else {
            bf16_t* o = (bf16_t*)out + at;
            float t4[4] = {v[0], v[1], v[2], v[3]};
            if (accumulate) {
                float old[4];
                ld4_bf16(o, old);
#pragma unroll
                for (int x = 0; x < 4; ++x) t4[x] += old[x];
            }
            st4_bf16(o, t4);
        }
    }
}

#ifndef GG_BF16_NW
#define GG_BF16_NW 4  // waves per workgroup of the bf16 variants (see the kernel)
#endif
#define GG_NW_OF(MODE, FP8) ((FP8) ? 8 : GG_BF16_NW)
#define GG_LAUNCH(MODE, EPI, F32, FP8)                                                                          \
    hipLaunchKernelGGL((gg_kernel<MODE, EPI, F32, FP8, GG_NW_OF(MODE, FP8)>),                                   \
                       dim3(ctx->num_cu > 0 ? ctx->num_cu : 256), dim3(GG_NW_OF(MODE, FP8) * 64),               \
                       0, (hipStream_t)stream, a)

// the four-wave bf16 kernel with operand P (GATH = 1) or Q (2) fetched through the row map
#define GG_LAUNCH_G(MODE, EPI, F32, GATH)                                                                       \
    hipLaunchKernelGGL((gg_kernel<MODE, EPI, F32, 0, 4, GATH>), dim3(ctx->num_cu > 0 ? ctx->num_cu : 256),      \
                       dim3(256), 0, (hipStream_t)stream, a)

// Arguments of a gathered operand: `ld` = its row length.  Limits: every byte offset into the unpermuted tensor, and
// GG_NO_ROW plus a column offset, must fit 32 bits; the map is read through a 32-bit record count; the division by k
// is a multiplication: with m = ceil(2^31 / k), (2 s + 1) m / 2^32 = (s + 1/2) / k + (2 s + 1) e / 2^32, 0 <= e < 1,
// whose first term lies at least 1 / (2 k) below the next integer, so the floor is s / k while (2 s + 1) 2 k < 2^32.
static moe_status gg_gather_args(moe_ctx* ctx, const char* who, gg_args& a, int T, const int32_t* src_of, int k, int ld,
                                 int64_t Rcap) {
    if (!src_of) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: src_of is NULL", who);
    if (T < 1 || k < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: need T >= 1 and k >= 1", who);
    if ((int64_t)T * ld * 2 > 0xE0000000LL || Rcap >= (1LL << 29) || (int64_t)T * k * k >= (1LL << 30))
        MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: T=%d rows of %d elements (or T*k*k, or Rcap) exceed the 32-bit offsets of the gathered fetch", who, T, ld);
    a.g_src_of = src_of;
    a.g_k = k;
    a.g_T = T;
    a.g_magic = (uint32_t)(((1ULL << 31) + (uint64_t)k - 1) / (uint64_t)k);
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_fwd_gather(moe_ctx* ctx, void* stream, const void* X, int T, const int32_t* src_of,
                                                  int k, const void* B, const int32_t* offsets, int E, int N, int K,
                                                  int64_t Rcap, moe_epilogue epi, const float* row_prob, void* C,
                                                  void* C_act) {
    if (!ctx) return MOE_ERR_ARG;
    if (GG_BF16_NW != 4) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd_gather: needs the four-wave bf16 body");
    if (row_prob && epi != MOE_EPI_SWIGLU)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_gather: row weights go with the SwiGLU epilogue");
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_fwd_gather", X, B, offsets, E, N, K, Rcap, MOE_BF16);
    if (st != MOE_OK) return st;
    if (epi == MOE_EPI_SWIGLU) {
        if (!C_act) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_gather: SWIGLU needs C_act");
        if (N % 16) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_gather: SWIGLU needs N %% 16 == 0");
    } else if (epi == MOE_EPI_NONE) {
        if (!C) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_gather: C is NULL");
    } else {
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_gather: bad epilogue");
    }
    if (K % 64) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd_gather: K=%d must be a multiple of 64", K);
    gg_args a = gg_make(ctx, X, B, offsets, E, N, K, Rcap, C);
    st = gg_gather_args(ctx, "moe_grouped_gemm_fwd_gather", a, T, src_of, k, K, Rcap);
    if (st != MOE_OK) return st;
    a.out_act = (bf16_t*)C_act;
    a.row_prob = row_prob;
    if (epi == MOE_EPI_SWIGLU) GG_LAUNCH_G(GG_FWD, GG_EPI_SWIGLU, false, 1);
    else GG_LAUNCH_G(GG_FWD, GG_EPI_STORE, false, 1);
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<fwd, gather>");
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_fwd(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                           const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                           moe_dtype dt, moe_epilogue epi,
                                           const float* a_scale, const float* b_scale,
                                           void* C, void* C_act) {
    return moe_grouped_gemm_fwd_weighted(ctx, stream, A, B, offsets, E, N, K, Rcap, dt, epi, a_scale, b_scale, nullptr,
                                         C, C_act);
}

extern "C" moe_status moe_grouped_gemm_fwd_weighted(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                                    const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                    moe_dtype dt, moe_epilogue epi,
                                                    const float* a_scale, const float* b_scale,
                                                    const float* row_prob, void* C, void* C_act) {
    return moe_grouped_gemm_fwd_quant(ctx, stream, A, B, offsets, E, N, K, Rcap, dt, epi, a_scale, b_scale, row_prob, C,
                                      C_act, nullptr, nullptr);
}

// the MXFP8 outputs of a quantising epilogue: 1x32 copy (q_row, e8_row), optional 32x1 copy (q_col, e8_col)
struct gg_mx_out {
    void* q_row;
    uint8_t* e8_row;
    void* q_col;
    uint8_t* e8_col;
};
static moe_status gg_mx_out_check(moe_ctx* ctx, const char* who, const gg_mx_out& o, moe_dtype dt, bool epi_ok, int64_t Rcap) {
    if (!o.q_row || !o.e8_row) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: q_row and e8_row are required", who);
    if ((o.q_col == nullptr) != (o.e8_col == nullptr)) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: q_col and e8_col go together", who);
    if (dt != MOE_MXFP8_E4M3 || !epi_ok)
        MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "%s: needs dt = MOE_MXFP8_E4M3 and the SwiGLU (forward) / SwiGLU-backward (Z_saved) epilogue", who);
    if (o.q_col && Rcap % 128) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: the 32x1 copy needs Rcap %% 128 == 0 (and 128-aligned experts)", who);
    return MOE_OK;
}

static moe_status gg_fwd_all(moe_ctx* ctx, void* stream, const void* A, const void* B, const int32_t* offsets, int E, int N,
                             int K, int64_t Rcap, moe_dtype dt, moe_epilogue epi, const float* a_scale, const float* b_scale,
                             const float* row_prob, void* C, void* C_act, void* act_q, float* act_q_scale,
                             const gg_mx_out* mxo);

extern "C" moe_status moe_grouped_gemm_fwd_quant(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                                 const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                 moe_dtype dt, moe_epilogue epi,
                                                 const float* a_scale, const float* b_scale,
                                                 const float* row_prob, void* C, void* C_act,
                                                 void* act_q, float* act_q_scale) {
    return gg_fwd_all(ctx, stream, A, B, offsets, E, N, K, Rcap, dt, epi, a_scale, b_scale, row_prob, C, C_act, act_q,
                      act_q_scale, nullptr);
}

extern "C" moe_status moe_grouped_gemm_fwd_quant_mx(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                                    const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                    const void* a_scale, const void* b_scale, const float* row_prob,
                                                    void* C, void* C_act, void* act_q_row, uint8_t* act_e8_row,
                                                    void* act_q_col, uint8_t* act_e8_col) {
    if (!ctx) return MOE_ERR_ARG;
    const gg_mx_out o = {act_q_row, act_e8_row, act_q_col, act_e8_col};
    return gg_fwd_all(ctx, stream, A, B, offsets, E, N, K, Rcap, MOE_MXFP8_E4M3, MOE_EPI_SWIGLU, (const float*)a_scale,
                      (const float*)b_scale, row_prob, C, C_act, nullptr, nullptr, &o);
}

static moe_status gg_fwd_all(moe_ctx* ctx, void* stream, const void* A, const void* B, const int32_t* offsets, int E, int N,
                             int K, int64_t Rcap, moe_dtype dt, moe_epilogue epi, const float* a_scale, const float* b_scale,
                             const float* row_prob, void* C, void* C_act, void* act_q, float* act_q_scale,
                             const gg_mx_out* mxo) {
    if (!ctx) return MOE_ERR_ARG;
    if ((act_q == nullptr) != (act_q_scale == nullptr))
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_quant: act_q and act_q_scale go together");
    if (act_q && (dt != MOE_FP8_E4M3 || epi != MOE_EPI_SWIGLU))
        MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd_quant: quantised output needs dt = MOE_FP8_E4M3 and the SwiGLU epilogue");
    if (mxo) {
        moe_status stq = gg_mx_out_check(ctx, "moe_grouped_gemm_fwd_quant_mx", *mxo, dt, epi == MOE_EPI_SWIGLU, Rcap);
        if (stq != MOE_OK) return stq;
    }
    if (dt == MOE_F32) {  // all-fp32 path (gemm_f32.hip)
        if (!A || !B || !offsets) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: NULL pointer");
        if (E < 1 || N < 1 || K < 1 || Rcap < 1 || Rcap > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: bad sizes");
        if (epi == MOE_EPI_SWIGLU ? (!C_act || N % 2) : (epi != MOE_EPI_NONE || !C || row_prob))
            MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd(f32): bad epilogue arguments");
        return moe_gg_f32_fwd(ctx, (hipStream_t)stream, A, B, offsets, E, N, K, Rcap, epi == MOE_EPI_SWIGLU, row_prob, C, C_act);
    }
    if (row_prob && epi != MOE_EPI_SWIGLU)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd_weighted: row weights go with the SwiGLU epilogue");
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_fwd", A, B, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    if (epi == MOE_EPI_SWIGLU) {
        if (!C_act) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: SWIGLU needs C_act");
        if (N % 16) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: SWIGLU needs N %% 16 == 0");
        if (dt != MOE_BF16 && N % 256) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: fp8 SWIGLU needs N %% 256 == 0");
    } else if (epi == MOE_EPI_NONE) {
        if (!C) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: C is NULL");
    } else {
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: bad epilogue");
    }
    const bool fp8 = dt != MOE_BF16, mx = dt == MOE_MXFP8_E4M3;
    if (fp8 && (!a_scale || !b_scale)) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd: fp8 needs a_scale and b_scale");
    if (!fp8 && K % 64) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_fwd: K=%d must be a multiple of 64", K);
    gg_args a = gg_make(ctx, A, B, offsets, E, N, K, Rcap, C);
    a.out_act = (bf16_t*)C_act;
    a.p_scale = a_scale;
    a.q_scale = b_scale;
    a.row_prob = row_prob;
    a.out_q = (uint8_t*)act_q;
    a.out_q_scale = act_q_scale;
    if (mxo) {
        a.out_q = (uint8_t*)mxo->q_row;
        a.out_q_e8 = mxo->e8_row;
        a.out_qc = (uint8_t*)mxo->q_col;
        a.out_qc_e8 = mxo->e8_col;
    }
    if (epi == MOE_EPI_SWIGLU) {
        if (mx) GG_LAUNCH(GG_FWD, GG_EPI_SWIGLU, false, 2);
        else if (fp8) GG_LAUNCH(GG_FWD, GG_EPI_SWIGLU, false, 1);
        else GG_LAUNCH(GG_FWD, GG_EPI_SWIGLU, false, 0);
    } else {
        if (mx) GG_LAUNCH(GG_FWD, GG_EPI_STORE, false, 2);
        else if (fp8) GG_LAUNCH(GG_FWD, GG_EPI_STORE, false, 1);
        else GG_LAUNCH(GG_FWD, GG_EPI_STORE, false, 0);
    }
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<fwd>");
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_dgrad_gather(moe_ctx* ctx, void* stream, const void* G, int T, const int32_t* src_of,
                                                    int k, const void* B, const int32_t* offsets, int E, int N, int K,
                                                    int64_t Rcap, const void* Z_saved, const float* row_prob, void* dA,
                                                    float* dprob_part) {
    if (!ctx) return MOE_ERR_ARG;
    if (GG_BF16_NW != 4) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad_gather: needs the four-wave bf16 body");
    if ((row_prob || dprob_part) && !Z_saved)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad_gather: row weights / dprob_part need Z_saved");
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_dgrad_gather", G, B, offsets, E, N, K, Rcap, MOE_BF16);
    if (st != MOE_OK) return st;
    if (!dA) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad_gather: dA is NULL");
    if (N % 64) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad_gather: N=%d must be a multiple of 64", N);
    gg_args a = gg_make(ctx, G, B, offsets, E, N, K, Rcap, dA);
    st = gg_gather_args(ctx, "moe_grouped_gemm_dgrad_gather", a, T, src_of, k, N, Rcap);
    if (st != MOE_OK) return st;
    a.Zsaved = (const bf16_t*)Z_saved;
    a.row_prob = row_prob;
    a.dprob_part = dprob_part;
    if (Z_saved) GG_LAUNCH_G(GG_DGRAD, GG_EPI_SWIGLU_BWD, false, 1);
    else GG_LAUNCH_G(GG_DGRAD, GG_EPI_STORE, false, 1);
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<dgrad, gather>");
    return MOE_OK;
}

extern "C" moe_status moe_grouped_gemm_dgrad(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                             const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                             moe_dtype dt, const void* Z_saved,
                                             const float* dc_scale, const float* b_scale, void* dA) {
    return moe_grouped_gemm_dgrad_weighted(ctx, stream, dC, B, offsets, E, N, K, Rcap, dt, Z_saved, dc_scale, b_scale,
                                           nullptr, dA, nullptr);
}

extern "C" moe_status moe_grouped_gemm_dgrad_weighted(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                                      const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                      moe_dtype dt, const void* Z_saved,
                                                      const float* dc_scale, const float* b_scale,
                                                      const float* row_prob, void* dA, float* dprob_part) {
    return moe_grouped_gemm_dgrad_quant(ctx, stream, dC, B, offsets, E, N, K, Rcap, dt, Z_saved, dc_scale, b_scale, row_prob,
                                        dA, dprob_part, nullptr, nullptr);
}

static moe_status gg_dgrad_all(moe_ctx* ctx, void* stream, const void* dC, const void* B, const int32_t* offsets, int E,
                               int N, int K, int64_t Rcap, moe_dtype dt, const void* Z_saved, const float* dc_scale,
                               const float* b_scale, const float* row_prob, void* dA, float* dprob_part, void* dz_q,
                               float* dz_q_scale, const gg_mx_out* mxo);

extern "C" moe_status moe_grouped_gemm_dgrad_quant(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                                   const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                   moe_dtype dt, const void* Z_saved,
                                                   const float* dc_scale, const float* b_scale,
                                                   const float* row_prob, void* dA, float* dprob_part,
                                                   void* dz_q, float* dz_q_scale) {
    return gg_dgrad_all(ctx, stream, dC, B, offsets, E, N, K, Rcap, dt, Z_saved, dc_scale, b_scale, row_prob, dA, dprob_part,
                        dz_q, dz_q_scale, nullptr);
}

extern "C" moe_status moe_grouped_gemm_dgrad_quant_mx(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                                      const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                      const void* Z_saved, const void* dc_scale, const void* b_scale,
                                                      const float* row_prob, void* dZ, float* dprob_part,
                                                      void* dz_q_row, uint8_t* dz_e8_row, void* dz_q_col, uint8_t* dz_e8_col) {
    if (!ctx) return MOE_ERR_ARG;
    const gg_mx_out o = {dz_q_row, dz_e8_row, dz_q_col, dz_e8_col};
    return gg_dgrad_all(ctx, stream, dC, B, offsets, E, N, K, Rcap, MOE_MXFP8_E4M3, Z_saved, (const float*)dc_scale,
                        (const float*)b_scale, row_prob, dZ, dprob_part, nullptr, nullptr, &o);
}

static moe_status gg_dgrad_all(moe_ctx* ctx, void* stream, const void* dC, const void* B, const int32_t* offsets, int E,
                               int N, int K, int64_t Rcap, moe_dtype dt, const void* Z_saved, const float* dc_scale,
                               const float* b_scale, const float* row_prob, void* dA, float* dprob_part, void* dz_q,
                               float* dz_q_scale, const gg_mx_out* mxo) {
    if (!ctx) return MOE_ERR_ARG;
    if (mxo) {
        moe_status stq = gg_mx_out_check(ctx, "moe_grouped_gemm_dgrad_quant_mx", *mxo, dt, Z_saved != nullptr, Rcap);
        if (stq != MOE_OK) return stq;
    }
    if ((dz_q == nullptr) != (dz_q_scale == nullptr))
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad_quant: dz_q and dz_q_scale go together");
    if (dz_q && (dt != MOE_FP8_E4M3 || !Z_saved))
        MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad_quant: quantised output needs dt = MOE_FP8_E4M3 and Z_saved");
    if (dt == MOE_F32) {  // all-fp32 path (gemm_f32.hip)
        if (!dC || !B || !offsets || !dA) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad: NULL pointer");
        if (E < 1 || N < 1 || K < 1 || Rcap < 1 || Rcap > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad: bad sizes");
        if (dprob_part) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad(f32): dprob_part is not built for fp32 operands");
        if (row_prob && !Z_saved) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad(f32): row weights need Z_saved");
        return moe_gg_f32_dgrad(ctx, (hipStream_t)stream, dC, B, offsets, E, N, K, Rcap, Z_saved, row_prob, dA);
    }
    if ((row_prob || dprob_part) && !Z_saved)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad_weighted: row weights / dprob_part need Z_saved");
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_dgrad", dC, B, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    if (!dA) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad: dA is NULL");
    const bool fp8 = dt != MOE_BF16, mx = dt == MOE_MXFP8_E4M3;
    if (fp8 && (!dc_scale || !b_scale)) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad: fp8 needs dc_scale and b_scale");
    if (!fp8 && N % 64) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_dgrad: N=%d must be a multiple of 64", N);
    gg_args a = gg_make(ctx, dC, B, offsets, E, N, K, Rcap, dA);
    a.Zsaved = (const bf16_t*)Z_saved;
    a.p_scale = dc_scale;
    a.q_scale = b_scale;
    a.row_prob = row_prob;
    a.dprob_part = dprob_part;
    a.out_q = (uint8_t*)dz_q;
    a.out_q_scale = dz_q_scale;
    if (mxo) {
        a.out_q = (uint8_t*)mxo->q_row;
        a.out_q_e8 = mxo->e8_row;
        a.out_qc = (uint8_t*)mxo->q_col;
        a.out_qc_e8 = mxo->e8_col;
    }
    if (Z_saved) {
        if (mx) GG_LAUNCH(GG_DGRAD, GG_EPI_SWIGLU_BWD, false, 2);
        else if (fp8) GG_LAUNCH(GG_DGRAD, GG_EPI_SWIGLU_BWD, false, 1);
        else GG_LAUNCH(GG_DGRAD, GG_EPI_SWIGLU_BWD, false, 0);
    } else {
        if (mx) GG_LAUNCH(GG_DGRAD, GG_EPI_STORE, false, 2);
        else if (fp8) GG_LAUNCH(GG_DGRAD, GG_EPI_STORE, false, 1);
        else GG_LAUNCH(GG_DGRAD, GG_EPI_STORE, false, 0);
    }
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<dgrad>");
    return MOE_OK;
}

static moe_status gg_wgrad_all(moe_ctx* ctx, void* stream, const void* A, const void* dC, const int32_t* offsets, int E,
                               int N, int K, int64_t Rcap, moe_dtype dt, const float* a_scale, const float* dc_scale,
                               int accumulate, moe_dtype out_dt, void* dB, int gath, int T, const int32_t* src_of, int k);

extern "C" moe_status moe_grouped_gemm_wgrad(moe_ctx* ctx, void* stream, const void* A, const void* dC,
                                             const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                             moe_dtype dt, const float* a_scale, const float* dc_scale,
                                             int accumulate, moe_dtype out_dt, void* dB) {
    return gg_wgrad_all(ctx, stream, A, dC, offsets, E, N, K, Rcap, dt, a_scale, dc_scale, accumulate, out_dt, dB, 0, 0,
                        nullptr, 0);
}

extern "C" moe_status moe_grouped_gemm_wgrad_gather(moe_ctx* ctx, void* stream, const void* A, const void* dC,
                                                    moe_gather which, int T, const int32_t* src_of, int k,
                                                    const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                                    int accumulate, moe_dtype out_dt, void* dB) {
    if (!ctx) return MOE_ERR_ARG;
    if (which != MOE_GATHER_A && which != MOE_GATHER_DC) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad_gather: bad `which`");
    if (GG_BF16_NW != 4) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wgrad_gather: needs the four-wave bf16 body");
    return gg_wgrad_all(ctx, stream, A, dC, offsets, E, N, K, Rcap, MOE_BF16, nullptr, nullptr, accumulate, out_dt, dB,
                        which == MOE_GATHER_A ? 2 : 1, T, src_of, k);
}

static moe_status gg_wgrad_all(moe_ctx* ctx, void* stream, const void* A, const void* dC, const int32_t* offsets, int E,
                               int N, int K, int64_t Rcap, moe_dtype dt, const float* a_scale, const float* dc_scale,
                               int accumulate, moe_dtype out_dt, void* dB, int gath, int T, const int32_t* src_of, int k) {
    if (!ctx) return MOE_ERR_ARG;
    if (dt == MOE_F32) {  // all-fp32 path (gemm_f32.hip)
        if (!A || !dC || !offsets || !dB) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: NULL pointer");
        if (E < 1 || N < 1 || K < 1 || Rcap < 1 || Rcap > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: bad sizes");
        if (out_dt != MOE_F32) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad(f32): out_dt must be MOE_F32");
        return moe_gg_f32_wgrad(ctx, (hipStream_t)stream, A, dC, offsets, E, N, K, Rcap, accumulate, dB);
    }
    moe_status st = gg_check_common(ctx, "moe_grouped_gemm_wgrad", dC, A, offsets, E, N, K, Rcap, dt);
    if (st != MOE_OK) return st;
    const bool mx = dt == MOE_MXFP8_E4M3, bw = dt == MOE_FP8_E4M3;
    if ((mx || bw) && (!a_scale || !dc_scale)) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: fp8 needs a_scale and dc_scale");
    if (!dB) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: dB is NULL");
    if (out_dt != MOE_BF16 && out_dt != MOE_F32) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad: out_dt must be bf16 or f32");
    gg_args a = gg_make(ctx, dC, A, offsets, E, N, K, Rcap, dB);
    a.accumulate = accumulate ? 1 : 0;
    a.tile_counter = (int*)((char*)ctx->ws + MOE_WS_TILE_COUNTER);
    moe_launch_fill_i32(a.tile_counter, 1, 0, (hipStream_t)stream);
    a.p_scale = dc_scale;
    a.q_scale = a_scale;
    // split contraction (bf16 operands): as many slices of partial tiles as the workspace holds behind its reserved head
    const size_t slice_bytes = (size_t)ceil_div64(N, GG_BM) * ceil_div64(K, GG_BN) * GG_BM * GG_BN * sizeof(float);
    const size_t ws_free = ctx->ws_bytes > MOE_WS_RESERVED ? ctx->ws_bytes - MOE_WS_RESERVED : 0;
    a.split_info = (int*)((char*)ctx->ws + MOE_WS_SPLIT_INFO);
    a.partials = (float*)((char*)ctx->ws + MOE_WS_RESERVED);
    a.split_cap = (!mx && !bw && GG_BF16_NW == 4) ? (int)(ws_free / slice_bytes < GG_MAX_SPLIT ? ws_free / slice_bytes : GG_MAX_SPLIT) : 0;
    if (gath) {  // (bf16 operands; P = dC, Q = A)
        st = gg_gather_args(ctx, "moe_grouped_gemm_wgrad_gather", a, T, src_of, k, gath == 2 ? K : N, Rcap);
        if (st != MOE_OK) return st;
    }
    if (gath == 2) {
        if (out_dt == MOE_F32) GG_LAUNCH_G(GG_WGRAD, GG_EPI_STORE, true, 2);
        else GG_LAUNCH_G(GG_WGRAD, GG_EPI_STORE, false, 2);
    } else if (gath == 1) {
        if (out_dt == MOE_F32) GG_LAUNCH_G(GG_WGRAD, GG_EPI_STORE, true, 1);
        else GG_LAUNCH_G(GG_WGRAD, GG_EPI_STORE, false, 1);
    } else if (mx) {
        if (out_dt == MOE_F32) GG_LAUNCH(GG_WGRAD, GG_EPI_STORE, true, 2);
        else GG_LAUNCH(GG_WGRAD, GG_EPI_STORE, false, 2);
    } else if (bw) {
        if (out_dt == MOE_F32) GG_LAUNCH(GG_WGRAD, GG_EPI_STORE, true, 1);
        else GG_LAUNCH(GG_WGRAD, GG_EPI_STORE, false, 1);
    } else {
        if (out_dt == MOE_F32) GG_LAUNCH(GG_WGRAD, GG_EPI_STORE, true, 0);
        else GG_LAUNCH(GG_WGRAD, GG_EPI_STORE, false, 0);
    }
    if (a.split_cap >= 2) {
        const dim3 grid((unsigned)(ceil_div64(N, GG_BM) * ceil_div64(K, GG_BN)), GG_MAX_SPLIT_EXPERTS);
        if (out_dt == MOE_F32)
            hipLaunchKernelGGL(gg_split_reduce_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, a.partials, a.split_info, N, K,
                               a.accumulate, dB);
        else
            hipLaunchKernelGGL(gg_split_reduce_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, a.partials, a.split_info, N, K,
                               a.accumulate, dB);
    }
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<wgrad>");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// Gate GEMM (Sec. 2.1.2 item 1): logits[T,E] = X[T,h] * Wr[E,h]^T, bf16 operands, fp32 accumulation and fp32
// output (the router works on fp32 logits, Sec. 5.1).  One group of T rows through the forward kernel with the
// fp32 store; the two-entry offsets array lives in the context's reserved workspace and is written by a
// one-thread kernel, so the call allocates and copies nothing.  With E <= 256 there is one column tile: T / 256
// workgroups have work, which is a quarter of the chip at T = 16384 -- small next to the layer, not tuned.
// ---------------------------------------------------------------------------
#define MOE_WS_GATE_OFFSETS 32  // byte offset of {0, T} in the reserved head of the workspace
__global__ void gate_offsets_kernel(int32_t* o, int T) {
    o[0] = 0;
    o[1] = T;
}

extern "C" moe_status moe_gate_gemm(moe_ctx* ctx, void* stream, const void* X, const void* Wr, int T, int E, int h,
                                    float* logits) {
    if (!ctx) return MOE_ERR_ARG;
    if (!logits) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_gate_gemm: logits is NULL");
    if (T < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_gate_gemm: T must be positive");
    int32_t* offsets = (int32_t*)((char*)ctx->ws + MOE_WS_GATE_OFFSETS);
    moe_status st = gg_check_common(ctx, "moe_gate_gemm", X, Wr, offsets, 1, E, h, T, MOE_BF16);
    if (st != MOE_OK) return st;
    if (h % 64) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_gate_gemm: h=%d must be a multiple of 64", h);
    hipLaunchKernelGGL(gate_offsets_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, offsets, T);
    gg_args a = gg_make(ctx, X, Wr, offsets, 1, E, h, T, logits);
    GG_LAUNCH(GG_FWD, GG_EPI_STORE, true, 0);
    MOE_LAUNCH_CHECK(ctx, "gg_kernel<gate>");
    return MOE_OK;
}
