// All-fp32 grouped GEMMs (dt = MOE_F32): the same three calls as gemm.hip with fp32 operands, fp32 FMA
// accumulation in increasing contraction index and fp32 results, for parity runs at the 1e-5 level on small
// layers (the tiny config is generated in fp32).  Correctness-first: one thread per output element, no tiling,
// no matrix instructions; the expert of a row is found by bisection over the offsets held in LDS.  Same
// conventions as the bf16 path: rows >= offsets[E] untouched, empty experts write zero weight gradients,
// inconsistent offsets raise the error word and nothing is written.
#include "common.h"

#define F32_THREADS 256
#define F32_MAX_E 1024

struct gf_args {
    const float* P;  // fwd: A, dgrad / wgrad: dC
    const float* Q;  // fwd / dgrad: W [E,N,K], wgrad: A
    const int32_t* offsets;
    int E, N, K;
    int64_t Rcap;
    float* out;      // fwd: C (may be NULL with SwiGLU), dgrad: dA or dZ, wgrad: dW
    float* out_act;  // fwd SwiGLU: activation [rows, N/2]
    const float* Zsaved;
    const float* row_prob;
    int accumulate;
    int* dev_err;
};

__device__ __forceinline__ float sigmoid32(float g) { return 1.0f / (1.0f + expf(-g)); }

// loads the offsets, checks them, returns false (after raising the error word) when they are inconsistent
__device__ __forceinline__ bool f32_offsets(const gf_args& a, int* offs) {
    __shared__ int bad;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    for (int e = threadIdx.x; e <= a.E; e += F32_THREADS) offs[e] = a.offsets[e];
    __syncthreads();
    for (int e = threadIdx.x; e < a.E; e += F32_THREADS)
        if (offs[e + 1] < offs[e]) bad = 1;
    if (threadIdx.x == 0 && (offs[0] < 0 || offs[a.E] > a.Rcap)) bad = 1;
    __syncthreads();
    if (bad && blockIdx.x == 0 && threadIdx.x == 0) atomicExch(a.dev_err, 1);
    return !bad;
}
__device__ __forceinline__ int f32_expert_of(const int* offs, int E, int64_t r) {
    int lo = 0, hi = E - 1;  // largest e with offs[e] <= r (empty experts share a start; the last of them owns the row)
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (offs[mid] <= r) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// EPI 0: C[r,n] = sum_k A[r,k] W[e,n,k].  EPI 1 (SwiGLU, N = 2f): thread (r, j < f) forms gate and up.
template <int EPI>
__global__ __launch_bounds__(F32_THREADS) void gf_fwd_kernel(const gf_args a) {
    __shared__ int offs[F32_MAX_E + 1];
    if (!f32_offsets(a, offs)) return;
    const int cols = EPI ? a.N / 2 : a.N;
    const int64_t idx = (int64_t)blockIdx.x * F32_THREADS + threadIdx.x;
    const int64_t r = idx / cols;
    const int j = (int)(idx % cols);
    if (r >= offs[a.E]) return;
    const int e = f32_expert_of(offs, a.E, r);
    const float* x = a.P + r * a.K;
    const float* w = a.Q + ((int64_t)e * a.N + j) * a.K;
    float g = 0.f;
    for (int k = 0; k < a.K; ++k) g = fmaf(x[k], w[k], g);
    if (EPI == 0) {
        a.out[r * a.N + j] = g;
    } else {
        const float* wu = w + (int64_t)cols * a.K;
        float u = 0.f;
        for (int k = 0; k < a.K; ++k) u = fmaf(x[k], wu[k], u);
        if (a.out) {
            a.out[r * a.N + j] = g;
            a.out[r * a.N + cols + j] = u;
        }
        const float pr = a.row_prob ? a.row_prob[r] : 1.0f;
        a.out_act[r * cols + j] = pr * (g * sigmoid32(g) * u);
    }
}

// dA[r,k] = sum_n dC[r,n] W[e,n,k];  with Zsaved: dZ[r,k] = dA up s (1 + g (1 - s)), dZ[r,K+k] = dA g s
__global__ __launch_bounds__(F32_THREADS) void gf_dgrad_kernel(const gf_args a) {
    __shared__ int offs[F32_MAX_E + 1];
    if (!f32_offsets(a, offs)) return;
    const int64_t idx = (int64_t)blockIdx.x * F32_THREADS + threadIdx.x;
    const int64_t r = idx / a.K;
    const int k = (int)(idx % a.K);
    if (r >= offs[a.E]) return;
    const int e = f32_expert_of(offs, a.E, r);
    const float* d = a.P + r * a.N;
    const float* w = a.Q + (int64_t)e * a.N * a.K + k;
    float acc = 0.f;
    for (int n = 0; n < a.N; ++n) acc = fmaf(d[n], w[(int64_t)n * a.K], acc);
    if (!a.Zsaved) {
        a.out[r * a.K + k] = acc;
    } else {
        const float g = a.Zsaved[r * 2 * a.K + k], u = a.Zsaved[r * 2 * a.K + a.K + k];
        const float s = sigmoid32(g);
        const float pr = a.row_prob ? a.row_prob[r] : 1.0f;
        a.out[r * 2 * a.K + k] = pr * acc * u * s * (1.0f + g * (1.0f - s));
        a.out[r * 2 * a.K + a.K + k] = pr * acc * g * s;
    }
}

// dW[e,n,k] = sum over the rows r of expert e of dC[r,n] A[r,k]
__global__ __launch_bounds__(F32_THREADS) void gf_wgrad_kernel(const gf_args a) {
    __shared__ int offs[F32_MAX_E + 1];
    if (!f32_offsets(a, offs)) return;
    const int64_t idx = (int64_t)blockIdx.x * F32_THREADS + threadIdx.x;
    const int64_t per = (int64_t)a.N * a.K;
    if (idx >= per * a.E) return;
    const int e = (int)(idx / per);
    const int n = (int)((idx % per) / a.K), k = (int)(idx % a.K);
    float acc = 0.f;
    for (int64_t r = offs[e]; r < offs[e + 1]; ++r) acc = fmaf(a.P[r * a.N + n], a.Q[r * a.K + k], acc);
    a.out[idx] = a.accumulate ? a.out[idx] + acc : acc;
}

static moe_status gf_launch_check(moe_ctx* ctx, const char* who, int64_t threads) {
    if (threads > (int64_t)0x7fffffff * F32_THREADS) MOE_FAIL(ctx, MOE_ERR_ARG, "%s: problem too large for the fp32 path", who);
    return MOE_OK;
}

moe_status moe_gg_f32_fwd(moe_ctx* ctx, hipStream_t s, const void* A, const void* B, const int32_t* offsets, int E, int N,
                          int K, int64_t Rcap, int swiglu, const float* row_prob, void* C, void* C_act) {
    if (E > F32_MAX_E) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_fwd(f32): E > %d", F32_MAX_E);
    gf_args a = {(const float*)A, (const float*)B, offsets, E, N, K, Rcap, (float*)C, (float*)C_act, nullptr, row_prob, 0,
                 ctx->dev_err};
    const int64_t threads = Rcap * (swiglu ? N / 2 : N);
    moe_status st = gf_launch_check(ctx, "moe_grouped_gemm_fwd(f32)", threads);
    if (st != MOE_OK) return st;
    const unsigned grid = (unsigned)ceil_div64(threads, F32_THREADS);
    if (swiglu) hipLaunchKernelGGL(gf_fwd_kernel<1>, dim3(grid), dim3(F32_THREADS), 0, s, a);
    else hipLaunchKernelGGL(gf_fwd_kernel<0>, dim3(grid), dim3(F32_THREADS), 0, s, a);
    MOE_LAUNCH_CHECK(ctx, "gf_fwd_kernel");
    return MOE_OK;
}

moe_status moe_gg_f32_dgrad(moe_ctx* ctx, hipStream_t s, const void* dC, const void* B, const int32_t* offsets, int E, int N,
                            int K, int64_t Rcap, const void* Z_saved, const float* row_prob, void* dA) {
    if (E > F32_MAX_E) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_dgrad(f32): E > %d", F32_MAX_E);
    gf_args a = {(const float*)dC, (const float*)B, offsets, E, N, K, Rcap, (float*)dA, nullptr, (const float*)Z_saved,
                 row_prob, 0, ctx->dev_err};
    const int64_t threads = Rcap * K;
    moe_status st = gf_launch_check(ctx, "moe_grouped_gemm_dgrad(f32)", threads);
    if (st != MOE_OK) return st;
    hipLaunchKernelGGL(gf_dgrad_kernel, dim3((unsigned)ceil_div64(threads, F32_THREADS)), dim3(F32_THREADS), 0, s, a);
    MOE_LAUNCH_CHECK(ctx, "gf_dgrad_kernel");
    return MOE_OK;
}

moe_status moe_gg_f32_wgrad(moe_ctx* ctx, hipStream_t s, const void* A, const void* dC, const int32_t* offsets, int E, int N,
                            int K, int64_t Rcap, int accumulate, void* dB) {
    if (E > F32_MAX_E) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_grouped_gemm_wgrad(f32): E > %d", F32_MAX_E);
    gf_args a = {(const float*)dC, (const float*)A, offsets, E, N, K, Rcap, (float*)dB, nullptr, nullptr, nullptr,
                 accumulate ? 1 : 0, ctx->dev_err};
    const int64_t threads = (int64_t)E * N * K;
    moe_status st = gf_launch_check(ctx, "moe_grouped_gemm_wgrad(f32)", threads);
    if (st != MOE_OK) return st;
    hipLaunchKernelGGL(gf_wgrad_kernel, dim3((unsigned)ceil_div64(threads, F32_THREADS)), dim3(F32_THREADS), 0, s, a);
    MOE_LAUNCH_CHECK(ctx, "gf_wgrad_kernel");
    return MOE_OK;
}
