// moe_route_topk: fused score function + top-k + weights + histogram (Sec. 2.1.2 item 2, Sec. 4.3.4).
//
// One 64-lane wavefront owns one token.  Lane l holds the logits of experts
// l, l+64, l+128, ... in registers; the max / sum of the score function and each
// of the k arg-max rounds are butterfly reductions over the wavefront, so a
// token costs one coalesced read of its E logits and no LDS traffic.  Selection
// is done on the raw logits (lower index wins ties), weights are computed for
// the k winners only.  A workgroup accumulates its tokens' histogram in LDS and
// adds it to the global counts once.
#include "common.h"

#define ROUTE_MAX_VPL 16          // values per lane -> E <= 1024
#define ROUTE_WAVES 4
#define ROUTE_TOKENS_PER_WAVE 8

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int VPL>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void route_topk_kernel(
    const float* __restrict__ logits, int T, int E, int k, int fn, int norm_topk, float scale,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_prob, int32_t* __restrict__ counts) {
    extern __shared__ int32_t hist[];  // [E]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist[e] = 0;
    __syncthreads();

    const int t0 = (blockIdx.x * ROUTE_WAVES + wave) * ROUTE_TOKENS_PER_WAVE;
    for (int tt = 0; tt < ROUTE_TOKENS_PER_WAVE; ++tt) {
        const int t = t0 + tt;
        if (t >= T) break;  // uniform per wave
        const float* l = logits + (int64_t)t * E;
        float v[VPL];
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            int e = lane + 64 * j;
            v[j] = e < E ? l[e] : -INFINITY;
        }
        float mx = 0.f, den = 1.f;
        if (fn == MOE_SCORE_SOFTMAX) {
            float m = v[0];
#pragma unroll
            for (int j = 1; j < VPL; ++j) m = fmaxf(m, v[j]);
            mx = wave_max(m);
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < VPL; ++j) s += (lane + 64 * j < E) ? expf(v[j] - mx) : 0.f;
            den = wave_sum(s);
        }
        // k rounds of arg-max over (logit desc, index asc)
        uint32_t taken = 0;
        float my_logit = 0.f;
        int my_idx = 0;
        for (int it = 0; it < k; ++it) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < VPL; ++j) {
                int e = lane + 64 * j;
                bool ok = e < E && !((taken >> j) & 1u);
                if (ok && (bi == 0x7fffffff || v[j] > bv)) { bv = v[j]; bi = e; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                float ov = __shfl_xor(bv, o);
                int oi = __shfl_xor(bi, o);
                bool take = (oi != 0x7fffffff) && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
                if (take) { bv = ov; bi = oi; }
            }
            if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
            if (lane == it) { my_logit = bv; my_idx = bi; }
        }
        float p = 0.f;
        if (lane < k) p = fn == MOE_SCORE_SOFTMAX ? expf(my_logit - mx) / den : 1.f / (1.f + expf(-my_logit));
        if (norm_topk) {
            float tot = wave_sum(lane < k ? p : 0.f);
            p = p / tot;
        }
        if (lane < k) {
            topk_idx[(int64_t)t * k + lane] = my_idx;
            topk_prob[(int64_t)t * k + lane] = p * scale;
            atomicAdd(&hist[my_idx], 1);
        }
    }
    __syncthreads();
    if (counts)
        for (int e = threadIdx.x; e < E; e += blockDim.x)
            if (hist[e]) atomicAdd(&counts[e], hist[e]);
}

extern "C" moe_status moe_route_topk(moe_ctx* ctx, void* stream, const float* logits, int T, int E, int k,
                                     moe_score fn, int norm_topk, float scale,
                                     int32_t* topk_idx, float* topk_prob, int32_t* counts) {
    if (!ctx) return MOE_ERR_ARG;
    if (!logits || !topk_idx || !topk_prob) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk: NULL pointer");
    if (T < 0 || E < 1 || E > 64 * ROUTE_MAX_VPL || k < 1 || k > 32 || k > E)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk: need T>=0, 1<=k<=min(E,32), E<=%d (T=%d E=%d k=%d)",
                 64 * ROUTE_MAX_VPL, T, E, k);
    if (fn != MOE_SCORE_SOFTMAX && fn != MOE_SCORE_SIGMOID) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk: bad score fn");
    hipStream_t s = (hipStream_t)stream;
    if (counts) moe_launch_fill_i32(counts, E, 0, s);
    if (T == 0) return MOE_OK;
    const int per_block = ROUTE_WAVES * ROUTE_TOKENS_PER_WAVE;
    dim3 grid((T + per_block - 1) / per_block), block(ROUTE_WAVES * 64);
    size_t shm = (size_t)E * sizeof(int32_t);
    const int vpl = (E + 63) / 64;
#define ROUTE_LAUNCH(V)                                                                                     \
    hipLaunchKernelGGL(route_topk_kernel<V>, grid, block, shm, s, logits, T, E, k, (int)fn, norm_topk, scale, \
                       topk_idx, topk_prob, counts)
    if (vpl <= 1) ROUTE_LAUNCH(1);
    else if (vpl <= 2) ROUTE_LAUNCH(2);
    else if (vpl <= 4) ROUTE_LAUNCH(4);
    else if (vpl <= 8) ROUTE_LAUNCH(8);
    else ROUTE_LAUNCH(16);
#undef ROUTE_LAUNCH
    MOE_LAUNCH_CHECK(ctx, "route_topk_kernel");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// moe_route_topk_grouped: the other branches of the fused score kernel (Sec. 4.3.4 item 1): group-limited
// top-k, the load-balancing expert bias (Sec. 7) and score scaling.
//   s_e = score(logits)_e;  c_e = s_e + bias_e decides, s_e weighs;
//   group score = sum of the k / topk_group largest c of the group; keep the topk_group best groups;
//   select the k largest c among the kept groups' experts; ties to the lower index throughout.
// Same wave-per-token layout as the plain kernel.  The decisions are taken on fp32 values that do not depend
// on the precision of a fast exponential: the score is evaluated in double and rounded to fp32 once, the bias
// add and the group sums (largest first) are single fp32 additions.  The group scores are formed by one lane
// per group from the wave's c values in LDS (each wave has its own region, so program order is all the
// synchronisation needed); groups and experts are then chosen by the same butterfly arg-max rounds.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// one round of arg-max over (value desc, index asc) across the wave; idx 0x7fffffff = no candidate
__device__ __forceinline__ void wave_argmax(float& bv, int& bi) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o);
        const int oi = __shfl_xor(bi, o);
        const bool take = (oi != 0x7fffffff) && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
        if (take) { bv = ov; bi = oi; }
    }
}

template <int VPL>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void route_topk_grouped_kernel(
    const float* __restrict__ logits, const float* __restrict__ bias, int T, int E, int k, int n_group, int topk_group,
    int fn, int norm_topk, float scale,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_prob, int32_t* __restrict__ counts) {
    extern __shared__ int32_t hist[];  // [E] histogram, then ROUTE_WAVES x [E] floats
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float* cw = (float*)(hist + E) + wave * E;
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist[e] = 0;
    __syncthreads();
    const int gs = E / n_group, m = k / topk_group;

    const int t0 = (blockIdx.x * ROUTE_WAVES + wave) * ROUTE_TOKENS_PER_WAVE;
    for (int tt = 0; tt < ROUTE_TOKENS_PER_WAVE; ++tt) {
        const int t = t0 + tt;
        if (t >= T) break;  // uniform per wave
        const float* l = logits + (int64_t)t * E;
        float v[VPL], sc[VPL], c[VPL];
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const int e = lane + 64 * j;
            v[j] = e < E ? l[e] : -INFINITY;
        }
        if (fn == MOE_SCORE_SOFTMAX) {
            float mf = v[0];
#pragma unroll
            for (int j = 1; j < VPL; ++j) mf = fmaxf(mf, v[j]);
            const double mx = (double)wave_max(mf);
            double part = 0.0;
#pragma unroll
            for (int j = 0; j < VPL; ++j) part += (lane + 64 * j < E) ? exp((double)v[j] - mx) : 0.0;
            const double den = wave_sum_f64(part);
#pragma unroll
            for (int j = 0; j < VPL; ++j) sc[j] = (float)(exp((double)v[j] - mx) / den);
        } else {
#pragma unroll
            for (int j = 0; j < VPL; ++j) sc[j] = (float)(1.0 / (1.0 + exp(-(double)v[j])));
        }
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const int e = lane + 64 * j;
            c[j] = (bias && e < E) ? sc[j] + bias[e] : sc[j];
        }

        // ---- groups to keep ----
        uint64_t keep = ~0ull;
        if (n_group > 1) {
#pragma unroll
            for (int j = 0; j < VPL; ++j) {
                const int e = lane + 64 * j;
                if (e < E) cw[e] = c[j];
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            // lane g: sum of the m largest c of group g, largest first; round r takes the best element that
            // comes after round r-1's pick in (value desc, index asc) order
            float gsum = -INFINITY;
            int gi = 0x7fffffff;
            if (lane < n_group) {
                float pv = INFINITY;
                int pi = -1;
                gsum = 0.f;
                for (int r = 0; r < m; ++r) {
                    float bv = -INFINITY;
                    int bi = 0x7fffffff;
                    for (int x = 0; x < gs; ++x) {
                        const float cv = cw[lane * gs + x];
                        const bool after = cv < pv || (cv == pv && x > pi);
                        if (after && (bi == 0x7fffffff || cv > bv)) { bv = cv; bi = x; }
                    }
                    gsum = r == 0 ? bv : gsum + bv;
                    pv = bv;
                    pi = bi;
                }
                gi = lane;
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            bool kept = false;
            for (int r = 0; r < topk_group; ++r) {
                float bv = kept ? -INFINITY : gsum;
                int bi = kept ? 0x7fffffff : gi;
                wave_argmax(bv, bi);
                if (bi == lane) kept = true;
            }
            keep = __ballot(kept);
        }

        // ---- k rounds of arg-max over c among the kept groups ----
        uint32_t taken = 0;
        float my_s = 0.f;
        int my_idx = 0;
        for (int it = 0; it < k; ++it) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < VPL; ++j) {
                const int e = lane + 64 * j;
                const bool ok = e < E && !((taken >> j) & 1u) && ((keep >> (e / gs)) & 1ull);
                if (ok && (bi == 0x7fffffff || c[j] > bv)) { bv = c[j]; bi = e; }
            }
            wave_argmax(bv, bi);
            float sv = 0.f;
#pragma unroll
            for (int j = 0; j < VPL; ++j)
                if (j == (bi >> 6)) sv = sc[j];
            sv = __shfl(sv, bi & 63);  // the winner's unbiased score
            if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
            if (lane == it) { my_s = sv; my_idx = bi; }
        }
        float p = lane < k ? my_s : 0.f;
        if (norm_topk) p = p / wave_sum(p);
        if (lane < k) {
            topk_idx[(int64_t)t * k + lane] = my_idx;
            topk_prob[(int64_t)t * k + lane] = p * scale;
            atomicAdd(&hist[my_idx], 1);
        }
    }
    __syncthreads();
    if (counts)
        for (int e = threadIdx.x; e < E; e += blockDim.x)
            if (hist[e]) atomicAdd(&counts[e], hist[e]);
}

extern "C" moe_status moe_route_topk_grouped(moe_ctx* ctx, void* stream, const float* logits, const float* expert_bias,
                                             int T, int E, int k, int n_group, int topk_group,
                                             moe_score fn, int norm_topk, float scale,
                                             int32_t* topk_idx, float* topk_prob, int32_t* counts) {
    if (!ctx) return MOE_ERR_ARG;
    if (!logits || !topk_idx || !topk_prob) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk_grouped: NULL pointer");
    if (T < 0 || E < 1 || E > 64 * ROUTE_MAX_VPL || k < 1 || k > 32 || k > E)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk_grouped: need T>=0, 1<=k<=min(E,32), E<=%d (T=%d E=%d k=%d)",
                 64 * ROUTE_MAX_VPL, T, E, k);
    if (n_group < 1 || n_group > 64 || E % n_group || topk_group < 1 || topk_group > n_group || k % topk_group ||
        k / topk_group > E / n_group)
        MOE_FAIL(ctx, MOE_ERR_ARG,
                 "moe_route_topk_grouped: need 1<=topk_group<=n_group<=64, E %% n_group == 0, k %% topk_group == 0 and "
                 "k/topk_group <= E/n_group (E=%d k=%d n_group=%d topk_group=%d)", E, k, n_group, topk_group);
    if (fn != MOE_SCORE_SOFTMAX && fn != MOE_SCORE_SIGMOID) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk_grouped: bad score fn");
    hipStream_t s = (hipStream_t)stream;
    if (counts) moe_launch_fill_i32(counts, E, 0, s);
    if (T == 0) return MOE_OK;
    const int per_block = ROUTE_WAVES * ROUTE_TOKENS_PER_WAVE;
    dim3 grid((T + per_block - 1) / per_block), block(ROUTE_WAVES * 64);
    size_t shm = (size_t)E * sizeof(int32_t) * (1 + ROUTE_WAVES);
    const int vpl = (E + 63) / 64;
#define ROUTE_LAUNCH(V)                                                                                            \
    hipLaunchKernelGGL(route_topk_grouped_kernel<V>, grid, block, shm, s, logits, expert_bias, T, E, k, n_group,   \
                       topk_group, (int)fn, norm_topk, scale, topk_idx, topk_prob, counts)
    if (vpl <= 1) ROUTE_LAUNCH(1);
    else if (vpl <= 2) ROUTE_LAUNCH(2);
    else if (vpl <= 4) ROUTE_LAUNCH(4);
    else if (vpl <= 8) ROUTE_LAUNCH(8);
    else ROUTE_LAUNCH(16);
#undef ROUTE_LAUNCH
    MOE_LAUNCH_CHECK(ctx, "route_topk_grouped_kernel");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// moe_route_topk_bwd: dL/dlogits from dL/dweights with the selection frozen (Sec. 2.1.2 item 2).
//   w_s = scale * q_s / D,  q_s = score of the s-th selected expert,  D = sum_s q_s (norm_topk) or 1
//   dq_s = scale * (dw_s / D - [norm] <dw, q> / D^2)
//   softmax: dl_j = p_j * ([j selected] dq_j - <dq, q>)      sigmoid: dl_j = [j selected] dq_j * q_j (1 - q_j)
// One wavefront per token, same register layout as the forward kernel; lane s < k holds slot s.
// ---------------------------------------------------------------------------
template <int VPL>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void route_topk_bwd_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ topk_idx, const float* __restrict__ dprob,
    int T, int E, int k, int fn, int norm_topk, float scale, float* __restrict__ dlogits) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * ROUTE_WAVES + wave) * ROUTE_TOKENS_PER_WAVE;
    for (int tt = 0; tt < ROUTE_TOKENS_PER_WAVE; ++tt) {
        const int t = t0 + tt;
        if (t >= T) break;  // uniform per wave
        const float* l = logits + (int64_t)t * E;
        float v[VPL];
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const int e = lane + 64 * j;
            v[j] = e < E ? l[e] : -INFINITY;
        }
        float mx = 0.f, den = 1.f;
        if (fn == MOE_SCORE_SOFTMAX) {
            float m = v[0];
#pragma unroll
            for (int j = 1; j < VPL; ++j) m = fmaxf(m, v[j]);
            mx = wave_max(m);
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < VPL; ++j) s += (lane + 64 * j < E) ? expf(v[j] - mx) : 0.f;
            den = wave_sum(s);
        }
        // slot s lives in lane s: its expert, its score q_s and the incoming gradient
        int my_idx = lane < k ? topk_idx[(int64_t)t * k + lane] : -1;
        if (my_idx < 0 || my_idx >= E) my_idx = -1;  // a slot that names no expert of this router contributes nothing
        const float dw = my_idx >= 0 ? dprob[(int64_t)t * k + lane] : 0.f;
        float q = 0.f;
        if (my_idx >= 0) {
            const float lg = l[my_idx];
            q = fn == MOE_SCORE_SOFTMAX ? expf(lg - mx) / den : 1.f / (1.f + expf(-lg));
        }
        float dq = scale * dw;
        if (norm_topk) {
            const float D = wave_sum(q);
            const float dwq = wave_sum(dw * q);
            dq = my_idx >= 0 ? scale * (dw / D - dwq / (D * D)) : 0.f;
        }
        const float dqq = wave_sum(dq * q);  // <dq, q>
        // every lane collects the dq of the selected experts it owns
        float gsel[VPL];
#pragma unroll
        for (int j = 0; j < VPL; ++j) gsel[j] = 0.f;
        for (int s = 0; s < k; ++s) {
            const int e = __shfl(my_idx, s);
            const float d = __shfl(dq, s);
            if (e >= 0 && (e & 63) == lane) {
#pragma unroll
                for (int j = 0; j < VPL; ++j)
                    if ((e >> 6) == j) gsel[j] += d;
            }
        }
        float* o = dlogits + (int64_t)t * E;
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const int e = lane + 64 * j;
            if (e < E) {
                float r;
                if (fn == MOE_SCORE_SOFTMAX) {
                    const float p = expf(v[j] - mx) / den;
                    r = p * (gsel[j] - dqq);
                } else {
                    const float sg = 1.f / (1.f + expf(-v[j]));
                    r = gsel[j] * sg * (1.f - sg);
                }
                o[e] = r;
            }
        }
    }
}

extern "C" moe_status moe_route_topk_bwd(moe_ctx* ctx, void* stream, const float* logits, const int32_t* topk_idx,
                                         const float* dprob, int T, int E, int k, moe_score fn, int norm_topk,
                                         float scale, float* dlogits) {
    if (!ctx) return MOE_ERR_ARG;
    if (!logits || !topk_idx || !dprob || !dlogits) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk_bwd: NULL pointer");
    if (T < 0 || E < 1 || E > 64 * ROUTE_MAX_VPL || k < 1 || k > 32 || k > E)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk_bwd: need T>=0, 1<=k<=min(E,32), E<=%d (T=%d E=%d k=%d)",
                 64 * ROUTE_MAX_VPL, T, E, k);
    if (fn != MOE_SCORE_SOFTMAX && fn != MOE_SCORE_SIGMOID) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_route_topk_bwd: bad score fn");
    if (T == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)stream;
    const int per_block = ROUTE_WAVES * ROUTE_TOKENS_PER_WAVE;
    dim3 grid((T + per_block - 1) / per_block), block(ROUTE_WAVES * 64);
    const int vpl = (E + 63) / 64;
#define ROUTE_BWD_LAUNCH(V)                                                                                       \
    hipLaunchKernelGGL(route_topk_bwd_kernel<V>, grid, block, 0, s, logits, topk_idx, dprob, T, E, k, (int)fn, norm_topk, \
                       scale, dlogits)
    if (vpl <= 1) ROUTE_BWD_LAUNCH(1);
    else if (vpl <= 2) ROUTE_BWD_LAUNCH(2);
    else if (vpl <= 4) ROUTE_BWD_LAUNCH(4);
    else if (vpl <= 8) ROUTE_BWD_LAUNCH(8);
    else ROUTE_BWD_LAUNCH(16);
#undef ROUTE_BWD_LAUNCH
    MOE_LAUNCH_CHECK(ctx, "route_topk_bwd_kernel");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// moe_aux_loss: load-balancing auxiliary loss and its gradient (Sec. 4.3.4 items 2 and 3, fused here into one
// pass over the logits; the Switch-Transformer form the paper cites):
//   p[t,:] = softmax(l[t,:]) or sigmoid(l[t,:]) / sum_j sigmoid(l[t,j])           (Sec. 2.1.2 item 2)
//   loss   = coeff E sum_e f_e P_e,  f_e = counts[e] / (T k),  P_e = (1/T) sum_t p[t,e]
//          = sum_t <w, p[t,:]>,      w_e = coeff E counts[e] / (T^2 k)
//   dl[t,j] = g p_j (w_j - <w, p>) (softmax),  g (1 - sg_j) p_j (w_j - <w, p>) (sigmoid),  g = dloss
// so both the loss and the gradient need only per-token quantities: one wavefront per token in the router's
// register layout; the per-token terms are summed in double, per workgroup, into the context's workspace and a
// one-wave kernel adds the partial sums in a fixed order (run-to-run identical, no floating-point atomics).
// ---------------------------------------------------------------------------
template <int VPL>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void aux_loss_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ counts, int T, int E, int fn, float wscale, float g,
    int accumulate, float* __restrict__ dlogits, double* __restrict__ partial) {
    extern __shared__ __attribute__((aligned(16))) float wsh[];  // [E] weights, then ROUTE_WAVES doubles
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < E; e += blockDim.x) wsh[e] = wscale * (float)counts[e];
    __syncthreads();
    float w[VPL];
#pragma unroll
    for (int j = 0; j < VPL; ++j) w[j] = lane + 64 * j < E ? wsh[lane + 64 * j] : 0.f;
    double acc = 0.0;
    const int t0 = (blockIdx.x * ROUTE_WAVES + wave) * ROUTE_TOKENS_PER_WAVE;
    for (int tt = 0; tt < ROUTE_TOKENS_PER_WAVE; ++tt) {
        const int t = t0 + tt;
        if (t >= T) break;  // uniform per wave
        const float* l = logits + (int64_t)t * E;
        float v[VPL], p[VPL], sg[VPL];
#pragma unroll
        for (int j = 0; j < VPL; ++j) v[j] = lane + 64 * j < E ? l[lane + 64 * j] : -INFINITY;
        float part = 0.f;
        if (fn == MOE_SCORE_SOFTMAX) {
            float m = v[0];
#pragma unroll
            for (int j = 1; j < VPL; ++j) m = fmaxf(m, v[j]);
            m = wave_max(m);
#pragma unroll
            for (int j = 0; j < VPL; ++j) { p[j] = lane + 64 * j < E ? expf(v[j] - m) : 0.f; part += p[j]; }
        } else {
#pragma unroll
            for (int j = 0; j < VPL; ++j) { sg[j] = lane + 64 * j < E ? 1.f / (1.f + expf(-v[j])) : 0.f; p[j] = sg[j]; part += p[j]; }
        }
        const float inv = 1.f / wave_sum(part);
        float d = 0.f;
#pragma unroll
        for (int j = 0; j < VPL; ++j) { p[j] *= inv; d += w[j] * p[j]; }
        d = wave_sum(d);  // <w, p[t,:]>
        acc += (double)d;
        if (dlogits) {
#pragma unroll
            for (int j = 0; j < VPL; ++j) {
                const int e = lane + 64 * j;
                if (e < E) {
                    float gr = g * p[j] * (w[j] - d);
                    if (fn != MOE_SCORE_SOFTMAX) gr *= 1.f - sg[j];
                    float* o = dlogits + (int64_t)t * E + e;
                    *o = accumulate ? *o + gr : gr;
                }
            }
        }
    }
    double* wpart = (double*)(wsh + ((E + 1) & ~1));
    if (lane == 0) wpart[wave] = acc;  // every lane holds the same sum
    __syncthreads();
    if (threadIdx.x == 0) {
        double sum = 0.0;
        for (int i = 0; i < ROUTE_WAVES; ++i) sum += wpart[i];
        partial[blockIdx.x] = sum;
    }
}

__global__ __launch_bounds__(64) void aux_loss_sum_kernel(const double* __restrict__ partial, int n, float* __restrict__ loss) {
    double a = 0.0;
    for (int i = threadIdx.x; i < n; i += 64) a += partial[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
    if (threadIdx.x == 0) *loss = (float)a;
}

extern "C" moe_status moe_aux_loss(moe_ctx* ctx, void* stream, const float* logits, const int32_t* counts,
                                   int T, int E, int k, moe_score fn, float coeff, float dloss, int accumulate,
                                   float* loss, float* dlogits) {
    if (!ctx) return MOE_ERR_ARG;
    if (!logits || !counts || !loss) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_aux_loss: NULL pointer");
    if (T < 1 || E < 1 || E > 64 * ROUTE_MAX_VPL || k < 1)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_aux_loss: need T>=1, 1<=E<=%d, k>=1 (T=%d E=%d k=%d)", 64 * ROUTE_MAX_VPL, T, E, k);
    if (fn != MOE_SCORE_SOFTMAX && fn != MOE_SCORE_SIGMOID) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_aux_loss: bad score fn");
    const int per_block = ROUTE_WAVES * ROUTE_TOKENS_PER_WAVE;
    const int nblocks = (T + per_block - 1) / per_block;
    if (MOE_WS_RESERVED + (size_t)nblocks * sizeof(double) > ctx->ws_bytes)
        MOE_FAIL(ctx, MOE_ERR_WORKSPACE, "moe_aux_loss: workspace %zu B < %zu B", ctx->ws_bytes,
                 MOE_WS_RESERVED + (size_t)nblocks * sizeof(double));
    hipStream_t s = (hipStream_t)stream;
    double* partial = (double*)((char*)ctx->ws + MOE_WS_RESERVED);
    const float wscale = (float)((double)coeff * E / ((double)T * T * k));
    const size_t shm = (size_t)((E + 1) & ~1) * sizeof(float) + ROUTE_WAVES * sizeof(double);
    const int vpl = (E + 63) / 64;
#define AUX_LAUNCH(V)                                                                                                \
    hipLaunchKernelGGL(aux_loss_kernel<V>, dim3(nblocks), dim3(ROUTE_WAVES * 64), shm, s, logits, counts, T, E, (int)fn, \
                       wscale, dloss, accumulate, dlogits, partial)
    if (vpl <= 1) AUX_LAUNCH(1);
    else if (vpl <= 2) AUX_LAUNCH(2);
    else if (vpl <= 4) AUX_LAUNCH(4);
    else if (vpl <= 8) AUX_LAUNCH(8);
    else AUX_LAUNCH(16);
#undef AUX_LAUNCH
    hipLaunchKernelGGL(aux_loss_sum_kernel, dim3(1), dim3(64), 0, s, partial, nblocks, loss);
    MOE_LAUNCH_CHECK(ctx, "aux_loss_kernel");
    return MOE_OK;
}
