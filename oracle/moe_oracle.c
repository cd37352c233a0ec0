/*
 * CPU oracle for the one-GPU MoE expert-layer path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, loop-over-tokens-and-experts statement of what the layer
 * computes, written from the paper's definitions.  It shares no code, header,
 * table or helper with the HIP library and must never be reached from the
 * product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg call it.
 *
 * The file is compiled twice, with -DREAL=double -DSFX=f64 (the parity
 * authority) and -DREAL=float -DSFX=f32 (the "plain fp32 CPU implementation"
 * whose time is reported beside the GPU's).  Integer steps do not depend on REAL.
 * OpenMP threads split only independent rows / experts; there is no blocking or
 * fusion.  One reordering exists: the dot-product loop of grouped_gemm_nt
 * carries "omp simd reduction(+)", so the compiler may add a dot product's terms in
 * several partial sums (vector lanes) instead of strictly left to right.  In the
 * fp64 build, the parity authority, that moves results by a few 1e-16 relative,
 * far below every bound used; the fp32 build is the timed baseline only.
 *
 * What each function follows:
 *   route_topk        Sec. 1.1 (p = Softmax(W_r x), sum over TopK) and Sec. 2.1.2
 *                     item 2 (softmax or sigmoid score, k highest per token).
 *   route_topk_grouped  Sec. 4.3.4 item 1 (group top-k, scaling) + Sec. 7 (expert bias); see its comment.
 *   permute_maps      Sec. 4.3.3 "Preprocessing": the row-ID map.
 *   permute_rows      Sec. 4.3.3 "Permute" (+ Sec. 5.4.1: zero padding fused in).
 *   grouped_gemm_nt   Sec. 2.1.4 / 4.3.2: one independent GEMM per expert over its
 *                     contiguous rows;  Sec. 4.1.2: E_i(x) = W2 phi(W1 x), no bias.
 *   swiglu(_bwd)      Sec. 2.1.4 gated activation phi; backward from the saved
 *                     pre-activation z (Sec. 4.1.2 last paragraph).
 *   grouped_gemm_nn   dgrad, grouped_gemm_tn: wgrad (Sec. 4.2.3 "W/D split";
 *                     Sec. 5.4.1: the wgrad contraction runs over the token dim).
 *   combine(_bwd)     Sec. 4.1.2 eq. (1); Sec. 4.3.3 "Unpermute": the k copies are
 *                     summed with the probabilities as weights; Sec. 2.1.1 stage 4:
 *                     the shared expert's output is added here.
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - top-k is selected on the raw fp32 logits (both score functions are strictly
 *     increasing), ties go to the lower expert index, slots are in descending order;
 *   - softmax weights are not renormalised unless norm_topk; sigmoid weights are
 *     s_i / sum over the k selected when norm_topk;
 *   - rows inside an expert keep the order of the flattened (token, slot) index;
 *   - expert ids outside [0,E) mean "not on this GPU": no row, row_of = -1;
 *   - SwiGLU: fc1 output is [gate(0:f) | up(f:2f)], phi = silu(gate) * up.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#define SFX f64
#endif
#define CAT_(a, b) a##_##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SFX)

/* ------------------------------------------------------------------------ */
/* Router: scores, top-k, combine weights, per-expert histogram              */
/* ------------------------------------------------------------------------ */
/* score: 0 softmax over all E, 1 sigmoid.  Returns 0, or -1 on bad arguments. */
int FN(orc_route_topk)(const float* logits, int T, int E, int k, int score, int norm_topk, double scale,
                       int32_t* topk_idx, REAL* topk_prob, int32_t* counts) {
    if (T < 0 || E < 1 || k < 1 || k > E) return -1;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    REAL* s = (REAL*)malloc(sizeof(REAL) * (size_t)E);
    char* taken = (char*)malloc((size_t)E);
    for (int t = 0; t < T; ++t) {
        const float* l = logits + (int64_t)t * E;
        /* scores over all E experts */
        if (score == 0) {
            REAL mx = (REAL)l[0];
            for (int e = 1; e < E; ++e) if ((REAL)l[e] > mx) mx = (REAL)l[e];
            REAL den = 0;
            for (int e = 0; e < E; ++e) { s[e] = (REAL)exp((double)((REAL)l[e] - mx)); den += s[e]; }
            for (int e = 0; e < E; ++e) s[e] /= den;
        } else {
            for (int e = 0; e < E; ++e) s[e] = (REAL)(1.0 / (1.0 + exp(-(double)l[e])));
        }
        /* k highest logits; strict '>' keeps the lowest index among equals */
        memset(taken, 0, (size_t)E);
        REAL sel_sum = 0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || l[e] > l[best])) best = e;
            taken[best] = 1;
            topk_idx[(int64_t)t * k + j] = best;
            sel_sum += s[best];
            counts[best] += 1;
        }
        for (int j = 0; j < k; ++j) {
            REAL w = s[topk_idx[(int64_t)t * k + j]];
            if (norm_topk) w /= sel_sum;
            topk_prob[(int64_t)t * k + j] = w * (REAL)scale;
        }
    }
    free(s);
    free(taken);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Router, the branches Sec. 4.3.4 item 1 lists for the fused score kernel:  */
/* group-limited top-k, the load-balancing expert bias (Sec. 7, "auxiliary-  */
/* loss-free balancing"), score scaling.                                     */
/* ------------------------------------------------------------------------ */
/* The paper names these branches and cites their sources; it does not restate them.  Reading taken (the
 * published DeepSeek-V3 router):
 *   s_e  = score function of the logits over all E experts (softmax or sigmoid);
 *   c_e  = s_e + bias_e decides the routing only; the combine weights use s_e;
 *   the E experts form n_group contiguous groups of E / n_group; a group's score is the sum of its
 *   k / topk_group largest c; the topk_group best groups stay, all other experts are excluded;
 *   the k largest c among the remaining experts are selected (slots in selection order);
 *   weight = s_e of the selected (divided by their sum when norm_topk) * scale.
 * Ties go to the lower index, for experts and for groups.  n_group = 1 (then topk_group = 1) and
 * bias = NULL reduce to the plain router.
 * Precision: the routing decisions are taken on fp32 values, as a fp32 router would (Sec. 5.1 keeps the
 * router in FP32): s_e is computed in double and rounded to fp32, c_e and the group sums are fp32
 * additions (group sums in descending order of c).  The weights are then formed in REAL from the fp32
 * scores. */
int FN(orc_route_topk_grouped)(const float* logits, const float* bias, int T, int E, int k, int n_group, int topk_group,
                               int score, int norm_topk, double scale,
                               int32_t* topk_idx, REAL* topk_prob, int32_t* counts) {
    if (T < 0 || E < 1 || k < 1 || k > E || n_group < 1 || E % n_group || topk_group < 1 || topk_group > n_group ||
        k % topk_group || k / topk_group > E / n_group || k > topk_group * (E / n_group))
        return -1;
    const int gs = E / n_group, m = k / topk_group;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    float* s = (float*)malloc(sizeof(float) * (size_t)E);
    float* c = (float*)malloc(sizeof(float) * (size_t)E);
    float* gscore = (float*)malloc(sizeof(float) * (size_t)n_group);
    char* taken = (char*)malloc((size_t)E);
    char* gkeep = (char*)malloc((size_t)n_group);
    for (int t = 0; t < T; ++t) {
        const float* l = logits + (int64_t)t * E;
        if (score == 0) {
            double mx = l[0], den = 0;
            for (int e = 1; e < E; ++e) if (l[e] > mx) mx = l[e];
            for (int e = 0; e < E; ++e) den += exp((double)l[e] - mx);
            for (int e = 0; e < E; ++e) s[e] = (float)(exp((double)l[e] - mx) / den);
        } else {
            for (int e = 0; e < E; ++e) s[e] = (float)(1.0 / (1.0 + exp(-(double)l[e])));
        }
        for (int e = 0; e < E; ++e) c[e] = bias ? s[e] + bias[e] : s[e];
        /* group scores: sum of the m largest c of the group, largest first */
        memset(taken, 0, (size_t)E);
        for (int g = 0; g < n_group; ++g) {
            float sum = 0.0f;
            for (int j = 0; j < m; ++j) {
                int best = -1;
                for (int e = g * gs; e < (g + 1) * gs; ++e)
                    if (!taken[e] && (best < 0 || c[e] > c[best])) best = e;
                taken[best] = 1;
                sum = j == 0 ? c[best] : sum + c[best];
            }
            gscore[g] = sum;
        }
        /* the topk_group best groups */
        memset(gkeep, 0, (size_t)n_group);
        for (int j = 0; j < topk_group; ++j) {
            int best = -1;
            for (int g = 0; g < n_group; ++g)
                if (!gkeep[g] && (best < 0 || gscore[g] > gscore[best])) best = g;
            gkeep[best] = 1;
        }
        /* k largest c among the experts of the kept groups */
        memset(taken, 0, (size_t)E);
        REAL sel_sum = 0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (gkeep[e / gs] && !taken[e] && (best < 0 || c[e] > c[best])) best = e;
            taken[best] = 1;
            topk_idx[(int64_t)t * k + j] = best;
            sel_sum += (REAL)s[best];
            counts[best] += 1;
        }
        for (int j = 0; j < k; ++j) {
            REAL w = (REAL)s[topk_idx[(int64_t)t * k + j]];
            if (norm_topk) w /= sel_sum;
            topk_prob[(int64_t)t * k + j] = w * (REAL)scale;
        }
    }
    free(s); free(c); free(gscore); free(taken); free(gkeep);
    return 0;
}

#ifdef ORC_INTEGER_PARTS
/* ------------------------------------------------------------------------ */
/* Row-ID map: stable counting sort of the (token, slot) pairs by expert     */
/* ------------------------------------------------------------------------ */
/* offsets[e] = first row of expert e, each expert's extent rounded up to `align`;
 * returns the total padded row count, or -1 if it exceeds Rcap / bad arguments. */
int64_t orc_permute_maps(const int32_t* idx, int T, int k, int E, int align, int64_t Rcap,
                         int32_t* row_of, int32_t* src_of, int32_t* offsets, int32_t* counts) {
    if (align < 1 || E < 1 || k < 1) return -1;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int64_t j = 0; j < (int64_t)T * k; ++j)
        if (idx[j] >= 0 && idx[j] < E) counts[idx[j]] += 1;
    int64_t run = 0;
    for (int e = 0; e < E; ++e) {
        offsets[e] = (int32_t)run;
        run += ((int64_t)counts[e] + align - 1) / align * align;
    }
    offsets[E] = (int32_t)run;
    if (run > Rcap) return -1;
    for (int64_t r = 0; r < Rcap; ++r) src_of[r] = -1;
    int32_t* fill = (int32_t*)calloc((size_t)E, sizeof(int32_t));
    for (int64_t j = 0; j < (int64_t)T * k; ++j) {
        int e = idx[j];
        if (e < 0 || e >= E) { row_of[j] = -1; continue; }
        int32_t r = offsets[e] + fill[e]++;
        row_of[j] = r;
        src_of[r] = (int32_t)j;
    }
    free(fill);
    return run;
}
#endif

/* Xp[r,:] = X[src_of[r] / k, :], pad rows (src_of < 0) are zero. */
void FN(orc_permute_rows)(const REAL* X, const int32_t* src_of, int64_t R, int k, int h, REAL* Xp) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        REAL* dst = Xp + r * h;
        if (src_of[r] < 0) { for (int c = 0; c < h; ++c) dst[c] = 0; continue; }
        const REAL* src = X + (int64_t)(src_of[r] / k) * h;
        for (int c = 0; c < h; ++c) dst[c] = src[c];
    }
}

/* expert that owns row r: offsets[e] <= r < offsets[e+1]; -1 if none */
static int owner_of(const int32_t* offsets, int E, int64_t r) {
    for (int e = 0; e < E; ++e)
        if (r >= offsets[e] && r < offsets[e + 1]) return e;
    return -1;
}

/* ------------------------------------------------------------------------ */
/* Expert GEMMs                                                              */
/* ------------------------------------------------------------------------ */
/* Forward: C[r,n] = sum_k A[r,k] * B[e(r),n,k].  rows==NULL: every row in
 * [offsets[0], offsets[E]) and C is [R,N] indexed by r; otherwise only the nrows
 * listed rows, C is [nrows,N] indexed by list position. */
void FN(orc_grouped_gemm_nt)(const REAL* A, const REAL* B, const int32_t* offsets, int E, int N, int K,
                             const int32_t* rows, int64_t nrows, REAL* C) {
    int64_t cnt = rows ? nrows : (int64_t)offsets[E] - offsets[0];
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < cnt; ++i) {
        int64_t r = rows ? rows[i] : offsets[0] + i;
        int e = owner_of(offsets, E, r);
        REAL* c = C + (rows ? i : r) * N;
        if (e < 0) { for (int n = 0; n < N; ++n) c[n] = 0; continue; }
        const REAL* a = A + r * K;
        const REAL* Be = B + (int64_t)e * N * K;
        for (int n = 0; n < N; ++n) {
            const REAL* b = Be + (int64_t)n * K;
            REAL acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int kk = 0; kk < K; ++kk) acc += a[kk] * b[kk];
            c[n] = acc;
        }
    }
}

/* dgrad: dA[r,k] = sum_n dC[r,n] * B[e(r),n,k].  Row subset as above. */
void FN(orc_grouped_gemm_nn)(const REAL* dC, const REAL* B, const int32_t* offsets, int E, int N, int K,
                             const int32_t* rows, int64_t nrows, REAL* dA) {
    int64_t cnt = rows ? nrows : (int64_t)offsets[E] - offsets[0];
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < cnt; ++i) {
        int64_t r = rows ? rows[i] : offsets[0] + i;
        int e = owner_of(offsets, E, r);
        REAL* da = dA + (rows ? i : r) * K;
        for (int kk = 0; kk < K; ++kk) da[kk] = 0;
        if (e < 0) continue;
        const REAL* dc = dC + r * N;
        const REAL* Be = B + (int64_t)e * N * K;
        for (int n = 0; n < N; ++n) {
            const REAL g = dc[n];
            const REAL* b = Be + (int64_t)n * K;
            for (int kk = 0; kk < K; ++kk) da[kk] += g * b[kk];
        }
    }
}

/* wgrad: dB[e,n,k] = sum over rows r of expert e of dC[r,n] * A[r,k]; the
 * contraction length is the expert's row count and may be zero (then dB_e = 0).
 * Only the window n in [n0,n0+nn), k in [k0,k0+kn) is produced; dB is [E,nn,kn]. */
void FN(orc_grouped_gemm_tn)(const REAL* dC, const REAL* A, const int32_t* offsets, int E, int N, int K,
                             int n0, int nn, int k0, int kn, REAL* dB) {
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int e = 0; e < E; ++e) {
        for (int n = 0; n < nn; ++n) {
            REAL* out = dB + ((int64_t)e * nn + n) * kn;
            for (int kk = 0; kk < kn; ++kk) out[kk] = 0;
            for (int64_t r = offsets[e]; r < offsets[e + 1]; ++r) {
                const REAL g = dC[r * N + n0 + n];
                const REAL* a = A + r * K + k0;
                for (int kk = 0; kk < kn; ++kk) out[kk] += g * a[kk];
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Gated activation                                                          */
/* ------------------------------------------------------------------------ */
static inline REAL sigm(REAL x) { return (REAL)(1.0 / (1.0 + exp(-(double)x))); }

/* Act[r,j] = silu(Z[r,j]) * Z[r,f+j],  silu(g) = g * sigmoid(g) */
void FN(orc_swiglu)(const REAL* Z, int64_t R, int f, REAL* Act) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int j = 0; j < f; ++j) {
            REAL g = Z[r * 2 * f + j], u = Z[r * 2 * f + f + j];
            Act[r * f + j] = g * sigm(g) * u;
        }
}

/* dZ[r,j]   = dAct * up * d silu(g)/dg,  d silu/dg = s (1 + g (1 - s)),  s = sigmoid(g)
 * dZ[r,f+j] = dAct * silu(g) */
void FN(orc_swiglu_bwd)(const REAL* dAct, const REAL* Z, int64_t R, int f, REAL* dZ) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int j = 0; j < f; ++j) {
            REAL g = Z[r * 2 * f + j], u = Z[r * 2 * f + f + j], d = dAct[r * f + j];
            REAL s = sigm(g);
            dZ[r * 2 * f + j] = d * u * s * (1 + g * (1 - s));
            dZ[r * 2 * f + f + j] = d * g * s;
        }
}

/* ------------------------------------------------------------------------ */
/* Unpermute + weighted combine, and its backward                            */
/* ------------------------------------------------------------------------ */
/* Y[t,:] = sum_s w[t,s] * O[row_of[t,s],:] (+ residual[t,:]);  prob==NULL: w = 1;
 * slots with row_of < 0 contribute nothing. */
void FN(orc_combine)(const REAL* O, const int32_t* row_of, const REAL* prob, const REAL* residual,
                     int T, int k, int h, REAL* Y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        REAL* y = Y + (int64_t)t * h;
        for (int c = 0; c < h; ++c) y[c] = residual ? residual[(int64_t)t * h + c] : 0;
        for (int s = 0; s < k; ++s) {
            int32_t r = row_of[(int64_t)t * k + s];
            if (r < 0) continue;
            REAL w = prob ? prob[(int64_t)t * k + s] : 1;
            const REAL* o = O + (int64_t)r * h;
            for (int c = 0; c < h; ++c) y[c] += w * o[c];
        }
    }
}

/* For L = <dY, Y>:  dO[row_of[t,s],:] = w[t,s] * dY[t,:],  dprob[t,s] = <dY[t,:], O[row_of[t,s],:]>.
 * Rows no (t,s) points at (padding) get dO = 0; skipped slots get dprob = 0. */
void FN(orc_combine_bwd)(const REAL* dY, const REAL* O, const int32_t* row_of, const REAL* prob,
                         int T, int k, int h, int64_t R, REAL* dO, REAL* dprob) {
    for (int64_t i = 0; i < R * h; ++i) dO[i] = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const REAL* g = dY + (int64_t)t * h;
        for (int s = 0; s < k; ++s) {
            int32_t r = row_of[(int64_t)t * k + s];
            if (r < 0) { if (dprob) dprob[(int64_t)t * k + s] = 0; continue; }
            REAL w = prob ? prob[(int64_t)t * k + s] : 1;
            REAL* d = dO + (int64_t)r * h;
            REAL acc = 0;
            for (int c = 0; c < h; ++c) {
                d[c] = w * g[c];
                if (O) acc += g[c] * O[(int64_t)r * h + c];
            }
            if (dprob) dprob[(int64_t)t * k + s] = acc;
        }
    }
}
