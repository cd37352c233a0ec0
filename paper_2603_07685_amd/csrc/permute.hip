// moe_permute / moe_unpermute_combine(+bwd): the row-ID map and the row moves
// (Sec. 4.3.3: preprocessing, permute, unpermute; Sec. 5.4.1: padding fused into permute).
//
// Row-ID map = stable counting sort of the T*k (token, slot) pairs by expert, with
// no atomics on positions so the map is bit-reproducible:
//   1. hist : one wavefront per chunk of PERMUTE_CHUNK consecutive pairs builds
//             that chunk's per-expert histogram (LDS) and stores it to the workspace;
//   2. scan : per expert, exclusive scan of the chunk histograms (chunk bases),
//             totals -> counts, padded exclusive scan over experts -> offsets;
//   3. rank : the same wavefront walks its chunk again, 64 pairs at a time; a
//             lane's rank among equal experts inside the 64 comes from ballots over
//             the bits of the expert id, the running per-expert count sits in LDS.
// Row moves are token-major: a workgroup reads one source row once and writes
// its k copies (permute), or reads the k expert rows once and writes one row
// (combine), 16 bytes per lane per access, fp32 accumulation in registers.
#include "common.h"
#include "layout.h"

#ifndef MOVE_THREADS
#define MOVE_THREADS 256
#endif

__device__ __forceinline__ u32x4_t mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    u32x4_t v = {a, b, c, d};
    return v;
}

// ---------------------------------------------------------------------------
// 1. per-chunk histograms
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void permute_hist_kernel(const int32_t* __restrict__ idx, int64_t pairs, int E,
                                                          int32_t* __restrict__ chunk_hist) {
    extern __shared__ int32_t lds[];
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) lds[e] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * PERMUTE_CHUNK;
    for (int i = 0; i < PERMUTE_CHUNK; i += 64) {
        int64_t j = base + i + lane;
        if (j < pairs) {
            int e = idx[j];
            if (e >= 0 && e < E) atomicAdd(&lds[e], 1);
        }
    }
    __syncthreads();
    for (int e = lane; e < E; e += 64) chunk_hist[(int64_t)blockIdx.x * E + e] = lds[e];
}

// ---------------------------------------------------------------------------
// 2. scans: chunk bases per expert, counts, padded offsets
// ---------------------------------------------------------------------------
#define SCAN_LDS_INTS 12288  // chunk histograms staged per pass (48 KB)
__global__ __launch_bounds__(1024) void permute_scan_kernel(int32_t* __restrict__ chunk_hist, int nchunks, int E,
                                                            int align, int32_t* __restrict__ counts,
                                                            int32_t* __restrict__ offsets) {
    // One workgroup.  The [nchunks][E] histogram table is brought into LDS with coalesced loads, a block of
    // chunks at a time; thread e then runs the exclusive scan of expert e down the block in LDS (the serial
    // chain is over LDS latency, not over dependent global loads) and the block is written back coalesced.
    __shared__ int32_t tab[SCAN_LDS_INTS];
    __shared__ int32_t tot[1024];
    const int tid = threadIdx.x;
    const int per_pass = SCAN_LDS_INTS / E;  // chunks per pass (E <= 1024 is checked by the caller)
    int32_t run = 0;
    for (int c0 = 0; c0 < nchunks; c0 += per_pass) {
        const int nc = min(per_pass, nchunks - c0);
        int32_t* g = chunk_hist + (int64_t)c0 * E;
        for (int i = tid; i < nc * E; i += 1024) tab[i] = g[i];
        __syncthreads();
        if (tid < E) {
            for (int c = 0; c < nc; ++c) {
                const int32_t v = tab[c * E + tid];
                tab[c * E + tid] = run;
                run += v;
            }
        }
        __syncthreads();
        for (int i = tid; i < nc * E; i += 1024) g[i] = tab[i];
        __syncthreads();
    }
    if (tid < E) {
        tot[tid] = run;
        if (counts) counts[tid] = run;
    }
    __syncthreads();
    if (tid == 0) {
        int64_t r = 0;
        for (int i = 0; i < E; ++i) {
            offsets[i] = (int32_t)r;
            r += ((int64_t)tot[i] + align - 1) / align * align;
        }
        offsets[E] = (int32_t)r;
    }
}

// ---------------------------------------------------------------------------
// 3. stable ranks -> row_of, src_of
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void permute_rank_kernel(const int32_t* __restrict__ idx, int64_t pairs, int E,
                                                          int nbits, const int32_t* __restrict__ chunk_base,
                                                          const int32_t* __restrict__ offsets,
                                                          int32_t* __restrict__ row_of, int32_t* __restrict__ src_of) {
    extern __shared__ int32_t run[];  // next free position of each expert for this chunk
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) run[e] = offsets[e] + chunk_base[(int64_t)blockIdx.x * E + e];
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * PERMUTE_CHUNK;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int i = 0; i < PERMUTE_CHUNK; i += 64) {
        int64_t j = base + i + lane;
        if (base + i >= pairs) break;  // uniform
        int e = j < pairs ? idx[j] : -1;
        bool valid = e >= 0 && e < E;
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            uint64_t m = __ballot((e >> b) & 1);
            peers &= ((e >> b) & 1) ? m : ~m;
        }
        const int rank = __popcll(peers & below);
        if (valid) {
            int row = run[e] + rank;
            row_of[j] = row;
            src_of[row] = (int32_t)j;
        } else if (j < pairs) {
            row_of[j] = -1;
        }
        __syncthreads();  // single wavefront: orders the LDS reads above before the update
        if (valid && rank == 0) run[e] += __popcll(peers);  // lowest lane of each group
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// permute: token-major row scatter + zero fill of padding rows
// ---------------------------------------------------------------------------
// grid = T token blocks followed by E padding blocks.
__global__ __launch_bounds__(MOVE_THREADS) void permute_rows_kernel(
    const u32x4_t* __restrict__ X, const int32_t* __restrict__ row_of, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ counts, int T, int k, int E, int vec_per_row, u32x4_t* __restrict__ Xp) {
    __shared__ int32_t rows[32 * 4];
    const int b = blockIdx.x;
    if (b < T) {
        for (int s = threadIdx.x; s < k; s += MOVE_THREADS) rows[s] = row_of[(int64_t)b * k + s];
        __syncthreads();
        const u32x4_t* src = X + (int64_t)b * vec_per_row;
        // four 16-byte pieces of the source row per thread are loaded before the first copy is written, so a
        // row of up to 16 KB is in flight at once instead of one piece per thread
        for (int c0 = threadIdx.x; c0 < vec_per_row; c0 += 4 * MOVE_THREADS) {
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * MOVE_THREADS;
                if (c < vec_per_row) v[u] = src[c];
            }
            for (int s = 0; s < k; ++s) {
                const int r = rows[s];
                if (r < 0) continue;
                u32x4_t* dst = Xp + (int64_t)r * vec_per_row;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u * MOVE_THREADS;
                    if (c < vec_per_row) __builtin_nontemporal_store(v[u], &dst[c]);
                }
            }
        }
    } else {
        const int e = b - T;
        const int64_t r0 = (int64_t)offsets[e] + counts[e], r1 = offsets[e + 1];
        const int64_t n = (r1 - r0) * vec_per_row;
        u32x4_t z = mk4(0, 0, 0, 0);
        u32x4_t* dst = Xp + r0 * vec_per_row;
        for (int64_t i = threadIdx.x; i < n; i += MOVE_THREADS) dst[i] = z;
    }
}

// ---------------------------------------------------------------------------
// combine: Y[t] = sum_s w[t,s] * O[row_of[t,s]] (+ residual[t]); fp32 accumulation
// ---------------------------------------------------------------------------
template <bool F32>
__device__ __forceinline__ void acc_vec(float (&a)[8], u32x4_t v, float w);
template <>
__device__ __forceinline__ void acc_vec<false>(float (&a)[8], u32x4_t v, float w) {
    a[0] += w * bf16_lo(v.x); a[1] += w * bf16_hi(v.x);
    a[2] += w * bf16_lo(v.y); a[3] += w * bf16_hi(v.y);
    a[4] += w * bf16_lo(v.z); a[5] += w * bf16_hi(v.z);
    a[6] += w * bf16_lo(v.w); a[7] += w * bf16_hi(v.w);
}
template <>
__device__ __forceinline__ void acc_vec<true>(float (&a)[8], u32x4_t v, float w) {
    a[0] += w * __uint_as_float(v.x); a[1] += w * __uint_as_float(v.y);
    a[2] += w * __uint_as_float(v.z); a[3] += w * __uint_as_float(v.w);
}

#define COMBINE_MAX_K 32

template <bool F32>
__global__ __launch_bounds__(MOVE_THREADS) void combine_kernel(
    const u32x4_t* __restrict__ O, const int32_t* __restrict__ row_of, const float* __restrict__ prob,
    const u32x4_t* __restrict__ residual, int T, int k, int vec_per_row, u32x4_t* __restrict__ Y) {
    __shared__ int32_t rows[COMBINE_MAX_K];
    __shared__ float wts[COMBINE_MAX_K];
    const int t = blockIdx.x;
    for (int s = threadIdx.x; s < k; s += MOVE_THREADS) {
        rows[s] = row_of[(int64_t)t * k + s];
        wts[s] = prob ? prob[(int64_t)t * k + s] : 1.0f;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < vec_per_row; c += MOVE_THREADS) {
        float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (residual) acc_vec<F32>(a, residual[(int64_t)t * vec_per_row + c], 1.0f);
        int s = 0;
        for (; s + 8 <= k; s += 8) {  // eight independent row reads in flight
            u32x4_t v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = rows[s + j];
                v[j] = r >= 0 ? __builtin_nontemporal_load(&O[(int64_t)r * vec_per_row + c]) : mk4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) acc_vec<F32>(a, v[j], wts[s + j]);
        }
        for (; s + 4 <= k; s += 4) {  // four independent row reads in flight
            int r0 = rows[s], r1 = rows[s + 1], r2 = rows[s + 2], r3 = rows[s + 3];
            u32x4_t z = mk4(0, 0, 0, 0);
            u32x4_t v0 = r0 >= 0 ? __builtin_nontemporal_load(&O[(int64_t)r0 * vec_per_row + c]) : z;
            u32x4_t v1 = r1 >= 0 ? __builtin_nontemporal_load(&O[(int64_t)r1 * vec_per_row + c]) : z;
            u32x4_t v2 = r2 >= 0 ? __builtin_nontemporal_load(&O[(int64_t)r2 * vec_per_row + c]) : z;
            u32x4_t v3 = r3 >= 0 ? __builtin_nontemporal_load(&O[(int64_t)r3 * vec_per_row + c]) : z;
            acc_vec<F32>(a, v0, wts[s]);
            acc_vec<F32>(a, v1, wts[s + 1]);
            acc_vec<F32>(a, v2, wts[s + 2]);
            acc_vec<F32>(a, v3, wts[s + 3]);
        }
        for (; s < k; ++s) {
            int r = rows[s];
            if (r >= 0) acc_vec<F32>(a, O[(int64_t)r * vec_per_row + c], wts[s]);
        }
        u32x4_t out;
        if (F32) {
            out = mk4(__float_as_uint(a[0]), __float_as_uint(a[1]), __float_as_uint(a[2]), __float_as_uint(a[3]));
        } else {
            out = mk4(pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(a[4], a[5]), pack_bf16(a[6], a[7]));
        }
        Y[(int64_t)t * vec_per_row + c] = out;
    }
}

// ---------------------------------------------------------------------------
// combine backward: dO[row_of[t,s]] = w[t,s] * dY[t];  dprob[t,s] = <dY[t], O[row_of[t,s]]>
// ---------------------------------------------------------------------------
template <bool F32>
__device__ __forceinline__ u32x4_t scale_vec(u32x4_t v, float w);
template <>
__device__ __forceinline__ u32x4_t scale_vec<false>(u32x4_t v, float w) {
    return mk4(pack_bf16(w * bf16_lo(v.x), w * bf16_hi(v.x)), pack_bf16(w * bf16_lo(v.y), w * bf16_hi(v.y)),
                      pack_bf16(w * bf16_lo(v.z), w * bf16_hi(v.z)), pack_bf16(w * bf16_lo(v.w), w * bf16_hi(v.w)));
}
template <>
__device__ __forceinline__ u32x4_t scale_vec<true>(u32x4_t v, float w) {
    return mk4(__float_as_uint(w * __uint_as_float(v.x)), __float_as_uint(w * __uint_as_float(v.y)),
                      __float_as_uint(w * __uint_as_float(v.z)), __float_as_uint(w * __uint_as_float(v.w)));
}
template <bool F32>
__device__ __forceinline__ float dot_vec(u32x4_t a, u32x4_t b);
template <>
__device__ __forceinline__ float dot_vec<false>(u32x4_t a, u32x4_t b) {
    return bf16_lo(a.x) * bf16_lo(b.x) + bf16_hi(a.x) * bf16_hi(b.x) + bf16_lo(a.y) * bf16_lo(b.y) +
           bf16_hi(a.y) * bf16_hi(b.y) + bf16_lo(a.z) * bf16_lo(b.z) + bf16_hi(a.z) * bf16_hi(b.z) +
           bf16_lo(a.w) * bf16_lo(b.w) + bf16_hi(a.w) * bf16_hi(b.w);
}
template <>
__device__ __forceinline__ float dot_vec<true>(u32x4_t a, u32x4_t b) {
    return __uint_as_float(a.x) * __uint_as_float(b.x) + __uint_as_float(a.y) * __uint_as_float(b.y) +
           __uint_as_float(a.z) * __uint_as_float(b.z) + __uint_as_float(a.w) * __uint_as_float(b.w);
}

template <bool F32>
__global__ __launch_bounds__(MOVE_THREADS) void combine_bwd_kernel(
    const u32x4_t* __restrict__ dY, const u32x4_t* __restrict__ O, const int32_t* __restrict__ row_of,
    const float* __restrict__ prob, int T, int k, int vec_per_row, u32x4_t* __restrict__ dO,
    float* __restrict__ dprob) {
    __shared__ int32_t rows[COMBINE_MAX_K];
    __shared__ float wts[COMBINE_MAX_K];
    __shared__ float part[COMBINE_MAX_K][MOVE_THREADS / 64];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int s = threadIdx.x; s < k; s += MOVE_THREADS) {
        rows[s] = row_of[(int64_t)t * k + s];
        wts[s] = prob ? prob[(int64_t)t * k + s] : 1.0f;
    }
    __syncthreads();
    const bool want_dot = dprob != nullptr && O != nullptr;
    // slots in chunks of 8: per 16-byte piece of dY[t] the 8 expert rows are read together (9 loads in flight per
    // thread) and the 8 scaled copies written; a slot's partial dot product stays in one register, summed over
    // the pieces in increasing order
    for (int s0 = 0; s0 < k; s0 += 8) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        for (int c = threadIdx.x; c < vec_per_row; c += MOVE_THREADS) {
            const u32x4_t g = dY[(int64_t)t * vec_per_row + c];
            u32x4_t o[8];
            if (want_dot) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int r = s0 + j < k ? rows[s0 + j] : -1;
                    if (r >= 0) o[j] = __builtin_nontemporal_load(&O[(int64_t)r * vec_per_row + c]);
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = s0 + j < k ? rows[s0 + j] : -1;
                if (r >= 0) {
                    if (want_dot) acc[j] += dot_vec<F32>(g, o[j]);
                    if (dO) __builtin_nontemporal_store(scale_vec<F32>(g, wts[s0 + j]), &dO[(int64_t)r * vec_per_row + c]);
                }
            }
        }
        if (dprob) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (s0 + j < k) {
                    float a = acc[j];
#pragma unroll
                    for (int o2 = 32; o2 > 0; o2 >>= 1) a += __shfl_xor(a, o2);
                    if (lane == 0) part[s0 + j][wave] = a;
                }
            }
        }
    }
    if (dprob) {
        __syncthreads();
        for (int s = threadIdx.x; s < k; s += MOVE_THREADS) {
            float a = 0.f;
            for (int w = 0; w < MOVE_THREADS / 64; ++w) a += part[s][w];
            dprob[(int64_t)t * k + s] = a;
        }
    }
}

// zero every row whose src_of is negative (padding)
__global__ __launch_bounds__(MOVE_THREADS) void zero_pad_rows_kernel(const int32_t* __restrict__ src_of, int64_t Rcap,
                                                                     int vec_per_row, u32x4_t* __restrict__ dO) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (MOVE_THREADS / 64) + wave;
    if (r >= Rcap || src_of[r] >= 0) return;
    u32x4_t z = mk4(0, 0, 0, 0);
    for (int c = lane; c < vec_per_row; c += 64) dO[r * vec_per_row + c] = z;
}

// ---------------------------------------------------------------------------
// host entry points
// ---------------------------------------------------------------------------
static int bits_for(int E) {
    int b = 0;
    while ((1 << b) < E) ++b;
    return b;
}

// Argument checks shared by moe_permute and moe_permute_static (err: where the message goes, 512 bytes, or NULL).
static moe_status permute_check(char* err, const void* X, moe_dtype dt, const int32_t* idx, int T, int k, int h, int E,
                                int align, const void* Xp, int64_t Rcap, const int32_t* row_of, const int32_t* src_of,
                                const int32_t* offsets, const int32_t* counts) {
#define PERMUTE_FAIL(code, ...)                        \
    do {                                               \
        if (err) snprintf(err, 512, __VA_ARGS__);      \
        return (code);                                 \
    } while (0)
    if (!idx || !row_of || !src_of || !offsets || !counts) PERMUTE_FAIL(MOE_ERR_ARG, "moe_permute: NULL map pointer");
    if ((X == nullptr) != (Xp == nullptr)) PERMUTE_FAIL(MOE_ERR_ARG, "moe_permute: X and Xp must both be given or both NULL");
    if (T < 0 || k < 1 || k > 32 || E < 1 || E > 1024 || align < 1 || h < 1)
        PERMUTE_FAIL(MOE_ERR_ARG, "moe_permute: need T>=0, 1<=k<=32, 1<=E<=1024, align>=1, h>=1");
    if (dt != MOE_BF16 && dt != MOE_F32) PERMUTE_FAIL(MOE_ERR_UNSUPPORTED, "moe_permute: dtype must be bf16 or f32");
    const size_t row_bytes = (size_t)h * moe_dtype_size(dt);
    if (X && row_bytes % 16) PERMUTE_FAIL(MOE_ERR_ARG, "moe_permute: row size %zu B is not a multiple of 16", row_bytes);
    const int64_t pairs = (int64_t)T * k;
    const int64_t need = pairs + (int64_t)E * (align - 1);
    if (Rcap < need) PERMUTE_FAIL(MOE_ERR_ARG, "moe_permute: Rcap=%lld < T*k+E*(align-1)=%lld", (long long)Rcap, (long long)need);
    if (Rcap > 0x7fffffffLL) PERMUTE_FAIL(MOE_ERR_ARG, "moe_permute: Rcap exceeds int32");
#undef PERMUTE_FAIL
    return MOE_OK;
}

// The launches of one permute call; chunk_hist = int32 [chunks, E] of device scratch (every entry is written by the
// histogram kernel before it is read: the buffer needs no clearing).
static void permute_launch(hipStream_t s, const void* X, moe_dtype dt, const int32_t* idx, int T, int k, int h, int E,
                           int align, void* Xp, int64_t Rcap, int32_t* row_of, int32_t* src_of, int32_t* offsets,
                           int32_t* counts, int32_t* chunk_hist) {
    const int64_t pairs = (int64_t)T * k;
    const int nchunks = (int)moe_permute_chunks(pairs);
    const size_t shm = (size_t)E * sizeof(int32_t);
    moe_launch_fill_i32(src_of, Rcap, -1, s);
    if (nchunks > 0) hipLaunchKernelGGL(permute_hist_kernel, dim3(nchunks), dim3(64), shm, s, idx, pairs, E, chunk_hist);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(1024), 0, s, chunk_hist, nchunks, E, align, counts, offsets);
    if (nchunks > 0)
        hipLaunchKernelGGL(permute_rank_kernel, dim3(nchunks), dim3(64), shm, s, idx, pairs, E, bits_for(E), chunk_hist,
                           offsets, row_of, src_of);
    if (X) {
        const int vec = (int)((size_t)h * moe_dtype_size(dt) / 16);
        hipLaunchKernelGGL(permute_rows_kernel, dim3(T + E), dim3(MOVE_THREADS), 0, s, (const u32x4_t*)X, row_of, offsets,
                           counts, T, k, E, vec, (u32x4_t*)Xp);
    }
}

extern "C" moe_status moe_permute(moe_ctx* ctx, void* stream, const void* X, moe_dtype dt,
                                  const int32_t* idx, int T, int k, int h, int E, int align,
                                  void* Xp, int64_t Rcap,
                                  int32_t* row_of, int32_t* src_of, int32_t* offsets, int32_t* counts) {
    if (!ctx) return MOE_ERR_ARG;
    const moe_status st = permute_check(ctx->err, X, dt, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts);
    if (st != MOE_OK) return st;
    const int64_t pairs = (int64_t)T * k;
    if (MOE_WS_RESERVED + moe_permute_ws_bytes(pairs, E) > ctx->ws_bytes)
        MOE_FAIL(ctx, MOE_ERR_WORKSPACE, "moe_permute: workspace %zu B < %zu B", ctx->ws_bytes,
                 MOE_WS_RESERVED + moe_permute_ws_bytes(pairs, E));
    permute_launch((hipStream_t)stream, X, dt, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts,
                   (int32_t*)((char*)ctx->ws + MOE_WS_RESERVED));
    MOE_LAUNCH_CHECK(ctx, "moe_permute kernels");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// moe_permute_static: moe_permute for callers that cannot allocate (no context, no hipMalloc anywhere on the path).
// The per-chunk histograms live in a file-scope device array instead of a context workspace.  Every GPU the library
// runs on holds its own copy of the array at its own address until the process ends; the address is looked up once
// per device, on the first call made with that device current, and kept.
// ---------------------------------------------------------------------------
#define PERMUTE_STATIC_BYTES (1u << 20)
#define PERMUTE_STATIC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[PERMUTE_STATIC_BYTES];
static void* scratch_ptr_of_device[PERMUTE_STATIC_MAX_DEVICES];  // host copies of the per-device addresses (0 = not yet looked up)

extern "C" moe_status moe_permute_static(void* stream, const void* X, moe_dtype dt,
                                         const int32_t* idx, int T, int k, int h, int E, int align,
                                         void* Xp, int64_t Rcap,
                                         int32_t* row_of, int32_t* src_of, int32_t* offsets, int32_t* counts) {
    char* err = moe_ctxless_error();  // this host thread's message buffer, read back with moe_last_error(NULL)
    err[0] = 0;
    const moe_status st = permute_check(err, X, dt, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts);
    if (st != MOE_OK) return st;
    const size_t need = moe_permute_ws_bytes((int64_t)T * k, E);
    if (need > PERMUTE_STATIC_BYTES) {
        snprintf(err, 512, "moe_permute_static: ceil(T*k/%d)*E*4 = %zu B exceeds the fixed scratch of %u B; use moe_permute",
                 PERMUTE_CHUNK, need, PERMUTE_STATIC_BYTES);
        return MOE_ERR_WORKSPACE;
    }
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= PERMUTE_STATIC_MAX_DEVICES) {
        snprintf(err, 512, "moe_permute_static: no current device below %d (%s)", PERMUTE_STATIC_MAX_DEVICES, hipGetErrorString(e));
        return MOE_ERR_HIP;
    }
    // (two host threads racing here both look up the same address and store the same value)
    void* ptr = __atomic_load_n(&scratch_ptr_of_device[dev], __ATOMIC_ACQUIRE);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            snprintf(err, 512, "moe_permute_static: hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
            return MOE_ERR_HIP;
        }
        __atomic_store_n(&scratch_ptr_of_device[dev], ptr, __ATOMIC_RELEASE);
    }
    permute_launch((hipStream_t)stream, X, dt, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts,
                   (int32_t*)ptr);
    e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(err, 512, "launch moe_permute_static kernels: %s", hipGetErrorString(e));
        return MOE_ERR_HIP;
    }
    return MOE_OK;
}

extern "C" moe_status moe_unpermute_combine(moe_ctx* ctx, void* stream, const void* O, moe_dtype dt,
                                            const int32_t* row_of, const float* prob, const void* residual,
                                            int T, int k, int h, void* Y) {
    if (!ctx) return MOE_ERR_ARG;
    if (!O || !row_of || !Y) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine: NULL pointer");
    if (T < 0 || k < 1 || k > COMBINE_MAX_K || h < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine: need T>=0, 1<=k<=32, h>=1");
    if (dt != MOE_BF16 && dt != MOE_F32) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_unpermute_combine: dtype must be bf16 or f32");
    const size_t row_bytes = (size_t)h * moe_dtype_size(dt);
    if (row_bytes % 16) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine: row size %zu B is not a multiple of 16", row_bytes);
    if (T == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)stream;
    const int vec = (int)(row_bytes / 16);
    if (dt == MOE_BF16)
        hipLaunchKernelGGL(combine_kernel<false>, dim3(T), dim3(MOVE_THREADS), 0, s, (const u32x4_t*)O, row_of, prob,
                           (const u32x4_t*)residual, T, k, vec, (u32x4_t*)Y);
    else
        hipLaunchKernelGGL(combine_kernel<true>, dim3(T), dim3(MOVE_THREADS), 0, s, (const u32x4_t*)O, row_of, prob,
                           (const u32x4_t*)residual, T, k, vec, (u32x4_t*)Y);
    MOE_LAUNCH_CHECK(ctx, "combine_kernel");
    return MOE_OK;
}

extern "C" moe_status moe_unpermute_combine_bwd(moe_ctx* ctx, void* stream, const void* dY, const void* O,
                                                moe_dtype dt, const int32_t* row_of, const int32_t* src_of,
                                                const float* prob, int T, int k, int h, int64_t Rcap,
                                                void* dO, float* dprob) {
    if (!ctx) return MOE_ERR_ARG;
    if (!dY || !row_of || !src_of) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine_bwd: NULL pointer");
    if (!dO && !dprob) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine_bwd: neither dO nor dprob requested");
    if (dprob && !O) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine_bwd: dprob needs O");
    if (T < 0 || k < 1 || k > COMBINE_MAX_K || h < 1 || Rcap < 0)
        MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine_bwd: need T>=0, 1<=k<=32, h>=1, Rcap>=0");
    if (dt != MOE_BF16 && dt != MOE_F32) MOE_FAIL(ctx, MOE_ERR_UNSUPPORTED, "moe_unpermute_combine_bwd: dtype must be bf16 or f32");
    const size_t row_bytes = (size_t)h * moe_dtype_size(dt);
    if (row_bytes % 16) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_unpermute_combine_bwd: row size %zu B is not a multiple of 16", row_bytes);
    hipStream_t s = (hipStream_t)stream;
    const int vec = (int)(row_bytes / 16);
    if (Rcap > 0 && dO)
        hipLaunchKernelGGL(zero_pad_rows_kernel, dim3((unsigned)ceil_div64(Rcap, MOVE_THREADS / 64)), dim3(MOVE_THREADS), 0,
                           s, src_of, Rcap, vec, (u32x4_t*)dO);
    if (T > 0) {
        if (dt == MOE_BF16)
            hipLaunchKernelGGL(combine_bwd_kernel<false>, dim3(T), dim3(MOVE_THREADS), 0, s, (const u32x4_t*)dY,
                               (const u32x4_t*)O, row_of, prob, T, k, vec, (u32x4_t*)dO, dprob);
        else
            hipLaunchKernelGGL(combine_bwd_kernel<true>, dim3(T), dim3(MOVE_THREADS), 0, s, (const u32x4_t*)dY,
                               (const u32x4_t*)O, row_of, prob, T, k, vec, (u32x4_t*)dO, dprob);
    }
    MOE_LAUNCH_CHECK(ctx, "combine_bwd kernels");
    return MOE_OK;
}

// ---------------------------------------------------------------------------
// eq. (2) helpers: routing weights per permuted row, and the way back for their gradients
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_row_prob_kernel(const float* __restrict__ prob,
                                                              const int32_t* __restrict__ src_of, int64_t Rcap,
                                                              float* __restrict__ row_prob) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= Rcap) return;
    const int32_t j = src_of[r];
    row_prob[r] = j >= 0 ? prob[j] : 0.0f;
}

__global__ __launch_bounds__(256) void scatter_row_dprob_kernel(const float* __restrict__ part, int parts,
                                                                const int32_t* __restrict__ row_of, int64_t pairs,
                                                                float* __restrict__ dprob) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= pairs) return;
    const int32_t r = row_of[j];
    float acc = 0.f;
    if (r >= 0)
        for (int q = 0; q < parts; ++q) acc += part[(int64_t)r * parts + q];
    dprob[j] = acc;
}

extern "C" moe_status moe_gather_row_prob(moe_ctx* ctx, void* stream, const float* prob, const int32_t* src_of,
                                          int64_t Rcap, float* row_prob) {
    if (!ctx) return MOE_ERR_ARG;
    if (!prob || !src_of || !row_prob) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_gather_row_prob: NULL pointer");
    if (Rcap < 0 || Rcap > 0x7fffffffLL) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_gather_row_prob: need 0 <= Rcap < 2^31");
    if (Rcap == 0) return MOE_OK;
    hipLaunchKernelGGL(gather_row_prob_kernel, dim3((unsigned)ceil_div64(Rcap, 256)), dim3(256), 0, (hipStream_t)stream,
                       prob, src_of, Rcap, row_prob);
    MOE_LAUNCH_CHECK(ctx, "gather_row_prob_kernel");
    return MOE_OK;
}

extern "C" moe_status moe_scatter_row_dprob(moe_ctx* ctx, void* stream, const float* dprob_part, int parts,
                                            const int32_t* row_of, int T, int k, float* dprob) {
    if (!ctx) return MOE_ERR_ARG;
    if (!dprob_part || !row_of || !dprob) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_scatter_row_dprob: NULL pointer");
    if (parts < 1 || T < 0 || k < 1) MOE_FAIL(ctx, MOE_ERR_ARG, "moe_scatter_row_dprob: need parts >= 1, T >= 0, k >= 1");
    const int64_t pairs = (int64_t)T * k;
    if (pairs == 0) return MOE_OK;
    hipLaunchKernelGGL(scatter_row_dprob_kernel, dim3((unsigned)ceil_div64(pairs, 256)), dim3(256), 0, (hipStream_t)stream,
                       dprob_part, parts, row_of, pairs, dprob);
    MOE_LAUNCH_CHECK(ctx, "scatter_row_dprob_kernel");
    return MOE_OK;
}
