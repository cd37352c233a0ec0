// Measurement aid, not part of the C ABI of the layer: the rate the matrix pipes of this very GPU sustain when
// nothing else happens -- every operand already in registers, no LDS, no memory -- for the two MFMA shapes the
// grouped GEMMs use (v_mfma_f32_16x16x32_bf16; v_mfma_scale_f32_32x32x64_f8f6f4 on E4M3 codes), on all-zero and on
// random operands.  On zeros the chip reaches its nominal rate; on random operands the sustained clock is set by
// the power limit, and that rate, not the nominal peak, is what a GEMM kernel on real data can approach.
// bench.py loads libmfma_ceiling.so and reports the four numbers beside its own ("box_reference").
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ inline uint32_t lcg(uint32_t& s) { s = s * 1664525u + 1013904223u; return s; }

// one wave per SIMD, 256 accumulators per lane, like the GEMM kernels' wave tile
template <int FP8>
__global__ __launch_bounds__(256, 1) void ceiling_kernel(float* out, int iters, int random) {
    uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
    float sum = 0.f;
    if (FP8) {
        f32x16_t acc[4][4];
        i32x8_t a[4], b[4];
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 4; ++j)
                for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;
        for (int i = 0; i < 4; ++i)
            for (int x = 0; x < 8; ++x) {   // finite E4M3 codes (exponent field 1111 avoided)
                uint32_t wa = lcg(seed) & 0xf7f7f7f7u, wb = lcg(seed) & 0xf7f7f7f7u;
                a[i][x] = random ? (int)wa : 0;
                b[i][x] = random ? (int)wb : 0;
            }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j], b[i], acc[i][j], 0, 0, 0, 120, 0, 120);
#pragma unroll
            for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(a[i]), "+v"(b[i]));   // (keeps the loop from being folded)
        }
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 4; ++j)
                for (int x = 0; x < 16; ++x) sum += acc[i][j][x];
    } else {
        f32x4_t acc[8][8];
        bf16x8_t a[8], b[8];
        for (int i = 0; i < 8; ++i)
            for (int j = 0; j < 8; ++j)
                for (int x = 0; x < 4; ++x) acc[i][j][x] = 0.f;
        for (int i = 0; i < 8; ++i)
            for (int x = 0; x < 8; ++x) {   // uniform in (-0.05, 0.05): the magnitude of the layer's operands
                a[i][x] = random ? (__bf16)(((int)(lcg(seed) >> 8) % 2001 - 1000) * 5e-5f) : (__bf16)0.f;
                b[i][x] = random ? (__bf16)(((int)(lcg(seed) >> 8) % 2001 - 1000) * 5e-5f) : (__bf16)0.f;
            }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j], b[i], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(a[i]), "+v"(b[i]));
        }
        for (int i = 0; i < 8; ++i)
            for (int j = 0; j < 8; ++j)
                for (int x = 0; x < 4; ++x) sum += acc[i][j][x];
    }
    out[blockIdx.x * 256 + threadIdx.x] = sum;
}

// fp8 = 0: bf16 16x16x32; 1: E4M3 32x32x64.  random = 0: zeros; 1: random operands.  ms: how long to measure
// (about; the launch is repeated).  Returns 0 and the rate in *tflops, or the HIP error code.  Uses the null stream,
// allocates and frees a 256 KB result buffer.
extern "C" int mfma_ceiling(int fp8, int random, int ms, float* tflops) {
    int dev = 0, cus = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return (int)err;
    err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (err != hipSuccess) return (int)err;
    float* out = nullptr;
    err = hipMalloc(&out, (size_t)cus * 256 * sizeof(float));
    if (err != hipSuccess) return (int)err;
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    const int iters = 4000;   // per wave and iteration: 64 x 16x16x32 bf16 MFMAs = 2^20 flop, or 16 x 32x32x64 fp8 = 2^21
    const double flop_per_launch = (fp8 ? 2097152.0 : 1048576.0) * iters * 4 * cus;   // 4 waves per workgroup, one per CU
    float t = 0.f;
    int reps = 2;
    for (int pass = 0; pass < 2; ++pass) {                        // pass 0 warms up and sizes pass 1
        hipEventRecord(e0, 0);
        for (int r = 0; r < reps; ++r) {
            if (fp8) hipLaunchKernelGGL(ceiling_kernel<1>, dim3(cus), dim3(256), 0, 0, out, iters, random);
            else hipLaunchKernelGGL(ceiling_kernel<0>, dim3(cus), dim3(256), 0, 0, out, iters, random);
        }
        hipEventRecord(e1, 0);
        err = hipEventSynchronize(e1);
        if (err != hipSuccess) break;
        hipEventElapsedTime(&t, e0, e1);
        if (pass == 0) {
            const int want = (int)(ms / (t / reps) + 0.5f);
            *tflops = (float)(flop_per_launch * reps / t / 1e9);
            reps = want < 1 ? 1 : (want > 400 ? 400 : want);
        } else {
            *tflops = (float)(flop_per_launch * reps / t / 1e9);
        }
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    hipFree(out);
    return (int)err;
}
