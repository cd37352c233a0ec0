// Context: device id, workspace, error reporting.
#include "common.h"

#include <new>

#include "layout.h"

__global__ void fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

void moe_launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t s) {
    if (n <= 0) return;
    int blocks = (int)(ceil_div64(n, 256) < 2048 ? ceil_div64(n, 256) : 2048);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks), dim3(256), 0, s, p, n, v);
}

extern "C" size_t moe_workspace_bytes(int T, int k, int E, int h, int f_max) {
    if (T < 0 || k < 1 || E < 1) return 0;
    // behind the reserved head the calls share one region (they are stream-ordered on a context): the row-ID map's
    // per-chunk histograms, or the fp32 partial tiles of a weight gradient whose contraction is split under a skewed
    // load: MOE_WS_SPLIT_SLICES copies of the larger of one expert's two weight gradients, in whole 256 x 256 tiles
    size_t bytes = moe_permute_ws_bytes((int64_t)T * k, E);
    if (h > 0 && f_max > 0) {
        const size_t t1 = (size_t)((2 * (int64_t)f_max + 255) / 256) * (size_t)((h + 255) / 256);   // fc1: [2f, h]
        const size_t split = (size_t)MOE_WS_SPLIT_SLICES * t1 * 256 * 256 * sizeof(float);
        if (split > bytes) bytes = split;
    }
    bytes += MOE_WS_RESERVED;
    return (bytes + 255) / 256 * 256;
}

extern "C" moe_status moe_ctx_create(moe_ctx** out, int device, size_t workspace_bytes) {
    if (!out) return MOE_ERR_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return MOE_ERR_ARG;
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return MOE_ERR_HIP;
    memset(c, 0, sizeof(*c));
    c->device = device;
    if (workspace_bytes < MOE_WS_RESERVED) workspace_bytes = MOE_WS_RESERVED;
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = hipMalloc(&c->ws, workspace_bytes);
    if (e == hipSuccess) e = hipMemset(c->ws, 0, workspace_bytes);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (c->ws) (void)hipFree(c->ws);
        delete c;
        return MOE_ERR_HIP;
    }
    c->ws_bytes = workspace_bytes;
    c->dev_err = (int*)c->ws;
    c->num_cu = prop.multiProcessorCount;
    *out = c;
    return MOE_OK;
}

extern "C" moe_status moe_ctx_destroy(moe_ctx* ctx) {
    if (!ctx) return MOE_OK;
    hipError_t e = hipSuccess;
    if (ctx->ws) e = hipFree(ctx->ws);
    delete ctx;
    return e == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

static thread_local char ctxless_err[512];
char* moe_ctxless_error() { return ctxless_err; }

extern "C" const char* moe_last_error(const moe_ctx* ctx) { return ctx ? ctx->err : ctxless_err; }

extern "C" moe_status moe_ctx_poll_error(moe_ctx* ctx, void* stream, int* device_error) {
    if (!ctx || !device_error) return MOE_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    MOE_HIP_CHECK(ctx, hipStreamSynchronize(s));
    int v = 0;
    MOE_HIP_CHECK(ctx, hipMemcpy(&v, ctx->dev_err, sizeof(int), hipMemcpyDeviceToHost));
    if (v != 0) {
        moe_launch_fill_i32(ctx->dev_err, 1, 0, s);
        MOE_HIP_CHECK(ctx, hipStreamSynchronize(s));
    }
    *device_error = v;
    return MOE_OK;
}
