// Measurement aids: what this device reaches with minimal kernels, to be reported next to the
// nominal peaks when the path's kernels are priced against a roofline.
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Streams n16 16-byte words with non-temporal loads; the sum keeps the loads alive.
__global__ __launch_bounds__(256) void calib_read_kernel(const v4i* __restrict__ p, size_t n16, int* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    v4i acc = {0, 0, 0, 0};
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x); i < n16; i += stride) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t j = i + (size_t)u * gridDim.x * blockDim.x;
            if (j < n16) acc += __builtin_nontemporal_load(p + j);
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x7fffffff) *sink = 1;
}

// One contiguous 4 KiB per workgroup, workgroups in address order: the store pattern that writes fastest here
// (a grid-stride loop over the same buffer, every workgroup hopping through all of it, reaches only 70 % of it).
__global__ __launch_bounds__(256) void calib_write_kernel(v4i* __restrict__ p, size_t n16) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const v4i v = {(int)threadIdx.x, 1, 2, 3};
    if (i < n16) p[i] = v;
}

// 16 independent 32x32 accumulators per wave, operands in registers: nothing but MFMA issue.
__global__ __launch_bounds__(256) void calib_mfma_i8_kernel(int iters, int seed, int* __restrict__ sink) {
    v16i acc[16];
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][r] = 0;
    const int t = threadIdx.x;
    const v4i x = {seed + t, seed * 3, seed * 5 + t, seed * 7}, y = {seed * 11, seed + 1, t * seed, seed * 13};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int a = 0; a < 16; ++a) acc[a] = __builtin_amdgcn_mfma_i32_32x32x32_i8(x, y, acc[a], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[a][r];
    if (s == 0x7fffffff) *sink = s;
}

// The same for the 4-bit form of v_mfma_f32_32x32x64_f8f6f4 (operand nibbles 0b0010 = 1.0, unit block scales):
// the instruction the co-activation kernel runs on.
typedef int v8i_c __attribute__((ext_vector_type(8)));
typedef float v16f_c __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void calib_mfma_fp4_kernel(int iters, int seed, int* __restrict__ sink) {
    v16f_c acc[16];
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
    const int t = threadIdx.x;
    const v8i_c x = {(seed + t) & 0x22222222, (seed * 3) & 0x22222222, (seed * 5 + t) & 0x22222222, (seed * 7) & 0x22222222, 0, 0, 0, 0};
    const v8i_c y = {(seed * 11) & 0x22222222, (seed + 1) & 0x22222222, (t * seed) & 0x22222222, (seed * 13) & 0x22222222, 0, 0, 0, 0};
    constexpr int unit = 0;                            // no block scales: the unscaled form, as the co-activation kernel issues it
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int a = 0; a < 16; ++a) acc[a] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x, y, acc[a], 4, 4, 0, unit, 0, unit);
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[a][r];
    if (s == -1.f) *sink = 1;
}

}  // namespace

swarm_status swarm_calibrate(swarm_ctx* ctx, int32_t what, void* buf, size_t bytes, int32_t reps, double* out) {
    SWARM_ENTER(ctx);
    if (!out || reps < 1) SWARM_REJECT(ctx, "calibrate: NULL out or reps < 1");
    if (ctx->capturing) SWARM_REJECT(ctx, "calibrate: not while recording");
    const bool mfma = what == SWARM_CAL_MFMA_I8 || what == SWARM_CAL_MFMA_FP4;
    if (!mfma) {
        if (!buf || bytes < 16 || (reinterpret_cast<uintptr_t>(buf) & 15)) SWARM_REJECT(ctx, "calibrate: buf must be 16-byte aligned, bytes >= 16");
    } else if (!buf) {
        SWARM_REJECT(ctx, "calibrate: buf must hold at least 4 bytes");
    }
    hipEvent_t e0, e1;
    SWARM_HIP(ctx, hipEventCreate(&e0));
    SWARM_HIP(ctx, hipEventCreate(&e1));
    const size_t n16 = bytes / 16;
    const unsigned blocks = 256 * 8;
    const int mfma_iters = 4096;
    auto launch = [&]() {
        if (what == SWARM_CAL_HBM_READ)
            hipLaunchKernelGGL(calib_read_kernel, dim3((unsigned)((n16 + 1023) / 1024 < blocks ? (n16 + 1023) / 1024 : blocks)), dim3(256), 0, ctx->stream, static_cast<const v4i*>(buf), n16, reinterpret_cast<int*>(ctx->dev_flags + 1));
        else if (what == SWARM_CAL_HBM_WRITE)
            hipLaunchKernelGGL(calib_write_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, ctx->stream, static_cast<v4i*>(buf), n16);
        else if (what == SWARM_CAL_MFMA_I8)
            hipLaunchKernelGGL(calib_mfma_i8_kernel, dim3(256 * 4), dim3(256), 0, ctx->stream, mfma_iters, 77, static_cast<int*>(buf));
        else
            hipLaunchKernelGGL(calib_mfma_fp4_kernel, dim3(256 * 4), dim3(256), 0, ctx->stream, mfma_iters, 77, static_cast<int*>(buf));
    };
    if (what != SWARM_CAL_HBM_READ && what != SWARM_CAL_HBM_WRITE && !mfma) {
        (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
        SWARM_REJECT(ctx, "calibrate: unknown measurement %d", what);
    }
    launch();                                              // warm-up
    hipError_t e = hipEventRecord(e0, ctx->stream);
    for (int r = 0; r < reps && e == hipSuccess; ++r) launch();
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) {
        snprintf(ctx->err, sizeof(ctx->err), "calibrate: %s", hipGetErrorString(e));
        return SWARM_EHIP;
    }
    const double s = (double)ms * 1e-3 / reps;
    if (what == SWARM_CAL_MFMA_I8) *out = 256.0 * 4 * 4 * (double)mfma_iters * 16 * 65536.0 / s / 1e12;   // TOP/s: 2 * 32 * 32 * 32 per instruction
    else if (what == SWARM_CAL_MFMA_FP4) *out = 256.0 * 4 * 4 * (double)mfma_iters * 16 * 131072.0 / s / 1e12;   // 2 * 32 * 32 * 64
    else *out = (double)(n16 * 16) / s / 1e9;                                                               // GB/s
    return SWARM_OK;
}
