// Two measured ceilings of the device the library runs on, as second denominators next to
// the published peaks: the rate of a dependency-free stream of the matrix instruction the
// scoring kernel uses, and the rate of a plain streaming read of device memory.
#include "internal.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int PROBE_MFMA_PER_LOOP = 8;

// Every wavefront issues `loops` x 8 v_mfma_f32_32x32x2_f32 (HALF: v_mfma_f32_32x32x16_f16) on eight
// independent accumulators (no memory traffic, no dependent issue): 4096 (32768) flop per instruction.
typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));

template <bool HALF>
__global__ __launch_bounds__(512) void mfma_rate_kernel(int loops, float seed, float *sink)
{
    floatx16 acc[PROBE_MFMA_PER_LOOP];
#pragma unroll
    for (int a = 0; a < PROBE_MFMA_PER_LOOP; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][e] = seed + (float)a;
    const float x = seed * (float)(threadIdx.x & 7), y = seed + 0.5f;
    probe_half8 xh, yh;
#pragma unroll
    for (int t = 0; t < 8; ++t) { xh[t] = (_Float16)(x + (float)t); yh[t] = (_Float16)(y * (float)(t + 1)); }
    for (int l = 0; l < loops; ++l) {
#pragma unroll
        for (int a = 0; a < PROBE_MFMA_PER_LOOP; ++a) {
            if (HALF) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xh, yh, acc[a], 0, 0, 0);
            else acc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[a], 0, 0, 0);
        }
    }
    float t = 0.0f;
#pragma unroll
    for (int a = 0; a < PROBE_MFMA_PER_LOOP; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[a][e];
    if (t == 12345.678f) sink[0] = t;          // keeps the loop alive; practically never taken
}

// Streaming read: every thread loads 16 bytes per iteration, grid-stride, and folds them.
__global__ __launch_bounds__(256) void read_rate_kernel(const int4 *__restrict__ src, size_t count, int *sink)
{
    int fold = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) {
        const int4 v = src[i];
        fold ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (fold == 0x5a5a5a5a) sink[0] = fold;
}

}  // namespace

extern "C" int mf_measure_ceilings(mf_ctx *ctx, const void *d_buffer, int64_t bytes, float out[8])
{
    if (!ctx || !out || (d_buffer && (bytes < 16 || ((uintptr_t)d_buffer & 15u)))) return MF_ERR_ARG;
    MF_HIP(hipSetDevice(ctx->device));
    for (int i = 0; i < 8; ++i) out[i] = 0.0f;
    const int cus = ctx->n_cus > 0 ? ctx->n_cus : 256;
    for (int half = 0; half < 2; ++half) {
        // two workgroups of eight wavefronts per compute unit, as the scoring kernel's occupancy allows
        const int loops = 20000, grid = cus * 2;
        auto launch = [&](int trips) {
            if (half) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(grid), dim3(512), 0, ctx->stream, trips, 1.0f, (float *)ctx->colmark);
            else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(grid), dim3(512), 0, ctx->stream, trips, 1.0f, (float *)ctx->colmark);
        };
        launch(200);
        MF_HIP(hipEventRecord(ctx->ev[0], ctx->stream));
        launch(loops);
        MF_HIP(hipEventRecord(ctx->ev[1], ctx->stream));
        MF_HIP(hipGetLastError());
        MF_HIP(hipStreamSynchronize(ctx->stream));
        float ms = 0.0f;
        MF_HIP(hipEventElapsedTime(&ms, ctx->ev[0], ctx->ev[1]));
        const double flop = (double)grid * 8.0 * (double)loops * PROBE_MFMA_PER_LOOP * (half ? 32768.0 : 4096.0);
        out[half ? 4 : 0] = (float)(flop / (ms * 1e-3) / 1e12);          // TFLOP/s
        out[half ? 5 : 1] = ms;
    }
    if (d_buffer) {
        const size_t count = (size_t)bytes / 16;
        const int grid = cus * 16;
        hipLaunchKernelGGL(read_rate_kernel, dim3(grid), dim3(256), 0, ctx->stream, (const int4 *)d_buffer, count,
                           ctx->colmark);
        MF_HIP(hipEventRecord(ctx->ev[0], ctx->stream));
        hipLaunchKernelGGL(read_rate_kernel, dim3(grid), dim3(256), 0, ctx->stream, (const int4 *)d_buffer, count,
                           ctx->colmark);
        MF_HIP(hipEventRecord(ctx->ev[1], ctx->stream));
        MF_HIP(hipGetLastError());
        MF_HIP(hipStreamSynchronize(ctx->stream));
        float ms = 0.0f;
        MF_HIP(hipEventElapsedTime(&ms, ctx->ev[0], ctx->ev[1]));
        out[2] = (float)((double)count * 16.0 / (ms * 1e-3) / 1e9);     // GB/s
        out[3] = ms;
    }
    return MF_OK;
}
