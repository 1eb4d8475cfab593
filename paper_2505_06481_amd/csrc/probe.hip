// Measurement aids, not part of the layer: what this GPU delivers for the two resources that
// bound the expert stage, so that a roofline fraction can be read against an achievable
// ceiling as well as against the data-sheet peak.
//   stream read   every workgroup reads its share of a buffer once with 16-byte loads, many
//                 loads in flight per lane: the HBM bandwidth a weight-streaming kernel can reach;
//   matrix loop   every wavefront issues v_mfma_f32_32x32x16_bf16 on register operands into 16
//                 independent accumulator tiles, no memory traffic: the matrix-core rate the
//                 chip sustains at the clock its power limit allows.
#include "mmoe_internal.h"

namespace mmoe {

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t n,
                                                         uint32_t* __restrict__ sink)
{
    constexpr int kUnroll = 8;
    size_t i = (size_t)blockIdx.x * 256 * kUnroll + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256 * kUnroll;
    u32x4 acc = {0, 0, 0, 0};
    for (; i + 256 * (kUnroll - 1) < n; i += stride) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u];
    }
    // never true for the caller's zero-filled buffer; keeps the loads alive
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[blockIdx.x] = 1;
}

__global__ __launch_bounds__(256, 1) void probe_mfma_kernel(int iters, float* __restrict__ sink)
{
    f32x16 acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
    // operands with a spread of exponents and mantissas, different in every lane
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (bf16_t)(0.01f * (float)((threadIdx.x * 7 + e * 13) % 61 - 30));
        b[e] = (bf16_t)(0.02f * (float)((threadIdx.x * 11 + e * 5) % 53 - 26));
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 16; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 16; ++t) s += acc[t][0];
    if (s == 12345.678f) sink[blockIdx.x] = s;  // keeps the accumulators alive
}

int run_probe(void* buf, size_t bytes, float* out, hipStream_t st)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return MMOE_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return MMOE_ERR_LAUNCH;
    }
    bool ok = true;
    const int reps = 5;
    // elapsed milliseconds of `reps` launches of `launch` on the stream, after one warm-up launch
    auto timed = [&](auto launch) -> float {
        float ms = 0.0f;
        launch();
        ok = ok && hipEventRecord(e0, st) == hipSuccess;
        for (int r = 0; r < reps; ++r) launch();
        ok = ok && hipEventRecord(e1, st) == hipSuccess;
        ok = ok && hipEventSynchronize(e1) == hipSuccess;
        ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
        return ms;
    };

    // stream read: the buffer minus a 1 MiB tail that serves as the sink
    const size_t n = (bytes - (1 << 20)) / 16;
    uint32_t* sink = (uint32_t*)((char*)buf + bytes - (1 << 20));
    const int grid_r = 256 * 16;
    float ms = timed([&] {
        hipLaunchKernelGGL(probe_read_kernel, dim3(grid_r), dim3(256), 0, st, (const u32x4*)buf, n, sink);
    });
    const size_t per_stride = (size_t)grid_r * 256 * 8;  // 16-byte pieces per grid stride; whole strides are read
    out[0] = ok ? (float)((double)(n / per_stride * per_stride) * 16.0 * reps / (ms * 1e-3) / 1e9) : 0.0f;  // GB/s

    // matrix loop: 1024 workgroups of four wavefronts (four rounds of one per compute unit)
    const int iters = 4096, grid_m = 1024;
    ms = timed([&] { hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid_m), dim3(256), 0, st, iters, (float*)sink); });
    const double flop = (double)grid_m * 4 * iters * 16 * (2.0 * 32 * 32 * 16) * reps;
    out[1] = ok ? (float)(flop / (ms * 1e-3) / 1e12) : 0.0f;  // TFLOP/s
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok) return MMOE_ERR_LAUNCH;
    return launch_status();
}

}  // namespace mmoe
