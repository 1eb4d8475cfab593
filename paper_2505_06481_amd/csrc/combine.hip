// Step C: Y[t,:] = sum_j topk_w[t,j] * Yg[inv_perm[t*k+j], :]  (section 3.2: the gate's
// weighted-averaging coefficients applied to the selected experts' outputs).
// Gather-side and therefore deterministic: one workgroup owns one output row, sums its k
// contributions in fp32 in ascending j and rounds once to the storage type.
#include "mmoe_internal.h"

namespace mmoe {

constexpr int kCombThreads = 256;

template <bool kBf16>
__global__ __launch_bounds__(kCombThreads) void combine_kernel(const f32x4* __restrict__ Yg,
                                                               const int32_t* __restrict__ inv_perm,
                                                               const float* __restrict__ topk_w,
                                                               void* __restrict__ Y, int d4, int k)
{
    const int t = blockIdx.x;
    int rows[kMaxTopK];
    float w[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j)
        if (j < k) {
            // without a permutation the expert outputs are indexed by pair id (self-grouping expert stage)
            rows[j] = inv_perm ? inv_perm[(size_t)t * k + j] : t * k + j;
            w[j] = topk_w[(size_t)t * k + j];
        }
    for (int c = threadIdx.x; c < d4; c += kCombThreads) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j)
            if (j < k) {
                f32x4 y = Yg[(size_t)rows[j] * d4 + c];
                acc += w[j] * y;
            }
        if (kBf16) {
            u32x2 o;
            o[0] = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
            o[1] = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
            reinterpret_cast<u32x2*>(Y)[(size_t)t * d4 + c] = o;
        } else {
            reinterpret_cast<f32x4*>(Y)[(size_t)t * d4 + c] = acc;
        }
    }
}

int launch_combine(const mmoe_shape& s, const float* Yg, const int32_t* inv_perm, const float* topk_w, void* Y,
                   hipStream_t st)
{
    dim3 grid(s.T), block(kCombThreads);
    if (s.dtype == MMOE_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, grid, block, 0, st, (const f32x4*)Yg, inv_perm, topk_w, Y,
                           s.d_model / 4, s.top_k);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, block, 0, st, (const f32x4*)Yg, inv_perm, topk_w, Y,
                           s.d_model / 4, s.top_k);
    return launch_status();
}

}  // namespace mmoe
