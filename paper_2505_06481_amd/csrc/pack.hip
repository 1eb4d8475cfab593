// One-time repacking of the expert pool: [S, R, C] -> [S, C, R] per matrix, so that the
// reduction dimension of each product is contiguous, which is what the matrix-core
// operand layout wants (each lane feeds 8 consecutive reduction elements of one row).
// Runs when the pool is loaded (section 3.1: the loader runs once, before serving), never
// on the serving path.
#include "mmoe_internal.h"

namespace mmoe {

constexpr int kTile = 64;

template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, T* __restrict__ out, int R,
                                                        int C)
{
    __shared__ T tile[kTile][kTile + 2];
    const size_t mat = (size_t)blockIdx.z * R * C;
    const int c0 = blockIdx.x * kTile, r0 = blockIdx.y * kTile;
    const int tx = threadIdx.x % kTile, ty = threadIdx.x / kTile;  // 64 x 4
    for (int i = ty; i < kTile; i += 4) {
        int r = r0 + i, c = c0 + tx;
        if (r < R && c < C) tile[i][tx] = in[mat + (size_t)r * C + c];
    }
    __syncthreads();
    for (int i = ty; i < kTile; i += 4) {
        int c = c0 + i, r = r0 + tx;
        if (r < R && c < C) out[mat + (size_t)c * R + r] = tile[tx][i];
    }
}

static void transpose(const void* in, void* out, int S, int R, int C, int dtype, hipStream_t st)
{
    dim3 grid((C + kTile - 1) / kTile, (R + kTile - 1) / kTile, S), block(256);
    if (dtype == MMOE_BF16)
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, block, 0, st, (const uint16_t*)in, (uint16_t*)out, R, C);
    else
        hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, st, (const float*)in, (float*)out, R, C);
}

int launch_pack(const mmoe_shape& s, const void* W1, const void* W3, const void* W2, void* W1p, void* W3p,
                void* W2p, hipStream_t st)
{
    transpose(W1, W1p, s.S, s.d_model, s.d_ff, s.dtype, st);
    if (W3) transpose(W3, W3p, s.S, s.d_model, s.d_ff, s.dtype, st);
    transpose(W2, W2p, s.S, s.d_ff, s.d_model, s.dtype, st);
    return launch_status();
}

}  // namespace mmoe
