// One-time repacking of the expert pool.  Runs when the pool is loaded (section 3.1: the
// loader runs once, before serving), never on the serving path.
//
// Every product of the expert stage is  out[r, n] = sum_k A[r, k] * W[n][k]  with W given
// "in x out", i.e. as W[k][n].
//
// fp32: W is transposed to [S, N, K] (reduction dimension contiguous).
//
// bf16: W is stored as matrix-core fragments.  A fragment is the 32-row x 16-k operand of
// v_mfma_f32_32x32x16_bf16 exactly as the 64 lanes hold it: 64 pieces of 16 bytes, piece
// `lane` = 8 consecutive k of row lane%32, for the lane half h = lane/32.  Fragments of one
// 32-row block follow each other along k, so a wavefront streams a block's weights with
// fully contiguous 1 KB loads straight into registers: no LDS, no shuffle.  The k values a
// fragment covers are permuted inside each run of 64 so that a lane's four consecutive
// fragments read 64 contiguous bytes of the activation row:
//     fragment ks = 4m + kk (kk < 4), lane half h  <->  k = 64m + 32h + 8kk + [0, 8).
// Element (n, k) of slot s lives at
//     ((((s*(N/32) + n/32) * (K/16) + ks) * 64 + 32h + n%32) * 8 + k%8.
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

// bf16 fragment packing: one thread writes one 16-byte piece.
__global__ __launch_bounds__(256) void pack_fragments_kernel(const uint16_t* __restrict__ in,
                                                             u32x4* __restrict__ out, int K, int N)
{
    // `in` is [S, K, N]; piece index = ((s*(N/32) + nb) * (K/16) + ks) * 64 + lane
    const size_t piece = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int lane = (int)(piece & 63);
    const size_t frag = piece >> 6;
    const int ks = (int)(frag % (size_t)(K / 16));
    const size_t blk = frag / (size_t)(K / 16);  // s*(N/32) + nb
    const int nb = (int)(blk % (size_t)(N / 32));
    const size_t s = blk / (size_t)(N / 32);
    const int n = nb * 32 + (lane & 31);
    const int k0 = (ks >> 2) * 64 + (lane >> 5) * 32 + (ks & 3) * 8;
    const uint16_t* src = in + (s * K + k0) * (size_t)N + n;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        w[e] = (uint32_t)src[(size_t)(2 * e) * N] | ((uint32_t)src[(size_t)(2 * e + 1) * N] << 16);
    out[piece] = u32x4{w[0], w[1], w[2], w[3]};
}

static void pack_fragments(const void* in, void* out, int S, int K, int N, hipStream_t st)
{
    const size_t pieces = (size_t)S * (N / 32) * (K / 16) * 64;  // a multiple of 256: K, N are multiples of 256
    hipLaunchKernelGGL(pack_fragments_kernel, dim3((unsigned)(pieces / 256)), dim3(256), 0, st, (const uint16_t*)in,
                       (u32x4*)out, K, N);
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
    if (s.dtype == MMOE_BF16) {
        pack_fragments(W1, W1p, s.S, s.d_model, s.d_ff, st);
        if (W3) pack_fragments(W3, W3p, s.S, s.d_model, s.d_ff, st);
        pack_fragments(W2, W2p, s.S, s.d_ff, s.d_model, st);
    } else {
        transpose(W1, W1p, s.S, s.d_model, s.d_ff, s.dtype, st);
        if (W3) transpose(W3, W3p, s.S, s.d_model, s.d_ff, s.dtype, st);
        transpose(W2, W2p, s.S, s.d_ff, s.d_model, s.dtype, st);
    }
    return launch_status();
}

}  // namespace mmoe
