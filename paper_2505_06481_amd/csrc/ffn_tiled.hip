// Step F, matrix-core-bound variant: the grouped expert FFN when slots hold many rows
// (prefill-shaped batches) -- Algorithm 2, "expert[iL][iE](act)"; the expert block is
// where the layer's time goes (section 5.1).
//
// Both products are  out[r, n] = sum_k A[r, k] * W[s][n][k]  over the packed pool, bf16
// inputs, fp32 accumulation on v_mfma_f32_32x32x16_bf16.  A workgroup computes a
// 128-row x 128-feature tile of one slot; the ragged row ranges come from the device
// array `offsets`, so the tile -> (slot, first row) map is resolved on the device and the
// host never waits for the histogram.
//
// Matrix-core operand roles: weights are the 32-row operand, tokens the 32-column one.
// A lane then owns, for one token, groups of 4 consecutive output features, which makes
// the gate/up pairing of SwiGLU lane-local and the stores 8 or 16 bytes wide.  For the
// gated product a workgroup's 128 weight rows are 64 rows of W1 and the same 64 rows of
// W3, interleaved per wavefront so that each lane holds matching gate and up values.
//
// LDS tiles are [row][64 k] bf16 (128 bytes a row), 16-byte pieces xor-swizzled with
// (row >> 1) & 7 so that both the staging writes and the operand reads are conflict-free.
#include "mmoe_internal.h"

namespace mmoe {

enum { kTModeReluH = 0, kTModeSwigluH = 1, kTModePlainF32 = 2 };

constexpr int kBM = 128;  // token rows per tile
constexpr int kBN = 128;  // weight rows per tile
constexpr int kBK = 64;
constexpr int kTThreads = 256;

__device__ __forceinline__ int swz(int row, int piece) { return row * 128 + ((piece ^ ((row >> 1) & 7)) << 4); }

__device__ __forceinline__ float silu_mul_t(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

template <int MODE>
__global__ __launch_bounds__(kTThreads) void tiled_kernel(const uint16_t* __restrict__ A,
                                                          const int32_t* __restrict__ offsets,
                                                          const uint16_t* __restrict__ W0,
                                                          const uint16_t* __restrict__ W1, void* __restrict__ out,
                                                          int K, int N, int S)
{
    __shared__ __attribute__((aligned(16))) char lds_a[kBM * kBK * 2];
    __shared__ __attribute__((aligned(16))) char lds_b[kBN * kBK * 2];
    __shared__ int sh_slot, sh_m0;

    // which slot and which rows does m-tile blockIdx.x cover?
    if (threadIdx.x == 0) {
        int mt = blockIdx.x, found = -1, m0 = 0, seen = 0;
        for (int s = 0; s < S; ++s) {
            int c = offsets[s + 1] - offsets[s];
            int nt = (c + kBM - 1) / kBM;
            if (mt < seen + nt) {
                found = s;
                m0 = (mt - seen) * kBM;
                break;
            }
            seen += nt;
        }
        sh_slot = found;
        sh_m0 = m0;
    }
    __syncthreads();
    const int s = sh_slot;
    if (s < 0) return;
    const int m0 = sh_m0;
    const int r0 = offsets[s];
    const int cnt = offsets[s + 1] - r0;

    constexpr int kFeat = MODE == kTModeSwigluH ? kBN / 2 : kBN;  // output features per tile
    const int n0 = blockIdx.y * kFeat;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;  // wavefront grid: 2 (tokens) x 2 (weight rows)

    // staging: thread copies pieces id = i*256 + tid, i < 4; row = id / 8, piece = id % 8
    const uint16_t* ga[4];
    const uint16_t* gb[4];
    int la[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int id = i * kTThreads + tid, row = id >> 3, pc = id & 7;
        int ar = min(m0 + row, cnt - 1);  // rows past the end re-read the last row; never stored
        ga[i] = A + (size_t)(r0 + ar) * K + pc * 8;
        // weight row of LDS row `row`: gated tiles interleave 32 rows of W1 with 32 rows of W3
        const uint16_t* wb;
        int feat;
        if (MODE == kTModeSwigluH) {
            int blk = row >> 5;              // 0..3: wavefront column wn = blk/2, gate/up = blk%2
            feat = (blk >> 1) * 32 + (row & 31);
            wb = (blk & 1) ? W1 : W0;
        } else {
            feat = row;
            wb = W0;
        }
        gb[i] = wb + ((size_t)s * N + n0 + feat) * K + pc * 8;
        la[i] = swz(row, pc);
    }

    f32x16 acc[2][2];  // [weight-row tile][token tile]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    u32x4 ra[4], rb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ra[i] = *reinterpret_cast<const u32x4*>(ga[i]);
        rb[i] = *reinterpret_cast<const u32x4*>(gb[i]);
    }
    const int nkt = K / kBK;
    for (int kt = 0; kt < nkt; ++kt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<u32x4*>(lds_a + la[i]) = ra[i];
            *reinterpret_cast<u32x4*>(lds_b + la[i]) = rb[i];
        }
        __syncthreads();
        if (kt + 1 < nkt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ra[i] = *reinterpret_cast<const u32x4*>(ga[i] + (size_t)(kt + 1) * kBK);
                rb[i] = *reinterpret_cast<const u32x4*>(gb[i] + (size_t)(kt + 1) * kBK);
            }
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int pc = kk * 2 + (lane >> 5);
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fa[j] = *reinterpret_cast<const bf16x8*>(lds_a + swz(wm * 64 + j * 32 + (lane & 31), pc));
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fb[i] = *reinterpret_cast<const bf16x8*>(lds_b + swz(wn * 64 + i * 32 + (lane & 31), pc));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i], fa[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator element e of lane l: weight row 8*(e/4) + 4*(l/32) + e%4, token column l%32
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = m0 + wm * 64 + j * 32 + (lane & 31);
        if (row >= cnt) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int sub = 8 * q + 4 * (lane >> 5);
            if (MODE == kTModeSwigluH) {
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = silu_mul_t(acc[0][j][4 * q + e], acc[1][j][4 * q + e]);
                u32x2 pk;
                pk[0] = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
                pk[1] = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
                const size_t at = (size_t)(r0 + row) * N + n0 + wn * 32 + sub;
                *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) = pk;
            } else {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const size_t at = (size_t)(r0 + row) * N + n0 + wn * 64 + i * 32 + sub;
                    if (MODE == kTModeReluH) {
                        float o[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = fmaxf(acc[i][j][4 * q + e], 0.0f);
                        u32x2 pk;
                        pk[0] = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
                        pk[1] = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
                        *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) = pk;
                    } else {
                        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out) + at) =
                            f32x4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    }
                }
            }
        }
    }
}

int launch_ffn_tiled(const mmoe_shape& s, const void* Xg, const int32_t* offsets, const void* W1p,
                     const void* W3p, const void* W2p, void* H, float* Yg, hipStream_t st, hipEvent_t mid)
{
    if (s.dtype != MMOE_BF16) return MMOE_ERR_DTYPE;
    const int P = s.T * s.top_k, d = s.d_model, f = s.d_ff;
    const int mtiles = (P + kBM - 1) / kBM + s.S;  // upper bound of sum_s ceil(count_s / kBM)
    dim3 block(kTThreads);
    const uint16_t* nul = nullptr;
    if (s.act == MMOE_SWIGLU)
        hipLaunchKernelGGL(tiled_kernel<kTModeSwigluH>, dim3(mtiles, f / (kBN / 2)), block, 0, st,
                           (const uint16_t*)Xg, offsets, (const uint16_t*)W1p, (const uint16_t*)W3p, H, d, f, s.S);
    else
        hipLaunchKernelGGL(tiled_kernel<kTModeReluH>, dim3(mtiles, f / kBN), block, 0, st, (const uint16_t*)Xg,
                           offsets, (const uint16_t*)W1p, nul, H, d, f, s.S);
    if (mid && hipEventRecord(mid, st) != hipSuccess) return MMOE_ERR_LAUNCH;
    hipLaunchKernelGGL(tiled_kernel<kTModePlainF32>, dim3(mtiles, d / kBN), block, 0, st, (const uint16_t*)H,
                       offsets, (const uint16_t*)W2p, nul, (void*)Yg, f, d, s.S);
    return launch_status();
}

}  // namespace mmoe
