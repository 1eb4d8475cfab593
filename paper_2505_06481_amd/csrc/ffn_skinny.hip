// Step F, weight-streaming variant: the grouped expert FFN when a slot sees only a few
// rows (decode-shaped batches) -- Algorithm 2, "expert[iL][iE](act)".  Each expert's
// weights are then read from HBM exactly once and that read is the whole cost, so the
// kernel is built around keeping many 16-byte loads of weights in flight per wavefront.
//
// Both products are of the form  out[r, n] = sum_k A[r, k] * W[s][n][k]  over the packed
// pool.  A workgroup owns a block of output features n of one slot and all rows of that
// slot; its four wavefronts split the reduction dimension and meet in LDS.  The weight rows
// are the row operand of a matrix-core instruction and the tokens its columns, so the
// weights pass through registers once however many tokens (up to 32 per pass) the slot holds.
// In the fused layer the token rows of the first product are read through the grouping
// permutation (row perm[r] / top_k of X) instead of from a gathered copy.
//
// Self-grouping mode (decode-sized batches of the fused layer): no grouping kernel runs at
// all.  The router has written slot[p] for every pair; a workgroup collects the pairs of its
// slot itself, in ascending pair id (which is the stable order of the grouped form), and the
// intermediates H and Yg are indexed by pair id instead of by grouped row.  Every row is still
// summed in the same order, so the layer's output is bit-identical to the staged path's.
//
// fp32 kernel (skinny_kernel): transposed pool [S, N, K], 16 features per workgroup,
// 16x16x4 matrix instructions, two 16-row token blocks per pass.  Reduction-index
// permutation: per 256-byte step of a row, lane group g = lane/16 loads the contiguous 64
// bytes [64g, 64g+64) as four 16-byte pieces q; piece q of every group feeds matrix
// instruction q.  Weights and activations use the same permutation, and a sum does not care
// in which order its terms are visited, so no shuffle is needed and every lane's global
// loads are contiguous.
//
// bf16 kernel (skinny_frag_kernel): fragment-packed pool, 32 features per workgroup,
// 32x32x16 matrix instructions, up to 32 rows per pass; see its own comment.
#include "mmoe_internal.h"

namespace mmoe {

// What a product writes: H = act(.) in the storage type (up product), plain fp32 rows of Yg (down
// product), or, for layers with top_k = 1, the layer's output rows themselves: 0 + w[token] * y in the
// storage type at row token (GateSink).
enum { kModeReluH = 0, kModeSwigluH = 1, kModePlainF32 = 2, kModeGeluH = 3, kModeGatedY = 4 };

constexpr int kSkThreads = 256;
constexpr int kSkWaves = 4;
constexpr int kSkMB = 2;  // 16-row token blocks per pass

template <typename T> struct Mma;
template <> struct Mma<float> {  // fp32, 16x16x4: one 16-byte piece = 4 elements = 4 instructions
    static __device__ __forceinline__ f32x4 run(u32x4 w, u32x4 x, f32x4 acc)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(w[c]), __uint_as_float(x[c]), acc, 0, 0, 0);
        return acc;
    }
};

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }
__device__ __forceinline__ float gelu(float a) { return 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f)); }

constexpr int kSelfMaxP = 1024;  // most pairs for which the expert kernels group by themselves

// Rows of one slot.  Grouped form: rows [r0, r0 + cnt) of the grouped order; input row of grouped
// row r is r itself, or perm[r] / kdiv (gather folded into the loads).  Self-grouping form: the
// pairs p with slot_of_pair[p] == s, ascending, collected here into `mine` by the first
// wavefront (ballot + popcount ranks); input row p / kdiv, output row p.
struct RowSet {
    int r0, cnt;
    const int32_t* perm;
    int kdiv;
    const int* mine;  // LDS list of pair ids, or null in the grouped form
    __device__ __forceinline__ int in_row(int rr) const
    {
        if (mine) return mine[rr] / kdiv;
        return perm ? perm[r0 + rr] / kdiv : r0 + rr;
    }
    __device__ __forceinline__ int out_row(int rr) const { return mine ? mine[rr] : r0 + rr; }
};

__device__ __forceinline__ RowSet slot_rows(const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
                                            int kdiv, const int32_t* __restrict__ slot_of_pair, int P, int s,
                                            int* mine, int* mine_cnt, SlotFilter filt)
{
    RowSet rs;
    rs.perm = perm;
    rs.kdiv = kdiv;
    rs.mine = nullptr;
    if (filt.skips(s)) {  // uniform over the workgroup: this launch leaves the slot to another one
        rs.r0 = 0;
        rs.cnt = 0;
        return rs;
    }
    if (!slot_of_pair) {
        rs.r0 = offsets[s];
        rs.cnt = offsets[s + 1] - rs.r0;
        return rs;
    }
    if (threadIdx.x < kWave) {
        int n = 0;
        for (int p0 = 0; p0 < P; p0 += kWave) {
            const int p = p0 + threadIdx.x;
            const bool hit = p < P && slot_of_pair[p] == s;
            const unsigned long long m = __ballot(hit);
            if (hit) mine[n + __popcll(m & ((1ull << threadIdx.x) - 1ull))] = p;
            n += __popcll(m);
        }
        if (threadIdx.x == 0) *mine_cnt = n;
    }
    __syncthreads();
    rs.r0 = 0;
    rs.cnt = *mine_cnt;
    rs.mine = mine;
    return rs;
}

// SPLITK: the four wavefronts split the reduction dimension of one 16-feature block and meet in
// LDS (long reductions).  !SPLITK: every wavefront owns a 16-feature block of its own and walks the
// whole reduction dimension (short reductions, where a quarter of K is one or two iterations: all
// latency, no pipelining): 64 features per workgroup, no LDS reduction, the token rows fetched a
// quarter as often per weight byte.
template <typename T, int NW, int KU, int MODE, bool SPLITK>
__global__ __launch_bounds__(kSkThreads) void skinny_kernel(const T* __restrict__ A,
                                                            const int32_t* __restrict__ perm, int kdiv,
                                                            const int32_t* __restrict__ offsets,
                                                            const int32_t* __restrict__ slot_of_pair, int P,
                                                            const T* __restrict__ W0, const T* __restrict__ W1,
                                                            void* __restrict__ out, int K, int N, SlotFilter filt,
                                                            const int32_t* __restrict__ sink_perm,
                                                            const float* __restrict__ sink_w)
{
    constexpr int EPB = 16 / (int)sizeof(T);  // elements per 16-byte piece
    constexpr int KSS = 16 * EPB;             // elements per 256-byte step
    __shared__ float red[kSkWaves][kSkMB][NW][kWave][4];
    __shared__ int mine[kSelfMaxP];
    __shared__ int mine_cnt;

    const int s = blockIdx.y;
    const RowSet rs = slot_rows(offsets, perm, kdiv, slot_of_pair, P, s, mine, &mine_cnt, filt);
    const int cnt = rs.cnt;
    if (cnt <= 0) return;  // uniform over the workgroup

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int n0 = SPLITK ? blockIdx.x * 16 : (blockIdx.x * kSkWaves + wave) * 16;
    const int li = lane & 15, g = lane >> 4;
    const int nit = K / (KSS * KU);
    constexpr int kFirst = SPLITK ? -1 : 0;        // first iteration of a wavefront: its index, or 0
    constexpr int kStride = SPLITK ? kSkWaves : 1;  // iterations between two of one wavefront

    const T* wrow[NW];
    wrow[0] = W0 + ((size_t)s * N + n0 + li) * K + g * (4 * EPB);
    if (NW == 2) wrow[NW - 1] = W1 + ((size_t)s * N + n0 + li) * K + g * (4 * EPB);

    for (int pass0 = 0; pass0 < cnt; pass0 += 16 * kSkMB) {
        const int nmb = min(kSkMB, (cnt - pass0 + 15) / 16);
        const T* arow[kSkMB];
#pragma unroll
        for (int mb = 0; mb < kSkMB; ++mb) {
            int rr = min(pass0 + mb * 16 + li, cnt - 1);  // rows past the end re-read the last one; never stored
            arow[mb] = A + (size_t)rs.in_row(rr) * K + g * (4 * EPB);
        }
        f32x4 acc[kSkMB][NW];
#pragma unroll
        for (int mb = 0; mb < kSkMB; ++mb)
#pragma unroll
            for (int w = 0; w < NW; ++w) acc[mb][w] = f32x4{0.f, 0.f, 0.f, 0.f};

        u32x4 wcur[NW][KU][4], wnxt[NW][KU][4];
        int it = kFirst < 0 ? wave : kFirst;
        if (it < nit) {
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int u = 0; u < KU; ++u)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        wcur[w][u][q] =
                            *reinterpret_cast<const u32x4*>(wrow[w] + (size_t)(it * KU + u) * KSS + q * EPB);
        }
        for (; it < nit; it += kStride) {
            u32x4 xa[kSkMB][KU][4];
#pragma unroll
            for (int mb = 0; mb < kSkMB; ++mb)
                if (mb < nmb) {
#pragma unroll
                    for (int u = 0; u < KU; ++u)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            xa[mb][u][q] =
                                *reinterpret_cast<const u32x4*>(arow[mb] + (size_t)(it * KU + u) * KSS + q * EPB);
                }
            const int itn = it + kStride;
            if (itn < nit) {  // the next weights: the youngest loads, still in flight during the math below
#pragma unroll
                for (int w = 0; w < NW; ++w)
#pragma unroll
                    for (int u = 0; u < KU; ++u)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            wnxt[w][u][q] =
                                *reinterpret_cast<const u32x4*>(wrow[w] + (size_t)(itn * KU + u) * KSS + q * EPB);
            }
#pragma unroll
            for (int mb = 0; mb < kSkMB; ++mb)
                if (mb < nmb) {
#pragma unroll
                    for (int u = 0; u < KU; ++u)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int w = 0; w < NW; ++w)
                                acc[mb][w] = Mma<T>::run(wcur[w][u][q], xa[mb][u][q], acc[mb][w]);
                }
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int u = 0; u < KU; ++u)
#pragma unroll
                    for (int q = 0; q < 4; ++q) wcur[w][u][q] = wnxt[w][u][q];
        }

        // accumulator element i of lane l is output feature n0 + 4*(l/16) + i of token column l%16
        auto finish = [&](int row, int l, const float (&v)[NW][4]) {
            float o[4];
            int orow = rs.out_row(row);
            float gw = 0.0f;
            if (MODE == kModeGatedY) {
                if (sink_perm) orow = sink_perm[orow];
                gw = sink_w[orow];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (MODE == kModeSwigluH) o[i] = silu_mul(v[0][i], v[NW - 1][i]);
                else if (MODE == kModeReluH) o[i] = fmaxf(v[0][i], 0.0f);
                else if (MODE == kModeGeluH) o[i] = gelu(v[0][i]);
                else if (MODE == kModeGatedY) o[i] = __builtin_fmaf(gw, v[0][i], 0.0f);
                else o[i] = v[0][i];
            }
            const size_t at = (size_t)orow * N + n0 + 4 * (l >> 4);
            if (MODE == kModePlainF32 || sizeof(T) == 4) {
                *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out) + at) = f32x4{o[0], o[1], o[2], o[3]};
            } else {
                u32x2 pk;
                pk[0] = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
                pk[1] = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
                *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) = pk;
            }
        };
        if (!SPLITK) {  // every wavefront finishes its own 16 features straight from its accumulators
#pragma unroll
            for (int mb = 0; mb < kSkMB; ++mb) {
                const int row = pass0 + mb * 16 + (lane & 15);
                if (mb < nmb && row < cnt) {
                    float v[NW][4];
#pragma unroll
                    for (int w = 0; w < NW; ++w)
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[w][i] = acc[mb][w][i];
                    finish(row, lane, v);
                }
            }
            continue;
        }
#pragma unroll
        for (int mb = 0; mb < kSkMB; ++mb)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int i = 0; i < 4; ++i) red[wave][mb][w][lane][i] = acc[mb][w][i];
        __syncthreads();
        for (int idx = threadIdx.x; idx < nmb * kWave; idx += kSkThreads) {
            const int mb = idx / kWave, l = idx % kWave;
            const int row = pass0 + mb * 16 + (l & 15);
            if (row < cnt) {
                float v[NW][4];
#pragma unroll
                for (int w = 0; w < NW; ++w)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        v[w][i] = (red[0][mb][w][l][i] + red[1][mb][w][l][i]) + (red[2][mb][w][l][i] + red[3][mb][w][l][i]);
                finish(row, l, v);
            }
        }
        __syncthreads();
    }
}

// ---- bf16 on the fragment-packed pool ----------------------------------------------------
// Workgroup = one 32-row block of weights (32 output features) of one slot, all rows of the
// slot.  The block's fragments lie one after the other in memory (1 KB each, 16 k per
// fragment), so the four wavefronts take runs of 4 fragments (64 k) in turn and every
// weight load is a fully contiguous 1 KB read that goes straight into the matrix-core
// operand registers.  Tokens are the 32-column operand: lane (token l%32, half h = l/32)
// reads the 64 contiguous bytes of its activation row that the run's permutation assigns
// to it.  Partial sums of the four wavefronts meet in LDS.
template <int NW, int KU, int MODE>
__global__ __launch_bounds__(kSkThreads) void skinny_frag_kernel(const uint16_t* __restrict__ A,
                                                                 const int32_t* __restrict__ perm, int kdiv,
                                                                 const int32_t* __restrict__ offsets,
                                                                 const int32_t* __restrict__ slot_of_pair, int P,
                                                                 const uint16_t* __restrict__ W0,
                                                                 const uint16_t* __restrict__ W1,
                                                                 void* __restrict__ out, int K, int N,
                                                                 SlotFilter filt,
                                                                 const int32_t* __restrict__ sink_perm,
                                                                 const float* __restrict__ sink_w)
{
    __shared__ float red[kSkWaves][NW][kWave][16];  // 16 KB per matrix
    __shared__ int mine[kSelfMaxP];
    __shared__ int mine_cnt;

    const int s = blockIdx.y;
    const int nb = blockIdx.x;
    const RowSet rs = slot_rows(offsets, perm, kdiv, slot_of_pair, P, s, mine, &mine_cnt, filt);
    const int cnt = rs.cnt;
    if (cnt <= 0) return;  // uniform over the workgroup

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int tok = lane & 31, h = lane >> 5;
    const int nit = K / (64 * KU);  // iterations of KU runs of 64 k

    // fragment ks of this block: element offset ((s*(N/32) + nb)*(K/16) + ks)*512 + lane*8
    const size_t blk = ((size_t)s * (N / 32) + nb) * (size_t)(K / 16) * 512 + (size_t)lane * 8;
    const uint16_t* wrow[NW];
    wrow[0] = W0 + blk;
    if (NW == 2) wrow[NW - 1] = W1 + blk;

    for (int pass0 = 0; pass0 < cnt; pass0 += 32) {
        const int rr = min(pass0 + tok, cnt - 1);  // tokens past the end re-read the last one; never stored
        const uint16_t* arow = A + (size_t)rs.in_row(rr) * K + h * 32;
        f32x16 acc[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[w][e] = 0.0f;

        u32x4 wcur[NW][KU][4], wnxt[NW][KU][4];
        int it = wave;
        if (it < nit) {
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int u = 0; u < KU; ++u)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        wcur[w][u][q] =
                            *reinterpret_cast<const u32x4*>(wrow[w] + ((size_t)(it * KU + u) * 4 + q) * 512);
        }
        for (; it < nit; it += kSkWaves) {
            u32x4 xa[KU][4];
#pragma unroll
            for (int u = 0; u < KU; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    xa[u][q] = *reinterpret_cast<const u32x4*>(arow + (size_t)(it * KU + u) * 64 + q * 8);
            const int itn = it + kSkWaves;
            if (itn < nit) {  // the next weights: the youngest loads, still in flight during the math below
#pragma unroll
                for (int w = 0; w < NW; ++w)
#pragma unroll
                    for (int u = 0; u < KU; ++u)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            wnxt[w][u][q] =
                                *reinterpret_cast<const u32x4*>(wrow[w] + ((size_t)(itn * KU + u) * 4 + q) * 512);
            }
#pragma unroll
            for (int u = 0; u < KU; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int w = 0; w < NW; ++w)
                        acc[w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wcur[w][u][q]),
                                                                         __builtin_bit_cast(bf16x8, xa[u][q]), acc[w],
                                                                         0, 0, 0);
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int u = 0; u < KU; ++u)
#pragma unroll
                    for (int q = 0; q < 4; ++q) wcur[w][u][q] = wnxt[w][u][q];
        }

#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[wave][w][lane][e] = acc[w][e];
        __syncthreads();
        // accumulator element e of lane l: feature 8*(e/4) + 4*(l/32) + e%4 of token column l%32.
        // Thread (l = tid%64, q = tid/64) finishes elements 4q .. 4q+3 of lane l: 4 consecutive features.
        {
            const int l = threadIdx.x & 63, q = threadIdx.x >> 6;
            const int row = pass0 + (l & 31);
            if (row < cnt) {
                float o[4];
                int orow = rs.out_row(row);
                float gw = 0.0f;
                if (MODE == kModeGatedY) {
                    if (sink_perm) orow = sink_perm[orow];
                    gw = sink_w[orow];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = 4 * q + i;
                    float v[NW];
#pragma unroll
                    for (int w = 0; w < NW; ++w)
                        v[w] = (red[0][w][l][e] + red[1][w][l][e]) + (red[2][w][l][e] + red[3][w][l][e]);
                    if (MODE == kModeSwigluH) o[i] = silu_mul(v[0], v[NW - 1]);
                    else if (MODE == kModeReluH) o[i] = fmaxf(v[0], 0.0f);
                    else if (MODE == kModeGeluH) o[i] = gelu(v[0]);
                    else if (MODE == kModeGatedY) o[i] = __builtin_fmaf(gw, v[0], 0.0f);
                    else o[i] = v[0];
                }
                const size_t at = (size_t)orow * N + nb * 32 + 8 * q + 4 * (l >> 5);
                if (MODE == kModePlainF32) {
                    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out) + at) = f32x4{o[0], o[1], o[2], o[3]};
                } else {
                    u32x2 pk;
                    pk[0] = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
                    pk[1] = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
                    *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) = pk;
                }
            }
        }
        __syncthreads();
    }
}

static int run_skinny_bf16(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                           const int32_t* slot_of_pair, const void* W1p, const void* W3p, const void* W2p, void* H,
                           float* Yg, hipStream_t st, hipEvent_t mid, SlotFilter filt, GateSink sink)
{
    const int32_t* nosink = nullptr;
    const float* now = nullptr;
    const int32_t* noperm = nullptr;
    const int d = s.d_model, f = s.d_ff, P = s.T * s.top_k;
    dim3 block(kSkThreads);
    dim3 g1(f / 32, s.S), g2(d / 32, s.S);
    const uint16_t* nul = nullptr;
    if (s.act == MMOE_SWIGLU)
        hipLaunchKernelGGL((skinny_frag_kernel<2, 1, kModeSwigluH>), g1, block, 0, st, (const uint16_t*)rows, perm,
                           s.top_k, offsets, slot_of_pair, P, (const uint16_t*)W1p, (const uint16_t*)W3p, H, d, f, filt,
                           nosink, now);
    else if (s.act == MMOE_GELU)
        hipLaunchKernelGGL((skinny_frag_kernel<1, 2, kModeGeluH>), g1, block, 0, st, (const uint16_t*)rows, perm,
                           s.top_k, offsets, slot_of_pair, P, (const uint16_t*)W1p, nul, H, d, f, filt, nosink, now);
    else
        hipLaunchKernelGGL((skinny_frag_kernel<1, 2, kModeReluH>), g1, block, 0, st, (const uint16_t*)rows, perm,
                           s.top_k, offsets, slot_of_pair, P, (const uint16_t*)W1p, nul, H, d, f, filt, nosink, now);
    if (mid && hipEventRecord(mid, st) != hipSuccess) return MMOE_ERR_LAUNCH;
    if (sink.w)
        hipLaunchKernelGGL((skinny_frag_kernel<1, 2, kModeGatedY>), g2, block, 0, st, (const uint16_t*)H, noperm, 1,
                           offsets, slot_of_pair, P, (const uint16_t*)W2p, nul, sink.Y, f, d, filt, sink.perm, sink.w);
    else
        hipLaunchKernelGGL((skinny_frag_kernel<1, 2, kModePlainF32>), g2, block, 0, st, (const uint16_t*)H, noperm, 1,
                           offsets, slot_of_pair, P, (const uint16_t*)W2p, nul, (void*)Yg, f, d, filt, nosink, now);
    return launch_status();
}

template <typename T, bool SPLITK>
static void launch_skinny_products(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                                   const int32_t* slot_of_pair, const void* W1p, const void* W3p, const void* W2p,
                                   void* H, float* Yg, hipStream_t st, hipEvent_t mid, SlotFilter filt, bool up,
                                   bool down, GateSink sink)
{
    const int32_t* nosink = nullptr;
    const float* now = nullptr;
    const int32_t* noperm = nullptr;
    const int d = s.d_model, f = s.d_ff, P = s.T * s.top_k;
    constexpr int kFeat = SPLITK ? 16 : 16 * kSkWaves;  // output features per workgroup
    dim3 block(kSkThreads);
    dim3 g1(f / kFeat, s.S), g2(d / kFeat, s.S);
    const T* nul = nullptr;
    if (up) {
        if (s.act == MMOE_SWIGLU)
            hipLaunchKernelGGL((skinny_kernel<T, 2, 1, kModeSwigluH, SPLITK>), g1, block, 0, st, (const T*)rows, perm,
                               s.top_k, offsets, slot_of_pair, P, (const T*)W1p, (const T*)W3p, H, d, f, filt,
                               nosink, now);
        else if (s.act == MMOE_GELU)
            hipLaunchKernelGGL((skinny_kernel<T, 1, 2, kModeGeluH, SPLITK>), g1, block, 0, st, (const T*)rows, perm,
                               s.top_k, offsets, slot_of_pair, P, (const T*)W1p, nul, H, d, f, filt, nosink, now);
        else
            hipLaunchKernelGGL((skinny_kernel<T, 1, 2, kModeReluH, SPLITK>), g1, block, 0, st, (const T*)rows, perm,
                               s.top_k, offsets, slot_of_pair, P, (const T*)W1p, nul, H, d, f, filt, nosink, now);
    }
    if (down && sink.w)
        hipLaunchKernelGGL((skinny_kernel<T, 1, 2, kModeGatedY, SPLITK>), g2, block, 0, st, (const T*)H, noperm, 1,
                           offsets, slot_of_pair, P, (const T*)W2p, nul, sink.Y, f, d, filt, sink.perm, sink.w);
    else if (down)
        hipLaunchKernelGGL((skinny_kernel<T, 1, 2, kModePlainF32, SPLITK>), g2, block, 0, st, (const T*)H, noperm, 1,
                           offsets, slot_of_pair, P, (const T*)W2p, nul, (void*)Yg, f, d, filt, nosink, now);
    (void)mid;
}

// A product whose reduction dimension gives a wavefront fewer than three iterations when split four
// ways keeps it whole (K <= 1024 for fp32).
static bool whole_k(int K) { return K <= 1024; }

template <typename T>
static int run_skinny(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                      const int32_t* slot_of_pair, const void* W1p, const void* W3p, const void* W2p, void* H, float* Yg,
                      hipStream_t st, hipEvent_t mid, SlotFilter filt, GateSink sink)
{
    if (whole_k(s.d_model))
        launch_skinny_products<T, false>(s, rows, perm, offsets, slot_of_pair, W1p, W3p, W2p, H, Yg, st, mid, filt, true,
                                         false, sink);
    else
        launch_skinny_products<T, true>(s, rows, perm, offsets, slot_of_pair, W1p, W3p, W2p, H, Yg, st, mid, filt, true,
                                        false, sink);
    if (mid && hipEventRecord(mid, st) != hipSuccess) return MMOE_ERR_LAUNCH;
    if (whole_k(s.d_ff))
        launch_skinny_products<T, false>(s, rows, perm, offsets, slot_of_pair, W1p, W3p, W2p, H, Yg, st, mid, filt, false,
                                         true, sink);
    else
        launch_skinny_products<T, true>(s, rows, perm, offsets, slot_of_pair, W1p, W3p, W2p, H, Yg, st, mid, filt, false,
                                        true, sink);
    return launch_status();
}

bool self_grouping(const mmoe_shape& s)
{
    return use_skinny(s) && (int64_t)s.T * s.top_k <= kSelfMaxP;
}

int launch_ffn_skinny(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                      const int32_t* slot_of_pair, const void* W1p, const void* W3p, const void* W2p, void* H,
                      float* Yg, hipStream_t st, hipEvent_t mid, SlotFilter filt, GateSink sink)
{
    if (slot_of_pair && (int64_t)s.T * s.top_k > kSelfMaxP) return MMOE_ERR_LIMIT;
    // gated output rows: one pick per token; the grouped form needs the permutation, the self-grouping form must not have one
    if (sink.w && (s.top_k != 1 || !sink.Y || (slot_of_pair != nullptr) != (sink.perm == nullptr))) return MMOE_ERR_DIM;
    if (s.dtype == MMOE_BF16)
        return run_skinny_bf16(s, rows, perm, offsets, slot_of_pair, W1p, W3p, W2p, H, Yg, st, mid, filt, sink);
    return run_skinny<float>(s, rows, perm, offsets, slot_of_pair, W1p, W3p, W2p, H, Yg, st, mid, filt, sink);
}

}  // namespace mmoe
