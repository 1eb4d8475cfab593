// Step R: per-variant gate, top-k selection and coefficients (Algorithm 2, "gate(act)";
// section 3.2).  Two launch shapes with the same arithmetic: small batches give a token to a
// workgroup whose wavefronts share out the experts (latency); large batches give a token to
// one wavefront that keeps the token row in registers and walks the experts (throughput).
//
// The logit is an fp32 sum in the fixed order the header states: lane l owns the
// elements i with (i div 4) mod 64 == l, which is exactly what a coalesced 4-element
// vector load per lane delivers; each lane folds its elements in ascending i with one
// fused multiply-add each; the 64 partial sums meet in an xor butterfly 32,16,...,1.
// fp32 addition is commutative, so both partners of an exchange compute the same sum and
// every lane ends with the same value.
//
// Logits are parked in LDS, then the k winners are found by wavefront arg-max
// reductions: lane l looks after experts l, l+64, ...; ties go to the lower index.
// Coefficients: softmax over the selected logits, or (gate over all experts) each selected
// expert's entry of the softmax over all E logits, whose normaliser is one more wavefront
// reduction over the parked logits.
#include "mmoe_internal.h"

namespace mmoe {

constexpr int kRouteWaves = 8;   // wavefronts per token: they share out the experts

template <typename T> struct Vec4;
template <> struct Vec4<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[4])
    {
        f32x4 t = *reinterpret_cast<const f32x4*>(p);
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    }
};
template <> struct Vec4<uint16_t> {
    static __device__ __forceinline__ void load(const uint16_t* p, float (&v)[4])
    {
        u32x2 t = *reinterpret_cast<const u32x2*>(p);
        v[0] = __uint_as_float(t[0] << 16);
        v[1] = __uint_as_float(t[0] & 0xFFFF0000u);
        v[2] = __uint_as_float(t[1] << 16);
        v[3] = __uint_as_float(t[1] & 0xFFFF0000u);
    }
};

// The k winners among E logits in LDS, found by one wavefront: lane l looks after experts
// l, l+64, l+128, l+192; k arg-max reductions, ties to the lower index; coefficients =
// softmax over the selected logits.
// With a table row `map_row` (= M[vid[t]], or null) the picks are also looked up in the expert
// map and slot[t*k + j] is written: step M folded into the router for batches whose expert stage
// groups the pairs itself.
__device__ __forceinline__ void select_topk(const float* __restrict__ lds_logit, int lane, int E, int k, int t,
                                            int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                            const int32_t* __restrict__ map_row, int32_t* __restrict__ slot, int S,
                                            int gate)
{
    constexpr int kPerLane = kMaxE / kWave;
    float mine[kPerLane];
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) {
        int e = lane + q * kWave;
        mine[q] = e < E ? lds_logit[e] : -INFINITY;
    }
    uint32_t taken = 0;
    float sel[kMaxTopK];
    int seli[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        if (j < k) {
            float bv = -INFINITY;
            int be = 0x7FFFFFFF;
#pragma unroll
            for (int q = 0; q < kPerLane; ++q) {  // ascending index: strict > keeps the lower one
                int e = lane + q * kWave;
                if (e < E && !(taken & (1u << q)) && (be == 0x7FFFFFFF || mine[q] > bv)) {
                    bv = mine[q];
                    be = e;
                }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                float ov = __shfl_xor(bv, off, kWave);
                int oe = __shfl_xor(be, off, kWave);
                bool other_valid = oe != 0x7FFFFFFF, self_valid = be != 0x7FFFFFFF;
                bool take = other_valid && (!self_valid || ov > bv || (ov == bv && oe < be));
                if (take) { bv = ov; be = oe; }
            }
            sel[j] = bv;
            seli[j] = be;
            if ((be & (kWave - 1)) == lane) taken |= 1u << (be / kWave);
        }
    }
    // gate over all experts: the normaliser is the sum of exp(logit - largest logit) over every expert
    // (sel[0] is the largest); fp32, lane-local in ascending expert index, then an xor butterfly
    float all = 0.0f;
    if (gate == MMOE_GATE_ALL) {
#pragma unroll
        for (int q = 0; q < kPerLane; ++q)
            if (lane + q * kWave < E) all += expf(mine[q] - sel[0]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) all += __shfl_xor(all, off, kWave);
    }
    if (lane == 0) {
        float z[kMaxTopK];
        float tot = 0.0f;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j)
            if (j < k) {
                z[j] = expf(sel[j] - sel[0]);
                tot += z[j];
            }
        if (gate == MMOE_GATE_ALL) tot = all;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j)
            if (j < k) {
                topk_idx[(size_t)t * k + j] = seli[j];
                topk_w[(size_t)t * k + j] = z[j] / tot;
                // the clamp keeps every later index in range even for an invalid table (results then undefined)
                if (map_row) slot[(size_t)t * k + j] = min(max(map_row[seli[j]], 0), S - 1);
            }
    }
}

// One workgroup per token; wavefront w scores experts w, w+8, ...  A token's dot product
// with one expert is never split between wavefronts, so the summation order is the
// contract's whatever the launch shape.  Four vectors per lane are fetched at a time to
// keep eight loads in flight.
template <typename T>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(
    const T* __restrict__ X, const int32_t* __restrict__ vid, const T* __restrict__ Wr,
    const float* __restrict__ br, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int Tn, int d,
    int V, int E, int k, const int32_t* __restrict__ M, int32_t* __restrict__ slot, int S, int gate)
{
    __shared__ float lds_logit[kMaxE];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int t = blockIdx.x;

    const int v = min(max(vid[t], 0), V - 1);  // out-of-range ids are the caller's error; stay in bounds
    const T* x = X + (size_t)t * d;
    const int nvec = d / 4;  // a multiple of 64: d is a multiple of 256

    for (int e = wave; e < E; e += kRouteWaves) {
        const T* w = Wr + ((size_t)v * E + e) * d;
        float acc = 0.0f;
        int q = lane;
        for (; q + 3 * kWave < nvec; q += 4 * kWave) {  // ascending i within the lane
            float xv[4][4], wv[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                Vec4<T>::load(x + 4 * (q + u * kWave), xv[u]);
                Vec4<T>::load(w + 4 * (q + u * kWave), wv[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc = __builtin_fmaf(xv[u][c], wv[u][c], acc);
        }
        for (; q < nvec; q += kWave) {
            float xv[4], wv[4];
            Vec4<T>::load(x + 4 * q, xv);
            Vec4<T>::load(w + 4 * q, wv);
#pragma unroll
            for (int c = 0; c < 4; ++c) acc = __builtin_fmaf(xv[c], wv[c], acc);
        }
        float p = acc;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) p = p + __shfl_xor(p, off, kWave);
        if (br) p = p + br[(size_t)v * E + e];
        if (lane == 0) lds_logit[e] = p;
    }
    __syncthreads();
    if (wave != 0) return;

    select_topk(lds_logit, lane, E, k, t, topk_idx, topk_w, M ? M + (size_t)v * E : nullptr, slot, S, gate);
}

// Four consecutive elements as loaded (bf16 stays packed until it is used, which halves the
// registers a pending load occupies).
template <typename T> struct Raw4;
template <> struct Raw4<float> {
    typedef f32x4 type;
    static __device__ __forceinline__ float get(const type& r, int q) { return r[q]; }
};
template <> struct Raw4<uint16_t> {
    typedef u32x2 type;
    static __device__ __forceinline__ float get(const type& r, int q)
    {
        return (q & 1) ? __uint_as_float(r[q >> 1] & 0xFFFF0000u) : __uint_as_float(r[q >> 1] << 16);
    }
};

// Throughput variant for large batches: one wavefront per token.  The token's elements
// stay in registers (NC chunks of 256, d = 256*NC exactly, so that every load of a pass is
// issued before the first one is waited for) and the wavefront walks the experts
// two at a time, so that the token row crosses the memory pipeline once instead of once
// per expert.  Each (token, expert) sum is formed by one wavefront in the contract's order:
// the results are bit-identical to route_kernel's.
constexpr int kRouteTokWaves = 4;
// batches at least this large use the wavefront-per-token kernel (measured crossover: between
// 1024 and 2048 tokens at d = 4096 and at d = 768)
constexpr int kRouteTokMinT = 2048;

template <typename T, int NC>
__global__ __launch_bounds__(kRouteTokWaves* kWave) void route_token_kernel(
    const T* __restrict__ X, const int32_t* __restrict__ vid, const T* __restrict__ Wr,
    const float* __restrict__ br, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int Tn, int d,
    int V, int E, int k, const int32_t* __restrict__ M, int32_t* __restrict__ slot, int S, int gate)
{
    __shared__ float lds_logit[kRouteTokWaves][kMaxE];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int t = blockIdx.x * kRouteTokWaves + wave;
    if (t >= Tn) return;  // uniform over the wavefront; no workgroup barrier below

    const int v = min(max(vid[t], 0), V - 1);
    const T* x = X + (size_t)t * d + 4 * lane;
    typedef typename Raw4<T>::type raw_t;
    raw_t xv[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) xv[c] = *reinterpret_cast<const raw_t*>(x + 256 * c);

    const T* wv0 = Wr + (size_t)v * E * d + 4 * lane;
    float* mylogit = lds_logit[wave];
    for (int e = 0; e < E; e += 2) {
        const bool two = e + 1 < E;
        const T* w0 = wv0 + (size_t)e * d;
        const T* w1 = wv0 + (size_t)(two ? e + 1 : e) * d;
        float a0 = 0.0f, a1 = 0.0f;
        raw_t p0[NC], p1[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            p0[c] = *reinterpret_cast<const raw_t*>(w0 + 256 * c);
            p1[c] = *reinterpret_cast<const raw_t*>(w1 + 256 * c);
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // ascending i within the lane
                const float xq = Raw4<T>::get(xv[c], q);
                a0 = __builtin_fmaf(xq, Raw4<T>::get(p0[c], q), a0);
                a1 = __builtin_fmaf(xq, Raw4<T>::get(p1[c], q), a1);
            }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            a0 = a0 + __shfl_xor(a0, off, kWave);
            a1 = a1 + __shfl_xor(a1, off, kWave);
        }
        if (br) {
            a0 = a0 + br[(size_t)v * E + e];
            if (two) a1 = a1 + br[(size_t)v * E + e + 1];
        }
        if (lane == 0) {
            mylogit[e] = a0;
            if (two) mylogit[e + 1] = a1;
        }
    }
    // lane 0's LDS writes before every lane's reads: one wavefront's LDS operations execute in
    // program order, the fence keeps the compiler from moving them
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    select_topk(mylogit, lane, E, k, t, topk_idx, topk_w, M ? M + (size_t)v * E : nullptr, slot, S, gate);
}

int launch_route(const mmoe_shape& s, const void* X, const int32_t* vid, const void* Wr, const float* br,
                 int32_t* topk_idx, float* topk_w, hipStream_t st, const int32_t* M, int32_t* slot)
{
    // Large batches of a common hidden size: a wavefront per token (the token row is read
    // once); otherwise a workgroup per token (lower latency, any d).
    const int nc = s.d_model / 256;
    const bool tok_nc = nc == 1 || nc == 2 || nc == 3 || nc == 4 || nc == 6 || nc == 8 || nc == 12 || nc == 16;
    if (s.T >= kRouteTokMinT && tok_nc && s.d_model % 256 == 0) {
        dim3 grid((s.T + kRouteTokWaves - 1) / kRouteTokWaves), block(kRouteTokWaves * kWave);
#define MMOE_ROUTE_TOK(NC)                                                                                          \
    case NC:                                                                                                        \
        if (s.dtype == MMOE_BF16)                                                                                   \
            hipLaunchKernelGGL((route_token_kernel<uint16_t, NC>), grid, block, 0, st, (const uint16_t*)X, vid,     \
                               (const uint16_t*)Wr, br, topk_idx, topk_w, s.T, s.d_model, s.V, s.E, s.top_k, M, slot, s.S, s.gate);       \
        else                                                                                                        \
            hipLaunchKernelGGL((route_token_kernel<float, NC>), grid, block, 0, st, (const float*)X, vid,           \
                               (const float*)Wr, br, topk_idx, topk_w, s.T, s.d_model, s.V, s.E, s.top_k, M, slot, s.S, s.gate);          \
        break
        switch (nc) {
            MMOE_ROUTE_TOK(1);
            MMOE_ROUTE_TOK(2);
            MMOE_ROUTE_TOK(3);
            MMOE_ROUTE_TOK(4);
            MMOE_ROUTE_TOK(6);
            MMOE_ROUTE_TOK(8);
            MMOE_ROUTE_TOK(12);
            default: MMOE_ROUTE_TOK(16);
        }
#undef MMOE_ROUTE_TOK
        return launch_status();
    }
    dim3 grid(s.T), block(kRouteWaves * kWave);
    if (s.dtype == MMOE_BF16)
        hipLaunchKernelGGL(route_kernel<uint16_t>, grid, block, 0, st, (const uint16_t*)X, vid,
                           (const uint16_t*)Wr, br, topk_idx, topk_w, s.T, s.d_model, s.V, s.E, s.top_k, M, slot, s.S, s.gate);
    else
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, st, (const float*)X, vid, (const float*)Wr, br,
                           topk_idx, topk_w, s.T, s.d_model, s.V, s.E, s.top_k, M, slot, s.S, s.gate);
    return launch_status();
}

}  // namespace mmoe
