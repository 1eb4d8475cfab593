// The initial expert loader's table (Algorithm 1; section 3.1): degree of similarity of every
// expert location, ranking, round-robin owners up to the expert capacity, per-layer slot tables.
//
// The cost is the first step: every model's experts are read once from HBM, which is the bound.
// For one location the flattened expert of model v is the concatenation of its matrices; the
// location's value is  sum_{i<j} sqrt( sum_t (a_i[t] - a_j[t])^2 ).  All V models are read in
// one pass (16 bytes per lane and model per step) and every pair's difference is formed from the
// registers, so the traffic is V reads per element whatever the number of pairs.
//
// Arithmetic: the difference of two stored values and its square are fp32 (a bf16 difference is
// exact in fp32 unless the exponents are 17 or more apart); squares are summed eight at a time in
// fp32 and then in fp64: per lane, across the wavefront (xor butterfly), across the workgroup's
// four wavefronts, and over the workgroups of a location in ascending order by a second kernel.
// No atomics: the result does not depend on the order in which workgroups run.
//
// The remaining steps are a few thousand integers: one workgroup ranks the locations by counting
// (rank = 1 + number of locations that are more similar, ties to the lower index), assigns owners
// and writes the tables.
#include "mmoe_internal.h"

namespace mmoe {

constexpr int kTabThreads = 256;
constexpr int kTabIters = 16;                              // 16-byte pieces per lane and model per workgroup
constexpr int kTabPieces = kTabThreads * kTabIters;        // pieces per workgroup
constexpr int kMaxPairs = kLoaderMaxV * (kLoaderMaxV - 1) / 2;

struct LoaderPtrs {
    const void* mat[kLoaderMaxV][3];
};

template <typename T> struct Piece;
template <> struct Piece<uint16_t> {  // 8 bf16 values
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void widen(const u32x4& r, float (&v)[8])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(r[i] << 16);
            v[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
        }
    }
};
template <> struct Piece<float> {  // 4 fp32 values
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void widen(const u32x4& r, float (&v)[4])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(r[i]);
    }
};

// grid (chunks of all matrices, L*E).  partial[(loc * nchunks + chunk) * npairs + pair].
template <typename T, int V>
__global__ __launch_bounds__(kTabThreads) void expert_distance_kernel(LoaderPtrs ptrs, int n_mats, int64_t e0, int64_t e1,
                                                                     int64_t e2, int c0, int c1,
                                                                     double* __restrict__ partial, int nchunks)
{
    constexpr int NP = V * (V - 1) / 2;
    constexpr int EL = Piece<T>::kElems;
    __shared__ double red[kTabThreads / kWave][NP > 0 ? NP : 1];
    const int loc = blockIdx.y, chunk = blockIdx.x;
    // chunk -> (matrix, first piece of the chunk inside the location's part of that matrix)
    const int m = chunk < c0 ? 0 : (chunk < c0 + c1 ? 1 : 2);
    const int64_t elems = m == 0 ? e0 : (m == 1 ? e1 : e2);
    const int64_t piece0 = (int64_t)(chunk - (m == 0 ? 0 : (m == 1 ? c0 : c0 + c1))) * kTabPieces;
    const int64_t pieces = elems / EL;
    const u32x4* src[V];
#pragma unroll
    for (int v = 0; v < V; ++v) src[v] = reinterpret_cast<const u32x4*>(ptrs.mat[v][m]) + (int64_t)loc * pieces;

    double acc[NP > 0 ? NP : 1];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = 0.0;
#pragma unroll 4
    for (int it = 0; it < kTabIters; ++it) {
        const int64_t q = piece0 + (int64_t)it * kTabThreads + threadIdx.x;
        if (q < pieces) {
            float val[V][EL];
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const u32x4 r = src[v][q];
                Piece<T>::widen(r, val[v]);
            }
            int p = 0;
#pragma unroll
            for (int i = 0; i < V; ++i)
#pragma unroll
                for (int j = i + 1; j < V; ++j) {
                    float s = 0.0f;
#pragma unroll
                    for (int t = 0; t < EL; ++t) {
                        const float df = val[i][t] - val[j][t];
                        s = __builtin_fmaf(df, df, s);
                    }
                    acc[p] += (double)s;
                    ++p;
                }
        }
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        double a = acc[p];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off, kWave);
        if (lane == 0) red[wave][p] = a;
    }
    __syncthreads();
    if (threadIdx.x < NP) {
        const int p = threadIdx.x;
        partial[((size_t)loc * nchunks + chunk) * NP + p] = (red[0][p] + red[1][p]) + (red[2][p] + red[3][p]);
    }
}

// One workgroup per location: the chunks' partial sums in a fixed order, the square root of every
// pair, the sum over the pairs.
__global__ __launch_bounds__(kTabThreads) void distance_finish_kernel(const double* __restrict__ partial, int nchunks,
                                                                     int npairs, double* __restrict__ distance)
{
    __shared__ double red[kTabThreads];
    const int loc = blockIdx.x;
    double total = 0.0;
    for (int p = 0; p < npairs; ++p) {  // uniform over the workgroup
        double a = 0.0;
        for (int c = threadIdx.x; c < nchunks; c += kTabThreads) a += partial[((size_t)loc * nchunks + c) * npairs + p];
        red[threadIdx.x] = a;
        __syncthreads();
        for (int half = kTabThreads / 2; half >= 1; half >>= 1) {
            if ((int)threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
            __syncthreads();
        }
        total += sqrt(red[0]);
        __syncthreads();
    }
    if (threadIdx.x == 0) distance[loc] = total;
}

// Ranking, owners and per-layer tables: one workgroup.
__global__ __launch_bounds__(kTabThreads) void expert_map_kernel(const double* __restrict__ distance, int V, int L, int E,
                                                                int capacity, int32_t* __restrict__ rank,
                                                                int32_t* __restrict__ owner, int32_t* __restrict__ M,
                                                                int32_t* __restrict__ S, int32_t* __restrict__ slot_src)
{
    __shared__ double d[kLoaderMaxLoc];
    __shared__ int own[kLoaderMaxLoc];
    const int N = L * E;
    for (int i = threadIdx.x; i < N; i += kTabThreads) d[i] = distance[i];
    __syncthreads();
    for (int i = threadIdx.x; i < N; i += kTabThreads) {
        const double di = d[i];
        int r = 1;  // 1-based: the most similar location has rank 1
        for (int j = 0; j < N; ++j) r += (d[j] < di || (d[j] == di && j < i)) ? 1 : 0;
        rank[i] = r;
        // round robin from the highest rank while capacity remains: rank 1 -> first model, 2 -> second, ...
        const int o = r <= capacity ? (r - 1) % V : -1;
        own[i] = o;
        owner[i] = o;
    }
    __syncthreads();
    // layer l: variant 0's locations take slots 0..E-1; the private slots of the other variants follow
    for (int l = threadIdx.x; l < L; l += kTabThreads) {
        int32_t* Ml = M + (size_t)l * V * E;
        int32_t* src = slot_src + (size_t)l * V * E * 2;
        for (int e = 0; e < E; ++e) {
            const int o = own[l * E + e];
            Ml[e] = e;
            src[2 * e] = o >= 0 ? o : 0;
            src[2 * e + 1] = e;
        }
        int nxt = E;
        for (int v = 1; v < V; ++v)
            for (int e = 0; e < E; ++e) {
                if (own[l * E + e] >= 0) {
                    Ml[v * E + e] = e;
                } else {
                    Ml[v * E + e] = nxt;
                    src[2 * nxt] = v;
                    src[2 * nxt + 1] = e;
                    ++nxt;
                }
            }
        S[l] = nxt;
        for (int s = nxt; s < V * E; ++s) {  // rows past the layer's last slot
            src[2 * s] = -1;
            src[2 * s + 1] = -1;
        }
    }
}

// Pool of one layer from the table: slot s of matrix m is a copy of the (variant, expert) that
// slot_src names ("load M[idx].expert[iL][iE] to GPU", Algorithm 1; here the variants already are in
// device memory, so the load is a device copy).  grid (chunks, S_l, n_mats), 16 bytes per lane and step.
__global__ __launch_bounds__(kTabThreads) void assemble_pool_kernel(LoaderPtrs ptrs, const int32_t* __restrict__ slot_src,
                                                                   int layer, int E, int64_t p0, int64_t p1, int64_t p2,
                                                                   u32x4* __restrict__ d0, u32x4* __restrict__ d1,
                                                                   u32x4* __restrict__ d2)
{
    const int s = blockIdx.y, m = blockIdx.z;
    const int v = slot_src[2 * s], e = slot_src[2 * s + 1];
    if (v < 0) return;  // uniform over the workgroup: a row past the layer's last slot
    const int64_t pieces = m == 0 ? p0 : (m == 1 ? p1 : p2);
    u32x4* dst = (m == 0 ? d0 : (m == 1 ? d1 : d2)) + (int64_t)s * pieces;
    const u32x4* src = reinterpret_cast<const u32x4*>(ptrs.mat[v][m]) + ((int64_t)layer * E + e) * pieces;
    for (int64_t q = (int64_t)blockIdx.x * kTabThreads + threadIdx.x; q < pieces; q += (int64_t)gridDim.x * kTabThreads)
        dst[q] = src[q];
}

int launch_assemble_pool(const mmoe_loader_shape& s, const void* const* mats, const int32_t* slot_src_layer, int layer,
                         int n_slots, void* const* pool, hipStream_t st)
{
    LoaderPtrs p = {};
    for (int v = 0; v < s.V; ++v)
        for (int m = 0; m < s.n_mats; ++m) p.mat[v][m] = mats[v * s.n_mats + m];
    const int el = s.dtype == MMOE_BF16 ? 8 : 4;
    int64_t pc[3] = {0, 0, 0};
    int64_t most = 0;
    for (int m = 0; m < s.n_mats; ++m) {
        pc[m] = s.mat_elems[m] / el;
        most = pc[m] > most ? pc[m] : most;
    }
    const int chunks = (int)((most + (int64_t)kTabThreads * 8 - 1) / ((int64_t)kTabThreads * 8));  // 8 pieces per thread
    hipLaunchKernelGGL(assemble_pool_kernel, dim3(chunks > 65535 ? 65535 : chunks, n_slots, s.n_mats), dim3(kTabThreads),
                       0, st, p, slot_src_layer, layer, s.E, pc[0], pc[1], pc[2], (u32x4*)pool[0],
                       (u32x4*)(s.n_mats > 1 ? pool[1] : nullptr), (u32x4*)(s.n_mats > 2 ? pool[2] : nullptr));
    return launch_status();
}

static int loader_chunks(const mmoe_loader_shape& s, int (&c)[3])
{
    const int el = s.dtype == MMOE_BF16 ? 8 : 4;
    int total = 0;
    for (int m = 0; m < 3; ++m) {
        c[m] = m < s.n_mats ? (int)((s.mat_elems[m] / el + kTabPieces - 1) / kTabPieces) : 0;
        total += c[m];
    }
    return total;
}

size_t loader_ws_bytes(const mmoe_loader_shape& s)
{
    int c[3];
    const int nch = loader_chunks(s, c);
    const int np = s.V * (s.V - 1) / 2;
    return align256((size_t)s.L * s.E * nch * (np > 0 ? np : 1) * sizeof(double));
}

template <typename T, int V>
static void launch_distance_v(const mmoe_loader_shape& s, const LoaderPtrs& p, const int (&c)[3], int nch,
                              double* partial, hipStream_t st)
{
    hipLaunchKernelGGL((expert_distance_kernel<T, V>), dim3(nch, s.L * s.E), dim3(kTabThreads), 0, st, p, s.n_mats,
                       s.mat_elems[0], s.mat_elems[1], s.mat_elems[2], c[0], c[1], partial, nch);
}

int launch_expert_distance(const mmoe_loader_shape& s, const void* const* mats, double* distance, double* partial,
                           hipStream_t st)
{
    LoaderPtrs p = {};
    for (int v = 0; v < s.V; ++v)
        for (int m = 0; m < s.n_mats; ++m) p.mat[v][m] = mats[v * s.n_mats + m];
    int c[3];
    const int nch = loader_chunks(s, c);
#define MMOE_DIST(VV)                                                                         \
    case VV:                                                                                  \
        if (s.dtype == MMOE_BF16) launch_distance_v<uint16_t, VV>(s, p, c, nch, partial, st); \
        else launch_distance_v<float, VV>(s, p, c, nch, partial, st);                         \
        break
    switch (s.V) {
        MMOE_DIST(1);
        MMOE_DIST(2);
        MMOE_DIST(3);
        MMOE_DIST(4);
        MMOE_DIST(5);
        MMOE_DIST(6);
        MMOE_DIST(7);
        default: MMOE_DIST(8);
    }
#undef MMOE_DIST
    hipLaunchKernelGGL(distance_finish_kernel, dim3(s.L * s.E), dim3(kTabThreads), 0, st, partial, nch,
                       s.V * (s.V - 1) / 2, distance);
    return launch_status();
}

int launch_expert_map(const mmoe_loader_shape& s, const double* distance, int32_t* rank, int32_t* owner, int32_t* M,
                      int32_t* S, int32_t* slot_src, hipStream_t st)
{
    hipLaunchKernelGGL(expert_map_kernel, dim3(1), dim3(kTabThreads), 0, st, distance, s.V, s.L, s.E, s.capacity, rank,
                       owner, M, S, slot_src);
    return launch_status();
}

}  // namespace mmoe
