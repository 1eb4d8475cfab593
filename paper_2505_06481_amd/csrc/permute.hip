// Steps M and G: expert-map lookup, slot histogram, exclusive scan, stable grouping of
// the (token, pick) pairs by pool slot, and the row gather (Algorithm 2, the map lookup
// that precedes the expert call; grouping is what lets one resident expert serve every
// token that hit it, whichever variant the token belongs to).
//
// Deterministic by construction: the rank of pair p inside its slot is the number of
// lower pair ids with the same slot, computed from wavefront ballots and integer
// prefix sums.  There are no cursors bumped by atomics and no waiting between
// workgroups: three short kernels (histogram, scan, scatter; two when the scatter workgroups can
// afford to sum the histograms themselves) and one gather.
//
// Work split: workgroup b owns pairs [b*2048, (b+1)*2048); inside it wavefront w owns a
// contiguous quarter, walked 64 pairs at a time in ascending order.
#include "mmoe_internal.h"
#include "tile_table.h"

namespace mmoe {

constexpr int kPermThreads = 256;
static_assert(kPermThreads == 256, "build_tile_lists is written for one workgroup of 256 threads");
constexpr int kPermWaves = kPermThreads / kWave;
constexpr int kPairsPerWave = kPermChunk / kPermWaves;  // 512
// Most grouping workgroups (of 2048 pairs) that each count the whole batch's slots themselves: the LDS
// atomics of one workgroup serialise on a few slot counters, so beyond two workgroups' worth of pairs
// the separate histogram kernel (2048 pairs per workgroup) is faster (measured at 8: 31 us against 18).
constexpr int kOwnHistMaxBlk = 2;
constexpr int kOwnScanMax = 1 << 14;  // most per-workgroup counts (workgroups x slots) a scatter workgroup sums by itself
static_assert(kMaxS % kPermThreads == 0, "slots per thread");

// slot[p] = M[vid[p / k]][topk_idx[p]]; per-workgroup histogram of the slots.
__global__ __launch_bounds__(kPermThreads) void slot_hist_kernel(
    const int32_t* __restrict__ vid, const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ M,
    int32_t* __restrict__ slot, int32_t* __restrict__ blk_counts, int P, int k, int V, int E, int S)
{
    __shared__ int hist[kMaxS];
    for (int s = threadIdx.x; s < S; s += kPermThreads) hist[s] = 0;
    __syncthreads();
    const int base = blockIdx.x * kPermChunk;
    for (int i = threadIdx.x; i < kPermChunk; i += kPermThreads) {
        int p = base + i;
        if (p < P) {
            // clamps keep every later index in range even for invalid ids (results then undefined)
            int v = min(max(vid[p / k], 0), V - 1);
            int e = min(max(topk_idx[p], 0), E - 1);
            int s = min(max(M[v * E + e], 0), S - 1);
            slot[p] = s;
            atomicAdd(&hist[s], 1);  // integer LDS atomic: the sum does not depend on order
        }
    }
    __syncthreads();
    for (int s = threadIdx.x; s < S; s += kPermThreads) blk_counts[(size_t)blockIdx.x * S + s] = hist[s];
}

// counts, offsets, and for every (workgroup, slot) the first output row of that workgroup's pairs.
__global__ __launch_bounds__(kPermThreads) void slot_scan_kernel(const int32_t* __restrict__ blk_counts,
                                                                 int32_t* __restrict__ blk_base,
                                                                 int32_t* __restrict__ counts,
                                                                 int32_t* __restrict__ offsets, int nblk, int S,
                                                                 TileJob tiles)
{
    __shared__ int tot[kMaxS];
    __shared__ int off[kMaxS + 1];
    for (int s = threadIdx.x; s < S; s += kPermThreads) {
        int run = 0;
        for (int b = 0; b < nblk; ++b) {
            int c = blk_counts[(size_t)b * S + s];
            blk_base[(size_t)b * S + s] = run;
            run += c;
        }
        tot[s] = run;
        counts[s] = run;
    }
    __syncthreads();
    if (threadIdx.x < kWave) {  // one wavefront scans the S totals, 64 at a time
        int carry = 0;
        for (int s0 = 0; s0 < S; s0 += kWave) {
            int s = s0 + threadIdx.x;
            int c = s < S ? tot[s] : 0;
            int incl = c;
#pragma unroll
            for (int dlt = 1; dlt < kWave; dlt <<= 1) {
                int o = __shfl_up(incl, dlt, kWave);
                if ((int)threadIdx.x >= dlt) incl += o;
            }
            if (s < S) off[s] = carry + incl - c;
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (threadIdx.x == 0) off[S] = carry;
    }
    __syncthreads();
    for (int s = threadIdx.x; s <= S; s += kPermThreads) offsets[s] = off[s];
    for (int s = threadIdx.x; s < S; s += kPermThreads) {
        int o = off[s];
        for (int b = 0; b < nblk; ++b) blk_base[(size_t)b * S + s] += o;
    }
    // the tile lists of the matrix-core expert kernels, from the offsets this workgroup has just written
    if (tiles.tab) {
        __syncthreads();
        build_tile_lists(offsets, tiles.tab, S, tiles.nt_up, tiles.nt_down, tiles.bm, tiles.L);
    }
}

// Stable placement of up to 64 pairs, one per lane, behind the pairs placed before them:
// lane l's peers are the lanes that hold the same slot, found with one ballot per bit of the
// slot id; its row is the slot's cursor plus the number of peers in lower lanes; the lowest
// peer then advances the cursor.  `cur` is this wavefront's private cursor row in LDS, and
// LDS operations of one wavefront execute in program order.
__device__ __forceinline__ void place_pairs(volatile int* cur, int s, bool valid, int lane, int sbits, int p,
                                            int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm)
{
    unsigned long long m = __ballot(valid);
    for (int b = 0; b < sbits; ++b) {
        const bool bit = (s >> b) & 1;
        const unsigned long long bal = __ballot(bit);
        m &= bit ? bal : ~bal;
    }
    const int rank = __popcll(m & ((1ull << lane) - 1ull));
    int base = 0;
    if (valid) {
        base = cur[s];
        const int r = base + rank;
        perm[r] = p;
        inv_perm[p] = r;
    }
    __builtin_amdgcn_wave_barrier();
    if (valid && rank == 0) cur[s] = base + __popcll(m);
    __builtin_amdgcn_wave_barrier();
}

// perm / inv_perm: stable ranks from ballots.  Where the first output row of this workgroup's pairs of
// every slot comes from:
//   kFromScan    `blk_base`, written by slot_scan_kernel;
//   kOwnScan     few workgroups, few slots, so the table of per-workgroup counts is small: every
//                workgroup sums that table itself, and the scan kernel and its launch are not needed;
//   kOwnHist     few workgroups, and slot[] already written by the router: every workgroup counts the
//                pairs in front of its own and the pairs of the whole batch itself (a read of P integers
//                and integer LDS atomics), and the histogram kernel is not needed either.
// In the last two the grid has one more workgroup, which places no pairs and writes counts, offsets and
// the tile lists instead.
enum { kFromScan = 0, kOwnScan = 1, kOwnHist = 2 };
template <int SRC>
__global__ __launch_bounds__(kPermThreads) void slot_scatter_kernel(const int32_t* __restrict__ slot,
                                                                    const int32_t* __restrict__ blk_base,
                                                                    const int32_t* __restrict__ blk_counts, int nblk,
                                                                    int32_t* __restrict__ counts,
                                                                    int32_t* __restrict__ offsets,
                                                                    int32_t* __restrict__ perm,
                                                                    int32_t* __restrict__ inv_perm, int P, int S,
                                                                    TileJob tiles)
{
    __shared__ int wtot[kPermWaves][kMaxS];  // pairs of each slot owned by each wavefront
    __shared__ int cursor[kPermWaves][kMaxS];
    constexpr bool SCAN = SRC != kFromScan;
    __shared__ int tot[SCAN ? kMaxS : 1];      // pairs of each slot in the whole batch, then its first row
    __shared__ int lower[SRC == kOwnHist ? kMaxS : 1];  // pairs of each slot in front of this workgroup's
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int sbits = 32 - __clz(max(S - 1, 1));  // bits of a slot id
    int before[kMaxS / kPermThreads];             // this workgroup's first row of slot threadIdx.x + 256 i
    if (SCAN) {
        const int b = blockIdx.x;  // nblk: the workgroup that writes the tables
        if (SRC == kOwnHist) {
            for (int sl = threadIdx.x; sl < S; sl += kPermThreads) {
                tot[sl] = 0;
                lower[sl] = 0;
            }
            __syncthreads();
            const int first = b * kPermChunk;  // this workgroup's first pair (the table writer's: unused)
            for (int p = threadIdx.x; p < P; p += kPermThreads) {
                const int sl = slot[p];
                atomicAdd(&tot[sl], 1);  // integer LDS atomics: the sums do not depend on order
                if (p < first) atomicAdd(&lower[sl], 1);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kMaxS / kPermThreads; ++i) {
                const int sl = threadIdx.x + i * kPermThreads;
                before[i] = sl < S ? lower[sl] : 0;
            }
        } else {
#pragma unroll
            for (int i = 0; i < kMaxS / kPermThreads; ++i) {
                const int sl = threadIdx.x + i * kPermThreads;
                int run = 0, mine = 0;
                if (sl < S)
                    for (int bb = 0; bb < nblk; ++bb) {
                        if (bb == b) mine = run;
                        run += blk_counts[(size_t)bb * S + sl];
                    }
                before[i] = mine;
                if (sl < S) tot[sl] = run;
            }
        }
        __syncthreads();
        if (b == nblk)
            for (int sl = threadIdx.x; sl < S; sl += kPermThreads) counts[sl] = tot[sl];
        __syncthreads();
        if (threadIdx.x < kWave) {  // exclusive scan of the S totals, 64 at a time; tot[s] becomes offsets[s]
            int carry = 0;
            for (int s0 = 0; s0 < S; s0 += kWave) {
                const int sl = s0 + threadIdx.x;
                const int c = sl < S ? tot[sl] : 0;
                int incl = c;
#pragma unroll
                for (int dlt = 1; dlt < kWave; dlt <<= 1) {
                    const int o = __shfl_up(incl, dlt, kWave);
                    if ((int)threadIdx.x >= dlt) incl += o;
                }
                if (sl < S) {
                    tot[sl] = carry + incl - c;
                    if (b == nblk) offsets[sl] = carry + incl - c;
                }
                carry += __shfl(incl, kWave - 1, kWave);
            }
            if (b == nblk && threadIdx.x == 0) offsets[S] = carry;
        }
        __syncthreads();
        if (b == nblk) {  // uniform over the workgroup
            if (tiles.tab) build_tile_lists(offsets, tiles.tab, S, tiles.nt_up, tiles.nt_down, tiles.bm, tiles.L);
            return;
        }
    }
    for (int i = threadIdx.x; i < kPermWaves * S; i += kPermThreads) wtot[i / S][i % S] = 0;
    __syncthreads();
    const int wbase = blockIdx.x * kPermChunk + wave * kPairsPerWave;
    for (int i = lane; i < kPairsPerWave; i += kWave) {
        int p = wbase + i;
        if (p < P) atomicAdd(&wtot[wave][slot[p]], 1);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kMaxS / kPermThreads; ++i) {
        const int s = threadIdx.x + i * kPermThreads;
        if (s < S) {
            int run = SCAN ? tot[s] + before[i] : blk_base[(size_t)blockIdx.x * S + s];
#pragma unroll
            for (int w = 0; w < kPermWaves; ++w) {
                cursor[w][s] = run;
                run += wtot[w][s];
            }
        }
    }
    __syncthreads();
    // From here on a wavefront touches only its own cursor row; LDS operations of one
    // wavefront execute in program order.
    volatile int* cur = cursor[wave];
    for (int i0 = 0; i0 < kPairsPerWave; i0 += kWave) {
        int p = wbase + i0 + lane;
        bool valid = p < P;
        int s = valid ? slot[p] : 0;
        place_pairs(cur, s, valid, lane, sbits, p, perm, inv_perm);
    }
}

// The three kernels above in one, for batches whose pairs fit one workgroup's chunk (decode):
// same ranks, same results, two launches fewer.
__global__ __launch_bounds__(kPermThreads) void slot_group_small_kernel(
    const int32_t* __restrict__ vid, const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ M,
    int32_t* __restrict__ slot, int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm, int P, int k, int V, int E, int S, TileJob tiles)
{
    __shared__ int wtot[kPermWaves][kMaxS];
    __shared__ int cursor[kPermWaves][kMaxS];
    __shared__ int tot[kMaxS];
    __shared__ int myslot[kPermChunk];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int sbits = 32 - __clz(max(S - 1, 1));  // bits of a slot id
    for (int i = threadIdx.x; i < kPermWaves * S; i += kPermThreads) wtot[i / S][i % S] = 0;
    __syncthreads();
    const int wbase = wave * kPairsPerWave;
    for (int i = lane; i < kPairsPerWave; i += kWave) {
        int p = wbase + i;
        if (p < P) {
            int v = min(max(vid[p / k], 0), V - 1);
            int e = min(max(topk_idx[p], 0), E - 1);
            int s = min(max(M[v * E + e], 0), S - 1);
            slot[p] = s;
            myslot[p] = s;
            atomicAdd(&wtot[wave][s], 1);
        }
    }
    __syncthreads();
    for (int s = threadIdx.x; s < S; s += kPermThreads) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < kPermWaves; ++w) run += wtot[w][s];
        tot[s] = run;
        counts[s] = run;
    }
    __syncthreads();
    if (threadIdx.x < kWave) {  // exclusive scan of the S totals, 64 at a time; tot[s] becomes offsets[s]
        int carry = 0;
        for (int s0 = 0; s0 < S; s0 += kWave) {
            int s = s0 + threadIdx.x;
            int c = s < S ? tot[s] : 0;
            int incl = c;
#pragma unroll
            for (int dlt = 1; dlt < kWave; dlt <<= 1) {
                int o = __shfl_up(incl, dlt, kWave);
                if ((int)threadIdx.x >= dlt) incl += o;
            }
            if (s < S) {
                tot[s] = carry + incl - c;
                offsets[s] = carry + incl - c;
            }
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (threadIdx.x == 0) offsets[S] = carry;
    }
    __syncthreads();
    for (int s = threadIdx.x; s < S; s += kPermThreads) {
        int run = tot[s];
#pragma unroll
        for (int w = 0; w < kPermWaves; ++w) {
            cursor[w][s] = run;
            run += wtot[w][s];
        }
    }
    __syncthreads();
    volatile int* cur = cursor[wave];
    for (int i0 = 0; i0 < kPairsPerWave; i0 += kWave) {
        int p = wbase + i0 + lane;
        bool valid = p < P;
        if (!__ballot(valid)) break;  // uniform over the wavefront
        int s = valid ? myslot[p] : 0;
        place_pairs(cur, s, valid, lane, sbits, p, perm, inv_perm);
    }
    if (tiles.tab) {  // uniform over the workgroup; the offsets were written before the barriers above
        __syncthreads();
        build_tile_lists(offsets, tiles.tab, S, tiles.nt_up, tiles.nt_down, tiles.bm, tiles.L);
    }
}

// Xg[r,:] = X[perm[r] / k, :], one wavefront per row, 16 bytes per lane per step.
__global__ __launch_bounds__(kPermThreads) void gather_rows_kernel(const u32x4* __restrict__ X,
                                                                   const int32_t* __restrict__ perm,
                                                                   u32x4* __restrict__ Xg, int P, int k,
                                                                   int row_vec)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int r = blockIdx.x * kPermWaves + threadIdx.x / kWave;
    if (r >= P) return;
    const int t = perm[r] / k;
    const u32x4* src = X + (size_t)t * row_vec;
    u32x4* dst = Xg + (size_t)r * row_vec;
    for (int i = lane; i < row_vec; i += kWave) dst[i] = src[i];
}

__global__ void validate_kernel(const int32_t* __restrict__ vid, const int32_t* __restrict__ M,
                                int32_t* __restrict__ flag, int T, int V, int E, int S)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    if (i < T) bad = vid[i] < 0 || vid[i] >= V;
    if (i < V * E) bad = bad || M[i] < 0 || M[i] >= S;
    if (bad) atomicOr(flag, 1);
}

__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

int launch_validate(const mmoe_shape& s, const int32_t* vid, const int32_t* M, int32_t* flag, hipStream_t st)
{
    int n = s.T > s.V * s.E ? s.T : s.V * s.E;
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    hipLaunchKernelGGL(validate_kernel, dim3((n + 255) / 256), dim3(256), 0, st, vid, M, flag, s.T, s.V, s.E,
                       s.S);
    return launch_status();
}

int launch_permute(const mmoe_shape& s, const void* X, const int32_t* vid, const int32_t* topk_idx,
                   const int32_t* M, int32_t* slot, int32_t* counts, int32_t* offsets, int32_t* perm,
                   int32_t* inv_perm, void* Xg, int32_t* blk_counts, int32_t* blk_base, int nblk, hipStream_t st,
                   int32_t* tile_tab, bool slot_ready)
{
    const int P = s.T * s.top_k;
    const TileJob tiles = tile_job(s, tile_tab);
    if (nblk == 1)
        hipLaunchKernelGGL(slot_group_small_kernel, dim3(1), dim3(kPermThreads), 0, st, vid, topk_idx, M, slot, counts,
                           offsets, perm, inv_perm, P, s.top_k, s.V, s.E, s.S, tiles);
    else if (slot_ready && nblk <= kOwnHistMaxBlk) {
        hipLaunchKernelGGL(slot_scatter_kernel<kOwnHist>, dim3(nblk + 1), dim3(kPermThreads), 0, st, slot, blk_base,
                           blk_counts, nblk, counts, offsets, perm, inv_perm, P, s.S, tiles);
    } else {
        hipLaunchKernelGGL(slot_hist_kernel, dim3(nblk), dim3(kPermThreads), 0, st, vid, topk_idx, M, slot,
                           blk_counts, P, s.top_k, s.V, s.E, s.S);
        if ((int64_t)nblk * s.S <= kOwnScanMax) {
            hipLaunchKernelGGL(slot_scatter_kernel<kOwnScan>, dim3(nblk + 1), dim3(kPermThreads), 0, st, slot, blk_base,
                               blk_counts, nblk, counts, offsets, perm, inv_perm, P, s.S, tiles);
        } else {
            hipLaunchKernelGGL(slot_scan_kernel, dim3(1), dim3(kPermThreads), 0, st, blk_counts, blk_base, counts,
                               offsets, nblk, s.S, tiles);
            hipLaunchKernelGGL(slot_scatter_kernel<kFromScan>, dim3(nblk), dim3(kPermThreads), 0, st, slot, blk_base,
                               blk_counts, nblk, counts, offsets, perm, inv_perm, P, s.S, TileJob());
        }
    }
    if (!Xg) return launch_status();
    const int row_vec = (int)((size_t)s.d_model * elem_size(s.dtype) / 16);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((P + kPermWaves - 1) / kPermWaves), dim3(kPermThreads), 0, st,
                       (const u32x4*)X, perm, (u32x4*)Xg, P, s.top_k, row_vec);
    return launch_status();
}

}  // namespace mmoe
