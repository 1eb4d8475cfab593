// Tile lists of the matrix-core expert kernels: layout, sizes, and the device code that writes
// them from the device-side `offsets` (run by one workgroup of 256 threads: either the kernel
// that finishes the grouping, or a kernel of its own when the caller brings the offsets).
#pragma once

#include "mmoe_internal.h"

namespace mmoe {

constexpr int kBMBig = 256;    // token rows per tile: large batches (one workgroup per compute unit)
constexpr int kBMSmall = 128;  // token rows per tile: batches with few tiles (two workgroups per compute unit)
constexpr int kXcds = 8;
constexpr int kNtGroup = 4;  // least number of feature tiles whose workgroups start back to back on the same token panel

// Tile lists, written by one workgroup from the device-side `offsets`.
//
// Row tiles.  A slot with c rows is u = ceil(c / 32) sub-tiles of 32 rows.  It is cut into
// mt = max(ceil(u / upt), ceil(u / h)) tiles whose heights differ by at most one sub-tile (upt = most
// sub-tiles of a tile, given per product by the host: a full tile's 8 or 4; h <= upt = the target height
// that the builder chooses per product from the counts, see build_tile_lists): the first u mod mt
// tiles have floor(u / mt) + 1 sub-tiles, the others floor(u / mt).  No slot has a short last tile (a tile of one sub-tile streams its weight panel
// for an eighth of the arithmetic), and no matrix instruction is spent on padding beyond the last
// partial sub-tile.
//
// Order.  tab[0], tab[1] = number of row tiles of the up and of the down product; four lists of int4 entries {slot, feature tile within
// the XCD, first row, rows}, one per (product, feature tiles per XCD): a product with NT feature
// tiles gives XCD x the tiles nt with nt mod 8 == x, that is ceil or floor of NT/8 of them; list
// entry `local` is the tile that the workgroup with id 8*local + x computes.  Entries are listed
// by (slot, group of feature tiles, row tile, feature tile within the group): workgroups start
// in id order, so the ones that share a token panel and the ones that share a weight panel run
// close enough in time to find the panel in L2.  The group is sized so that the workgroups
// resident on an XCD at one time form a block of row tiles x feature tiles that is as square as
// the slot allows (8 x 4 for a slot of 8 row tiles, 4 x 8 for one of 4).
// Target heights of a row tile that the table builder may choose from, in quarters of a 32-row
// sub-tile: from a full tile (4 upt) down to five eighths of one.
__host__ __device__ inline int min_height_q(int upt) { return (5 * upt + 1) / 2; }
constexpr int kMaxHeightCands = 16;

struct TileLists {
    int hdr;        // int32 index of tab[0]
    int list[2][2]; // [product: up, down][0: ceil(NT/8) per XCD, 1: floor] -> int4 index into tab
    int cap[2];     // entries reserved per list of each product
    int upt[2];     // most 32-row sub-tiles of a row tile, per product
    int rows_cap[2]; // most row tiles of each product
    size_t bytes;
};

inline TileLists tile_lists(int P, int S, int nt_up, int nt_down, int upt_up, int upt_down)
{
    TileLists L;
    L.hdr = 0;
    L.upt[0] = upt_up;
    L.upt[1] = upt_down;
    // Row tiles the lists have room for: an eighth more than full tiles can need, which is
    // sum_s ceil(ceil(c_s / 32) / upt) <= P / (32 upt) + S.  The grid of a product is sized by this bound
    // (the host does not know the counts), and a workgroup without a tile still waits for a compute unit
    // before it can leave, so the room for lower target heights is kept small.
    auto most_tiles = [&](int upt) { const int full = (P + 32 * upt - 1) / (32 * upt) + S; return full + (full + 7) / 8; };
    L.rows_cap[0] = most_tiles(upt_up);
    L.rows_cap[1] = most_tiles(upt_down);
    L.cap[0] = L.rows_cap[0] * ((nt_up + kXcds - 1) / kXcds);
    L.cap[1] = L.rows_cap[1] * ((nt_down + kXcds - 1) / kXcds);
    int at = 16;  // int4 units; the header takes the first 256 bytes
    for (int p = 0; p < 2; ++p)
        for (int c = 0; c < 2; ++c) {
            L.list[p][c] = at;
            at += L.cap[p];
        }
    L.bytes = (size_t)at * 16;
    return L;
}

// One workgroup of 256 threads; every thread of it must call.  `offsets` must be visible to the
// whole workgroup (written before a workgroup barrier, or by an earlier kernel).
// Slots that `filt` skips get no tiles.
__device__ __forceinline__ void build_tile_lists(const int32_t* offsets, int32_t* __restrict__ tab, int S, int nt_up,
                                                 int nt_down, int bm, TileLists L, SlotFilter filt = SlotFilter())
{
    __shared__ int cnt_s[kMaxS];       // rows of each slot
    __shared__ int off_s[kMaxS];       // first row of each slot
    __shared__ int base[kMaxS + 1];    // row tiles of the slots before each slot
    __shared__ int part[256];
    __shared__ int cand[kMaxHeightCands];  // row tiles of the whole batch at every candidate height
    __shared__ int chosen_hq;
    const int tid = threadIdx.x;
    const int conc = bm == kBMBig ? 32 : 64;   // workgroups resident on one XCD
    for (int s = tid; s < S; s += 256) {
        const int o = offsets[s];
        off_s[s] = o;
        cnt_s[s] = filt.skips(s) ? 0 : offsets[s + 1] - o;
    }
    __syncthreads();
    int4* lists = reinterpret_cast<int4*>(tab);
    for (int p = 0; p < 2; ++p) {
        const int NT = p == 0 ? nt_up : nt_down;
        const int upt = L.upt[p];
        // Target height.  A slot of u sub-tiles is cut into max(ceil(u / upt), ceil(u / h)) tiles, h the
        // target height, the same for all slots.  h is chosen here, from the counts, so that the product's
        // tiles fill whole rounds of the chip: with `conc` workgroups resident per XCD a product of M row
        // tiles takes about ceil(M NT / (8 conc)) rounds of one tile each, a tile costing a fixed part
        // (half a sub-tile's worth of time: prologue and epilogue) plus its height.  Lower targets also
        // bring the slots' tile heights closer together.  The cut decides where tiles begin, not what a
        // row's result is.
        const int hq_hi = 4 * upt, hq_lo = min_height_q(upt), ncand = hq_hi - hq_lo + 1;  // <= kMaxHeightCands
        auto tiles_at = [&](int u, int hq) { return max((u + upt - 1) / upt, (4 * u + hq - 1) / hq); };
        __syncthreads();  // the lists of the product before have been written: cand is free
        if (tid < kMaxHeightCands) cand[tid] = 0;
        if (tid == 0) chosen_hq = 0;
        __syncthreads();
        {   // thread = (candidate c, one of 16 groups of slots): integer sums, so their order does not matter
            const int c = tid % kMaxHeightCands;
            int tiles = 0, units = 0;
            for (int s = tid / kMaxHeightCands; s < S; s += 256 / kMaxHeightCands) {
                const int u = (cnt_s[s] + 31) >> 5;
                units += u;
                if (c < ncand) tiles += tiles_at(u, hq_hi - c);
            }
            if (tiles) atomicAdd(&cand[c], tiles);
            if (c == 0 && units) atomicAdd(&chosen_hq, units);  // sub-tiles of the whole batch, for now
        }
        __syncthreads();
        if (tid == 0) {
            const int U = chosen_hq;
            int best = 0;
            float best_cost = 0.0f;
            for (int c = 0; c < ncand; ++c) {
                const int M = cand[c];
                if (M == 0 || M > L.rows_cap[p]) break;  // no rows at all, or more tiles than the lists hold
                const int rounds = (M * NT + kXcds * conc - 1) / (kXcds * conc);
                const float cost = (float)rounds * (0.5f + (float)U / (float)M);
                if (c == 0 || cost < best_cost) {
                    best = c;
                    best_cost = cost;
                }
            }
            chosen_hq = hq_hi - best;
        }
        __syncthreads();
        const int hq = chosen_hq;
        // exclusive prefix sum of the row tiles per slot: a run of slots per thread, then a scan of the runs
        auto tiles_of = [&](int s) { return tiles_at((cnt_s[s] + 31) >> 5, hq); };
        const int chunk = (S + 255) / 256;
        const int s_lo = min(tid * chunk, S), s_hi = min(s_lo + chunk, S);
        int mine = 0;
        for (int s = s_lo; s < s_hi; ++s) mine += tiles_of(s);
        __syncthreads();  // the lists of the product before have been written: base and part are free
        part[tid] = mine;
        __syncthreads();
        if (tid < kWave) {  // inclusive scan of the 256 runs by the first wavefront: four per lane, then across the lanes
            int v[4], sum = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sum += part[4 * tid + i];
                v[i] = sum;
            }
            int incl = sum;
#pragma unroll
            for (int dlt = 1; dlt < kWave; dlt <<= 1) {
                const int o = __shfl_up(incl, dlt, kWave);
                if (tid >= dlt) incl += o;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) part[4 * tid + i] = incl - sum + v[i];
        }
        __syncthreads();
        int run = part[tid] - mine;
        for (int s = s_lo; s < s_hi; ++s) {
            base[s] = run;
            run += tiles_of(s);
        }
        const int total_m = part[255];
        if (tid == 0) {
            base[S] = total_m;
            tab[L.hdr + p] = total_m;
        }
        __syncthreads();
        for (int c = 0; c < 2; ++c) {
            if (c == 1 && NT % kXcds == 0) break;  // every XCD has the same number of feature tiles: one list
            const int nt_x = c == 0 ? (NT + kXcds - 1) / kXcds : NT / kXcds;
            const int n = total_m * nt_x;
            for (int e = tid; e < n; e += 256) {
                int lo = 0, hi = S;  // largest s with base[s]*nt_x <= e (empty slots have equal bounds)
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (base[mid] * nt_x <= e) lo = mid; else hi = mid;
                }
                const int s = lo, mt = base[s + 1] - base[s];
                const int rem = e - base[s] * nt_x;
                // groups of g feature tiles; inside a group the feature tile runs fastest
                const int g = min(nt_x, max(kNtGroup, conc / mt));
                const int grp = rem / (g * mt), within = rem - grp * (g * mt);
                const int g_sz = min(g, nt_x - grp * g);
                const int i = within / g_sz, ntl = grp * g + within - i * g_sz;
                // row tile i of the slot: the first `extra` tiles are one sub-tile taller
                const int u = (cnt_s[s] + 31) >> 5, h = u / mt, extra = u - h * mt;
                const int row0 = 32 * (i * h + min(i, extra));
                const int rows = 32 * (h + (i < extra ? 1 : 0));
                lists[L.list[p][c] + e] = make_int4(s, ntl, off_s[s] + row0, min(rows, cnt_s[s] - row0));
            }
        }
    }
}


// What the grouping kernels need to write the lists themselves (null `tab`: they do not).
struct TileJob {
    int32_t* tab;
    int nt_up, nt_down, bm;
    TileLists L;
};

// The job for this shape (host side; defined beside the matrix-core kernels).  Null `tab`: no job.
TileJob tile_job(const mmoe_shape& s, int32_t* tab);

}  // namespace mmoe
