// Step F, matrix-core-bound variant: the grouped expert FFN when slots hold many rows
// (prefill-shaped batches) -- Algorithm 2, "expert[iL][iE](act)"; the expert block is
// where the layer's time goes (section 5.1).
//
// Both products are  out[r, n] = sum_k A[r, k] * W[s][n][k]  over the packed pool, bf16
// inputs, fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//
// Tile: 256 token rows x 256 weight rows x 64 k per step, one workgroup of four
// wavefronts per compute unit.  Each wavefront owns all 256 token rows and 64 weight rows
// (for the gated product: 32 rows of W1 and the same 32 rows of W3, so that SiLU(gate)*up
// is lane-local): 8 x 2 accumulator tiles of 32x32, 256 accumulator registers.  Weights are
// the 32-row matrix-core operand and tokens the 32-column one, hence a lane owns, for one
// token, groups of 4 consecutive output features and stores 8 or 16 bytes at a time.
//
// Memory pipeline: the pool is stored as matrix-core fragments, so a wavefront loads its
// weight operands straight from global memory into registers (16 bytes per lane, 1 KB per
// instruction, contiguous), four steps ahead of their use.  Token rows are copied global ->
// LDS without passing registers (global_load_lds, 16 bytes per lane) into a four-stage ring
// of LDS tiles, [row][64 k] bf16 (128 bytes a row) with the 16-byte pieces xor-swizzled by
// (row >> 1) & 7, two steps ahead, and are read back as fragments; one barrier per step.
//
// Ragged groups: row ranges come from the device array `offsets`.  A one-workgroup
// preparation kernel turns them into lists of tiles; the product kernels map their
// workgroup id to (slot, row tile, feature tile) through those lists, so the host never
// waits for the histogram.  Workgroup ids are dealt round-robin to the 8 XCDs by the
// hardware; the id -> tile map gives XCD x the feature tiles nt with nt mod 8 == x, so the
// workgroups resident on one XCD share weight and activation panels in that XCD's L2 and
// every XCD sees the same mix of row tiles.
#include <type_traits>

#include "mmoe_internal.h"
#include "tile_table.h"

namespace mmoe {

// What a product writes: H = act(.) in bf16 (up product), plain fp32 rows of Yg (down product), or,
// for layers with top_k = 1, the layer's output rows: 0 + w[token] * y in bf16 at row token (GateSink).
enum { kTModeReluH = 0, kTModeSwigluH = 1, kTModePlainF32 = 2, kTModeGeluH = 3, kTModeGatedY = 4 };

constexpr int kBN = 256;  // weight rows per tile: four wavefronts of two 32-row blocks (128 with one block each)
constexpr int kBK = 64;
constexpr int kStagesA = 4;    // LDS ring of token tiles

typedef __attribute__((address_space(3))) void* lptr_t;

// silu(g) * u with the hardware exponential and reciprocal (about 1 ulp each; the result is
// rounded to bf16 right after).  A full-precision division here costs more matrix-core idle
// time at the end of every tile than it is worth.
__device__ __forceinline__ float silu_mul_t(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

__global__ __launch_bounds__(256) void tile_table_kernel(const int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ tab, int S, int nt_up, int nt_down,
                                                         int bm, TileLists L, SlotFilter filt)
{
    build_tile_lists(offsets, tab, S, nt_up, nt_down, bm, L, filt);
}

template <int MODE, int BM, int NB>
__global__ __launch_bounds__(256, BM == kBMBig ? 1 : 2) void tiled_kernel(const uint16_t* __restrict__ A,
                                                       const int32_t* __restrict__ perm, int kdiv,
                                                            const int32_t* __restrict__ tab, int hdr, int list_hi,
                                                            int list_lo, const uint16_t* __restrict__ W0,
                                                            const uint16_t* __restrict__ W1,
                                                            void* __restrict__ out, int K, int N, int NT,
                                                            const int32_t* __restrict__ sink_perm,
                                                            const float* __restrict__ sink_w)
{
    constexpr int kTileBytes = BM * kBK * 2;  // one step of the token operand (32 KB for 256 rows)
    __shared__ __attribute__((aligned(1024))) char lds_a[kStagesA * kTileBytes];

    // ---- workgroup id -> tile ------------------------------------------------------------
    // XCD x (= workgroup id mod 8) owns the feature tiles nt with nt mod 8 == x, for every slot
    // and row tile: every XCD gets the same mix of full and partial row tiles, and all row
    // tiles that share a weight panel run on the XCD whose L2 holds it.  One 16-byte entry of
    // the prepared list says which tile this workgroup computes.
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int nt_x = (NT - xcd + kXcds - 1) / kXcds;  // feature tiles owned by this XCD
    const int4* list = reinterpret_cast<const int4*>(tab) + (nt_x == (NT + kXcds - 1) / kXcds ? list_hi : list_lo);
    const int total_m = tab[hdr];
    const int4 ent = list[local];                     // in bounds for every workgroup of the grid
    if (local >= total_m * nt_x) return;              // uniform over the workgroup
    const int s = ent.x;
    const int nt = ent.y * kXcds + xcd;
    const int r0 = ent.z;                             // first row of the tile
    const int cnt = ent.w;                            // rows of the tile that exist (1..256)

    // NB = 32-row weight blocks per wavefront: 2 (256 weight rows per tile), or 1 (128: twice as many
    // tiles for a product that would otherwise leave compute units without work; not for the gated
    // product, whose wavefronts pair a gate block with an up block)
    static_assert(NB == 2 || (NB == 1 && MODE != kTModeSwigluH), "weight blocks per wavefront");
    constexpr int kFeat = MODE == kTModeSwigluH ? kBN / 2 : 128 * NB;  // output features per tile
    const int n0 = nt * kFeat;

    constexpr int kWaves = 4;         // one per SIMD
    constexpr int kThreads = kWaves * 64;
    constexpr int kNJ = BM / 32;      // 32-row token sub-tiles per wavefront (all rows of the tile)
    // 16-k slices between a weight fragment's load and its use: what the registers allow
    constexpr int kBAhead = (BM == kBMBig || NB == 1) ? 16 : 8;
    constexpr int kNP = BM * 8 / kThreads;  // 16-byte pieces of a token tile per thread
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps bases in scalar registers
    const int lr = lane & 31;
    const int wn = wave;              // which 64 weight rows of the tile

    // ---- token operand: global -> LDS ------------------------------------------------------------
    // Piece id = i*kThreads + tid (i < kNP) of a [256 rows][8 pieces of 16 bytes] tile: 8
    // consecutive threads read one row's 128 contiguous bytes.  Rows past the end of the group
    // re-read its last row (they are multiplied but never stored).
    // Grouped row r is row r of A, or, when a permutation is given, row perm[r] / kdiv of A (the
    // gather of the token rows folded into this product's loads).
    const char* a_base = reinterpret_cast<const char*>(A);
    uint32_t a_row[kNP];  // byte offset of the row each piece comes from
#pragma unroll
    for (int i = 0; i < kNP; ++i) {
        const int row = i * (kThreads / 8) + (tid >> 3);
        const int r = r0 + min(row, cnt - 1);
        a_row[i] = (uint32_t)(perm ? perm[r] / kdiv : r) * (uint32_t)K * 2u;
    }
    // Copy instruction i of a wavefront writes its 64 pieces to 1 KB of consecutive LDS addresses
    // (M0 + 16*lane), 8 rows of 128 bytes, so the swizzle is applied on the global side: the lane
    // that fills physical piece q of a row fetches logical piece q ^ ((row >> 1) & 7).
    uint32_t a_goff[kNP];
#pragma unroll
    for (int i = 0; i < kNP; ++i) a_goff[i] = a_row[i] + (((tid & 7) ^ ((tid >> 4) & 7)) << 4);
    // The copies are written in assembly so that the compiler's wait-count bookkeeping does not
    // see them (it would drain every load in flight before each LDS read); the waits that order
    // them are written out next to the barriers.  M0 is only used here.
    auto copy_a = [&](int stage, int kt) {
        const char* ab = a_base + (size_t)kt * (kBK * 2);
#pragma unroll
        for (int i = 0; i < kNP; ++i) {
            const uint32_t dst =
                (uint32_t)(uintptr_t)(lptr_t)(lds_a + stage * kTileBytes + (i * kThreads + wave * 64) * 16);
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :
                         : "v"(a_goff[i]), "s"(ab), "s"(dst)
                         : "m0", "memory");
        }
    };
    // ---- weight operand: fragment-packed pool -> registers ------------------------------------------
    // A wavefront owns weight rows [64 wn, 64 wn + 64) of the tile, two 32-row blocks; for the
    // gated product they are block (n0 + 32 wn)/32 of W1 (gate) and the same block of W3 (up), so
    // that a lane holds matching gate and up values.  Fragment ks of a block is 1 KB at ks*1024.
    const size_t frag_bytes_per_block = (size_t)(K / 16) * 1024;
    const char* wb[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const uint16_t* w = (MODE == kTModeSwigluH && i == 1) ? W1 : W0;
        const int nb = MODE == kTModeSwigluH ? (n0 + wn * 32) / 32 : (n0 + wn * (32 * NB) + i * 32) / 32;
        wb[i] = reinterpret_cast<const char*>(w) + ((size_t)s * (N / 32) + nb) * frag_bytes_per_block + lane * 16;
    }

    // ---- token fragments from LDS ------------------------------------------------------------------
    // Slice kk (16 k) of a step: lane (row lane%32, half h = lane/32) reads logical piece 4h + kk,
    // the 8 k values that the packed weight fragment pairs with it.
    int frag_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        frag_off[kk] = lr * 128 + ((((lane >> 5) * 4 + kk) ^ ((lr >> 1) & 7)) << 4);

    // Gated output rows (GateSink): the coefficient of this lane's token column of every sub-tile, and
    // the output row (token) of every row this lane stores in the epilogue.  Two dependent loads each;
    // short-lived 128-row tiles start them here, behind the main loop's own loads, tall tiles (no
    // registers to spare in the main loop, and an epilogue that is a hundredth of the tile) when
    // the main loop is over.
    constexpr int kSinkLpr = 4;   // lanes per stored row of 32 bf16 features (the epilogue's kLpr)
    constexpr int kSinkRpi = 16;  // rows per store instruction (its kRpi)
    constexpr bool kEarlySink = BM == kBMSmall;
    float gate_w[kNJ];
    int sink_row[kNJ][32 / kSinkRpi];
    auto fetch_sink = [&]() {
#pragma unroll
        for (int j = 0; j < kNJ; ++j) {
            gate_w[j] = sink_w[sink_perm[r0 + min(j * 32 + lr, cnt - 1)]];
#pragma unroll
            for (int it = 0; it < 32 / kSinkRpi; ++it)
                sink_row[j][it] = sink_perm[r0 + min(j * 32 + it * kSinkRpi + lane / kSinkLpr, cnt - 1)];
        }
    };
    if (MODE == kTModeGatedY && kEarlySink) fetch_sink();

    f32x16 acc[kNJ][NB];  // [token sub-tile][weight block]
#pragma unroll
    for (int j = 0; j < kNJ; ++j)
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.0f;

    // Main loop, instantiated for NJ = number of this wavefront's 32-row token sub-tiles that
    // hold rows (all 8 for every tile but the last one of a slot).
    //
    // Pipeline (k step t = 64 k = four 16-k slices; step t's tokens live in LDS stage t mod 4):
    //   weights   slice g is loaded straight into registers kBAhead slices (four steps) before
    //             use; these are ordinary loads and the compiler inserts their waits;
    //   tokens    the copies of step t+4 are issued right after the barrier of step t, into the
    //             stage that step t has just finished with, and must have landed by the barrier
    //             of step t+2; token fragments roll through one set of registers: as soon as the
    //             two matrix instructions that use fragment j have been issued, fragment j of
    //             the next slice is fetched into it;
    //   barrier   one per step, in the middle of its last slice: by then every wavefront's
    //             reads of the step's stage have returned (only the first NJ/2 fetches of the
    //             next stage may be in flight), so nobody waits for LDS.
    // The loop is unrolled by kBAhead/4 steps so that the ring of weight registers is indexed
    // statically.
    //
    // What orders the copies.  The compiler does not see them, so the wait that makes them
    // land is written out next to every barrier: s_waitcnt vmcnt(N) returns when at most N of
    // this wavefront's vector-memory instructions are outstanding, and they complete in issue
    // order.  Rule at every such wait: only the most recent group of kNP copies may still be in
    // flight, every older one has landed.  That holds if at least N vector-memory instructions
    // were issued after the last copy of the second most recent group: the kNP copies of the most
    // recent group plus weight-fragment loads, whose place in the instruction stream the compiler
    // chooses.  Their count is therefore not taken on trust: tests/test_tiled_wait_counts.py
    // reads the compiler's assembly output for this file and checks the rule at every written-out
    // wait of every instantiation, along every path that reaches it.
    // What orders the LDS reads.  Before a stage is handed back to the copies, the fragments
    // of that stage that are still to be used are made operands of an (empty) asm statement in
    // front of the barrier, so the compiler itself waits for exactly those reads and for nothing
    // younger (the NH fetches of the next stage stay in flight across the barrier).
    const int nkt = K / kBK;         // even: K is a multiple of 256
    const int last = nkt - 1;
    const int last_slice = K / 16 - 1;
    auto run = [&](auto njc) {
        constexpr int NJ = decltype(njc)::value;
        constexpr int NH = NJ / 2;  // fetches of the next stage issued before the barrier
        struct BFrags {
            u32x4 b[NB];
        };
        bf16x8 fa[NJ];
        auto frag_ptr = [&](int stage, int kk) { return lds_a + stage * kTileBytes + frag_off[kk]; };
        auto load_bf = [&](BFrags& fr, int g) {
            const size_t o = (size_t)min(g, last_slice) * 1024;  // past the end: a harmless reload
#pragma unroll
            for (int i = 0; i < NB; ++i) fr.b[i] = *reinterpret_cast<const u32x4*>(wb[i] + o);
        };
        // one token sub-tile against both weight blocks, then its fragment of the next slice
        auto mma_roll = [&](int j, const BFrags& fb, const char* next) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb.b[i]), fa[j],
                                                                    acc[j][i], 0, 0, 0);
            fa[j] = *reinterpret_cast<const bf16x8*>(next + j * 32 * 128);
        };
        // a slice whose successor lies in the same LDS stage
        auto slice = [&](BFrags& fb, const char* next, int g_reload) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) mma_roll(j, fb, next);
            load_bf(fb, g_reload);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x020, NB, 0);
        };

        BFrags bq[kBAhead];
        // prologue: copies of steps 0..3 into the four stages, then the first weight fragments;
        // the wait leaves at most the copies of step 3 in flight
        copy_a(0, 0);
        copy_a(1, min(1, last));
        copy_a(2, min(2, last));
        copy_a(3, min(3, last));
#pragma unroll
        for (int g = 0; g < kBAhead; ++g) load_bf(bq[g], g);
        static_assert(kNP + NB * kBAhead <= 63, "vmcnt is a 6-bit counter");
        __builtin_amdgcn_sched_barrier(0);  // the weight loads are issued before the wait, not after it
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kNP + NB * kBAhead) : "memory");
        {
            const char* p0 = frag_ptr(0, 0);
#pragma unroll
            for (int j = 0; j < NJ; ++j) fa[j] = *reinterpret_cast<const bf16x8*>(p0 + j * 32 * 128);
        }

        int st = 0;  // LDS stage of step kt
        constexpr int kUnroll = kBAhead / 4;  // steps per trip: the weight ring is indexed statically
        int kt = 0;
        do {  // at least one trip (K >= 256): the prologue's loads have nowhere to sink to
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int t = kt + u;
                const int stn = st == kStagesA - 1 ? 0 : st + 1;
                const int g = 4 * t;
                slice(bq[(4 * u + 0) % kBAhead], frag_ptr(st, 1), g + kBAhead);
                slice(bq[(4 * u + 1) % kBAhead], frag_ptr(st, 2), g + kBAhead + 1);
                slice(bq[(4 * u + 2) % kBAhead], frag_ptr(st, 3), g + kBAhead + 2);
                // last slice of the step: its fragments are in flight or in registers
                {
                    BFrags& fb = bq[(4 * u + 3) % kBAhead];
                    const char* next = frag_ptr(stn, 0);
#pragma unroll
                    for (int j = 0; j < NH; ++j) mma_roll(j, fb, next);
#pragma unroll
                    for (int j = 0; j < NH; ++j) {
                        __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    // Stage st goes back to the copies after this barrier.  Its fragments that are still
                    // to be used (sub-tiles NH.. of this slice) become operands here, so the compiler
                    // waits for those reads; every other read of the stage has been consumed by a matrix
                    // instruction above.  The NH fetches just issued read the next stage and stay in flight.
#pragma unroll
                    for (int j = NH; j < NJ; ++j) asm volatile("" ::"v"(fa[j]));
                    // This wavefront's copies of step t+2 were issued two steps ago, after the barrier of
                    // step t-2 (for t < 2: in the prologue); since then it has issued the kNP copies of
                    // step t+3 and, in the order written here, 8*NB weight-fragment loads (NB in the rest
                    // of that slice, 4*NB in step t-1, 3*NB in this step): a wait that leaves at most
                    // kWaitN = min(16, kNP + 8*NB - 4) instructions outstanding leaves the copies of step
                    // t+2 landed, and after the barrier every wavefront may read that step, whose first
                    // fragments are fetched before the next barrier.
                    constexpr int kWaitN = kNP + 8 * NB - 4 < 16 ? kNP + 8 * NB - 4 : 16;
                    static_assert(kWaitN >= kNP, "the copies of step t+3 stay in flight");
                    static_assert(kNP + NB * kBAhead + 3 * NB >= kWaitN, "first step: after the copies of step 2");
                    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kWaitN) : "memory");
                    copy_a(st, min(t + 4, last));  // tokens of step t+4; past the end: a harmless reload
#pragma unroll
                    for (int j = NH; j < NJ; ++j) mma_roll(j, fb, next);
                    load_bf(fb, g + kBAhead + 3);
#pragma unroll
                    for (int q = 0; q < NJ - NH; ++q) {
                        __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x020, NB, 0);
                }
                st = stn;
            }
            kt += kUnroll;
        } while (kt < nkt);
        // no copy may still be on its way into LDS when the epilogue reuses it or the workgroup ends
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    switch (min(kNJ, (cnt + 31) / 32)) {  // uniform over the workgroup
        case 8: if constexpr (kNJ >= 8) run(std::integral_constant<int, 8>{}); break;
        case 7: if constexpr (kNJ >= 8) run(std::integral_constant<int, 7>{}); break;
        case 6: if constexpr (kNJ >= 8) run(std::integral_constant<int, 6>{}); break;
        case 5: if constexpr (kNJ >= 8) run(std::integral_constant<int, 5>{}); break;
        case 4: run(std::integral_constant<int, 4>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        default: run(std::integral_constant<int, 1>{}); break;
    }

    // ---- epilogue -------------------------------------------------------------------------------
    // Accumulator element e of lane l is weight row 8*(e/4) + 4*(l/32) + e%4 of token column
    // l%32: a lane holds scattered 4-feature groups of one token.  Each wavefront therefore
    // passes its results through a private LDS patch, 32 tokens x 32 features at a time, and
    // reads them back row by row, so that every global store instruction writes whole
    // contiguous row segments (128 bytes for fp32 output, 64 for bf16).
    constexpr int kEsz = MODE == kTModePlainF32 ? 4 : 2;
    constexpr int kRowB = 32 * kEsz;                  // bytes of one staged row
    constexpr int kPitch = kRowB + 16;                // padded: conflict-free 16-byte column writes
    constexpr int kLpr = kRowB / 16;                  // lanes that read one row back
    constexpr int kRpi = 64 / kLpr;                   // rows per read-back instruction
    static_assert(MODE != kTModeGatedY || (kLpr == kSinkLpr && kRpi == kSinkRpi), "the sink rows follow the stores");
    constexpr int kChunks = MODE == kTModeSwigluH ? 1 : NB;       // 32-feature chunks this wavefront stores
    const int wfeat = MODE == kTModeSwigluH ? wn * 32 : wn * (32 * NB);
    // the patches reuse the token ring: every wavefront has left the main loop
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    char* ebuf = lds_a + wave * (32 * (32 * 4 + 16));
    char* const obase = reinterpret_cast<char*>(out) + ((size_t)r0 * N + n0 + wfeat) * kEsz +
                        (size_t)(lane / kLpr) * N * kEsz + (lane % kLpr) * 16;
    if (MODE == kTModeGatedY && !kEarlySink) fetch_sink();
    char* const ybase = reinterpret_cast<char*>(out) + (size_t)(n0 + wfeat) * kEsz + (lane % kLpr) * 16;
    // o[4q + e]: the 16 finished values of this lane for token sub-tile j, feature chunk c
    auto emit = [&](int j, int c, const float (&o)[16]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            char* at = ebuf + lr * kPitch + (8 * q + 4 * (lane >> 5)) * kEsz;
            if (kEsz == 4) {
                *reinterpret_cast<f32x4*>(at) = f32x4{o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]};
            } else {
                u32x2 pk;
                pk[0] = (uint32_t)f32_to_bf16_bits(o[4 * q]) | ((uint32_t)f32_to_bf16_bits(o[4 * q + 1]) << 16);
                pk[1] = (uint32_t)f32_to_bf16_bits(o[4 * q + 2]) | ((uint32_t)f32_to_bf16_bits(o[4 * q + 3]) << 16);
                *reinterpret_cast<u32x2*>(at) = pk;
            }
        }
#pragma unroll
        for (int it = 0; it < 32 / kRpi; ++it) {
            const int row = it * kRpi + lane / kLpr;
            const u32x4 v = *reinterpret_cast<const u32x4*>(ebuf + row * kPitch + (lane % kLpr) * 16);
            if (j * 32 + row < cnt) {
                char* dst = MODE == kTModeGatedY ? ybase + ((size_t)sink_row[j][it % (32 / kSinkRpi)] * N + c * 32) * kEsz
                                                 : obase + ((size_t)(j * 32 + it * kRpi) * N + c * 32) * kEsz;
                *reinterpret_cast<u32x4*>(dst) = v;
            }
        }
    };
#pragma unroll
    for (int j = 0; j < kNJ; ++j) {
        if (j * 32 >= cnt) break;  // uniform over the workgroup
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            float o[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                if (MODE == kTModeSwigluH) o[e] = silu_mul_t(acc[j][0][e], acc[j][NB - 1][e]);
                else if (MODE == kTModeReluH) o[e] = fmaxf(acc[j][c][e], 0.0f);
                else if (MODE == kTModeGeluH) o[e] = 0.5f * acc[j][c][e] * (1.0f + erff(acc[j][c][e] * 0.70710678118654752440f));
                else if (MODE == kTModeGatedY) o[e] = __builtin_fmaf(gate_w[j], acc[j][c][e], 0.0f);
                else o[e] = acc[j][c][e];
            }
            emit(j, c, o);
        }
    }
}

// Weight blocks per wavefront of a product with N output features: 2, or 1 (tiles of 128 weight
// rows, twice as many of them) when 128-row token tiles are in use and the product would otherwise
// have fewer tiles than the chip holds workgroups at a time.  Shape only.
constexpr int kNb1Room = 512;  // two workgroups of 128-row tiles on each of 256 compute units
static int planned_nb(const mmoe_shape& s, int bm, int N, bool gated)
{
    if (gated || bm != kBMSmall) return 2;
    const int64_t P = (int64_t)s.T * s.top_k;
    return ((P + bm - 1) / bm) * (N / kBN) < kNb1Room ? 1 : 2;
}

static void tiled_nts(const mmoe_shape& s, int bm, int& nt_up, int& nt_down, int& nb_up, int& nb_down)
{
    nb_up = planned_nb(s, bm, s.d_ff, s.act == MMOE_SWIGLU);
    nb_down = planned_nb(s, bm, s.d_model, false);
    nt_up = s.act == MMOE_SWIGLU ? s.d_ff / (kBN / 2) : s.d_ff / (128 * nb_up);
    nt_down = s.d_model / (128 * nb_down);
}

// Tile height: 128 rows (two workgroups per compute unit, so one's prologue and epilogue hide
// behind the other's main loop) when a tile is short-lived -- a short reduction in the up
// product, or slots with few rows -- and 256 rows (deeper weight prefetch, half the weight
// traffic per row) otherwise.  The host knows P and S, not the counts.  Measured with each
// height forced: on the Switch shape (d = 768) 128 rows win at every batch size up to 16384
// tokens; on the Mixtral shape (d = 4096) they win up to 59 rows per slot (384 tokens) and
// lose from 79 rows per slot (512 tokens) on.
int planned_tile_rows(const mmoe_shape& s)
{
    if (s.tile_rows) return s.tile_rows;  // forced for this call (checked by check_shape: 128 or 256)
    const int64_t P = (int64_t)s.T * s.top_k;
    return (s.d_model <= 1024 || P < (int64_t)64 * s.S) ? kBMSmall : kBMBig;
}

// Most sub-tiles of a row tile: a full tile.  (Shorter tiles for products with few tiles were
// measured on the Switch shape and lose: every tile streams its whole weight panel, and a step of
// a short tile is over before the copies issued two steps earlier have landed.)
static int planned_upt(const mmoe_shape&, int bm, int) { return bm / 32; }

// Everything the launches of one shape share: tile height, weight blocks per wavefront and feature
// tiles of both products, and the tile lists' layout.
struct TiledPlan {
    int bm, nt_up, nt_down, nb_up, nb_down;
    TileLists L;
};

static TiledPlan tiled_plan(const mmoe_shape& s)
{
    TiledPlan p;
    p.bm = planned_tile_rows(s);
    tiled_nts(s, p.bm, p.nt_up, p.nt_down, p.nb_up, p.nb_down);
    p.L = tile_lists(s.T * s.top_k, s.S, p.nt_up, p.nt_down, planned_upt(s, p.bm, p.nt_up),
                     planned_upt(s, p.bm, p.nt_down));
    return p;
}

size_t tiled_table_bytes(const mmoe_shape& s)
{
    // the most entries any plan of this shape can have: the shortest tiles, the narrowest feature tiles
    const int nt_up = s.act == MMOE_SWIGLU ? s.d_ff / (kBN / 2) : s.d_ff / 128;
    return align256(tile_lists(s.T * s.top_k, s.S, nt_up, s.d_model / 128, 1, 1).bytes);
}

template <int MODE, int BM, int NB>
static void launch_product(const TiledPlan& p, int prod, const void* A, const int32_t* perm, int kdiv, const int32_t* tab,
                           const void* W0, const void* W1, void* out, int K, int N, hipStream_t st,
                           GateSink sink = GateSink())
{
    hipLaunchKernelGGL((tiled_kernel<MODE, BM, NB>), dim3(p.L.cap[prod] * kXcds), dim3(256), 0, st, (const uint16_t*)A,
                       perm, kdiv, tab, p.L.hdr + prod, p.L.list[prod][0], p.L.list[prod][1], (const uint16_t*)W0,
                       (const uint16_t*)W1, out, K, N, prod == 0 ? p.nt_up : p.nt_down, sink.perm, sink.w);
}

// one weight block per wavefront exists for 128-row tiles only (planned_nb)
template <int MODE>
static void launch_plain_product(const TiledPlan& p, int prod, const void* A, const int32_t* perm, int kdiv,
                                 const int32_t* tab, const void* W0, void* out, int K, int N, hipStream_t st,
                                 GateSink sink = GateSink())
{
    const int nb = prod == 0 ? p.nb_up : p.nb_down;
    if (p.bm == kBMBig) launch_product<MODE, kBMBig, 2>(p, prod, A, perm, kdiv, tab, W0, nullptr, out, K, N, st, sink);
    else if (nb == 2) launch_product<MODE, kBMSmall, 2>(p, prod, A, perm, kdiv, tab, W0, nullptr, out, K, N, st, sink);
    else launch_product<MODE, kBMSmall, 1>(p, prod, A, perm, kdiv, tab, W0, nullptr, out, K, N, st, sink);
}

TileJob tile_job(const mmoe_shape& s, int32_t* tab)
{
    const TiledPlan p = tiled_plan(s);
    TileJob j;
    j.tab = tab;
    j.nt_up = p.nt_up;
    j.nt_down = p.nt_down;
    j.bm = p.bm;
    j.L = p.L;
    return j;
}

int launch_ffn_tiled(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                     const void* W1p, const void* W3p, const void* W2p, void* H, float* Yg, int32_t* tab,
                     hipStream_t st, hipEvent_t mid, bool tab_ready, SlotFilter filt, GateSink sink)
{
    if (s.dtype != MMOE_BF16) return MMOE_ERR_DTYPE;
    const int P = s.T * s.top_k, d = s.d_model, f = s.d_ff;
    if ((int64_t)P * (d > f ? d : f) >= ((int64_t)1 << 31)) return MMOE_ERR_LIMIT;  // 32-bit byte offsets inside a panel
    const TiledPlan p = tiled_plan(s);
    if (!tab_ready)
        hipLaunchKernelGGL(tile_table_kernel, dim3(1), dim3(256), 0, st, offsets, tab, s.S, p.nt_up, p.nt_down, p.bm, p.L,
                           filt);
    if (s.act == MMOE_SWIGLU) {
        if (p.bm == kBMBig)
            launch_product<kTModeSwigluH, kBMBig, 2>(p, 0, rows, perm, s.top_k, tab, W1p, W3p, H, d, f, st);
        else
            launch_product<kTModeSwigluH, kBMSmall, 2>(p, 0, rows, perm, s.top_k, tab, W1p, W3p, H, d, f, st);
    } else if (s.act == MMOE_GELU) {
        launch_plain_product<kTModeGeluH>(p, 0, rows, perm, s.top_k, tab, W1p, H, d, f, st);
    } else {
        launch_plain_product<kTModeReluH>(p, 0, rows, perm, s.top_k, tab, W1p, H, d, f, st);
    }
    if (mid && hipEventRecord(mid, st) != hipSuccess) return MMOE_ERR_LAUNCH;
    if (sink.w) {
        if (s.top_k != 1 || !sink.perm || !sink.Y) return MMOE_ERR_DIM;
        launch_plain_product<kTModeGatedY>(p, 1, H, nullptr, 1, tab, W2p, sink.Y, f, d, st, sink);
    } else {
        launch_plain_product<kTModePlainF32>(p, 1, H, nullptr, 1, tab, W2p, Yg, f, d, st);
    }
    return launch_status();
}

}  // namespace mmoe
