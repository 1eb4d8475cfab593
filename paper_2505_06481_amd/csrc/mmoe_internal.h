// Internal declarations shared by the HIP translation units of libmmoe (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mmoe.h"

namespace mmoe {

constexpr int kWave = 64;
constexpr int kMaxTopK = 8;
constexpr int kMaxE = 256;
constexpr int kMaxS = 1024;
constexpr int kPermChunk = 2048;  // pairs per workgroup in the grouping kernels
constexpr int kLoaderMaxV = 8;       // variants the expert-map builder compares in one pass
constexpr int kLoaderMaxLoc = 4096;  // expert locations (layers x experts) it ranks

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even (hardware conversion on gfx950)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x)
{
    bf16_t h = (bf16_t)x;
    return __builtin_bit_cast(uint16_t, h);
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline size_t elem_size(int dtype) { return dtype == MMOE_BF16 ? 2 : 4; }

// Which slots one launch of the expert stage works on: all of them (`flag` null), or those whose
// flag equals `want` (a launch for the resident slots, a later one for the slots just fetched).
struct SlotFilter {
    const uint8_t* flag = nullptr;  // DEVICE [S]
    int want = 0;
    __host__ __device__ bool skips(int s) const { return flag && flag[s] != want; }
};

// Where the rows of the down product go.  Default (`w` null): row r of Yg, fp32.  With `w` (layers
// with top_k = 1, whose combination is a single product per element): row token(r) of Y in the storage
// type, holding 0 + w[token] * y -- the value the combination kernel computes for one pick -- so that
// kernel and the round trip of Yg through memory are not needed.
struct GateSink {
    void* Y = nullptr;              // DEVICE [T, d_model] dtype
    const float* w = nullptr;       // DEVICE topk_w [T]
    const int32_t* perm = nullptr;  // grouped row -> pair id (= token when top_k = 1); null: rows are indexed by pair id
};

// Sub-buffers of the caller's workspace used by mmoe_layer_forward (byte offsets).
struct WsLayout {
    size_t topk_idx, topk_w, slot, counts, offsets, perm, inv_perm, blk_counts, blk_base, tile_tab, resident, H, Yg,
        total;
    int nblk;
};
WsLayout ws_layout(const mmoe_shape& s);

int check_shape(const mmoe_shape* s);

// true when the expert stage uses the weight-streaming kernels (few rows per slot)
bool use_skinny(const mmoe_shape& s);

// Kernel launchers (one per translation unit).  All return an mmoe_status.
// `M` and `slot` both given: the router also writes slot[p] = M[vid[t]][topk_idx[p]] (step M).
int launch_route(const mmoe_shape& s, const void* X, const int32_t* vid, const void* Wr, const float* br,
                 int32_t* topk_idx, float* topk_w, hipStream_t st, const int32_t* M = nullptr,
                 int32_t* slot = nullptr);
// `Xg` null: everything but the row gather (the fused layer reads token rows through `perm`).
// `tile_tab` given: the kernel that finishes the grouping also writes the tile lists of the
// matrix-core expert kernels there (launch_ffn_tiled is then called with tab_ready).
// `slot_ready`: the router has already written slot[] (launch_route with M and slot): the lookup is not
// repeated where the grouping can do without its histogram kernel.
int launch_permute(const mmoe_shape& s, const void* X, const int32_t* vid, const int32_t* topk_idx,
                   const int32_t* M, int32_t* slot, int32_t* counts, int32_t* offsets, int32_t* perm,
                   int32_t* inv_perm, void* Xg, int32_t* blk_counts, int32_t* blk_base, int nblk,
                   hipStream_t st, int32_t* tile_tab = nullptr, bool slot_ready = false);
// Expert stage.  Row r of the grouped input is rows[r] when `perm` is null (rows = Xg), and
// rows[perm[r] / top_k] otherwise (rows = X: the gather is folded into the up product's loads).
// `mid`, when not null, is recorded between the up product (+ activation) and the down product.
// `sink` with `w` set: the down product writes the layer's output rows itself (see GateSink), Yg is unused.
// `slot_of_pair` given (self-grouping, only when self_grouping(s)): no grouping has run; every
// workgroup collects the pairs of its slot from slot_of_pair[P] itself, rows = X, and H and Yg are
// indexed by pair id; `perm` and `offsets` are then unused.
int launch_ffn_skinny(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                      const int32_t* slot_of_pair, const void* W1p, const void* W3p, const void* W2p, void* H,
                      float* Yg, hipStream_t st, hipEvent_t mid = nullptr, SlotFilter filt = SlotFilter(),
                      GateSink sink = GateSink());
// true when the fused layer skips the grouping kernels (streaming expert kernels, few pairs)
bool self_grouping(const mmoe_shape& s);
// `tab`: tiled_table_bytes() of scratch for the row-tile table.
// `tab_ready`: the grouping kernels have already written the tile lists into `tab`.
int launch_ffn_tiled(const mmoe_shape& s, const void* rows, const int32_t* perm, const int32_t* offsets,
                     const void* W1p, const void* W3p, const void* W2p, void* H, float* Yg, int32_t* tab,
                     hipStream_t st, hipEvent_t mid = nullptr, bool tab_ready = false,
                     SlotFilter filt = SlotFilter(), GateSink sink = GateSink());
size_t tiled_table_bytes(const mmoe_shape& s);
int planned_tile_rows(const mmoe_shape& s);  // tile height launch_ffn_tiled would use for this shape
// `inv_perm` null: Yg is indexed by pair id.
int launch_combine(const mmoe_shape& s, const float* Yg, const int32_t* inv_perm, const float* topk_w,
                   void* Y, hipStream_t st);
int launch_pack(const mmoe_shape& s, const void* W1, const void* W3, const void* W2, void* W1p, void* W3p,
                void* W2p, hipStream_t st);
int run_probe(void* buf, size_t bytes, float* out, hipStream_t st);
int launch_validate(const mmoe_shape& s, const int32_t* vid, const int32_t* M, int32_t* flag, hipStream_t st);

// expert-map builder (one translation unit)
size_t loader_ws_bytes(const mmoe_loader_shape& s);
int launch_expert_distance(const mmoe_loader_shape& s, const void* const* mats, double* distance, double* partial,
                           hipStream_t st);
int launch_assemble_pool(const mmoe_loader_shape& s, const void* const* mats, const int32_t* slot_src_layer, int layer,
                         int n_slots, void* const* pool, hipStream_t st);
int launch_expert_map(const mmoe_loader_shape& s, const double* distance, int32_t* rank, int32_t* owner, int32_t* M,
                      int32_t* S, int32_t* slot_src, hipStream_t st);

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? MMOE_OK : MMOE_ERR_LAUNCH;
}

}  // namespace mmoe
