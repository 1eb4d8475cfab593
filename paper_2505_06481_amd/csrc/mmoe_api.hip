// C-ABI entry points of libmmoe: argument checks, workspace carving, stage sequencing.
// Every step of the layer runs in the HIP kernels of the other translation units.
#include <mutex>

#include "mmoe_internal.h"

namespace mmoe {

int check_shape(const mmoe_shape* s)
{
    if (!s) return MMOE_ERR_NULL;
    if (s->T <= 0 || s->d_model <= 0 || s->d_ff <= 0 || s->V <= 0 || s->E <= 0 || s->S <= 0 || s->top_k <= 0)
        return MMOE_ERR_DIM;
    if (s->dtype != MMOE_F32 && s->dtype != MMOE_BF16) return MMOE_ERR_DTYPE;
    if (s->act != MMOE_RELU && s->act != MMOE_SWIGLU && s->act != MMOE_GELU) return MMOE_ERR_DTYPE;
    if (s->gate != MMOE_GATE_SELECTED && s->gate != MMOE_GATE_ALL) return MMOE_ERR_DTYPE;
    if (s->tile_rows != 0 && s->tile_rows != 128 && s->tile_rows != 256) return MMOE_ERR_DIM;
    if (s->top_k > s->E || s->top_k > kMaxTopK) return MMOE_ERR_TOPK;
    if (s->d_model % 256 != 0 || s->d_ff % 256 != 0) return MMOE_ERR_MULTIPLE;
    if (s->E > kMaxE || s->S > kMaxS) return MMOE_ERR_LIMIT;
    int64_t P = (int64_t)s->T * s->top_k;
    int64_t widest = s->d_model > s->d_ff ? s->d_model : s->d_ff;
    if (P > (int64_t)1 << 30 || P * widest >= ((int64_t)1 << 35)) return MMOE_ERR_LIMIT;
    // the matrix-core expert kernels address a panel with 32-bit byte offsets
    if (!use_skinny(*s) && P * widest >= ((int64_t)1 << 31)) return MMOE_ERR_LIMIT;
    return MMOE_OK;
}

WsLayout ws_layout(const mmoe_shape& s)
{
    WsLayout L;
    size_t P = (size_t)s.T * s.top_k, es = elem_size(s.dtype);
    L.nblk = (int)((P + kPermChunk - 1) / kPermChunk);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    L.topk_idx = take(P * 4);
    L.topk_w = take(P * 4);
    L.slot = take(P * 4);
    L.counts = take((size_t)s.S * 4);
    L.offsets = take((size_t)(s.S + 1) * 4);
    L.perm = take(P * 4);
    L.inv_perm = take(P * 4);
    L.blk_counts = take((size_t)L.nblk * s.S * 4);
    L.blk_base = take((size_t)L.nblk * s.S * 4);
    L.tile_tab = take(tiled_table_bytes(s));
    L.resident = take((size_t)s.S);
    L.H = take(P * s.d_ff * es);
    L.Yg = take(P * s.d_model * 4);
    L.total = off;
    return L;
}

bool use_skinny(const mmoe_shape& s)
{
    // fp32 always streams (fp32 MFMA, full precision).  bf16 streams when a slot sees few
    // rows: the weights are then read once from HBM and that read is the bound.  The
    // streaming kernel takes 32 rows of a slot per pass over its weights, so it only pays
    // while the fullest slot stays near that.  Measured with each kernel forced: on the
    // Mixtral shape (352 MB a slot) it wins up to an average of 16 rows per slot and loses
    // quickly beyond (1.21 ms against 0.83 ms at 40); on the Switch shape (9 MB a slot, a
    // second pass finds the weights in cache) up to 32.
    if (s.dtype == MMOE_F32) return true;
    const int64_t P = (int64_t)s.T * s.top_k;
    const bool small_experts = (int64_t)s.d_model * s.d_ff <= ((int64_t)4 << 20);
    return P <= (int64_t)(small_experts ? 32 : 16) * s.S;
}

static inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

}  // namespace mmoe

using namespace mmoe;

extern "C" {

size_t mmoe_workspace_bytes(const mmoe_shape* shape)
{
    if (check_shape(shape) != MMOE_OK) return 0;
    return ws_layout(*shape).total;
}

const char* mmoe_strerror(int status)
{
    switch (status) {
        case MMOE_OK: return "success";
        case MMOE_ERR_NULL: return "a required pointer is NULL";
        case MMOE_ERR_DIM: return "a dimension is not positive";
        case MMOE_ERR_TOPK: return "top_k exceeds E or the supported maximum of 8";
        case MMOE_ERR_DTYPE: return "unknown dtype, activation or gate mode";
        case MMOE_ERR_W3: return "W3 must be given for SWIGLU and must be NULL for RELU and GELU";
        case MMOE_ERR_WORKSPACE: return "workspace missing or smaller than mmoe_workspace_bytes()";
        case MMOE_ERR_ALIGN: return "a pointer is not sufficiently aligned (16 bytes; workspace 256)";
        case MMOE_ERR_MULTIPLE: return "d_model and d_ff must be multiples of 256";
        case MMOE_ERR_LIMIT: return "E, S or the problem size exceeds the library's limits";
        case MMOE_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
        case MMOE_ERR_STATIC_LIMIT:
            return "the shape needs more scratch than mmoe_layer_forward_static holds "
                   "(MMOE_STATIC_WORKSPACE_BYTES); use mmoe_layer_forward with a workspace";
        default: return "unknown status";
    }
}

int mmoe_pack_weights(const mmoe_shape* shape, const void* W1, const void* W3, const void* W2, void* W1p,
                      void* W3p, void* W2p, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!W1 || !W2 || !W1p || !W2p) return MMOE_ERR_NULL;
    bool gated = shape->act == MMOE_SWIGLU;
    if (gated != (W3 != nullptr) || gated != (W3p != nullptr)) return MMOE_ERR_W3;
    if (misaligned(W1, 16) || misaligned(W2, 16) || misaligned(W3, 16) || misaligned(W1p, 16) ||
        misaligned(W2p, 16) || misaligned(W3p, 16))
        return MMOE_ERR_ALIGN;
    return launch_pack(*shape, W1, W3, W2, W1p, W3p, W2p, (hipStream_t)stream);
}

int mmoe_route(const mmoe_shape* shape, const void* X, const int32_t* vid, const void* Wr, const float* br,
               int32_t* topk_idx, float* topk_w, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!X || !vid || !Wr || !topk_idx || !topk_w) return MMOE_ERR_NULL;
    if (misaligned(X, 16) || misaligned(Wr, 16) || misaligned(vid, 4) || misaligned(br, 4) ||
        misaligned(topk_idx, 4) || misaligned(topk_w, 4))
        return MMOE_ERR_ALIGN;
    return launch_route(*shape, X, vid, Wr, br, topk_idx, topk_w, (hipStream_t)stream);
}

int mmoe_remap_permute(const mmoe_shape* shape, const void* X, const int32_t* vid, const int32_t* topk_idx,
                       const int32_t* M, int32_t* slot, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv_perm, void* Xg, void* ws, size_t ws_bytes, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!X || !vid || !topk_idx || !M || !slot || !counts || !offsets || !perm || !inv_perm || !Xg)
        return MMOE_ERR_NULL;
    WsLayout L = ws_layout(*shape);
    size_t need = 2 * align256((size_t)L.nblk * shape->S * 4);
    if (!ws || ws_bytes < need) return MMOE_ERR_WORKSPACE;
    if (misaligned(ws, 256) || misaligned(X, 16) || misaligned(Xg, 16) || misaligned(vid, 4) ||
        misaligned(topk_idx, 4) || misaligned(M, 4) || misaligned(slot, 4) || misaligned(counts, 4) ||
        misaligned(offsets, 4) || misaligned(perm, 4) || misaligned(inv_perm, 4))
        return MMOE_ERR_ALIGN;
    int32_t* blk_counts = (int32_t*)ws;
    int32_t* blk_base = (int32_t*)((char*)ws + need / 2);
    return launch_permute(*shape, X, vid, topk_idx, M, slot, counts, offsets, perm, inv_perm, Xg, blk_counts,
                          blk_base, L.nblk, (hipStream_t)stream);
}

int mmoe_expert_ffn(const mmoe_shape* shape, const void* Xg, const int32_t* offsets, const void* W1p,
                    const void* W3p, const void* W2p, float* Yg, void* ws, size_t ws_bytes, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!Xg || !offsets || !W1p || !W2p || !Yg) return MMOE_ERR_NULL;
    if ((shape->act == MMOE_SWIGLU) != (W3p != nullptr)) return MMOE_ERR_W3;
    const size_t h_bytes = align256((size_t)shape->T * shape->top_k * shape->d_ff * elem_size(shape->dtype));
    const size_t need = h_bytes + tiled_table_bytes(*shape);
    if (!ws || ws_bytes < need) return MMOE_ERR_WORKSPACE;
    if (misaligned(ws, 256) || misaligned(Xg, 16) || misaligned(W1p, 16) || misaligned(W3p, 16) ||
        misaligned(W2p, 16) || misaligned(Yg, 16) || misaligned(offsets, 4))
        return MMOE_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (use_skinny(*shape)) return launch_ffn_skinny(*shape, Xg, nullptr, offsets, nullptr, W1p, W3p, W2p, ws, Yg, st);
    return launch_ffn_tiled(*shape, Xg, nullptr, offsets, W1p, W3p, W2p, ws, Yg, (int32_t*)((char*)ws + h_bytes),
                            st);
}

int mmoe_combine(const mmoe_shape* shape, const float* Yg, const int32_t* inv_perm, const float* topk_w,
                 void* Y, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!Yg || !inv_perm || !topk_w || !Y) return MMOE_ERR_NULL;
    if (misaligned(Yg, 16) || misaligned(Y, 16) || misaligned(inv_perm, 4) || misaligned(topk_w, 4))
        return MMOE_ERR_ALIGN;
    return launch_combine(*shape, Yg, inv_perm, topk_w, Y, (hipStream_t)stream);
}

int mmoe_layer_forward_events(const mmoe_shape* shape, const void* X, const int32_t* vid, const void* Wr,
                              const float* br, const int32_t* M, const void* W1p, const void* W3p,
                              const void* W2p, void* Y, void* ws, size_t ws_bytes, void* stream,
                              void* const* events)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!X || !vid || !Wr || !M || !W1p || !W2p || !Y) return MMOE_ERR_NULL;
    if ((shape->act == MMOE_SWIGLU) != (W3p != nullptr)) return MMOE_ERR_W3;
    WsLayout L = ws_layout(*shape);
    if (!ws || ws_bytes < L.total) return MMOE_ERR_WORKSPACE;
    if (misaligned(ws, 256) || misaligned(X, 16) || misaligned(Wr, 16) || misaligned(W1p, 16) ||
        misaligned(W3p, 16) || misaligned(W2p, 16) || misaligned(Y, 16) || misaligned(vid, 4) ||
        misaligned(br, 4) || misaligned(M, 4))
        return MMOE_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    auto mark = [&](int i) -> int {
        if (!events || !events[i]) return MMOE_OK;
        return hipEventRecord((hipEvent_t)events[i], st) == hipSuccess ? MMOE_OK : MMOE_ERR_LAUNCH;
    };
    char* w = (char*)ws;
    int32_t* topk_idx = (int32_t*)(w + L.topk_idx);
    float* topk_w = (float*)(w + L.topk_w);
    int32_t* offsets = (int32_t*)(w + L.offsets);
    int32_t* inv_perm = (int32_t*)(w + L.inv_perm);
    float* Yg = (float*)(w + L.Yg);
    hipEvent_t mid = events ? (hipEvent_t)events[MMOE_EV_FFN_UP] : nullptr;  // may be null
    // One pick per token: the combination is one product per element, and the down product's epilogue
    // applies it and writes Y itself (same arithmetic as the combination kernel: bit-identical).
    const bool fold = shape->top_k == 1;
    GateSink sink;
    if (fold) {
        sink.Y = Y;
        sink.w = topk_w;
    }

    if ((rc = mark(MMOE_EV_START))) return rc;
    if (self_grouping(*shape)) {
        // Decode-sized batches: four launches.  The router looks the picks up in the expert map, the
        // expert kernels collect the pairs of their slot themselves and index H and Yg by pair id, the
        // combination reads them by pair id: no grouping kernel, bit-identical output.
        int32_t* slot = (int32_t*)(w + L.slot);
        if ((rc = launch_route(*shape, X, vid, Wr, br, topk_idx, topk_w, st, M, slot))) return rc;
        if ((rc = mark(MMOE_EV_ROUTE))) return rc;
        if ((rc = mark(MMOE_EV_PERMUTE))) return rc;
        rc = launch_ffn_skinny(*shape, X, nullptr, nullptr, slot, W1p, W3p, W2p, w + L.H, Yg, st, mid, SlotFilter(), sink);
        if (rc) return rc;
        if ((rc = mark(MMOE_EV_FFN_DOWN))) return rc;
        if (!fold && (rc = launch_combine(*shape, Yg, nullptr, topk_w, Y, st))) return rc;
        return mark(MMOE_EV_COMBINE);
    }
    // the router also looks its picks up in the expert map (step M): the grouping starts from slot[]
    if ((rc = launch_route(*shape, X, vid, Wr, br, topk_idx, topk_w, st, M, (int32_t*)(w + L.slot)))) return rc;
    if ((rc = mark(MMOE_EV_ROUTE))) return rc;
    // no gathered copy of the token rows: the up product reads X through perm
    int32_t* perm = (int32_t*)(w + L.perm);
    const bool tiled = !use_skinny(*shape);
    int32_t* tile_tab = (int32_t*)(w + L.tile_tab);
    rc = launch_permute(*shape, X, vid, topk_idx, M, (int32_t*)(w + L.slot), (int32_t*)(w + L.counts), offsets,
                        perm, inv_perm, nullptr, (int32_t*)(w + L.blk_counts), (int32_t*)(w + L.blk_base), L.nblk,
                        st, tiled ? tile_tab : nullptr, true);
    if (rc) return rc;
    if ((rc = mark(MMOE_EV_PERMUTE))) return rc;
    sink.perm = perm;
    if (!tiled)
        rc = launch_ffn_skinny(*shape, X, perm, offsets, nullptr, W1p, W3p, W2p, w + L.H, Yg, st, mid, SlotFilter(), sink);
    else
        rc = launch_ffn_tiled(*shape, X, perm, offsets, W1p, W3p, W2p, w + L.H, Yg, tile_tab, st, mid, true,
                              SlotFilter(), sink);
    if (rc) return rc;
    if ((rc = mark(MMOE_EV_FFN_DOWN))) return rc;
    if (!fold && (rc = launch_combine(*shape, Yg, inv_perm, topk_w, Y, st))) return rc;
    return mark(MMOE_EV_COMBINE);
}

int mmoe_layer_forward_paged(const mmoe_shape* shape, const void* X, const int32_t* vid, const void* Wr,
                             const float* br, const int32_t* M, void* W1p, void* W3p, void* W2p,
                             const uint8_t* resident, const void* const* host_W1p, const void* const* host_W3p,
                             const void* const* host_W2p, void* Y, void* ws, size_t ws_bytes, void* stream,
                             void* copy_stream, uint8_t* fetched)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!X || !vid || !Wr || !M || !W1p || !W2p || !Y || !resident || !host_W1p || !host_W2p) return MMOE_ERR_NULL;
    const bool gated = shape->act == MMOE_SWIGLU;
    if (gated != (W3p != nullptr) || gated != (host_W3p != nullptr)) return MMOE_ERR_W3;
    WsLayout L = ws_layout(*shape);
    if (!ws || ws_bytes < L.total) return MMOE_ERR_WORKSPACE;
    if (misaligned(ws, 256) || misaligned(X, 16) || misaligned(Wr, 16) || misaligned(W1p, 16) ||
        misaligned(W3p, 16) || misaligned(W2p, 16) || misaligned(Y, 16) || misaligned(vid, 4) ||
        misaligned(br, 4) || misaligned(M, 4))
        return MMOE_ERR_ALIGN;
    if (!copy_stream || copy_stream == stream) return MMOE_ERR_NULL;  // the copies need a stream of their own
    const int S = shape->S;
    for (int s = 0; s < S; ++s)
        if (!resident[s] && (!host_W1p[s] || !host_W2p[s] || (gated && !host_W3p[s]))) return MMOE_ERR_NULL;
    hipStream_t st = (hipStream_t)stream, cp = (hipStream_t)copy_stream;
    char* w = (char*)ws;
    int32_t* topk_idx = (int32_t*)(w + L.topk_idx);
    float* topk_w = (float*)(w + L.topk_w);
    int32_t* counts = (int32_t*)(w + L.counts);
    int32_t* offsets = (int32_t*)(w + L.offsets);
    int32_t* perm = (int32_t*)(w + L.perm);
    int32_t* inv_perm = (int32_t*)(w + L.inv_perm);
    uint8_t* res_dev = (uint8_t*)(w + L.resident);
    float* Yg = (float*)(w + L.Yg);

    hipEvent_t ev_start = nullptr, ev_copied = nullptr;
    if (hipEventCreateWithFlags(&ev_start, hipEventDisableTiming) != hipSuccess) return MMOE_ERR_LAUNCH;
    if (hipEventCreateWithFlags(&ev_copied, hipEventDisableTiming) != hipSuccess) {
        hipEventDestroy(ev_start);
        return MMOE_ERR_LAUNCH;
    }
    auto done = [&](int code) {
        hipEventDestroy(ev_start);
        hipEventDestroy(ev_copied);
        return code;
    };
    // everything queued on `stream` before this call may still read the pool: the copies wait for it
    if (hipEventRecord(ev_start, st) != hipSuccess || hipStreamWaitEvent(cp, ev_start, 0) != hipSuccess)
        return done(MMOE_ERR_LAUNCH);
    // gate, expert-map lookup, grouping; then the host learns which slots this batch touches
    if (hipMemcpyAsync(res_dev, resident, (size_t)S, hipMemcpyHostToDevice, st) != hipSuccess)
        return done(MMOE_ERR_LAUNCH);
    if ((rc = launch_route(*shape, X, vid, Wr, br, topk_idx, topk_w, st))) return done(rc);
    rc = launch_permute(*shape, X, vid, topk_idx, M, (int32_t*)(w + L.slot), counts, offsets, perm, inv_perm, nullptr,
                        (int32_t*)(w + L.blk_counts), (int32_t*)(w + L.blk_base), L.nblk, st);
    if (rc) return done(rc);
    int32_t host_counts[kMaxS];
    if (hipMemcpyAsync(host_counts, counts, (size_t)S * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return done(MMOE_ERR_LAUNCH);
    // misses: the requested variant's own expert is brought in from host memory (Algorithm 2's miss
    // branch), into the slot's place in the pool, on the copy stream
    const size_t mat_bytes = (size_t)shape->d_model * shape->d_ff * elem_size(shape->dtype);
    int n_missed = 0;
    for (int s = 0; s < S; ++s) {
        const bool miss = !resident[s] && host_counts[s] > 0;
        if (fetched) fetched[s] = miss ? 1 : 0;
        if (!miss) continue;
        ++n_missed;
        bool ok = hipMemcpyAsync((char*)W1p + s * mat_bytes, host_W1p[s], mat_bytes, hipMemcpyHostToDevice, cp) == hipSuccess;
        ok = ok && hipMemcpyAsync((char*)W2p + s * mat_bytes, host_W2p[s], mat_bytes, hipMemcpyHostToDevice, cp) == hipSuccess;
        if (gated)
            ok = ok && hipMemcpyAsync((char*)W3p + s * mat_bytes, host_W3p[s], mat_bytes, hipMemcpyHostToDevice, cp) == hipSuccess;
        if (!ok) return done(MMOE_ERR_LAUNCH);
    }
    if (n_missed && hipEventRecord(ev_copied, cp) != hipSuccess) return done(MMOE_ERR_LAUNCH);
    // hits first (they overlap the copies), then the slots that have just arrived
    const bool tiled = !use_skinny(*shape);
    int32_t* tile_tab = (int32_t*)(w + L.tile_tab);
    const bool fold = shape->top_k == 1;  // the down product writes Y itself (see mmoe_layer_forward_events)
    GateSink sink;
    if (fold) {
        sink.Y = Y;
        sink.w = topk_w;
        sink.perm = perm;
    }
    for (int pass = 0; pass < (n_missed ? 2 : 1); ++pass) {
        SlotFilter filt;
        filt.flag = res_dev;
        filt.want = pass == 0 ? 1 : 0;
        if (pass == 1 && hipStreamWaitEvent(st, ev_copied, 0) != hipSuccess) return done(MMOE_ERR_LAUNCH);
        if (!tiled)
            rc = launch_ffn_skinny(*shape, X, perm, offsets, nullptr, W1p, W3p, W2p, w + L.H, Yg, st, nullptr, filt,
                                   sink);
        else
            rc = launch_ffn_tiled(*shape, X, perm, offsets, W1p, W3p, W2p, w + L.H, Yg, tile_tab, st, nullptr, false,
                                  filt, sink);
        if (rc) return done(rc);
    }
    if (!fold && (rc = launch_combine(*shape, Yg, inv_perm, topk_w, Y, st))) return done(rc);
    return done(n_missed);
}

int mmoe_layer_forward(const mmoe_shape* shape, const void* X, const int32_t* vid, const void* Wr,
                       const float* br, const int32_t* M, const void* W1p, const void* W3p, const void* W2p,
                       void* Y, void* ws, size_t ws_bytes, void* stream)
{
    return mmoe_layer_forward_events(shape, X, vid, Wr, br, M, W1p, W3p, W2p, Y, ws, ws_bytes, stream, nullptr);
}

// ---- the layer for callers that cannot allocate --------------------------------------------
// Same kernels as mmoe_layer_forward; the intermediates live in a fixed array in device memory
// that is part of the loaded code object instead of in a caller's workspace.  Each GPU holds its
// own copy of the array at its own address; the address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[MMOE_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until looked up

// Device address of `scratch` on the current device (looked up on the first call on that device).
int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MMOE_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MMOE_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MMOE_OK;
}
}  // namespace

int mmoe_layer_forward_static(const mmoe_shape* shape, const void* X, const int32_t* vid, const void* Wr,
                              const float* br, const int32_t* M, const void* W1p, const void* W3p,
                              const void* W2p, void* Y, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (ws_layout(*shape).total > (size_t)MMOE_STATIC_WORKSPACE_BYTES) return MMOE_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    return mmoe_layer_forward_events(shape, X, vid, Wr, br, M, W1p, W3p, W2p, Y, ws,
                                     (size_t)MMOE_STATIC_WORKSPACE_BYTES, stream, nullptr);
}

int mmoe_expert_plan(const mmoe_shape* shape, int* streaming, int* tile_rows)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!streaming || !tile_rows) return MMOE_ERR_NULL;
    *streaming = use_skinny(*shape) ? 1 : 0;
    *tile_rows = *streaming ? 32 : planned_tile_rows(*shape);
    return MMOE_OK;
}

int mmoe_probe_ceilings(void* buf, size_t bytes, float* out, void* stream)
{
    if (!buf || !out) return MMOE_ERR_NULL;
    if (bytes < ((size_t)64 << 20)) return MMOE_ERR_WORKSPACE;
    if (misaligned(buf, 256)) return MMOE_ERR_ALIGN;
    return run_probe(buf, bytes, out, (hipStream_t)stream);
}

static int check_loader_shape(const mmoe_loader_shape* s)
{
    if (!s) return MMOE_ERR_NULL;
    if (s->V <= 0 || s->L <= 0 || s->E <= 0 || s->n_mats <= 0 || s->capacity < 0) return MMOE_ERR_DIM;
    if (s->dtype != MMOE_F32 && s->dtype != MMOE_BF16) return MMOE_ERR_DTYPE;
    if (s->V > kLoaderMaxV || s->n_mats > 3 || (int64_t)s->L * s->E > kLoaderMaxLoc) return MMOE_ERR_LIMIT;
    for (int m = 0; m < s->n_mats; ++m) {
        if (s->mat_elems[m] <= 0) return MMOE_ERR_DIM;
        if (s->mat_elems[m] % 256 != 0) return MMOE_ERR_MULTIPLE;
        if (s->mat_elems[m] > ((int64_t)1 << 40)) return MMOE_ERR_LIMIT;
    }
    return MMOE_OK;
}

size_t mmoe_loader_workspace_bytes(const mmoe_loader_shape* shape)
{
    if (check_loader_shape(shape) != MMOE_OK) return 0;
    return loader_ws_bytes(*shape);
}

int mmoe_expert_distance(const mmoe_loader_shape* shape, const void* const* mats, double* distance, void* ws,
                         size_t ws_bytes, void* stream)
{
    int rc = check_loader_shape(shape);
    if (rc) return rc;
    if (!mats || !distance) return MMOE_ERR_NULL;
    for (int i = 0; i < shape->V * shape->n_mats; ++i) {
        if (!mats[i]) return MMOE_ERR_NULL;
        if (misaligned(mats[i], 16)) return MMOE_ERR_ALIGN;
    }
    if (!ws || ws_bytes < loader_ws_bytes(*shape)) return MMOE_ERR_WORKSPACE;
    if (misaligned(ws, 256) || misaligned(distance, 8)) return MMOE_ERR_ALIGN;
    return launch_expert_distance(*shape, mats, distance, (double*)ws, (hipStream_t)stream);
}

int mmoe_build_expert_map(const mmoe_loader_shape* shape, const double* distance, int32_t* rank, int32_t* owner,
                          int32_t* M, int32_t* S, int32_t* slot_src, void* stream)
{
    int rc = check_loader_shape(shape);
    if (rc) return rc;
    if (!distance || !rank || !owner || !M || !S || !slot_src) return MMOE_ERR_NULL;
    if (misaligned(distance, 8) || misaligned(rank, 4) || misaligned(owner, 4) || misaligned(M, 4) ||
        misaligned(S, 4) || misaligned(slot_src, 4))
        return MMOE_ERR_ALIGN;
    return launch_expert_map(*shape, distance, rank, owner, M, S, slot_src, (hipStream_t)stream);
}

int mmoe_assemble_pool(const mmoe_loader_shape* shape, const void* const* mats, const int32_t* slot_src, int32_t layer,
                       int32_t n_slots, void* const* pool, void* stream)
{
    int rc = check_loader_shape(shape);
    if (rc) return rc;
    if (!mats || !slot_src || !pool) return MMOE_ERR_NULL;
    if (layer < 0 || layer >= shape->L || n_slots <= 0 || n_slots > shape->V * shape->E) return MMOE_ERR_DIM;
    for (int i = 0; i < shape->V * shape->n_mats; ++i)
        if (!mats[i]) return MMOE_ERR_NULL;
    for (int m = 0; m < shape->n_mats; ++m) {
        if (!pool[m]) return MMOE_ERR_NULL;
        if (misaligned(pool[m], 16)) return MMOE_ERR_ALIGN;
    }
    if (misaligned(slot_src, 4)) return MMOE_ERR_ALIGN;
    return launch_assemble_pool(*shape, mats, slot_src + (size_t)layer * shape->V * shape->E * 2, layer, n_slots, pool,
                                (hipStream_t)stream);
}

int mmoe_validate_inputs(const mmoe_shape* shape, const int32_t* vid, const int32_t* M, void* ws,
                         size_t ws_bytes, void* stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!vid || !M) return MMOE_ERR_NULL;
    if (!ws || ws_bytes < 256) return MMOE_ERR_WORKSPACE;
    if (misaligned(ws, 256)) return MMOE_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    rc = launch_validate(*shape, vid, M, (int32_t*)ws, st);
    if (rc) return rc;
    int32_t flag = 0;
    if (hipMemcpyAsync(&flag, ws, 4, hipMemcpyDeviceToHost, st) != hipSuccess) return MMOE_ERR_LAUNCH;
    if (hipStreamSynchronize(st) != hipSuccess) return MMOE_ERR_LAUNCH;
    return flag ? 1 : 0;
}

}  // extern "C"
