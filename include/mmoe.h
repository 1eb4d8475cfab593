/*
 * mmoe -- forward pass of one multi-model MoE layer on AMD MI355X (gfx950).
 *
 * Several fine-tuned variants of one MoE model are served from a single
 * consolidated pool of experts (paper, section 3.1: similar experts of the
 * variants are loaded once and shared; Algorithm 1 emits the expert map).  At
 * inference (Algorithm 2, the per-layer body; Figure 3) the requested variant's
 * own gate scores the token, the top experts are selected, each selected
 * (variant, expert) is looked up in the map, the resident expert for that
 * location is applied -- possibly another variant's when the location is
 * consolidated, the variant's own otherwise -- and the results are combined
 * with the gate's coefficients (section 3.2).
 *
 * This library evaluates that layer for a batch that mixes tokens of several
 * variants.  Every token carries its variant id; the map is the table
 * M[v][e] -> pool slot; the pool holds each resident expert once.
 *
 * Conventions
 *   T tokens, d = d_model, f = d_ff, V variants, E experts per variant,
 *   k = top_k, S pool slots, P = T*k (token, pick) pairs, pair id p = t*k + j.
 *   All tensors are dense and row-major.  "dtype" is the storage type of X, Wr,
 *   the pool, H and Y; every product is accumulated in fp32.
 *
 * Pointers
 *   Every pointer except mmoe_shape* is a DEVICE pointer owned by the caller.
 *   The library never allocates, frees or keeps device memory; scratch comes
 *   from the caller's workspace `ws` (at least mmoe_workspace_bytes(), 256-byte
 *   aligned).  Inputs are read-only, outputs are fully overwritten.  `stream`
 *   is a hipStream_t passed as void*; every call is asynchronous on it and
 *   never synchronises the host (mmoe_validate_inputs excepted).
 *
 * Errors
 *   0 on success, a negative mmoe_status otherwise.  Only host-checkable faults
 *   are detected: null pointers, bad dimensions, unsupported combinations,
 *   small workspace, misalignment, launch failures.  Device data is not
 *   validated on the hot path: vid[t] outside [0,V), M[v][e] outside [0,S) or
 *   non-finite logits give undefined results (use mmoe_validate_inputs).
 *
 * Limits
 *   d_model and d_ff multiples of 256; E <= 256; top_k <= min(E, 8); S <= 1024;
 *   P*max(d,f) < 2^35, and < 2^31 for bf16 batches large enough for the matrix-core expert
 *   kernels (P > 16*S, or 32*S when d*f <= 4 Mi): otherwise MMOE_ERR_LIMIT.  SWIGLU needs W3, RELU and GELU need W3 == NULL.
 */
#ifndef MMOE_H
#define MMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MMOE_F32 = 0, MMOE_BF16 = 1 } mmoe_dtype;
typedef enum { MMOE_RELU = 0, MMOE_SWIGLU = 1, MMOE_GELU = 2 } mmoe_act;
/*
 * How the gate's coefficients are formed (section 3.2: "the gate network generates weighted
 * averaging coefficients for each expert, and ... the top experts are selected"; the paper gives
 * no formula, and its two model families differ):
 *   MMOE_GATE_SELECTED  softmax over the k selected logits; the coefficients of a token sum to 1
 *                       (k = 1 gives exactly 1).  The Mixtral-style top-2 gate.
 *   MMOE_GATE_ALL       softmax over all E logits; every selected expert keeps its own probability,
 *                       nothing is renormalised, so the coefficients sum to less than 1 unless
 *                       k = E.  The Switch-style top-1 gate (section 4.3's model family).
 * The selection itself (k largest logits, ties to the lower index) is the same in both.
 */
typedef enum { MMOE_GATE_SELECTED = 0, MMOE_GATE_ALL = 1 } mmoe_gate;

typedef enum {
    MMOE_OK = 0,
    MMOE_ERR_NULL = -1,      /* a required pointer is NULL                               */
    MMOE_ERR_DIM = -2,       /* a dimension is not positive                              */
    MMOE_ERR_TOPK = -3,      /* top_k > E or top_k > 8                                   */
    MMOE_ERR_DTYPE = -4,     /* unknown dtype, activation or gate code                   */
    MMOE_ERR_W3 = -5,        /* W3 missing for SWIGLU, or given for RELU / GELU          */
    MMOE_ERR_WORKSPACE = -6, /* ws is NULL or ws_bytes too small                         */
    MMOE_ERR_ALIGN = -7,     /* a tensor pointer is not 16-byte (ws: 256-byte) aligned   */
    MMOE_ERR_MULTIPLE = -8,  /* d_model or d_ff is not a multiple of 256                 */
    MMOE_ERR_LIMIT = -9,     /* E, S or the problem size exceeds the limits above        */
    MMOE_ERR_LAUNCH = -10,   /* the HIP runtime refused a kernel launch                  */
    MMOE_ERR_STATIC_LIMIT = -11 /* the shape needs more than MMOE_STATIC_WORKSPACE_BYTES     */
} mmoe_status;

typedef struct {
    int32_t T;       /* tokens in the batch                      */
    int32_t d_model; /* hidden size d                            */
    int32_t d_ff;    /* expert inner size f                      */
    int32_t V;       /* model variants                           */
    int32_t E;       /* experts per variant                      */
    int32_t S;       /* slots in the consolidated pool           */
    int32_t top_k;   /* experts selected per token               */
    int32_t dtype;   /* mmoe_dtype                               */
    int32_t act;     /* mmoe_act                                 */
    int32_t gate;    /* mmoe_gate                                */
    int32_t tile_rows; /* tuning, normally 0: token rows per tile of the matrix-core expert kernels.
                          0 chooses by shape: 128 rows (two workgroups per compute unit) when tiles are
                          short-lived (d_model <= 1024, or fewer than 64 rows per slot on average), 256
                          rows otherwise.  128 or 256 forces that height for the call.  Either height sums
                          every output element in the same order: the results are bit-identical.  Any
                          other value: MMOE_ERR_DIM.  Ignored by shapes that use the streaming kernels. */
} mmoe_shape;

/* Host only, pure.  Workspace (bytes) sufficient for every call below, 0 if the shape is invalid. */
size_t mmoe_workspace_bytes(const mmoe_shape *shape);

/* Host only.  Text for a status code (static storage). */
const char *mmoe_strerror(int status);

/*
 * One-time repacking of the pool, done when the pool is loaded (the paper's
 * loader runs once, offline, before serving: section 3.1).  The boundary's
 * plain layout is "in x out": W1, W3 [S, d, f] and W2 [S, f, d].  The expert
 * kernels read the packed pool that this call writes; each packed matrix has as
 * many elements as the plain one.  With out[n] = sum_k x[k] W[k][n], N outputs, K inputs:
 *   fp32: the transpose [S, N, K] (reduction dimension contiguous);
 *   bf16: matrix-core fragments.  Element (n, k) of slot s is stored at
 *         ((((s*(N/32) + n/32)*(K/16) + ks)*64 + 32*h + n%32)*8 + k%8
 *         with m = k/64, h = (k%64)/32, kk = (k%32)/8, ks = 4*m + kk:
 *         the 64 pieces of 16 bytes that follow each other are exactly the 32-row x 16-k
 *         operand of v_mfma_f32_32x32x16_bf16 as its 64 lanes hold it.
 * W3/W3p are NULL for RELU and GELU.  Outputs must not overlap inputs.
 */
int mmoe_pack_weights(const mmoe_shape *shape, const void *W1, const void *W3, const void *W2,
                      void *W1p, void *W3p, void *W2p, void *stream);

/*
 * Step R -- gate of the requested variant (Algorithm 2, "gate(act)"; section 3.2).
 *   logit[t,e] = <X[t,:], Wr[vid[t],e,:]> (+ br[vid[t],e])
 *   the k largest logits are selected, ties to the lower expert index, listed in
 *   selection (descending) order; w[t,j] = softmax over the k selected logits
 *   (MMOE_GATE_SELECTED) or entry j's probability in the softmax over all E logits (MMOE_GATE_ALL).
 * The logit is an fp32 sum in a fixed order, so that the selected indices are
 * reproducible bit for bit: element i belongs to lane (i div 4) mod 64; a lane
 * accumulates its elements in ascending i with one fused multiply-add each,
 * starting from +0; the 64 partial sums are combined by the butterfly
 * "for off in 32,16,8,4,2,1: p[l] = p[l] + p[l xor off]"; the bias is added last.
 *   X [T,d] dtype; vid [T] int32; Wr [V,E,d] dtype; br [V,E] fp32 or NULL;
 *   topk_idx [T,k] int32 out; topk_w [T,k] fp32 out.
 */
int mmoe_route(const mmoe_shape *shape, const void *X, const int32_t *vid, const void *Wr,
               const float *br, int32_t *topk_idx, float *topk_w, void *stream);

/*
 * Steps M and G -- expert-map lookup and grouping by pool slot (Algorithm 2, the
 * "map[iL][iE]" lookup; section 3.2: a hit uses the resident expert whoever owns it,
 * a miss the requested variant's own, which here is a private slot).
 *   slot[p] = M[vid[t]][topk_idx[p]];  counts[s] = #{p : slot[p] = s};
 *   offsets = exclusive prefix sum of counts, offsets[S] = P;
 *   perm = pair ids sorted by (slot, p) (stable);  inv_perm[perm[r]] = r;
 *   Xg[r,:] = X[perm[r] / k, :].
 * Deterministic: no result depends on the order in which threads run.
 *   M [V,E] int32 in [0,S);  slot, perm, inv_perm [P];  counts [S];  offsets [S+1];
 *   Xg [P,d] dtype.  Uses `ws`.
 */
int mmoe_remap_permute(const mmoe_shape *shape, const void *X, const int32_t *vid,
                       const int32_t *topk_idx, const int32_t *M, int32_t *slot, int32_t *counts,
                       int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *Xg, void *ws,
                       size_t ws_bytes, void *stream);

/*
 * Step F -- the resident experts applied to their groups (Algorithm 2,
 * "expert[iL][iE](act)"; section 3.2: a Mixtral expert has 3*d*f parameters).
 * For every slot s and row r in [offsets[s], offsets[s+1]):
 *   SWIGLU: Yg[r,:] = (silu(Xg[r,:] W1[s]) * (Xg[r,:] W3[s])) W2[s],  silu(a) = a/(1+exp(-a))
 *   RELU:   Yg[r,:] = relu(Xg[r,:] W1[s]) W2[s]
 *   GELU:   Yg[r,:] = gelu(Xg[r,:] W1[s]) W2[s],  gelu(a) = a/2 (1 + erf(a / sqrt 2))
 * Products accumulate in fp32; the hidden activation is stored in `dtype`
 * (rounded to nearest even for bf16) between the two products.
 *   Xg [P,d] dtype; offsets [S+1] int32 (device); W1p, W3p, W2p: PACKED pool
 *   (see mmoe_pack_weights);  Yg [P,d] fp32 out.  Uses `ws` for the hidden activation.
 */
int mmoe_expert_ffn(const mmoe_shape *shape, const void *Xg, const int32_t *offsets,
                    const void *W1p, const void *W3p, const void *W2p, float *Yg, void *ws,
                    size_t ws_bytes, void *stream);

/*
 * Step C -- combination with the gate's coefficients (section 3.2):
 *   Y[t,:] = sum_{j<k} topk_w[t,j] * Yg[inv_perm[t*k+j], :], fp32, ascending j,
 * rounded once to `dtype`.  Gather-side: no atomics, deterministic.
 *   Yg [P,d] fp32; inv_perm [P]; topk_w [T,k] fp32; Y [T,d] dtype out.
 */
int mmoe_combine(const mmoe_shape *shape, const float *Yg, const int32_t *inv_perm,
                 const float *topk_w, void *Y, void *stream);

/*
 * The whole layer, R -> M -> G -> F -> C, on one stream with no host
 * synchronisation; intermediates live in `ws`.  Arguments as above; the pool is
 * the PACKED one.  Y [T,d] dtype out.  The gathered copy Xg is not materialised: the
 * expert stage reads row perm[r] / k of X where the staged call reads row r of Xg; the
 * result is bit-identical to the staged calls'.
 */
int mmoe_layer_forward(const mmoe_shape *shape, const void *X, const int32_t *vid, const void *Wr,
                       const float *br, const int32_t *M, const void *W1p, const void *W3p,
                       const void *W2p, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * The layer with part of the pool in host memory: Algorithm 2's miss branch (section 3.2: on a
 * miss the requested variant's own expert is loaded from the host; section 5.1: the copy is what a
 * miss costs).  resident[s] (HOST array of S flags) says whether slot s of the DEVICE pool holds
 * its expert; for every other slot host_W1p[s], host_W3p[s], host_W2p[s] (HOST arrays of S
 * pointers) point to the slot's PACKED matrices in PINNED host memory (the layout
 * mmoe_pack_weights writes, one slot each).  The call
 *   - runs the gate, the map lookup and the grouping, then SYNCHRONISES `stream` once to learn
 *     which slots the batch touches (the copies to issue depend on the routing);
 *   - copies every touched non-resident slot into its place in the device pool on `copy_stream`
 *     (a second stream of the default priority, not `stream`);
 *   - applies the resident experts to their groups while the copies run, then the fetched ones,
 *     and combines: Y is bit-identical to mmoe_layer_forward on a fully resident pool.
 * The pool's non-resident slots are scratch until fetched; a fetched slot stays valid afterwards,
 * and fetched[s] (HOST out, may be NULL) tells the caller which ones arrived, so that it can mark
 * them resident for later calls (the paper leaves open what is evicted).  Returns the number
 * of slots fetched (>= 0) or a negative status.  Everything queued on `stream` before the call may
 * still read the pool: the copies wait for it.
 */
int mmoe_layer_forward_paged(const mmoe_shape *shape, const void *X, const int32_t *vid, const void *Wr,
                             const float *br, const int32_t *M, void *W1p, void *W3p, void *W2p,
                             const uint8_t *resident, const void *const *host_W1p,
                             const void *const *host_W3p, const void *const *host_W2p, void *Y, void *ws,
                             size_t ws_bytes, void *stream, void *copy_stream, uint8_t *fetched);

/*
 * mmoe_layer_forward for callers that cannot allocate device memory or hand over a workspace:
 * code that runs under HIP graph capture, tight serving loops (one decode step after the
 * other), harnesses that forbid allocation.  Same arguments without `ws`; same kernels, same
 * results bit for bit.  The intermediates live in a fixed array of
 * MMOE_STATIC_WORKSPACE_BYTES in device memory that belongs to the library's code object (each
 * GPU the library runs on holds its own copy until the process ends).  The call allocates and
 * frees nothing.  A shape with mmoe_workspace_bytes() above that size is refused with
 * MMOE_ERR_STATIC_LIMIT before anything is launched (64 MiB covers decode-shaped batches: up to
 * about 700 tokens of the Mixtral shape, 6000 of the Switch shape).
 * Every call on one GPU uses that GPU's one array, whatever the stream: two calls that overlap
 * in time on one GPU race; order them (same stream, or events).  Nothing in the array has to
 * start at zero: every intermediate is written before it is read, so the contents left by an
 * earlier call do not matter.  The array's address is looked up on the first call on each
 * device; make that call outside of any stream capture.
 */
#define MMOE_STATIC_WORKSPACE_BYTES (64u << 20)
int mmoe_layer_forward_static(const mmoe_shape *shape, const void *X, const int32_t *vid,
                              const void *Wr, const float *br, const int32_t *M, const void *W1p,
                              const void *W3p, const void *W2p, void *Y, void *stream);

/*
 * mmoe_layer_forward with timing marks, for benchmarks and profilers.  `events` is a HOST
 * array of MMOE_NUM_EVENTS hipEvent_t (as void*), created by the caller with timing
 * enabled; events[MMOE_EV_START] is recorded on `stream` before the first kernel and
 * events[i] right after the last kernel of stage i, so that the elapsed time between two
 * consecutive events is the duration of one stage (the expert stage is split into its up
 * product + activation and its down product: one kernel each).  A NULL entry is skipped (a
 * caller that wants one kernel's duration passes the two events around it); NULL `events`
 * makes this identical to mmoe_layer_forward.  The results do not depend on `events`.
 */
enum {
    MMOE_EV_START = 0,
    MMOE_EV_ROUTE = 1,    /* after step R                                         */
    MMOE_EV_PERMUTE = 2,  /* after steps M and G                                  */
    MMOE_EV_FFN_UP = 3,   /* after H = act(Xg W1 [, Xg W3])                       */
    MMOE_EV_FFN_DOWN = 4, /* after Yg = H W2                                      */
    MMOE_EV_COMBINE = 5,  /* after step C                                         */
    MMOE_NUM_EVENTS = 6
};
int mmoe_layer_forward_events(const mmoe_shape *shape, const void *X, const int32_t *vid,
                              const void *Wr, const float *br, const int32_t *M, const void *W1p,
                              const void *W3p, const void *W2p, void *Y, void *ws, size_t ws_bytes,
                              void *stream, void *const *events);

/*
 * Host only, pure: which expert-stage kernels
 * mmoe_expert_ffn and mmoe_layer_forward will use for this shape.  *streaming = 1: the
 * weight-streaming kernels (every fp32 shape; bf16 with few rows per slot), *tile_rows = 32
 * (rows of a slot per pass over its weights); *streaming = 0: the matrix-core kernels with
 * tiles of *tile_rows (128 or 256) token rows.  The choice depends on the shape only.
 */
int mmoe_expert_plan(const mmoe_shape *shape, int *streaming, int *tile_rows);

/*
 * Measurement aid, SYNCHRONISES the stream; not part of the layer.  Measures what this GPU
 * delivers for the two resources that bound the expert stage: out[0] = GB/s of a pure
 * streaming read of `buf` (DEVICE memory, `bytes` >= 64 MiB, 256-byte aligned, zero-filled by
 * the caller; its last MiB is written), out[1] = TFLOP/s of a loop of
 * v_mfma_f32_32x32x16_bf16 on register operands with no memory traffic.  `out` is a HOST
 * array of two floats.  Benchmarks print these beside the data-sheet peaks.
 */
int mmoe_probe_ceilings(void* buf, size_t bytes, float* out, void* stream);

/*
 * The initial expert loader's table (Algorithm 1; section 3.1), run once, offline, before
 * serving.  V fine-tuned variants of one MoE model, L layers of E experts; the expert block of
 * a location (layer, expert) is the concatenation of its n_mats matrices.
 *   1. degree of similarity of a location: the L2 distance between the flattened experts that
 *      two variants hold there, summed over all variant-to-variant combinations (unordered pairs;
 *      the listing's sum over ordered pairs is twice this and ranks identically);
 *   2. locations are ranked, the lowest distance first (rank 1), ties to the lower l*E + e;
 *   3. from rank 1 on, while fewer than `capacity` locations are taken, the location is given to
 *      the variants in turn: rank r goes to variant (r - 1) mod V (the section's text: with two
 *      models the odd ranks go to the first model; the listing's "count mod |M|" read with
 *      0-based lists starts one variant later).  Such a location is CONSOLIDATED: one resident
 *      expert, the owner's, used by every variant;
 *   4. any other location keeps every variant's own expert (the paper loads it on a miss; here
 *      it is a private slot of the pool).
 * The per-layer table of the forward pass follows: variant 0's locations take slots 0..E-1
 * (shared or private alike), the private slots of variants 1.. follow in (variant, expert) order.
 */
typedef struct {
    int32_t V;            /* variants, 1..8                                             */
    int32_t L;            /* layers                                                     */
    int32_t E;            /* experts per layer; L*E <= 4096                             */
    int32_t n_mats;       /* matrices of an expert block, 1..3                          */
    int64_t mat_elems[3]; /* elements of each matrix per location, multiples of 256     */
    int32_t dtype;        /* mmoe_dtype                                                 */
    int32_t capacity;     /* expert capacity C: locations to consolidate (>= 0)         */
} mmoe_loader_shape;

/* Host only, pure.  Workspace (bytes) for mmoe_expert_distance, 0 if the shape is invalid. */
size_t mmoe_loader_workspace_bytes(const mmoe_loader_shape *shape);

/*
 * Step 1.  `mats` is a HOST array of V*n_mats DEVICE pointers: mats[v*n_mats + m] is matrix m of
 * variant v for every location, [L, E, mat_elems[m]] row-major, 16-byte aligned.
 * distance [L, E] float64 (DEVICE) out.  Differences and squares are fp32, sums fp64, in a fixed
 * order (no atomics).  Reads every stored element once.  Uses `ws`.
 */
int mmoe_expert_distance(const mmoe_loader_shape *shape, const void *const *mats, double *distance,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * Steps 2 to 4, all DEVICE pointers.  distance [L, E] float64 in (finite).  Out: rank [L, E] int32
 * (1-based); owner [L, E] int32 (variant of a consolidated location, -1 otherwise); M [L, V, E]
 * int32 (the layer's table for mmoe_layer_forward); S [L] int32 (slots of each layer's pool);
 * slot_src [L, V*E, 2] int32: (variant, expert) whose weights fill each slot of the layer's pool,
 * rows past S[l] are (-1, -1).
 */
int mmoe_build_expert_map(const mmoe_loader_shape *shape, const double *distance, int32_t *rank,
                          int32_t *owner, int32_t *M, int32_t *S, int32_t *slot_src, void *stream);

/*
 * The loader's last step for one layer: the consolidated pool itself ("load M[idx].expert[iL][iE] to
 * GPU", Algorithm 1).  With the variants already in device memory the load is a device copy:
 * pool[m][s] (HOST array of n_mats DEVICE pointers, each [n_slots, mat_elems[m]] in the plain
 * layout) = matrix m of the (variant, expert) that slot_src names for slot s of `layer`.
 * slot_src is the whole [L, V*E, 2] array written by mmoe_build_expert_map (DEVICE); n_slots = S[layer]
 * (the caller reads S back to size the pool).  Follow with mmoe_pack_weights.
 */
int mmoe_assemble_pool(const mmoe_loader_shape *shape, const void *const *mats, const int32_t *slot_src,
                       int32_t layer, int32_t n_slots, void *const *pool, void *stream);

/*
 * Debugging aid, SYNCHRONISES the stream: checks on the device that every vid[t] is in
 * [0,V) and every M[v][e] in [0,S).  Returns 0 if so, 1 if not, a negative status on
 * argument errors.  `ws` needs 256 bytes.
 */
int mmoe_validate_inputs(const mmoe_shape *shape, const int32_t *vid, const int32_t *M, void *ws,
                         size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MMOE_H */
