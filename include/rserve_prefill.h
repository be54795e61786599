/*
 * rserve_prefill.h -- C ABI of the chunked-prefill decoder-layer library for AMD MI355X (gfx950).
 *
 * What the library computes.  RServe (arXiv 2509.24381) schedules the language model's prefill
 * in token-budgeted chunks; its Algorithm 2 (section 3.3) ends in BatchExecute(S), one forward
 * pass of the language model over a micro-batch S that holds the schedulable tokens of one or
 * more requests.  Chunked prefill (section 2.1.1 and section 2.2.1) means: the prompt is split
 * into chunks that are processed one after another, and a chunk depends on earlier chunks only
 * through the KV cache they left behind.  This library is that forward pass for ONE decoder
 * layer at a time:
 *
 *     h = rmsnorm(x) -> q,k,v = h Wqkv^T (+b) -> RoPE(q,k) at absolute positions P..P+T-1
 *     -> append k~,v to the request's KV cache -> causal GQA attention of the chunk against the
 *     whole cache -> r = x + o Wo^T -> y = r + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T,  h2 = rmsnorm(r)
 *
 * with bf16 storage (inputs, weights, KV cache - optionally 8-bit, see rs_kv_alloc_fp8 -, outputs) and fp32
 * accumulation.  The paper does
 * not spell out the layer; it is the pre-norm decoder block of the model family the paper serves
 * (section 4.1.1), with sequential 1-D rotary positions.
 *
 * Conventions shared by every call
 *  - Every `void*` named dev / documented "device" is GPU memory owned by the CALLER (typically a
 *    PyTorch tensor).  The library owns only host-side handles (rs_ctx, rs_kv), pinned host staging
 *    for per-call descriptors, and one device buffer it allocates in rs_ctx_create (the RoPE
 *    cos/sin table).  rs_prefill_* allocate nothing.
 *  - Slabs (weights, KV, workspace) must be 256-byte aligned; x and y 16-byte aligned.
 *  - All work is enqueued on the caller's HIP stream (`hip_stream`, a hipStream_t passed as
 *    void*, NULL = the null stream) and the call returns without waiting.  Host-side state
 *    (cache lengths) is advanced at enqueue time.  The caller orders streams: two calls whose work
 *    overlaps on the GPU must not share an rs_kv or a workspace (one rs_ctx may serve several
 *    streams).  The host side is not thread-safe: one thread at a time per rs_ctx.
 *  - rs_prefill_* calls are not for HIP graph capture: every call builds its descriptors (cache lengths, work items,
 *    page numbers) on the host and stages them through pinned memory that later calls reuse, and it may wait on an
 *    event of its own; on a capturing stream the call returns RS_ESTATE and records nothing.  A replay would also be meaningless: each call's
 *    shape depends on the cache lengths it finds.  Between the kernels of consecutive calls the stream idles for a few
 *    microseconds, so there is little for a graph to win.
 *  - Errors are decided on the host BEFORE anything is launched; on any status other than RS_OK
 *    nothing was enqueued and no state changed (RS_EHIP excepted: a launch itself failed).
 *  - bf16 matrices are row-major.  "torch layout" for a weight means [out_features, in_features].
 */
#ifndef RSERVE_PREFILL_H
#define RSERVE_PREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rs_status {
    RS_OK = 0,
    RS_EINVAL = -1,     /* null / misaligned pointer, negative size, bad layer index, duplicate request, shape the kernels do not support */
    RS_ECAPACITY = -2,  /* chunk does not fit the KV cache capacity or the RoPE table (max_pos) */
    RS_EWORKSPACE = -3, /* workspace smaller than rs_workspace_bytes() for this call */
    RS_ESTATE = -4,     /* handle used with a context, pool or kind of cache it does not belong to; pool destroyed while in use */
    RS_EHIP = -5        /* a HIP runtime call failed; see rs_last_error() */
} rs_status;

/* Shape of one decoder layer and the limits of one call. */
typedef struct rs_layer_cfg {
    int hidden;               /* H; multiple of 64 */
    int n_q_heads;            /* Hq */
    int n_kv_heads;           /* Hkv; divides Hq */
    int head_dim;             /* d; 64 or 128 */
    int mlp_inter;            /* I; multiple of 64 */
    float rms_eps;            /* added to mean(x^2) inside the square root */
    float rope_theta;         /* RoPE base; angle of pair j at position n is n * theta^(-2j/d) */
    int qkv_bias;             /* nonzero: rs_layer_weights.b_qkv is used */
    int max_tokens_per_call;  /* upper bound on the rows of one rs_prefill_* call (the token budget B of Algorithm 2) */
    int max_requests;         /* upper bound on R in rs_prefill_batch */
    int max_pos;              /* RoPE table length: cache length after any call must stay <= max_pos */
} rs_layer_cfg;

/* Device pointers to one layer's parameters (bf16).
 * In torch layout: ln1_g[H], w_qkv[(Hq+2Hkv)*d, H] = rows of Wq, then Wk, then Wv, b_qkv[(Hq+2Hkv)*d] or NULL,
 * w_o[H, Hq*d], ln2_g[H], w_gate_up[2I, H] = rows of W_gate then W_up, w_down[H, I].
 * rs_prefill_* take the PACKED form produced by rs_weights_pack (same struct, pointers into the packed slab). */
typedef struct rs_layer_weights {
    const void* ln1_g;
    const void* w_qkv;
    const void* b_qkv;
    const void* w_o;
    const void* ln2_g;
    const void* w_gate_up;
    const void* w_down;
} rs_layer_weights;

typedef struct rs_ctx rs_ctx; /* layer shape + RoPE table + descriptor staging; host handle */
typedef struct rs_kv rs_kv;   /* one request's KV cache over n_layers layers; host handle over caller-owned device memory */

/* Create / destroy a context for one layer shape on the current HIP device.
 * Allocates the RoPE cos/sin table (max_pos * d/2 * 8 bytes of device memory) and pinned staging for
 * per-call request descriptors.  RS_EINVAL if the shape is outside what the kernels support (see rs_layer_cfg).
 * On a host without a GPU the context is still created (host-only): every argument check works, and any call that
 * would have to launch returns RS_EHIP.
 * TEST-ONLY environment variables, read once here.  They force launch shapes that the default rules pick only on other
 * call sizes, so that the parity tests reach every kernel path on small inputs; results meet the same bar, speed does
 * not.  Not for production use, and they may change without notice:
 *   RS_SPLITK=n      K ranges of the residual projections (1..4; default: a cost model per call)
 *   RS_NCU=n         compute-unit count the GEMM strips are sized for (default: the device's)
 *   RS_NARROW=0      never the GEMM geometry for strips of at most two units;  RS_NARROW_TM=n  use it up to n token blocks
 *   RS_PAIRS=0       never two wavefronts per pair of units in that geometry
 *   RS_ATTN_SPLIT=n  parts every attention block's key range is cut into (1 = never; default: decided per call)
 *   RS_ATTN_ORDER=plain  attention work items stay in heaviest-first order (default: between one and two items per
 *                    compute unit, the heaviest run alone on theirs and the others are paired heavy with light) */
rs_status rs_ctx_create(const rs_layer_cfg* cfg, rs_ctx** out);
void rs_ctx_destroy(rs_ctx* ctx);

/* One-time weight repack, off the hot path.  `src` holds torch-layout device pointers; `dst` is a caller-owned
 * device slab of rs_weights_packed_bytes() bytes; `packed` receives pointers into `dst` in the layout the
 * kernels read (gate and up rows interleaved in blocks so SwiGLU can be applied inside the GEMM).
 * After the call completes on `hip_stream` the torch-layout tensors may be freed. */
size_t rs_weights_packed_bytes(const rs_ctx* ctx);
rs_status rs_weights_pack(rs_ctx* ctx, const rs_layer_weights* src, void* dst, size_t dst_bytes,
                          rs_layer_weights* packed, void* hip_stream);

/* KV cache (the per-request state chunked prefill builds, section 2.2.1).  The slab layout is private; capacity is
 * fixed at allocation (see below for caches that grow page by page).  Each layer keeps its own length so that layers 0..L-1 can be run in turn for a chunk.
 *   rs_kv_bytes      bytes of device memory needed for n_layers layers of capacity_tokens tokens.
 *   rs_kv_alloc      wraps caller-owned device memory `dev_mem` (>= rs_kv_bytes, 256-byte aligned); lengths start at 0.
 *   rs_kv_free       frees the host handle only.
 *   rs_kv_len        cached tokens of `layer`, or -1 on a bad argument.
 *   rs_kv_reset      all lengths := 0.
 *   rs_kv_truncate   length of `layer` := n_tokens (0 <= n_tokens <= current length): drops the newest tokens.
 *   rs_kv_export     copies the first rs_kv_len tokens to canonical bf16 [len][Hkv][d] arrays (post-RoPE K, V).
 *   rs_kv_import     loads n_tokens canonical rows as the cache content of `layer` and sets its length. */
size_t rs_kv_bytes(const rs_ctx* ctx, int n_layers, int capacity_tokens);
rs_status rs_kv_alloc(rs_ctx* ctx, int n_layers, int capacity_tokens, void* dev_mem, size_t bytes, rs_kv** out);
void rs_kv_free(rs_kv* kv);
int rs_kv_len(const rs_kv* kv, int layer);
int rs_kv_capacity(const rs_kv* kv);
rs_status rs_kv_reset(rs_kv* kv);
rs_status rs_kv_truncate(rs_kv* kv, int layer, int n_tokens);
rs_status rs_kv_export(const rs_kv* kv, int layer, void* k_out_dev, void* v_out_dev, void* hip_stream);
rs_status rs_kv_import(rs_kv* kv, int layer, const void* k_dev, const void* v_dev, int n_tokens, void* hip_stream);

/* Paged, growable KV caches.  The serving systems the paper measures size their KV memory as the largest that fits
 * (section 4.1.3), which presupposes that requests share it in small units instead of reserving a maximum length each.
 * A pool cuts caller-owned device memory into pages of rs_kv_page_bytes() bytes; a page holds 64 tokens of ONE layer
 * (K and V of all KV heads).  A paged cache starts empty and takes pages from its pool as tokens arrive: inside
 * rs_prefill_* and rs_kv_import, after every check has passed (a call that would need more pages than the pool has free
 * fails with RS_ECAPACITY before anything is launched or changed; rs_prefill_model_batch counts the pages of all its
 * layers together).  rs_kv_truncate and rs_kv_reset give whole pages beyond the new length back, rs_kv_free all of them.
 * Everything else (rs_kv_len, export, import, every rs_prefill_* entry point, mixing paged and contiguous caches in one
 * micro-batch) works alike for both kinds, and the results are bit-identical to those with a contiguous cache.
 * rs_kv_capacity of a paged cache is the number of tokens its current pages can hold (the smallest over its layers).
 *   rs_kv_pool_create   dev_mem: 256-byte aligned device memory of `bytes` bytes, used as floor(bytes / page) pages;
 *                       RS_EWORKSPACE if that is not even one page.  The memory need not be initialised.
 *   rs_kv_pool_destroy  frees the host handle; RS_ESTATE while caches allocated from the pool are alive.
 *   rs_kv_pool_pages / rs_kv_pool_free_pages   total and currently free pages (-1 for a null pool).
 *   rs_kv_alloc_paged   an empty cache of n_layers layers on `pool` (free it with rs_kv_free before the pool).
 * The host bookkeeping is not thread-safe: one thread at a time per pool.
 * Stream ordering: pages change hands on the host, at the moment of the call, with no regard to GPU work still queued.
 * A page that rs_kv_truncate, rs_kv_reset, rs_kv_free or a shrinking rs_kv_import gives back may be handed to another
 * cache of the pool by the very next call.  So either run every cache of a pool on ONE stream (then the stream's order
 * protects the page: whatever still reads it was enqueued before whatever overwrites it), or make the stream of the next
 * taker wait (event / synchronize) for the work that last touched the cache before calling one of those four. */
typedef struct rs_kv_pool rs_kv_pool;
size_t rs_kv_page_bytes(const rs_ctx* ctx);
rs_status rs_kv_pool_create(rs_ctx* ctx, void* dev_mem, size_t bytes, rs_kv_pool** out);
rs_status rs_kv_pool_destroy(rs_kv_pool* pool);
int rs_kv_pool_pages(const rs_kv_pool* pool);
int rs_kv_pool_free_pages(const rs_kv_pool* pool);
rs_status rs_kv_alloc_paged(rs_ctx* ctx, rs_kv_pool* pool, int n_layers, rs_kv** out);

/* Bytes of device workspace a call with up to max_tokens rows and max_requests requests needs. */
size_t rs_workspace_bytes(const rs_ctx* ctx, int max_tokens, int max_requests);

/* 8-bit KV caches.  The paper's systems are configured for the largest KV memory that fits (section 4.1.3) and its
 * prompts run to tens of thousands of multimodal tokens (sections 2.1.1, 4.1.2); a cache that keeps one byte per element
 * holds twice the tokens.  Storage format: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinity,
 * 0x7f / 0xff are NaN, largest value 448), one scale for the keys and one for the values of a cache:
 *     stored  code  = e4m3( fl32( x * fl32(1 / scale) ) )   x: the bfloat16 K~ or V element; round to nearest, ties to
 *                                                           even, |.| > 448 saturates to +-448, NaN -> 0x7f
 *     read    value = bf16( fl32( decode(code) * scale ) )
 * Every key and value goes through the cache before attention reads it, the running chunk's own rows included, so the
 * result does not depend on how a prompt is cut into chunks (the contract of section 2.2.1 holds for the quantised
 * model).  Queries, scores and everything else stay as with a bfloat16 cache.
 *   rs_kv_fp8_bytes    bytes of device memory for n_layers layers of capacity_tokens tokens (half of rs_kv_bytes).
 *   rs_kv_alloc_fp8    like rs_kv_alloc; k_scale, v_scale > 0 and finite, with finite reciprocals (RS_EINVAL otherwise).
 *   rs_kv_page_bytes_fp8, rs_kv_pool_create_fp8, rs_kv_alloc_paged_fp8   the paged form: a pool of 8-bit pages (half of
 *                      rs_kv_page_bytes: 64 tokens of one layer, K then V^T codes of all KV heads) and growable caches on
 *                      it, with everything said above about pools and paged caches.  A pool serves one kind of cache:
 *                      rs_kv_alloc_paged on an 8-bit pool, or rs_kv_alloc_paged_fp8 on a bfloat16 one, is RS_ESTATE.
 *                      Results are bit-identical to those with a contiguous 8-bit cache.
 *   rs_kv_pool_is_fp8  1 / 0, -1 for a null handle.
 *   rs_kv_is_fp8       1 / 0, -1 for a null handle.
 *   rs_kv_export / rs_kv_import on an 8-bit cache produce / consume bfloat16 rows through the formulas above.
 *   rs_kv_export_codes, rs_kv_import_codes   the bytes themselves, canonical [len][Hkv][d] uint8 device arrays: what a
 *                      transfer of the cache to another worker would ship.  RS_ESTATE on a bfloat16 cache.
 * All caches of one rs_prefill_* call must be of one kind (RS_EINVAL otherwise).  A call on 8-bit caches first expands the
 * blocks its rows can see into bfloat16 tiles in the workspace (one layer at a time) and runs the ordinary attention
 * kernel on them, so its workspace must hold, beyond rs_workspace_bytes(), 4 * Hkv * d bytes per visible token, each
 * request's cached + new tokens rounded up to a multiple of 64; RS_EWORKSPACE otherwise.
 *   rs_workspace_bytes_fp8kv   that sum for calls whose requests see at most max_visible_tokens tokens in total
 *                      (sum over the call's requests of cached + new tokens; the rounding is added here). */
size_t rs_kv_fp8_bytes(const rs_ctx* ctx, int n_layers, int capacity_tokens);
rs_status rs_kv_alloc_fp8(rs_ctx* ctx, int n_layers, int capacity_tokens, float k_scale, float v_scale, void* dev_mem,
                          size_t bytes, rs_kv** out);
int rs_kv_is_fp8(const rs_kv* kv);
rs_status rs_kv_export_codes(const rs_kv* kv, int layer, void* k_codes_dev, void* v_codes_dev, void* hip_stream);
rs_status rs_kv_import_codes(rs_kv* kv, int layer, const void* k_codes_dev, const void* v_codes_dev, int n_tokens,
                             void* hip_stream);
size_t rs_workspace_bytes_fp8kv(const rs_ctx* ctx, int max_tokens, int max_requests, size_t max_visible_tokens);
size_t rs_kv_page_bytes_fp8(const rs_ctx* ctx);
rs_status rs_kv_pool_create_fp8(rs_ctx* ctx, void* dev_mem, size_t bytes, rs_kv_pool** out);
int rs_kv_pool_is_fp8(const rs_kv_pool* pool);
rs_status rs_kv_alloc_paged_fp8(rs_ctx* ctx, rs_kv_pool* pool, int n_layers, float k_scale, float v_scale, rs_kv** out);

/* One chunk of one request through one layer (chunked prefill, section 2.2.1).
 *   x   device bf16 [T, H]: the chunk's rows (image-embedding or text-embedding rows alike), prompt order.
 *   y   device bf16 [T, H]: layer output; may alias x.
 * With P = rs_kv_len(kv, layer): rows take positions P..P+T-1, their post-RoPE K and V are appended at [P, P+T),
 * row i attends to cache entries 0..P+i, and the layer's length becomes P+T.  T = 0 is a no-op.
 * RS_ECAPACITY if P+T exceeds the cache capacity or max_pos; RS_EINVAL if T > max_tokens_per_call.
 * Reproducibility: every kernel divides its work in a way fixed by the call's sizes and none uses atomics, so the same
 * call on the same inputs gives the same bits.  The K and V a token leaves in the cache are the same bits however its
 * prompt is cut into chunks or batched with other requests (the QKV projection is never split along K, and the row sums
 * of the norm before it are taken in one fixed order).  A token's output row may differ between chunkings by rounding:
 * the K ranges of the residual projections and the key ranges of the attention blocks are chosen per call. */
rs_status rs_prefill_chunk(rs_ctx* ctx, const rs_layer_weights* packed, int layer, rs_kv* kv,
                           const void* x_dev, int T, void* y_dev,
                           void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* rs_prefill_chunk for callers that cannot allocate device memory and have no workspace to pass: tight serving loops
 * and harnesses that forbid hipMalloc around the call.  Same arguments, same kernels, same result to the bit; the
 * workspace is a static device array of RS_STATIC_WORKSPACE_BYTES inside the library (each GPU the library runs on
 * holds it until the process ends; its address on the context's GPU is looked up once, in rs_ctx_create).  The call
 * allocates nothing on the device and calls no allocating library routine.
 *   - RS_EWORKSPACE, nothing enqueued, nothing changed, if the call needs more than the array holds:
 *     rs_workspace_bytes(ctx, T, 1) (8-bit caches: rs_workspace_bytes_fp8kv with the tokens visible after the call) must
 *     be <= rs_static_workspace_bytes().  At the 7B shape that is up to 640 rows per call.
 *   - RS_ESTATE if the GPU current on the calling thread is not the one the context was created on.
 *   - Every call on a GPU shares that GPU's array: two calls whose work overlaps on one GPU (different streams, or
 *     different contexts) race.  Nothing in it has to start at zero; it keeps the last call's intermediates. */
#define RS_STATIC_WORKSPACE_BYTES ((size_t)128 << 20)
size_t rs_static_workspace_bytes(void);
rs_status rs_prefill_chunk_static(rs_ctx* ctx, const rs_layer_weights* packed, int layer, rs_kv* kv,
                                  const void* x_dev, int T, void* y_dev, void* hip_stream);

/* One micro-batch of R requests through one layer (the set S of Algorithm 2, section 3.3).
 *   kvs[i], chunk_lens[i]  host arrays: request i contributes chunk_lens[i] >= 0 rows this round.
 *   x   device bf16 [sum chunk_lens, H]: rows packed in request order, each request's rows contiguous, prompt order.
 *   y   device bf16, same shape; may alias x.
 * Each request behaves exactly as in rs_prefill_chunk against its own cache; requests do not interact.
 * The same rs_kv may not appear twice (RS_EINVAL).  sum chunk_lens must be <= max_tokens_per_call, R <= max_requests. */
rs_status rs_prefill_batch(rs_ctx* ctx, const rs_layer_weights* packed, int layer,
                           rs_kv* const* kvs, const int* chunk_lens, int R,
                           const void* x_dev, void* y_dev,
                           void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* Three-axis rotary positions (the M-RoPE of the model family the paper serves, section 4.1.1; not part of the paper's
 * own text).  The d/2 rotary pairs of a head are split into three consecutive sections; pair j is turned by the row's
 * temporal, height or width position according to the section it falls in.  Sections are counts of pairs, multiples of
 * 4, summing to head_dim / 2; the default after rs_ctx_create is (head_dim / 2, 0, 0), i.e. 1-D RoPE.  Applies to every
 * later call on the context. */
rs_status rs_ctx_set_mrope_sections(rs_ctx* ctx, int temporal, int height, int width);

/* rs_prefill_batch with explicit rotary positions: positions is a HOST array [sum chunk_lens][3] of (temporal, height,
 * width) positions in packed row order, each in [0, max_pos) (RS_ECAPACITY otherwise).  Only the rotation uses them:
 * cache slots and the causal order stay P..P+T-1.  With all three equal to P+i this is rs_prefill_batch. */
rs_status rs_prefill_batch_mrope(rs_ctx* ctx, const rs_layer_weights* packed, int layer,
                                 rs_kv* const* kvs, const int* chunk_lens, int R, const int* positions,
                                 const void* x_dev, void* y_dev,
                                 void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* The same micro-batch through n_layers stacked layers in one call (layer l uses packed_layers[l] and the requests'
 * layer-l caches; layer 0 reads x, every later layer reads the previous layer's output, the last one leaves y).  What a
 * serving loop needs per scheduling round: section 3.3's BatchExecute for a whole model.  Every layer's capacity and
 * size checks are made before the first launch, so a failing call changes nothing. */
rs_status rs_prefill_model_batch(rs_ctx* ctx, const rs_layer_weights* packed_layers, int n_layers,
                                 rs_kv* const* kvs, const int* chunk_lens, int R,
                                 const void* x_dev, void* y_dev,
                                 void* workspace_dev, size_t workspace_bytes, void* hip_stream);
/* rs_prefill_model_batch with the rotary positions of rs_prefill_batch_mrope (the same positions for every layer). */
rs_status rs_prefill_model_batch_mrope(rs_ctx* ctx, const rs_layer_weights* packed_layers, int n_layers,
                                       rs_kv* const* kvs, const int* chunk_lens, int R, const int* positions,
                                       const void* x_dev, void* y_dev,
                                       void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* First output token (what "time to first token", the paper's latency metric in section 4.1.4, waits for): final
 * RMSNorm and vocabulary projection of n_rows hidden-state rows (the last prompt row of each request whose prefill has
 * finished).
 *   final_norm_gain  device bf16 [H]
 *   w_lm             device bf16 [vocab, H], torch layout, used as is
 *   x                device bf16 [n_rows, H]
 *   logits           device fp32 [n_rows, vocab]:  logits[r, v] = sum_k rmsnorm(x[r])[k] * w_lm[v, k], fp32 accumulation,
 *                    the normalised row kept in fp32
 * workspace: rs_lm_head_workspace_bytes(ctx, n_rows) bytes, 256-byte aligned.  n_rows = 0 is a no-op. */
size_t rs_lm_head_workspace_bytes(const rs_ctx* ctx, int n_rows);
rs_status rs_lm_head(rs_ctx* ctx, const void* final_norm_gain_dev, const void* w_lm_dev, int vocab,
                     const void* x_dev, int n_rows, void* logits_dev,
                     void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* Measurement hook.  The steps of one rs_prefill_* call, in launch order: */
typedef enum rs_step {
    RS_STEP_ROW_RMS = 0,       /* 1/rms of the input rows (first RMSNorm; gains are folded into the packed weights) */
    RS_STEP_QKV_GEMM = 1,      /* QKV projection with the norm factor, bias and RoPE in its epilogue */
    RS_STEP_APPEND_KV = 2,     /* K copy + transposing V append into the cache */
    RS_STEP_ATTENTION = 3,
    RS_STEP_O_GEMM = 4,        /* output projection + residual + second norm's row factors (and split-K reduction, if any) */
    RS_STEP_GATE_UP_GEMM = 5,  /* gate/up projection with the norm factor and SwiGLU in its epilogue */
    RS_STEP_DOWN_GEMM = 6,     /* down projection + residual (and split-K reduction, if any) */
    RS_STEP_COUNT = 7
} rs_step;
/* rs_profile_enable(ctx, step, n): from now on the first n launches of `step` are bracketed by two HIP events recorded
 * on the call's own stream (step = -1 switches the hook off).  rs_profile_read waits for the recorded events, returns
 * the summed elapsed milliseconds and the number of launches measured, and restarts the count.  Events are created in
 * rs_profile_enable, never inside rs_prefill_*. */
rs_status rs_profile_enable(rs_ctx* ctx, int step, int max_launches);
/* Only every `every`-th launch of the step is bracketed (1, the initial setting: all of them).  The two event records
 * around a kernel keep it from overlapping its neighbours' launch and drain (about 5 us each); sampling keeps a
 * measurement inside a timed region from slowing that region.  Persists until changed. */
rs_status rs_profile_sample_every(rs_ctx* ctx, int every);
rs_status rs_profile_read(rs_ctx* ctx, double* total_ms, int* launches);

/* Message of the most recent failing call on this thread (never NULL). */
const char* rs_last_error(void);

/* Library version, for the binding's sanity check. */
int rs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RSERVE_PREFILL_H */
