// Host side of the C ABI declared in include/rserve_prefill.h: argument checks, per-call descriptors and the
// kernel sequence of one decoder layer over one chunk / micro-batch.  All device work goes to the caller's stream.
#include "../../include/rserve_prefill.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "attention.h"
#include "common.h"
#include "elementwise.h"
#include "kv_fp8.h"
#include "gemm_strip.h"
#include "last_error.h"

namespace {

thread_local std::string g_last_error = "";

void set_last_error(const char* fmt, va_list ap) {
    char buf[512];
    vsnprintf(buf, sizeof(buf), fmt, ap);
    g_last_error = buf;
}

rs_status fail(rs_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    set_last_error(fmt, ap);
    va_end(ap);
    return st;
}

#define RS_HIP(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail(RS_EHIP, "%s: %s", #expr, hipGetErrorString(e_));       \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr int RING_SLOTS = 32;
constexpr int RING_CHECKPOINT = 8;

// Workspace of rs_prefill_chunk_static.  In host code the array's name is only a handle for hipGetSymbolAddress: each GPU
// holds its own copy at its own address, which static_workspace_lookup fetches once per device (with that device
// current) and every later use goes through.
static __device__ __align__(256) unsigned char g_static_workspace[RS_STATIC_WORKSPACE_BYTES];
constexpr int MAX_DEVICES = 64;
void* g_static_workspace_addr[MAX_DEVICES] = {};   // per device; written under g_static_workspace_mutex
std::mutex g_static_workspace_mutex;

// The address of the current device's copy of the array (the device must be `dev`); looked up on first use.
hipError_t static_workspace_lookup(int dev, void** out) {
    std::lock_guard<std::mutex> lock(g_static_workspace_mutex);
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_static_workspace_addr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_workspace));
        if (e != hipSuccess) return e;
        g_static_workspace_addr[dev] = p;
    }
    *out = g_static_workspace_addr[dev];
    return hipSuccess;
}

}  // namespace

rs_status rs_internal_fail(rs_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    set_last_error(fmt, ap);
    va_end(ap);
    return st;
}

struct rs_ctx {
    rs_layer_cfg cfg;
    int qkv_dim, q_dim, kv_dim, group;
    float2* rope_dev = nullptr;  // [max_pos][d/2] (cos, sin)
    // pinned staging ring for per-call descriptors
    char* pinned[RING_SLOTS] = {};
    char* pinned_dev[RING_SLOTS] = {};  // the same buffers as the device addresses them
    // A slot may be overwritten once the first kernel of the call that used it has run.  Recording an event behind that
    // kernel in every call would tell, but an event record holds the stream up for about 6 us; so events are recorded only
    // at checkpoints: after every RING_CHECKPOINT-th use, and - on the stream that is being left - whenever the caller's
    // stream changes.  Uses are numbered; the first checkpoint at or after use u is on u's stream and behind its kernel.
    hipEvent_t slot_done[RING_SLOTS] = {};
    long slot_recorded_at[RING_SLOTS];   // the use number slot_done[slot] was last recorded at (-1: never)
    size_t slot_bytes = 0;
    long use_count = 0;                   // uses so far; use u occupies slot u % RING_SLOTS
    hipStream_t last_stream = nullptr;
    int splitk_override = 0;  // RS_SPLITK environment variable (0 = heuristic)
    int mrope_b0 = 0, mrope_b1 = 0;  // rotary pair j turns with axis 0 below b0, axis 1 below b1, axis 2 above (set in rs_ctx_create)
    int attn_plain_order = 0; // RS_ATTN_ORDER=plain: attention items stay heaviest-first (no pairing by compute unit)
    int attn_split = 0;       // RS_ATTN_SPLIT environment variable: parts a block's key range is cut into (0: decided per call)
    int gemm_pairs = 1;       // RS_PAIRS environment variable: 0 never lets two wavefronts of a GEMM workgroup split a pair of units
    int gemm_narrow = 1;      // RS_NARROW environment variable: 0 never uses the narrow GEMM geometry; otherwise launches of at most
    int narrow_max_tiles_m = 1;  // narrow_max_tiles_m (RS_NARROW_TM) token blocks whose strips would hold at most 2 units use it
    int n_cu = 256;           // compute units of the device: the number of strips a GEMM launch is cut into
    bool has_device = false;  // false: created on a host without a GPU; argument checks work, launches return RS_EHIP
    int device = -1;          // the GPU that was current in rs_ctx_create
    void* static_ws = nullptr;  // that GPU's copy of the static workspace (rs_prefill_chunk_static)
    int lm_rows = 0;          // rows per launch of the first-token head (0: its LDS size not yet set, see rs_lm_head)
    // measurement hook: HIP events around every launch of one step of the layer
    int prof_step = -1;
    int prof_count = 0;
    int prof_every = 1;       // measure every n-th launch of the step
    int prof_seen = 0;        // launches of the step seen since rs_profile_enable
    bool prof_take = false;   // the launch in progress is being measured
    std::vector<hipEvent_t> prof_events;  // (start, stop) pairs
};

// A pool of fixed-size pages in caller-owned device memory.  A page holds 64 tokens of ONE layer: the K tiles [64][d] of
// all KV heads followed by their V^T tiles [d][64].  The free list lives on the host.
struct rs_kv_pool {
    rs_ctx* ctx;
    char* base;
    size_t page_bytes;
    int n_pages;
    bool fp8 = false;              // pages of E4M3 bytes (half the size) for 8-bit caches
    int n_caches = 0;              // paged caches alive on this pool
    std::vector<int> free_pages;   // stack: the back is handed out next
};

struct rs_kv {
    rs_ctx* ctx;
    int n_layers;
    int cap;  // contiguous: capacity in tokens, multiple of 64; paged: unused (see capacity())
    char* base;
    size_t k_bytes;      // one layer's K
    size_t layer_bytes;  // K + V^T
    std::vector<int> len;
    rs_kv_pool* pool = nullptr;             // paged caches only
    std::vector<std::vector<int>> pages;    // paged: pages[layer][block]
    bool fp8 = false;                       // one E4M3 byte per element (contiguous caches only); k_bytes counts bytes
    float k_scale = 1.0f, v_scale = 1.0f;   // 8-bit caches: value = decode(code) * scale
    bool paged() const { return pool != nullptr; }
    uint8_t* kc_of(int layer) const { return reinterpret_cast<uint8_t*>(base + (size_t)layer * layer_bytes); }
    uint8_t* vc_of(int layer) const { return reinterpret_cast<uint8_t*>(base + (size_t)layer * layer_bytes + k_bytes); }
    bf16* k_of(int layer) const { return reinterpret_cast<bf16*>(base + (size_t)layer * layer_bytes); }
    bf16* vt_of(int layer) const { return reinterpret_cast<bf16*>(base + (size_t)layer * layer_bytes + k_bytes); }
    // new pages layer `layer` needs before it can hold n_tokens
    int pages_missing(int layer, long n_tokens) const {
        return paged() ? std::max<long>(0, (n_tokens + 63) / 64 - (long)pages[layer].size()) : 0;
    }
    void take_pages(int layer, long n_tokens) {  // the caller has checked that the pool has enough
        for (int k = pages_missing(layer, n_tokens); k > 0; --k) {
            pages[layer].push_back(pool->free_pages.back());
            pool->free_pages.pop_back();
        }
    }
    void give_back_pages(int layer, long n_tokens) {  // keeps the pages that hold the first n_tokens
        const size_t keep = (size_t)((n_tokens + 63) / 64);
        while (pages[layer].size() > keep) {
            pool->free_pages.push_back(pages[layer].back());
            pages[layer].pop_back();
        }
    }
    // the cache of `layer` as the kernels see it (row0 / T / P left to the caller; `pages` is a device pointer or a marker)
    ReqDesc view(int layer, const int* dev_pages) const {
        ReqDesc d{};
        d.cap = cap;
        d.hkv = ctx->cfg.n_kv_heads;
        if (paged()) {
            d.kcache = reinterpret_cast<bf16*>(pool->base);
            d.pages = dev_pages;
        } else {
            d.kcache = k_of(layer);
            d.vtcache = vt_of(layer);
        }
        return d;
    }
};

namespace {

struct DescSizes {
    size_t reqs, items, vblocks, rowpos, pagetab, mitems, fp8, total;
};

constexpr int ATT_MIN_PART_TILES = 8;      // a part is worth a workgroup and its share of the merge from about 500 keys
constexpr int ATT_MIN_SPLIT_TILES = 16;    // no block of the call is split unless the longest walks at least 1024 keys
// slots of the split buffer: blocks are split only when there are fewer of them than compute units, into about two
// workgroups per unit in total (sized for the 256 units of an MI355X; a block that finds no free slots stays whole)
size_t attn_split_slots(const rs_ctx*) { return 768; }

DescSizes desc_sizes(const rs_ctx* c, int max_tokens, int max_requests) {
    DescSizes d;
    const size_t n_items = ((size_t)(max_tokens * (size_t)c->group + ATT_ROWS - 1) / ATT_ROWS + max_requests) * c->cfg.n_kv_heads +
                           attn_split_slots(c);
    const size_t n_vb = (size_t)max_tokens / 64 + 2 * (size_t)max_requests + 1;
    d.reqs = align_up(sizeof(ReqDesc) * std::max(max_requests, 1), 256);
    d.items = align_up(sizeof(AttnItem) * n_items, 256);
    d.vblocks = align_up(sizeof(KVBlockItem) * n_vb, 256);
    d.rowpos = align_up(3 * sizeof(int) * (size_t)std::max(max_tokens, 1), 256);  // (temporal, height, width) per row
    // block -> page numbers of the paged caches in the call: at most max_pos / 64 + 1 blocks per request
    d.pagetab = align_up(sizeof(int) * (size_t)std::max(max_requests, 1) * ((size_t)c->cfg.max_pos / 64 + 2), 256);
    d.mitems = align_up(sizeof(AttnMergeItem) * attn_split_slots(c), 256);
    d.fp8 = align_up(sizeof(Fp8CacheDesc) * std::max(max_requests, 1), 256);
    d.total = d.reqs + d.items + d.vblocks + d.rowpos + d.pagetab + d.mitems + d.fp8;
    return d;
}

// Strips per 256-row block of a GEMM with `units` 32-feature units: one workgroup per compute unit when there is enough
// width, never more strips than units.
int strips_for(const rs_ctx* c, int tiles_m, int splits, int units) {
    return std::max(1, std::min(units, c->n_cu / std::max(1, tiles_m * splits)));
}

// Whether a launch qualifies for the narrow kernel geometry: few token blocks, no strip wider than the narrow tile.
bool use_narrow(const rs_ctx* c, int tiles_m, int splits, int units, int max_tiles_m = 0) {
    if (!c->gemm_narrow || tiles_m > std::max(max_tiles_m, c->narrow_max_tiles_m)) return false;
    const int strips = strips_for(c, tiles_m, splits, units);
    return (units + strips - 1) / strips <= GS_NARROW_NT;
}

// Estimated duration (shader clocks) of a residual GEMM cut into `splits` K ranges.  Constants fitted to measurements
// on MI355X: a step of K = 64 costs 256 clocks of matrix-pipe issue per unit plus about 350 of barrier and issue overhead,
// a tile about 20000 for pipeline fill and epilogue, and the reduction kernel moves its bytes at about 2 TB/s.
double gemm_cost_clocks(const rs_ctx* c, int M, int units, int k_steps, int splits) {
    const int tiles_m = (M + GS_BM - 1) / GS_BM;
    const int strips = strips_for(c, tiles_m, splits, units);
    const int waves = (tiles_m * strips * splits + c->n_cu - 1) / c->n_cu;  // rounds of workgroups over the chip
    const int ups = (units + strips - 1) / strips;
    const int ntiles = (ups + GS_MAX_NT - 1) / GS_MAX_NT;
    const double nt = (double)ups / ntiles;
    const int steps = (k_steps + splits - 1) / splits;
    // (a step of the wide geometry also moves 32 KB of token fragments per workgroup whatever the tile's width: with three
    // units or fewer that, not the MFMAs, sets its duration - about 1200 clocks measured; without this floor calls of 257
    // to 768 rows kept the O projection unsplit, 3 to 8 us slower than in two or three K ranges)
    double step = 256.0 * nt + 350.0;
    if (!use_narrow(c, tiles_m, splits, units)) step = std::max(step, 1200.0);
    double clocks = (double)waves * ntiles * (steps * step + 20000.0);
    if (splits > 1) clocks += (double)M * units * 32.0 * (4.0 * splits + 4.0) / 2.0e12 * 1.4e9;
    return clocks;
}

int choose_splitk(const rs_ctx* c, int M, int units, int k_steps) {
    if (c->splitk_override > 0) return std::min(std::min(c->splitk_override, 4), std::max(1, k_steps));  // (the workspace holds 4 planes)
    int best = 1;
    double best_cost = gemm_cost_clocks(c, M, units, k_steps, 1);
    for (int s = 2; s <= 4 && k_steps / s >= 8; ++s) {
        const double cost = gemm_cost_clocks(c, M, units, k_steps, s);
        if (cost < 0.97 * best_cost) {
            best = s;
            best_cost = cost;
        }
    }
    return best;
}

struct WorkspaceLayout {
    size_t qkv, xf, attn, r, act, partial, attn_split, inv_rms1, inv_rms2, rowss, desc, total;
};

WorkspaceLayout ws_layout(const rs_ctx* c, int T, int R) {
    const rs_layer_cfg& f = c->cfg;
    WorkspaceLayout w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    const size_t t = (size_t)std::max(T, 1);
    const size_t tp = align_up(t, 32);  // fragment-major buffers hold whole blocks of 32 tokens
    w.qkv = take(t * c->qkv_dim * 2);
    w.xf = take(tp * f.hidden * 2);
    w.attn = take(tp * c->q_dim * 2);
    w.r = take(tp * f.hidden * 2);
    w.act = take(tp * f.mlp_inter * 2);
    w.partial = take(4 * t * f.hidden * 4);  // up to 4 split-K partial planes of [T, H] fp32
    w.attn_split = take(attn_split_slots(c) * (size_t)ATT_ROWS * (f.head_dim + 2) * 4);  // partial results of split key ranges
    w.inv_rms1 = take(tp * 4);
    w.inv_rms2 = take(tp * 4);
    w.rowss = take(tp * (f.hidden / 32) * 4);
    w.desc = take(desc_sizes(c, T, R).total);
    w.total = off;
    return w;
}

// bytes of the bfloat16 copy of an 8-bit cache's first n_tokens (whole 64-token blocks, K and V^T of all KV heads)
size_t fp8_expansion_bytes(const rs_ctx* c, long n_tokens) {
    return (size_t)2 * align_up((size_t)n_tokens, 64) * c->kv_dim * 2;
}

// *columns_out (optional) receives the number of workgroup columns of the launch: strips times the wavefronts that split a
// strip's units, i.e. the number of parts the residual epilogue leaves in GemmArgs::rowss.
template <int EPI>
rs_status launch_gemm(const rs_ctx* c, GemmArgs a, int splits, hipStream_t st, int* columns_out = nullptr) {
    a.tiles_m = (a.M + GS_BM - 1) / GS_BM;
    const int units = a.N / 32;
    const int steps = a.K / GS_BK;
    a.steps_per_split = (steps + splits - 1) / splits;
    splits = (steps + a.steps_per_split - 1) / a.steps_per_split;  // no empty K range
    // A call of 129 to 256 rows whose strips would hold one pair of units each: blocks of 128 rows, two wavefronts along
    // the rows and two along the pair (16 KB of token fragments per step and workgroup instead of 32; measured: QKV 40 -> 35
    // us at 256 rows; up to 128 rows, where half the wavefronts of a 256-row block idle anyway, it is slower).
    if (c->gemm_narrow && c->gemm_pairs && a.M > GS_BM / 2 && a.M <= GS_BM && units % 2 == 0) {
        const int tiles_m = (a.M + GS_BM / 2 - 1) / (GS_BM / 2);
        const int strips = strips_for(c, tiles_m, splits, units / 2);
        if (strips == units / 2) {
            a.tiles_m = tiles_m;
            a.strips = strips;
            if (columns_out) *columns_out = 2 * strips;
            hipLaunchKernelGGL((gemm_strip_kernel<EPI, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD, 2>), dim3(tiles_m * strips, splits),
                               dim3(256), GS_NARROW_LDS_BYTES, st, a);
            RS_HIP(hipGetLastError());
            return RS_OK;
        }
    }
    a.strips = strips_for(c, a.tiles_m, splits, units);
    if (columns_out) *columns_out = a.strips;
    dim3 grid(a.tiles_m * a.strips, splits);
    // (the QKV projection, which is never split along K, also takes the narrow geometry on two token blocks: 43 -> 38 us
    // at 320 rows, no change at 512; the residual projections of such calls are better off split along K in the wide one)
    if (use_narrow(c, a.tiles_m, splits, units, EPI == EPI_QKV_ROPE ? 2 : 0))
        hipLaunchKernelGGL((gemm_strip_kernel<EPI, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD>), grid, dim3(256),
                           GS_NARROW_LDS_BYTES, st, a);
    else
        hipLaunchKernelGGL(gemm_strip_kernel<EPI>, grid, dim3(256), GS_LDS_BYTES, st, a);
    RS_HIP(hipGetLastError());
    return RS_OK;
}

// out = resid + X W^T, through split-K partials when the unsplit launch would leave compute units idle.  X is fragment-
// major; resid and out are row-major or fragment-major as flagged.  When inv_rms_out is given, the RMSNorm factor of the
// next GEMM's input, rsqrt(mean(out[m,:]^2) + eps) per row, is prepared in one of two forms: the split-K reduction writes
// it to inv_rms_out (*rowss_parts_out = 0); an unsplit launch leaves *rowss_parts_out > 0 partial sums of squares per row
// in rowss, which the next GEMM closes itself (GemmArgs::rowss).
// With `defer` (the layers of one rs_prefill_model_batch call) a split-K launch leaves its reduction to the next layer's
// first kernel: *defer then describes the pending sum (splits > 0) and `out` has not been written yet.
struct PendingReduce {
    int splits = 0;             // 0: nothing pending
    const float* partial = nullptr;
    const bf16* resid = nullptr;   // fragment-major
    bf16* out = nullptr;           // row-major
};
rs_status gemm_residual(const rs_ctx* c, const bf16* X, const bf16* W, const bf16* resid, int resid_frag, bf16* out,
                        int out_frag, int M, int N, int K, float* partial, float* inv_rms_out, float* rowss, int* rowss_parts_out,
                        hipStream_t st, PendingReduce* defer = nullptr) {
    GemmArgs a{};
    a.X = X; a.W = W; a.out = out; a.ldo = N; a.out_frag = out_frag; a.resid = resid; a.ldr = N; a.resid_frag = resid_frag;
    a.partial = partial;
    a.M = M; a.N = N; a.K = K;
    const float eps = c->cfg.rms_eps;
    int splits = choose_splitk(c, M, N / 32, K / GS_BK);
    if (splits > 1) {
        const int sps = (K / GS_BK + splits - 1) / splits;
        splits = (K / GS_BK + sps - 1) / sps;
    }
    if (rowss_parts_out) *rowss_parts_out = 0;
    if (splits == 1) {
        a.rowss = inv_rms_out ? rowss : nullptr;
        return launch_gemm<EPI_RESIDUAL>(c, a, 1, st, inv_rms_out ? rowss_parts_out : nullptr);
    }
    rs_status s = launch_gemm<EPI_PARTIAL>(c, a, splits, st);
    if (s != RS_OK) return s;
    if (defer && resid_frag && !out_frag && !inv_rms_out) {
        defer->splits = splits; defer->partial = partial; defer->resid = resid; defer->out = out;
        return RS_OK;
    }
    if (M <= 512)  // few rows: a workgroup per row instead of per four
        hipLaunchKernelGGL(splitk_reduce_residual_kernel<4>, dim3(M), dim3(256), 0, st, (const float*)partial, splits, resid, N,
                           resid_frag, out, N, out_frag, M, N, inv_rms_out, eps);
    else
        hipLaunchKernelGGL(splitk_reduce_residual_kernel<1>, dim3((M + 3) / 4), dim3(256), 0, st, (const float*)partial, splits, resid, N,
                           resid_frag, out, N, out_frag, M, N, inv_rms_out, eps);
    RS_HIP(hipGetLastError());
    return RS_OK;
}

// Brackets one step of the layer with HIP events on the call's stream when that step is being measured.
struct StepTimer {
    rs_ctx* c;
    hipStream_t st;
    void begin(int step) const {
        if (c->prof_step != step) return;
        c->prof_take = (c->prof_seen++ % c->prof_every == 0) && 2 * (c->prof_count + 1) <= (int)c->prof_events.size();
        if (c->prof_take) (void)hipEventRecord(c->prof_events[2 * c->prof_count], st);
    }
    void end(int step) const {
        if (c->prof_step != step || !c->prof_take) return;
        (void)hipEventRecord(c->prof_events[2 * c->prof_count + 1], st);
        ++c->prof_count;
        c->prof_take = false;
    }
};

template <int D>
rs_status launch_attention_path(const rs_ctx* c, bf16* qkv, bf16* attn, const ReqDesc* d_reqs,
                                const AttnItem* d_items, int n_items, const KVBlockItem* d_vb, int n_vb, bool any_paged,
                                float* split_buf, const AttnMergeItem* d_mitems, int n_mitems, const Fp8CacheDesc* d_fp8, int n_reqs,
                                int n_xblocks, hipStream_t st, const StepTimer& tm) {
    const rs_layer_cfg& f = c->cfg;
    tm.begin(RS_STEP_APPEND_KV);
    if (d_fp8) {  // 8-bit caches: quantise the new rows into them, then expand what the rows can see for the attention kernel
        hipLaunchKernelGGL(append_kv_fp8_kernel<D>, dim3(n_vb, f.n_kv_heads), dim3(256), 0, st, (const bf16*)qkv, c->qkv_dim,
                           d_reqs, d_fp8, d_vb, f.n_q_heads, f.n_kv_heads);
        RS_HIP(hipGetLastError());
        hipLaunchKernelGGL(kv_expand_fp8_kernel<D>, dim3(n_xblocks, f.n_kv_heads), dim3(256), 0, st, d_reqs, d_fp8, n_reqs);
    } else {
        hipLaunchKernelGGL(append_kv_kernel<D>, dim3(n_vb, f.n_kv_heads), dim3(256), 0, st, (const bf16*)qkv, c->qkv_dim,
                           d_reqs, d_vb, f.n_q_heads, f.n_kv_heads);
    }
    RS_HIP(hipGetLastError());
    tm.end(RS_STEP_APPEND_KV);
    const float scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)D));
    tm.begin(RS_STEP_ATTENTION);
    if (any_paged)
        hipLaunchKernelGGL((attn_prefill_pipelined_kernel<D, true>), dim3(n_items), dim3(256), 0, st, d_reqs, d_items,
                           (const bf16*)qkv, c->qkv_dim, attn, c->q_dim, c->group, scale_log2e, split_buf);
    else
        hipLaunchKernelGGL((attn_prefill_pipelined_kernel<D, false>), dim3(n_items), dim3(256), 0, st, d_reqs, d_items,
                           (const bf16*)qkv, c->qkv_dim, attn, c->q_dim, c->group, scale_log2e, split_buf);
    RS_HIP(hipGetLastError());
    if (n_mitems > 0) {
        hipLaunchKernelGGL(attn_merge_kernel<D>, dim3(n_mitems, ATT_MERGE_Y), dim3(256), 0, st, d_reqs, d_mitems, (const float*)split_buf, attn,
                           c->q_dim, c->group, scale_log2e);
        RS_HIP(hipGetLastError());
    }
    tm.end(RS_STEP_ATTENTION);
    return RS_OK;
}

// Runs an 8-bit cache's export or import kernel over tokens [0, n): in one launch for a contiguous cache, in windows of
// KV_PAGE_WINDOW blocks (whose page numbers ride in the kernel arguments) for a paged one.
template <class Launch>
void for_each_fp8_window(const rs_kv* kv, int layer, int n, Launch&& launch) {
    Fp8CacheDesc fc{};
    fc.hkv = kv->ctx->cfg.n_kv_heads;
    fc.k_scale = kv->k_scale; fc.v_scale = kv->v_scale;
    fc.k_inv = 1.0f / kv->k_scale; fc.v_inv = 1.0f / kv->v_scale;
    KVPageWindow win{};
    if (!kv->paged()) {
        fc.kc = kv->kc_of(layer); fc.vc = kv->vc_of(layer); fc.cap = kv->cap;
        launch(fc, win, 0, 0, n);
        return;
    }
    fc.kc = reinterpret_cast<uint8_t*>(kv->pool->base);
    fc.pages = reinterpret_cast<const int*>(kv->pool->base);   // non-null marker: the numbers come from the window
    const int window_tokens = KV_PAGE_WINDOW * 64;
    for (int t0 = 0; t0 < n; t0 += window_tokens) {
        const int nt = std::min(window_tokens, n - t0);
        const int b0 = t0 / 64, nb = (nt + 63) / 64;
        for (int b = 0; b < nb; ++b) win.page[b] = kv->pages[layer][b0 + b];
        launch(fc, win, b0, t0, nt);
    }
}

// Tokens [0, len) of an 8-bit cache's layer as bfloat16 values or as codes (whichever pair of outputs is given).
rs_status fp8_export(const rs_kv* kv, int layer, bf16* k_out, bf16* v_out, uint8_t* kc_out, uint8_t* vc_out, hipStream_t st) {
    const int kv_dim = kv->ctx->kv_dim;
    const bool d128 = kv->ctx->cfg.head_dim == 128;
    for_each_fp8_window(kv, layer, kv->len[layer], [&](const Fp8CacheDesc& fc, const KVPageWindow& win, int b0, int t0, int nt) {
        const int blocks = (int)std::min<size_t>(((size_t)nt * kv_dim + 255) / 256, 4096);
        if (d128)
            hipLaunchKernelGGL(kv_fp8_export_kernel<128>, dim3(blocks), dim3(256), 0, st, fc, win, b0, k_out, v_out, kc_out, vc_out, t0, nt);
        else
            hipLaunchKernelGGL(kv_fp8_export_kernel<64>, dim3(blocks), dim3(256), 0, st, fc, win, b0, k_out, v_out, kc_out, vc_out, t0, nt);
    });
    RS_HIP(hipGetLastError());
    return RS_OK;
}

// Fills tokens [0, n) of an 8-bit cache's layer from bfloat16 values or from codes (the caller has checked n against the
// capacity and, for a paged cache, taken the pages).
rs_status fp8_import(rs_kv* kv, int layer, const bf16* k_in, const bf16* v_in, const uint8_t* kc_in, const uint8_t* vc_in, int n,
                     hipStream_t st) {
    const int kv_dim = kv->ctx->kv_dim;
    const bool d128 = kv->ctx->cfg.head_dim == 128;
    for_each_fp8_window(kv, layer, n, [&](const Fp8CacheDesc& fc, const KVPageWindow& win, int b0, int t0, int nt) {
        const int blocks = (int)std::min<size_t>((align_up((size_t)nt, 64) * kv_dim + 255) / 256, 4096);
        if (d128)
            hipLaunchKernelGGL(kv_fp8_import_kernel<128>, dim3(blocks), dim3(256), 0, st, fc, win, b0, k_in, v_in, kc_in, vc_in, t0, nt);
        else
            hipLaunchKernelGGL(kv_fp8_import_kernel<64>, dim3(blocks), dim3(256), 0, st, fc, win, b0, k_in, v_in, kc_in, vc_in, t0, nt);
    });
    RS_HIP(hipGetLastError());
    return RS_OK;
}

// The checks rs_kv_import and rs_kv_import_codes share, in the order they are reported; changes nothing.
rs_status import_check(const rs_kv* kv, int layer, int n_tokens) {
    if (layer < 0 || layer >= kv->n_layers) return fail(RS_EINVAL, "layer %d out of range", layer);
    if (n_tokens < 0) return fail(RS_EINVAL, "n_tokens is negative");
    if (!kv->paged() && n_tokens > kv->cap) return fail(RS_ECAPACITY, "%d tokens exceed cache capacity %d", n_tokens, kv->cap);
    if (n_tokens > kv->ctx->cfg.max_pos) return fail(RS_ECAPACITY, "%d tokens exceed max_pos %d", n_tokens, kv->ctx->cfg.max_pos);
    if (kv->paged() && kv->pages_missing(layer, n_tokens) > (int)kv->pool->free_pages.size())
        return fail(RS_ECAPACITY, "the import needs %d new KV pages, the pool has %zu free", kv->pages_missing(layer, n_tokens),
                    kv->pool->free_pages.size());
    return RS_OK;
}

// Every check of one layer's call; changes nothing.  *total_out receives the number of rows.
// Runs the export or import kernel over tokens [0, n): in one launch for a contiguous cache, in windows of
// KV_PAGE_WINDOW blocks (whose page numbers ride in the kernel arguments) for a paged one.
template <class Launch>
rs_status for_each_kv_window(const rs_kv* kv, int layer, int n, Launch&& launch) {
    KVPageWindow win{};
    if (!kv->paged()) {
        launch(kv->view(layer, nullptr), win, 0, 0, n);
        return RS_OK;
    }
    const int window_tokens = KV_PAGE_WINDOW * 64;
    for (int t0 = 0; t0 < n; t0 += window_tokens) {
        const int nt = std::min(window_tokens, n - t0);
        const int b0 = t0 / 64, nb = (nt + 63) / 64;
        for (int b = 0; b < nb; ++b) win.page[b] = kv->pages[layer][b0 + b];
        launch(kv->view(layer, reinterpret_cast<const int*>(kv->pool->base)), win, b0, t0, nt);  // non-null marker: paged
    }
    return RS_OK;
}

// pages a call would take from each pool
typedef std::vector<std::pair<rs_kv_pool*, long>> PoolNeed;
void add_need(PoolNeed& need, rs_kv_pool* pool, long n) {
    if (n <= 0) return;
    for (auto& e : need)
        if (e.first == pool) {
            e.second += n;
            return;
        }
    need.emplace_back(pool, n);
}
rs_status check_need(const PoolNeed& need) {
    for (const auto& e : need)
        if (e.second > (long)e.first->free_pages.size())
            return fail(RS_ECAPACITY, "the call needs %ld new KV pages, the pool has %zu free", e.second, e.first->free_pages.size());
    return RS_OK;
}

rs_status prefill_check(rs_ctx* ctx, const rs_layer_weights* w, int layer, rs_kv* const* kvs, const int* lens, int R,
                        const void* x, void* y, void* ws, size_t ws_bytes, int* total_out, const int* positions3 = nullptr,
                        PoolNeed* pages_needed = nullptr) {
    if (!ctx) return fail(RS_EINVAL, "ctx is null");
    if (!w) return fail(RS_EINVAL, "weights are null");
    const rs_layer_cfg& f = ctx->cfg;
    if (!w->ln1_g || !w->w_qkv || !w->w_o || !w->ln2_g || !w->w_gate_up || !w->w_down)
        return fail(RS_EINVAL, "a weight pointer is null");
    if (f.qkv_bias && !w->b_qkv) return fail(RS_EINVAL, "cfg.qkv_bias is set but b_qkv is null");
    if (R < 0) return fail(RS_EINVAL, "R = %d is negative", R);
    if (R > f.max_requests) return fail(RS_EINVAL, "R = %d exceeds max_requests = %d", R, f.max_requests);
    if (R > 0 && (!kvs || !lens)) return fail(RS_EINVAL, "kvs / chunk_lens is null");
    long total = 0;
    for (int i = 0; i < R; ++i) {
        if (!kvs[i]) return fail(RS_EINVAL, "kvs[%d] is null", i);
        if (kvs[i]->ctx != ctx) return fail(RS_ESTATE, "kvs[%d] belongs to another context", i);
        if (layer < 0 || layer >= kvs[i]->n_layers) return fail(RS_EINVAL, "layer %d out of range for kvs[%d]", layer, i);
        if (lens[i] < 0) return fail(RS_EINVAL, "chunk_lens[%d] = %d is negative", i, lens[i]);
        total += lens[i];
    }
    if (total > f.max_tokens_per_call)
        return fail(RS_EINVAL, "%ld rows exceed max_tokens_per_call = %d", total, f.max_tokens_per_call);
    {
        std::vector<const rs_kv*> sorted(kvs, kvs + R);
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end())
            return fail(RS_EINVAL, "the same rs_kv appears twice in one micro-batch");
    }
    for (int i = 1; i < R; ++i)
        if (kvs[i]->fp8 != kvs[0]->fp8)
            return fail(RS_EINVAL, "kvs[%d]: the caches of one call must all be bfloat16 or all be 8-bit", i);
    for (int i = 0; i < R; ++i) {
        const long after = (long)kvs[i]->len[layer] + lens[i];
        if (!kvs[i]->paged() && after > kvs[i]->cap)
            return fail(RS_ECAPACITY, "request %d: %ld tokens exceed cache capacity %d", i, after, kvs[i]->cap);
        if (after > f.max_pos) return fail(RS_ECAPACITY, "request %d: %ld tokens exceed max_pos %d", i, after, f.max_pos);
    }
    if (pages_needed) {  // the caller adds up several layers; one layer's call checks its own need here
        for (int i = 0; i < R; ++i)
            if (kvs[i]->paged()) add_need(*pages_needed, kvs[i]->pool, kvs[i]->pages_missing(layer, (long)kvs[i]->len[layer] + lens[i]));
    } else {
        PoolNeed need;
        for (int i = 0; i < R; ++i)
            if (kvs[i]->paged()) add_need(need, kvs[i]->pool, kvs[i]->pages_missing(layer, (long)kvs[i]->len[layer] + lens[i]));
        const rs_status ps = check_need(need);
        if (ps != RS_OK) return ps;
    }
    *total_out = (int)total;
    if (total == 0) return RS_OK;
    const int T = (int)total;
    if (positions3)
        for (long i = 0; i < 3 * total; ++i)
            if (positions3[i] < 0 || positions3[i] >= f.max_pos)
                return fail(RS_ECAPACITY, "rotary position %d of row %ld is outside [0, max_pos = %d)", positions3[i], i / 3, f.max_pos);
    if (!x || !y) return fail(RS_EINVAL, "x / y is null");
    if (!aligned(x, 16) || !aligned(y, 16)) return fail(RS_EINVAL, "x / y must be 16-byte aligned");
    if (!ws) return fail(RS_EINVAL, "workspace is null");
    if (!aligned(ws, 256)) return fail(RS_EINVAL, "workspace must be 256-byte aligned");
    const WorkspaceLayout L = ws_layout(ctx, T, R);
    size_t expansion = 0;  // 8-bit caches: bfloat16 copies of the blocks the call's rows can see
    for (int i = 0; i < R; ++i)
        if (kvs[i]->fp8 && lens[i] > 0) expansion += fp8_expansion_bytes(ctx, (long)kvs[i]->len[layer] + lens[i]);
    if (ws_bytes < L.total + expansion)
        return fail(RS_EWORKSPACE, "workspace has %zu bytes, this call needs %zu%s", ws_bytes, L.total + expansion,
                    expansion ? " (rs_workspace_bytes_fp8kv: the 8-bit caches are expanded there)" : "");
    // (a caller that adds up the page need of several layers reports that shortage before the missing device)
    if (!pages_needed && !ctx->has_device) return fail(RS_EHIP, "no HIP device: the context was created on a host without a GPU");
    return RS_OK;
}

// Enqueues one layer's call (arguments already checked by prefill_check) and advances the cache lengths.
// `pending_in` (layers after the first of rs_prefill_model_batch): the previous layer's down projection left its split-K
// sum pending; x is then that layer's output buffer, not yet written, and this layer's first kernel produces it.
// `pending_out`: this layer may leave its own down projection pending in the same way (the next layer follows at once).
rs_status prefill_enqueue(rs_ctx* ctx, const rs_layer_weights* w, int layer, rs_kv* const* kvs, const int* lens, int R, int T,
                          const void* x, void* y, void* ws, void* stream, const int* positions3 = nullptr,
                          const PendingReduce* pending_in = nullptr, PendingReduce* pending_out = nullptr) {
    const rs_layer_cfg& f = ctx->cfg;
    const WorkspaceLayout L = ws_layout(ctx, T, R);
    {   // a call recorded into a HIP graph would replay with stale descriptors: refuse it, before anything changes
        hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(reinterpret_cast<hipStream_t>(stream), &capturing) != hipSuccess) (void)hipGetLastError();
        else if (capturing != hipStreamCaptureStatusNone) return fail(RS_ESTATE, "the stream is capturing a HIP graph");
    }

    // Pages taken below go back to their pools if a later host-side check refuses the call (nothing may change on a
    // status other than RS_OK); from the first launch on they stay.
    struct PageRollback {
        struct Entry { rs_kv* kv; int layer; int len; };
        std::vector<Entry> taken;
        bool armed = true;
        ~PageRollback() {
            if (!armed) return;
            for (auto it = taken.rbegin(); it != taken.rend(); ++it) it->kv->give_back_pages(it->layer, it->len);
        }
    } rollback;

    // ---- host descriptors
    std::vector<ReqDesc> reqs;
    std::vector<AttnItem> items;
    std::vector<KVBlockItem> vbs;
    std::vector<int> rowpos;
    std::vector<int> pagetab;
    std::vector<Fp8CacheDesc> fp8s;
    int n_xblocks = 0;
    size_t expansion_off = L.total;
    rowpos.reserve(3 * (size_t)T);
    const DescSizes ds = desc_sizes(ctx, T, R);
    char* wsb = reinterpret_cast<char*>(ws);
    const int* d_pagetab = reinterpret_cast<const int*>(wsb + L.desc + ds.reqs + ds.items + ds.vblocks + ds.rowpos);
    const int g = ctx->group;
    int row0 = 0;
    for (int i = 0; i < R; ++i) {
        const int Ti = lens[i];
        if (Ti == 0) continue;
        rs_kv* kv = kvs[i];
        const int P = kv->len[layer];
        if (kv->paged() && kv->pages_missing(layer, (long)P + Ti) > 0) rollback.taken.push_back({kv, layer, P});
        kv->take_pages(layer, (long)P + Ti);   // (paged caches; prefill_check has made sure the pool has them)
        ReqDesc d = kv->view(layer, d_pagetab + pagetab.size());
        d.row0 = row0; d.T = Ti; d.P = P;
        if (kv->fp8) {  // the kernels append to the 8-bit cache and attend to its expansion in the workspace
            Fp8CacheDesc fc{};
            if (kv->paged()) {   // the 8-bit kernels look the pages up; attention reads the (contiguous) expansion
                fc.kc = reinterpret_cast<uint8_t*>(kv->pool->base);
                fc.pages = d.pages;
                d.pages = nullptr;
            } else {
                fc.kc = kv->kc_of(layer); fc.vc = kv->vc_of(layer); fc.cap = kv->cap;
            }
            fc.xb0 = n_xblocks; fc.hkv = f.n_kv_heads;
            fc.k_scale = kv->k_scale; fc.v_scale = kv->v_scale;
            fc.k_inv = 1.0f / kv->k_scale; fc.v_inv = 1.0f / kv->v_scale;
            fp8s.push_back(fc);
            const size_t plane = fp8_expansion_bytes(ctx, (long)P + Ti) / 2;
            d.kcache = reinterpret_cast<bf16*>(wsb + expansion_off);
            d.vtcache = reinterpret_cast<bf16*>(wsb + expansion_off + plane);
            d.cap = (int)align_up((size_t)P + Ti, 64);
            expansion_off += 2 * plane;
            n_xblocks += d.cap / 64;
        }
        if (kv->paged()) pagetab.insert(pagetab.end(), kv->pages[layer].begin(), kv->pages[layer].end());
        const int ri = (int)reqs.size();
        reqs.push_back(d);
        const int nqb = (Ti * g + ATT_ROWS - 1) / ATT_ROWS;
        for (int qb = 0; qb < nqb; ++qb) {
            const int t_max = std::min(Ti - 1, (qb * ATT_ROWS + ATT_ROWS - 1) / g);
            const int nkb = (P + t_max + 1 + ATT_KEYS - 1) / ATT_KEYS;
            for (int c = 0; c < f.n_kv_heads; ++c) items.push_back(AttnItem{ri, c, qb, nkb, 0, -1, 0, 0});
        }
        for (int b = P / 64; b <= (P + Ti - 1) / 64; ++b) vbs.push_back(KVBlockItem{ri, b});
        for (int t = 0; t < Ti; ++t)
            for (int ax = 0; ax < 3; ++ax) rowpos.push_back(positions3 ? positions3[3 * (size_t)(row0 + t) + ax] : P + t);
        row0 += Ti;
    }
    // Fewer blocks than compute units: cut the key ranges so that up to two workgroups per compute unit exist, not more (a
    // third round of workgroups costs more than the shorter parts save: 512 rows on 16384 cached tokens 201 us with 5 parts,
    // 175 with 4).  A part has at least ATT_MIN_PART_TILES tiles, so every row of the block sees
    // keys in each part: the rows of a block span at most 128 positions, i.e. only the last three tiles can be hidden from
    // some of them.
    std::vector<AttnMergeItem> mitems;
    if (!items.empty()) {
        const int blocks = (int)items.size();
        int want = ctx->attn_split;
        if (want == 0) {
            // (the merge is a second kernel of about 6 us, i.e. six tiles of a block's walk; measured at the 7B shape, 64 rows
            // on 2048 cached tokens: 43 us of attention unsplit, 25 in 4 parts; 512 rows on 1536: 50 -> 40)
            int longest = 0;
            for (const AttnItem& it : items) longest = std::max(longest, it.nkb);
            want = (blocks < ctx->n_cu && longest >= ATT_MIN_SPLIT_TILES)
                       ? std::min(ATT_MAX_PARTS, std::max(1, 2 * ctx->n_cu / blocks)) : 1;
            if (want > 1) {
                // What the call's longest walk would shrink by, in tiles (blocks under two parts' worth stay whole and may
                // then be the longest).  Splitting pays from 7 tiles when the chip is nearly empty and from 12 when the
                // blocks alone nearly fill it (fitted: 1024 rows on 512 cached tokens lose 1 us with a gain of 9 tiles, on
                // 1024 cached tokens they win 6 us with a gain of 16; 64 rows on 960 win 6 us with a gain of 8).
                int longest_after = 0;
                for (const AttnItem& it : items) {
                    const int parts = std::min(want, it.nkb / ATT_MIN_PART_TILES);
                    longest_after = std::max(longest_after, parts < 2 ? it.nkb : (it.nkb + parts - 1) / parts);
                }
                if ((long)(longest - longest_after) * ctx->n_cu < 7L * ctx->n_cu + 5L * blocks) want = 1;
            }
        }
        if (want > 1) {
            std::vector<AttnItem> cut;
            int slots = 0;
            const int slot_cap = (int)attn_split_slots(ctx);
            for (const AttnItem& it : items) {
                const int parts = std::min(want, it.nkb / ATT_MIN_PART_TILES);
                if (parts < 2 || slots + parts > slot_cap) {
                    cut.push_back(it);
                    continue;
                }
                mitems.push_back(AttnMergeItem{it.req, it.kvh, it.qblock, parts, slots, 0, 0, 0});
                for (int p = 0; p < parts; ++p) {
                    AttnItem part = it;
                    part.kb0 = (int)((long)p * it.nkb / parts);
                    part.nkb = (int)((long)(p + 1) * it.nkb / parts);
                    part.slot = slots++;
                    cut.push_back(part);
                }
            }
            items.swap(cut);
        }
    }
    // heaviest work first: the tail of the launch is then made of short items
    std::stable_sort(items.begin(), items.end(),
                     [](const AttnItem& a, const AttnItem& b) { return a.nkb - a.kb0 > b.nkb - b.kb0; });
    // Between one and two workgroups per compute unit every item is resident from the first clock, and on an empty chip the
    // dispatcher hands workgroup k and workgroup k + n_cu to the same compute unit (measured: 448 workgroups of this
    // footprint leave exactly workgroups 192 .. 255 alone on theirs).  A lone workgroup walks its tiles faster than two that
    // share the matrix pipe, and a pair lasts as long as both walks together, so the launch ends soonest when the heaviest
    // items are the lone ones and the rest are paired heavy with light.  Only the order of independent items changes.
    const int n_items_now = (int)items.size();
    if (n_items_now > ctx->n_cu && n_items_now <= 2 * ctx->n_cu && !ctx->attn_plain_order) {
        const int paired = n_items_now - ctx->n_cu, lone = ctx->n_cu - paired;
        std::vector<AttnItem> placed(items.size());
        for (int k = 0; k < lone; ++k) placed[paired + k] = items[k];
        // (the light partners are taken from the tail in runs of one item per KV head, in the head order of the front: the
        //  blocks of a head then stay on the XCDs, workgroup index mod 8, whose L2 already holds that head's K and V)
        const int run = ctx->cfg.n_kv_heads;
        const bool by_head = n_items_now % run == 0 && paired % run == 0;
        for (int k = 0; k < paired; ++k) {
            placed[k] = items[lone + k];
            placed[ctx->n_cu + k] = by_head ? items[n_items_now - run * (k / run + 1) + k % run] : items[n_items_now - 1 - k];
        }
        items.swap(placed);
    }

    if (sizeof(ReqDesc) * reqs.size() > ds.reqs || sizeof(AttnItem) * items.size() > ds.items ||
        sizeof(KVBlockItem) * vbs.size() > ds.vblocks || sizeof(int) * rowpos.size() > ds.rowpos ||
        sizeof(int) * pagetab.size() > ds.pagetab || sizeof(AttnMergeItem) * mitems.size() > ds.mitems ||
        sizeof(Fp8CacheDesc) * fp8s.size() > ds.fp8 || (!fp8s.empty() && fp8s.size() != reqs.size()) ||
        ds.total > ctx->slot_bytes)
        return fail(RS_EINVAL, "internal: descriptor sizing");

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const long use = ctx->use_count;
    const int slot = (int)(use % RING_SLOTS);
    if (use > 0 && st != ctx->last_stream) {  // leaving a stream: a checkpoint behind its last use, unless there is one
        const int prev = (int)((use - 1) % RING_SLOTS);
        if (ctx->slot_recorded_at[prev] != use - 1) {
            if (hipEventRecord(ctx->slot_done[prev], ctx->last_stream) != hipSuccess) {
                (void)hipGetLastError();       // (the stream is gone: wait for everything instead)
                RS_HIP(hipDeviceSynchronize());
                RS_HIP(hipEventRecord(ctx->slot_done[prev], st));
            }
            ctx->slot_recorded_at[prev] = use - 1;
        }
    }
    if (use >= RING_SLOTS) {  // the slot's previous use: wait for the first checkpoint at or after it
        const long old = use - RING_SLOTS;
        bool waited = false;
        for (long u = old; u < old + RING_CHECKPOINT && !waited; ++u)
            if (ctx->slot_recorded_at[u % RING_SLOTS] == u) {
                RS_HIP(hipEventSynchronize(ctx->slot_done[u % RING_SLOTS]));
                waited = true;
            }
        if (!waited) return fail(RS_EINVAL, "internal: no checkpoint behind use %ld of the descriptor ring", old);
    }
    char* stage = ctx->pinned[slot];
    memcpy(stage, reqs.data(), sizeof(ReqDesc) * reqs.size());
    memcpy(stage + ds.reqs, items.data(), sizeof(AttnItem) * items.size());
    memcpy(stage + ds.reqs + ds.items, vbs.data(), sizeof(KVBlockItem) * vbs.size());
    memcpy(stage + ds.reqs + ds.items + ds.vblocks, rowpos.data(), sizeof(int) * rowpos.size());
    memcpy(stage + ds.reqs + ds.items + ds.vblocks + ds.rowpos, pagetab.data(), sizeof(int) * pagetab.size());
    memcpy(stage + ds.reqs + ds.items + ds.vblocks + ds.rowpos + ds.pagetab, mitems.data(), sizeof(AttnMergeItem) * mitems.size());
    memcpy(stage + ds.reqs + ds.items + ds.vblocks + ds.rowpos + ds.pagetab + ds.mitems, fp8s.data(), sizeof(Fp8CacheDesc) * fp8s.size());
    // (the first kernel below copies the staged descriptors into the workspace; the slot is free again once it has run)
    const ReqDesc* d_reqs = reinterpret_cast<const ReqDesc*>(wsb + L.desc);
    const AttnItem* d_items = reinterpret_cast<const AttnItem*>(wsb + L.desc + ds.reqs);
    const KVBlockItem* d_vb = reinterpret_cast<const KVBlockItem*>(wsb + L.desc + ds.reqs + ds.items);
    const int* d_rowpos = reinterpret_cast<const int*>(wsb + L.desc + ds.reqs + ds.items + ds.vblocks);
    const AttnMergeItem* d_mitems =
        reinterpret_cast<const AttnMergeItem*>(wsb + L.desc + ds.reqs + ds.items + ds.vblocks + ds.rowpos + ds.pagetab);
    float* attn_split = reinterpret_cast<float*>(wsb + L.attn_split);
    const Fp8CacheDesc* d_fp8 = fp8s.empty() ? nullptr :
        reinterpret_cast<const Fp8CacheDesc*>(wsb + L.desc + ds.reqs + ds.items + ds.vblocks + ds.rowpos + ds.pagetab + ds.mitems);

    bf16* qkv = reinterpret_cast<bf16*>(wsb + L.qkv);
    bf16* xf = reinterpret_cast<bf16*>(wsb + L.xf);
    bf16* attn = reinterpret_cast<bf16*>(wsb + L.attn);
    bf16* r = reinterpret_cast<bf16*>(wsb + L.r);
    bf16* act = reinterpret_cast<bf16*>(wsb + L.act);
    float* partial = reinterpret_cast<float*>(wsb + L.partial);
    float* inv_rms1 = reinterpret_cast<float*>(wsb + L.inv_rms1);
    float* inv_rms2 = reinterpret_cast<float*>(wsb + L.inv_rms2);
    float* rowss = reinterpret_cast<float*>(wsb + L.rowss);
    const bf16* xb = reinterpret_cast<const bf16*>(x);
    bf16* yb = reinterpret_cast<bf16*>(y);
    const int H = f.hidden, I = f.mlp_inter;
    rs_status s;
    const StepTimer tm{ctx, st};

    rollback.armed = false;   // every host-side check has passed: from here on the call is launched
    // 1/rms of every input row (the first RMSNorm; its gain lives in the packed W_qkv)
    tm.begin(RS_STEP_ROW_RMS);
    // and, in the same pass, x in the GEMMs' fragment-major token-operand layout
    const int desc_chunks = (int)(ds.total / 16);
    if (pending_in && pending_in->splits > 0) {
        // (the pending sum reads the previous layer's r and partial planes, which this layer overwrites only later)
        ReduceSource red{pending_in->partial, pending_in->splits, pending_in->resid, pending_in->out};
        hipLaunchKernelGGL(rms_and_fragment_major_kernel<true>, dim3((T + 7) / 8 + (desc_chunks + 255) / 256), dim3(256), 0, st, xb, xf,
                           inv_rms1, T, H, f.rms_eps, reinterpret_cast<const uint4*>(ctx->pinned_dev[slot]),
                           reinterpret_cast<uint4*>(wsb + L.desc), desc_chunks, red);
    } else {
        hipLaunchKernelGGL(rms_and_fragment_major_kernel<false>, dim3((T + 7) / 8 + (desc_chunks + 255) / 256), dim3(256), 0, st, xb, xf,
                           inv_rms1, T, H, f.rms_eps, reinterpret_cast<const uint4*>(ctx->pinned_dev[slot]),
                           reinterpret_cast<uint4*>(wsb + L.desc), desc_chunks, ReduceSource{});
    }
    RS_HIP(hipGetLastError());
    if (use % RING_CHECKPOINT == RING_CHECKPOINT - 1) {
        RS_HIP(hipEventRecord(ctx->slot_done[slot], st));
        ctx->slot_recorded_at[slot] = use;
    } else {
        ctx->slot_recorded_at[slot] = -1;   // (what was recorded here belonged to the slot's previous use)
    }
    ctx->last_stream = st;
    ctx->use_count = use + 1;
    tm.end(RS_STEP_ROW_RMS);
    // qkv = rope( (x Wqkv'^T) / rms + b )
    tm.begin(RS_STEP_QKV_GEMM);
    {
        GemmArgs a{};
        a.X = xf; a.W = (const bf16*)w->w_qkv; a.out = qkv; a.ldo = ctx->qkv_dim;
        a.bias = f.qkv_bias ? (const bf16*)w->b_qkv : nullptr;
        a.row_scale = inv_rms1; a.row_pos = d_rowpos; a.rope_cs = (const float2*)ctx->rope_dev;
        a.rope_cols = ctx->q_dim + ctx->kv_dim; a.head_dim = f.head_dim;
        a.mrope_b0 = ctx->mrope_b0; a.mrope_b1 = ctx->mrope_b1;
        a.M = T; a.N = ctx->qkv_dim; a.K = H;
        if ((s = launch_gemm<EPI_QKV_ROPE>(ctx, a, 1, st)) != RS_OK) return s;
    }
    tm.end(RS_STEP_QKV_GEMM);
    // cache append, attention
    if (f.head_dim == 128)
        s = launch_attention_path<128>(ctx, qkv, attn, d_reqs, d_items, (int)items.size(), d_vb, (int)vbs.size(), !pagetab.empty() && fp8s.empty(),
                                       attn_split, d_mitems, (int)mitems.size(), d_fp8, (int)reqs.size(), n_xblocks, st, tm);
    else
        s = launch_attention_path<64>(ctx, qkv, attn, d_reqs, d_items, (int)items.size(), d_vb, (int)vbs.size(), !pagetab.empty() && fp8s.empty(),
                                      attn_split, d_mitems, (int)mitems.size(), d_fp8, (int)reqs.size(), n_xblocks, st, tm);
    if (s != RS_OK) return s;
    // r = x + attn Wo^T, and 1/rms of every row of r (the second RMSNorm; its gain lives in the packed W_gate_up)
    tm.begin(RS_STEP_O_GEMM);
    int rowss_parts = 0;
    if ((s = gemm_residual(ctx, attn, (const bf16*)w->w_o, xb, 0, r, 1, T, H, ctx->q_dim, partial, inv_rms2, rowss, &rowss_parts, st)) != RS_OK) return s;
    tm.end(RS_STEP_O_GEMM);
    // act = silu((r Wg'^T) / rms) * ((r Wu'^T) / rms)
    tm.begin(RS_STEP_GATE_UP_GEMM);
    {
        GemmArgs a{};
        a.X = r; a.W = (const bf16*)w->w_gate_up; a.out = act; a.ldo = I; a.out_frag = 1;
        a.row_scale = inv_rms2;
        if (rowss_parts > 0) {   // the output projection ran unsplit: its per-column sums of squares, closed in this kernel
            a.rowss = rowss; a.rowss_parts = rowss_parts; a.rms_eps = f.rms_eps;
        }
        a.M = T; a.N = 2 * I; a.K = H;
        if ((s = launch_gemm<EPI_SWIGLU>(ctx, a, 1, st)) != RS_OK) return s;
    }
    tm.end(RS_STEP_GATE_UP_GEMM);
    // y = r + act Wd^T
    tm.begin(RS_STEP_DOWN_GEMM);
    if ((s = gemm_residual(ctx, act, (const bf16*)w->w_down, r, 1, yb, 0, T, H, I, partial, nullptr, nullptr, nullptr, st, pending_out)) != RS_OK) return s;
    tm.end(RS_STEP_DOWN_GEMM);

    for (int i = 0; i < R; ++i) kvs[i]->len[layer] += lens[i];
    return RS_OK;
}

rs_status prefill_impl(rs_ctx* ctx, const rs_layer_weights* w, int layer, rs_kv* const* kvs, const int* lens, int R,
                       const void* x, void* y, void* ws, size_t ws_bytes, void* stream, const int* positions3 = nullptr) {
    int T = 0;
    const rs_status s = prefill_check(ctx, w, layer, kvs, lens, R, x, y, ws, ws_bytes, &T, positions3);
    if (s != RS_OK || T == 0) return s;
    return prefill_enqueue(ctx, w, layer, kvs, lens, R, T, x, y, ws, stream, positions3);
}

}  // namespace

// =============================================================================================== C ABI
extern "C" {

const char* rs_last_error(void) { return g_last_error.c_str(); }
int rs_version(void) { return 1; }

rs_status rs_ctx_create(const rs_layer_cfg* cfg, rs_ctx** out) {
    if (!cfg || !out) return fail(RS_EINVAL, "cfg / out is null");
    *out = nullptr;
    const rs_layer_cfg& f = *cfg;
    if (f.hidden <= 0 || f.n_q_heads <= 0 || f.n_kv_heads <= 0 || f.mlp_inter <= 0 || f.max_tokens_per_call <= 0 ||
        f.max_requests <= 0 || f.max_pos <= 0)
        return fail(RS_EINVAL, "sizes must be positive");
    if (f.head_dim != 64 && f.head_dim != 128) return fail(RS_EINVAL, "head_dim must be 64 or 128");
    if (f.n_q_heads % f.n_kv_heads) return fail(RS_EINVAL, "n_kv_heads must divide n_q_heads");
    const int q_dim = f.n_q_heads * f.head_dim, kv_dim = f.n_kv_heads * f.head_dim, qkv_dim = q_dim + 2 * kv_dim;
    if (f.hidden % 64) return fail(RS_EINVAL, "hidden must be a multiple of 64");
    if (f.mlp_inter % 64) return fail(RS_EINVAL, "mlp_inter must be a multiple of 64");
    if (!(f.rms_eps >= 0.0f) || !(f.rope_theta > 0.0f)) return fail(RS_EINVAL, "rms_eps / rope_theta out of range");
    if ((size_t)f.max_tokens_per_call * (size_t)std::max(qkv_dim, f.mlp_inter) * 2 >= (size_t)1 << 31)
        return fail(RS_EINVAL, "max_tokens_per_call too large for 32-bit row offsets");
    if ((size_t)f.max_tokens_per_call * (size_t)f.hidden * 4 >= (size_t)1 << 31)
        return fail(RS_EINVAL, "max_tokens_per_call * hidden too large for 32-bit offsets into a split-K plane");
    if ((size_t)std::max(2 * f.mlp_inter, qkv_dim) * (size_t)f.hidden * 2 >= (size_t)1 << 31 ||
        (size_t)f.hidden * (size_t)f.mlp_inter * 2 >= (size_t)1 << 31)
        return fail(RS_EINVAL, "weight matrix too large for 32-bit row offsets");

    rs_ctx* c = new rs_ctx();
    c->cfg = f;
    c->q_dim = q_dim; c->kv_dim = kv_dim; c->qkv_dim = qkv_dim; c->group = f.n_q_heads / f.n_kv_heads;
    c->mrope_b0 = c->mrope_b1 = f.head_dim / 2;  // 1-D RoPE: every pair turns with the first axis
    if (const char* e = getenv("RS_SPLITK")) c->splitk_override = atoi(e);
    if (const char* e = getenv("RS_PAIRS")) c->gemm_pairs = atoi(e);
    if (const char* e = getenv("RS_NARROW")) c->gemm_narrow = atoi(e);
    if (const char* e = getenv("RS_NARROW_TM")) c->narrow_max_tiles_m = atoi(e);
    if (const char* e = getenv("RS_ATTN_SPLIT")) c->attn_split = std::max(0, std::min(atoi(e), ATT_MAX_PARTS));
    if (const char* e = getenv("RS_ATTN_ORDER")) c->attn_plain_order = strcmp(e, "plain") == 0;
    auto cleanup = [&](rs_status s) { rs_ctx_destroy(c); return s; };

    c->slot_bytes = desc_sizes(c, f.max_tokens_per_call, f.max_requests).total;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) {
        (void)hipGetLastError();
        *out = c;  // host-only context: every check that precedes a launch still works
        return RS_OK;
    }
    c->has_device = true;

    // RoPE table from fp64 angles
    const int half = f.head_dim / 2;
    std::vector<float2> table((size_t)f.max_pos * half);
    std::vector<double> inv_freq(half);
    for (int j = 0; j < half; ++j) inv_freq[j] = std::pow((double)f.rope_theta, -2.0 * j / f.head_dim);
    for (int p = 0; p < f.max_pos; ++p)
        for (int j = 0; j < half; ++j) {
            const double ang = (double)p * inv_freq[j];
            table[(size_t)p * half + j] = make_float2((float)std::cos(ang), (float)std::sin(ang));
        }
    hipError_t e = hipMalloc((void**)&c->rope_dev, table.size() * sizeof(float2));
    if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipMalloc(rope table): %s", hipGetErrorString(e)));
    e = hipMemcpy(c->rope_dev, table.data(), table.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipMemcpy(rope table): %s", hipGetErrorString(e)));

    for (int i = 0; i < RING_SLOTS; ++i) {
        e = hipHostMalloc((void**)&c->pinned[i], c->slot_bytes, hipHostMallocDefault);
        if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipHostMalloc: %s", hipGetErrorString(e)));
        e = hipHostGetDevicePointer((void**)&c->pinned_dev[i], c->pinned[i], 0);
        if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipHostGetDevicePointer: %s", hipGetErrorString(e)));
        e = hipEventCreateWithFlags(&c->slot_done[i], hipEventDisableTiming);
        if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipEventCreate: %s", hipGetErrorString(e)));
        c->slot_recorded_at[i] = -1;
    }
    int dev = 0, n_cu = 0;
    e = hipGetDevice(&dev);
    if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipGetDevice: %s", hipGetErrorString(e)));
    c->device = dev;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n_cu > 0) c->n_cu = n_cu;
    e = static_workspace_lookup(dev, &c->static_ws);
    if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipGetSymbolAddress(static workspace): %s", hipGetErrorString(e)));
    if (const char* e = getenv("RS_NCU")) {  // test hook: fewer, wider strips exercise every tile width on small shapes
        if (atoi(e) > 0) c->n_cu = atoi(e);
    }
    // kernels that use more than 64 KB of LDS must opt in
    e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_QKV_ROPE>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_RESIDUAL>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_SWIGLU>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_PARTIAL>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_QKV_ROPE, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_RESIDUAL, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_SWIGLU, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_PARTIAL, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_QKV_ROPE, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_RESIDUAL, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_SWIGLU, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_strip_kernel<EPI_PARTIAL, GS_NARROW_NT, GS_NARROW_SLOTS, 1, GS_NARROW_XD, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, GS_NARROW_LDS_BYTES);
    // (the pipelined attention kernel keeps its LDS in static arrays; these references make the launch stubs exist)
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_prefill_pipelined_kernel<128, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 0);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_prefill_pipelined_kernel<64, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 0);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_prefill_pipelined_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 0);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_prefill_pipelined_kernel<64, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 0);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_merge_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, 0);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_merge_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, 0);
    if (e != hipSuccess) return cleanup(fail(RS_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e)));
    *out = c;
    return RS_OK;
}

void rs_ctx_destroy(rs_ctx* c) {
    if (!c) return;
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    if (c->rope_dev) (void)hipFree(c->rope_dev);
    for (int i = 0; i < RING_SLOTS; ++i) {
        if (c->slot_done[i]) (void)hipEventDestroy(c->slot_done[i]);
        if (c->pinned[i]) (void)hipHostFree(c->pinned[i]);
    }
    delete c;
}

size_t rs_weights_packed_bytes(const rs_ctx* c) {
    if (!c) return 0;
    const rs_layer_cfg& f = c->cfg;
    const size_t H = f.hidden, I = f.mlp_inter;
    size_t b = 0;
    b += align_up(H * 2, 256) * 2;                    // gains
    b += align_up((size_t)c->qkv_dim * H * 2, 256);   // w_qkv
    b += align_up((size_t)c->qkv_dim * 2, 256);       // b_qkv
    b += align_up(H * c->q_dim * 2, 256);             // w_o
    b += align_up(2 * I * H * 2, 256);                // w_gate_up
    b += align_up(H * I * 2, 256);                    // w_down
    return b;
}

rs_status rs_weights_pack(rs_ctx* c, const rs_layer_weights* src, void* dst, size_t dst_bytes, rs_layer_weights* packed,
                          void* stream) {
    if (!c || !src || !dst || !packed) return fail(RS_EINVAL, "null argument");
    const rs_layer_cfg& f = c->cfg;
    if (!src->ln1_g || !src->w_qkv || !src->w_o || !src->ln2_g || !src->w_gate_up || !src->w_down)
        return fail(RS_EINVAL, "a source weight pointer is null");
    if (f.qkv_bias && !src->b_qkv) return fail(RS_EINVAL, "cfg.qkv_bias is set but b_qkv is null");
    if (!aligned(dst, 256)) return fail(RS_EINVAL, "dst must be 256-byte aligned");
    if (!aligned(src->w_gate_up, 16) || !aligned(src->w_qkv, 16) || !aligned(src->ln1_g, 16) || !aligned(src->ln2_g, 16))
        return fail(RS_EINVAL, "source weights must be 16-byte aligned");
    if (dst_bytes < rs_weights_packed_bytes(c)) return fail(RS_EWORKSPACE, "dst has %zu bytes, need %zu", dst_bytes, rs_weights_packed_bytes(c));
    if (!c->has_device) return fail(RS_EHIP, "no HIP device");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const size_t H = f.hidden, I = f.mlp_inter;
    char* p = reinterpret_cast<char*>(dst);
    auto copy = [&](const void* s, size_t bytes, const void** slot) -> hipError_t {
        *slot = p;
        hipError_t e = hipMemcpyAsync(p, s, bytes, hipMemcpyDeviceToDevice, st);
        p += align_up(bytes, 256);
        return e;
    };
    rs_layer_weights o{};
    RS_HIP(copy(src->ln1_g, H * 2, &o.ln1_g));
    RS_HIP(copy(src->ln2_g, H * 2, &o.ln2_g));
    // W_qkv with the first norm's gain folded into its columns
    o.w_qkv = p;
    hipLaunchKernelGGL(pack_rows_kernel, dim3(c->qkv_dim), dim3(256), 0, st, (const bf16*)src->w_qkv, (const bf16*)src->ln1_g,
                       reinterpret_cast<bf16*>(p), f.hidden, (int)PACK_QKV_ROPE, f.head_dim, c->q_dim + c->kv_dim);
    RS_HIP(hipGetLastError());
    p += align_up((size_t)c->qkv_dim * H * 2, 256);
    if (f.qkv_bias) {
        RS_HIP(copy(src->b_qkv, (size_t)c->qkv_dim * 2, &o.b_qkv));
    } else {
        p += align_up((size_t)c->qkv_dim * 2, 256);
    }
    RS_HIP(copy(src->w_o, H * c->q_dim * 2, &o.w_o));
    // W_gate / W_up interleaved in 16-row blocks (one unit = 16 gate rows + their up rows), second norm gain folded in
    o.w_gate_up = p;
    hipLaunchKernelGGL(pack_rows_kernel, dim3(2 * f.mlp_inter), dim3(256), 0, st, (const bf16*)src->w_gate_up,
                       (const bf16*)src->ln2_g, reinterpret_cast<bf16*>(p), f.hidden, (int)PACK_GATE_UP, f.mlp_inter, 0);
    RS_HIP(hipGetLastError());
    p += align_up(2 * I * H * 2, 256);
    RS_HIP(copy(src->w_down, H * I * 2, &o.w_down));
    *packed = o;
    return RS_OK;
}

size_t rs_kv_bytes(const rs_ctx* c, int n_layers, int capacity_tokens) {
    if (!c || n_layers <= 0 || capacity_tokens <= 0) return 0;
    const size_t cap = align_up((size_t)capacity_tokens, 64);
    const size_t plane = align_up(cap * c->kv_dim * 2, 256);
    return 2 * plane * n_layers;
}

rs_status rs_kv_alloc(rs_ctx* c, int n_layers, int capacity_tokens, void* dev_mem, size_t bytes, rs_kv** out) {
    if (!c || !out) return fail(RS_EINVAL, "ctx / out is null");
    *out = nullptr;
    if (n_layers <= 0 || capacity_tokens <= 0) return fail(RS_EINVAL, "n_layers and capacity_tokens must be positive");
    if (!dev_mem || !aligned(dev_mem, 256)) return fail(RS_EINVAL, "dev_mem must be a 256-byte aligned device pointer");
    const size_t need = rs_kv_bytes(c, n_layers, capacity_tokens);
    if (bytes < need) return fail(RS_EWORKSPACE, "KV slab has %zu bytes, need %zu", bytes, need);
    rs_kv* kv = new rs_kv();
    kv->ctx = c;
    kv->n_layers = n_layers;
    kv->cap = (int)align_up((size_t)capacity_tokens, 64);
    kv->base = reinterpret_cast<char*>(dev_mem);
    kv->k_bytes = align_up((size_t)kv->cap * c->kv_dim * 2, 256);
    kv->layer_bytes = 2 * kv->k_bytes;
    kv->len.assign(n_layers, 0);
    *out = kv;
    return RS_OK;
}

static bool fp8_scales_ok(float k_scale, float v_scale) {
    return k_scale > 0.0f && v_scale > 0.0f && std::isfinite(k_scale) && std::isfinite(v_scale) && std::isfinite(1.0f / k_scale) &&
           std::isfinite(1.0f / v_scale);
}

size_t rs_kv_fp8_bytes(const rs_ctx* c, int n_layers, int capacity_tokens) {
    if (!c || n_layers <= 0 || capacity_tokens <= 0) return 0;
    const size_t cap = align_up((size_t)capacity_tokens, 64);
    const size_t plane = align_up(cap * c->kv_dim, 256);
    return 2 * plane * n_layers;
}

rs_status rs_kv_alloc_fp8(rs_ctx* c, int n_layers, int capacity_tokens, float k_scale, float v_scale, void* dev_mem, size_t bytes,
                          rs_kv** out) {
    if (!c || !out) return fail(RS_EINVAL, "ctx / out is null");
    *out = nullptr;
    if (n_layers <= 0 || capacity_tokens <= 0) return fail(RS_EINVAL, "n_layers and capacity_tokens must be positive");
    if (!fp8_scales_ok(k_scale, v_scale))
        return fail(RS_EINVAL, "k_scale = %g and v_scale = %g must be positive, finite and have a finite reciprocal", k_scale, v_scale);
    if (!dev_mem || !aligned(dev_mem, 256)) return fail(RS_EINVAL, "dev_mem must be a 256-byte aligned device pointer");
    const size_t need = rs_kv_fp8_bytes(c, n_layers, capacity_tokens);
    if (bytes < need) return fail(RS_EWORKSPACE, "KV slab has %zu bytes, need %zu", bytes, need);
    rs_kv* kv = new rs_kv();
    kv->ctx = c;
    kv->n_layers = n_layers;
    kv->cap = (int)align_up((size_t)capacity_tokens, 64);
    kv->base = reinterpret_cast<char*>(dev_mem);
    kv->k_bytes = align_up((size_t)kv->cap * c->kv_dim, 256);
    kv->layer_bytes = 2 * kv->k_bytes;
    kv->len.assign(n_layers, 0);
    kv->fp8 = true;
    kv->k_scale = k_scale;
    kv->v_scale = v_scale;
    *out = kv;
    return RS_OK;
}

int rs_kv_is_fp8(const rs_kv* kv) { return kv ? (kv->fp8 ? 1 : 0) : -1; }

size_t rs_kv_page_bytes(const rs_ctx* c) {
    if (!c) return 0;
    return (size_t)2 * c->cfg.n_kv_heads * 64 * c->cfg.head_dim * 2;
}

size_t rs_kv_page_bytes_fp8(const rs_ctx* c) { return rs_kv_page_bytes(c) / 2; }

static rs_status pool_create(rs_ctx* c, void* dev_mem, size_t bytes, bool fp8, rs_kv_pool** out);
rs_status rs_kv_pool_create(rs_ctx* c, void* dev_mem, size_t bytes, rs_kv_pool** out) { return pool_create(c, dev_mem, bytes, false, out); }
rs_status rs_kv_pool_create_fp8(rs_ctx* c, void* dev_mem, size_t bytes, rs_kv_pool** out) { return pool_create(c, dev_mem, bytes, true, out); }
int rs_kv_pool_is_fp8(const rs_kv_pool* p) { return p ? (p->fp8 ? 1 : 0) : -1; }

static rs_status pool_create(rs_ctx* c, void* dev_mem, size_t bytes, bool fp8, rs_kv_pool** out) {
    if (!c || !out) return fail(RS_EINVAL, "ctx / out is null");
    *out = nullptr;
    if (!dev_mem || !aligned(dev_mem, 256)) return fail(RS_EINVAL, "dev_mem must be a 256-byte aligned device pointer");
    const size_t pb = fp8 ? rs_kv_page_bytes_fp8(c) : rs_kv_page_bytes(c);
    const size_t n = bytes / pb;
    if (n == 0) return fail(RS_EWORKSPACE, "the pool's memory (%zu bytes) is smaller than one page (%zu bytes)", bytes, pb);
    if (n > (size_t)0x7fffffff) return fail(RS_EINVAL, "more than 2^31 - 1 pages");
    rs_kv_pool* p = new rs_kv_pool();
    p->ctx = c;
    p->base = reinterpret_cast<char*>(dev_mem);
    p->page_bytes = pb;
    p->fp8 = fp8;
    p->n_pages = (int)n;
    p->free_pages.resize(n);
    for (size_t i = 0; i < n; ++i) p->free_pages[i] = (int)(n - 1 - i);  // page 0 is handed out first
    *out = p;
    return RS_OK;
}

rs_status rs_kv_pool_destroy(rs_kv_pool* p) {
    if (!p) return RS_OK;
    if (p->n_caches != 0) return fail(RS_ESTATE, "%d caches still use this pool", p->n_caches);
    delete p;
    return RS_OK;
}

int rs_kv_pool_pages(const rs_kv_pool* p) { return p ? p->n_pages : -1; }
int rs_kv_pool_free_pages(const rs_kv_pool* p) { return p ? (int)p->free_pages.size() : -1; }

static rs_status alloc_paged(rs_ctx* c, rs_kv_pool* pool, int n_layers, bool fp8, float k_scale, float v_scale, rs_kv** out);
rs_status rs_kv_alloc_paged(rs_ctx* c, rs_kv_pool* pool, int n_layers, rs_kv** out) {
    return alloc_paged(c, pool, n_layers, false, 1.0f, 1.0f, out);
}
rs_status rs_kv_alloc_paged_fp8(rs_ctx* c, rs_kv_pool* pool, int n_layers, float k_scale, float v_scale, rs_kv** out) {
    return alloc_paged(c, pool, n_layers, true, k_scale, v_scale, out);
}

static rs_status alloc_paged(rs_ctx* c, rs_kv_pool* pool, int n_layers, bool fp8, float k_scale, float v_scale, rs_kv** out) {
    if (!c || !out) return fail(RS_EINVAL, "ctx / out is null");
    *out = nullptr;
    if (!pool) return fail(RS_EINVAL, "pool is null");
    if (pool->ctx != c) return fail(RS_ESTATE, "the pool belongs to another context");
    if (pool->fp8 != fp8)
        return fail(RS_ESTATE, "the pool holds %s pages, the cache asked for is %s", pool->fp8 ? "8-bit" : "bfloat16", fp8 ? "8-bit" : "bfloat16");
    if (n_layers <= 0) return fail(RS_EINVAL, "n_layers must be positive");
    if (fp8 && !fp8_scales_ok(k_scale, v_scale))
        return fail(RS_EINVAL, "k_scale = %g and v_scale = %g must be positive, finite and have a finite reciprocal", k_scale, v_scale);
    rs_kv* kv = new rs_kv();
    kv->ctx = c;
    kv->n_layers = n_layers;
    kv->cap = 0;
    kv->base = nullptr;
    kv->k_bytes = kv->layer_bytes = 0;
    kv->len.assign(n_layers, 0);
    kv->pool = pool;
    kv->fp8 = fp8;
    kv->k_scale = k_scale;
    kv->v_scale = v_scale;
    kv->pages.assign(n_layers, std::vector<int>());
    ++pool->n_caches;
    *out = kv;
    return RS_OK;
}

void rs_kv_free(rs_kv* kv) {
    if (!kv) return;
    if (kv->paged()) {
        for (int l = 0; l < kv->n_layers; ++l) kv->give_back_pages(l, 0);
        --kv->pool->n_caches;
    }
    delete kv;
}

int rs_kv_len(const rs_kv* kv, int layer) {
    if (!kv || layer < 0 || layer >= kv->n_layers) return -1;
    return kv->len[layer];
}

int rs_kv_capacity(const rs_kv* kv) {
    if (!kv) return -1;
    if (!kv->paged()) return kv->cap;
    size_t fewest = kv->pages[0].size();
    for (const auto& pl : kv->pages) fewest = std::min(fewest, pl.size());
    return (int)(fewest * 64);
}

rs_status rs_kv_reset(rs_kv* kv) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    std::fill(kv->len.begin(), kv->len.end(), 0);
    if (kv->paged())
        for (int l = 0; l < kv->n_layers; ++l) kv->give_back_pages(l, 0);
    return RS_OK;
}

rs_status rs_kv_truncate(rs_kv* kv, int layer, int n_tokens) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    if (layer < 0 || layer >= kv->n_layers) return fail(RS_EINVAL, "layer %d out of range", layer);
    if (n_tokens < 0 || n_tokens > kv->len[layer]) return fail(RS_EINVAL, "n_tokens = %d outside [0, %d]", n_tokens, kv->len[layer]);
    kv->len[layer] = n_tokens;
    if (kv->paged()) kv->give_back_pages(layer, n_tokens);
    return RS_OK;
}

rs_status rs_kv_export(const rs_kv* kv, int layer, void* k_out, void* v_out, void* stream) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    if (layer < 0 || layer >= kv->n_layers) return fail(RS_EINVAL, "layer %d out of range", layer);
    const int n = kv->len[layer];
    if (n == 0) return RS_OK;
    if (!k_out || !v_out) return fail(RS_EINVAL, "k_out / v_out is null");
    if (!kv->ctx->has_device) return fail(RS_EHIP, "no HIP device");
    const rs_layer_cfg& f = kv->ctx->cfg;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int kv_dim = kv->ctx->kv_dim;
    if (kv->fp8) return fp8_export(kv, layer, (bf16*)k_out, (bf16*)v_out, nullptr, nullptr, st);
    for_each_kv_window(kv, layer, n, [&](const ReqDesc& rq, const KVPageWindow& win, int b0, int t0, int nt) {
        const size_t total = (size_t)nt * kv_dim;
        const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
        if (f.head_dim == 128)
            hipLaunchKernelGGL(kv_export_kernel<128>, dim3(blocks), dim3(256), 0, st, rq, win, b0, (bf16*)k_out, (bf16*)v_out, t0, nt);
        else
            hipLaunchKernelGGL(kv_export_kernel<64>, dim3(blocks), dim3(256), 0, st, rq, win, b0, (bf16*)k_out, (bf16*)v_out, t0, nt);
    });
    RS_HIP(hipGetLastError());
    return RS_OK;
}

rs_status rs_kv_import(rs_kv* kv, int layer, const void* k, const void* v, int n_tokens, void* stream) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    {
        const rs_status s = import_check(kv, layer, n_tokens);
        if (s != RS_OK) return s;
    }
    if (n_tokens == 0) {
        kv->len[layer] = 0;
        if (kv->paged()) kv->give_back_pages(layer, 0);
        return RS_OK;
    }
    if (!k || !v) return fail(RS_EINVAL, "k / v is null");
    if (!kv->ctx->has_device) return fail(RS_EHIP, "no HIP device");
    const rs_layer_cfg& f = kv->ctx->cfg;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int kv_dim = kv->ctx->kv_dim;
    if (kv->paged()) {
        kv->take_pages(layer, n_tokens);
        kv->give_back_pages(layer, n_tokens);
    }
    if (kv->fp8) {
        const rs_status s = fp8_import(kv, layer, (const bf16*)k, (const bf16*)v, nullptr, nullptr, n_tokens, st);
        if (s == RS_OK) kv->len[layer] = n_tokens;
        return s;
    }
    for_each_kv_window(kv, layer, n_tokens, [&](const ReqDesc& rq, const KVPageWindow& win, int b0, int t0, int nt) {
        const size_t total = align_up((size_t)nt, 64) * kv_dim;
        const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
        if (f.head_dim == 128)
            hipLaunchKernelGGL(kv_import_kernel<128>, dim3(blocks), dim3(256), 0, st, rq, win, b0, (const bf16*)k, (const bf16*)v, t0, nt);
        else
            hipLaunchKernelGGL(kv_import_kernel<64>, dim3(blocks), dim3(256), 0, st, rq, win, b0, (const bf16*)k, (const bf16*)v, t0, nt);
    });
    RS_HIP(hipGetLastError());
    kv->len[layer] = n_tokens;
    return RS_OK;
}

rs_status rs_kv_export_codes(const rs_kv* kv, int layer, void* k_codes, void* v_codes, void* stream) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    if (!kv->fp8) return fail(RS_ESTATE, "not an 8-bit cache");
    if (layer < 0 || layer >= kv->n_layers) return fail(RS_EINVAL, "layer %d out of range", layer);
    if (kv->len[layer] == 0) return RS_OK;
    if (!k_codes || !v_codes) return fail(RS_EINVAL, "k_codes / v_codes is null");
    if (!kv->ctx->has_device) return fail(RS_EHIP, "no HIP device");
    return fp8_export(kv, layer, nullptr, nullptr, (uint8_t*)k_codes, (uint8_t*)v_codes, reinterpret_cast<hipStream_t>(stream));
}

rs_status rs_kv_import_codes(rs_kv* kv, int layer, const void* k_codes, const void* v_codes, int n_tokens, void* stream) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    if (!kv->fp8) return fail(RS_ESTATE, "not an 8-bit cache");
    {
        const rs_status s = import_check(kv, layer, n_tokens);
        if (s != RS_OK) return s;
    }
    if (n_tokens == 0) {
        kv->len[layer] = 0;
        if (kv->paged()) kv->give_back_pages(layer, 0);
        return RS_OK;
    }
    if (!k_codes || !v_codes) return fail(RS_EINVAL, "k_codes / v_codes is null");
    if (!kv->ctx->has_device) return fail(RS_EHIP, "no HIP device");
    if (kv->paged()) {
        kv->take_pages(layer, n_tokens);
        kv->give_back_pages(layer, n_tokens);
    }
    const rs_status s = fp8_import(kv, layer, nullptr, nullptr, (const uint8_t*)k_codes, (const uint8_t*)v_codes, n_tokens,
                                   reinterpret_cast<hipStream_t>(stream));
    if (s == RS_OK) kv->len[layer] = n_tokens;
    return s;
}

rs_status rs_profile_enable(rs_ctx* c, int step, int max_launches) {
    if (!c) return fail(RS_EINVAL, "ctx is null");
    if (step < -1 || step >= RS_STEP_COUNT) return fail(RS_EINVAL, "step %d out of range", step);
    if (step >= 0 && max_launches <= 0) return fail(RS_EINVAL, "max_launches must be positive");
    if (step >= 0 && !c->has_device) return fail(RS_EHIP, "no HIP device");
    c->prof_step = step;
    c->prof_count = 0;
    c->prof_seen = 0;
    c->prof_take = false;
    while (step >= 0 && (int)c->prof_events.size() < 2 * max_launches) {
        hipEvent_t e;
        RS_HIP(hipEventCreate(&e));
        c->prof_events.push_back(e);
    }
    return RS_OK;
}

rs_status rs_profile_sample_every(rs_ctx* c, int every) {
    if (!c) return fail(RS_EINVAL, "ctx is null");
    if (every <= 0) return fail(RS_EINVAL, "every = %d must be positive", every);
    c->prof_every = every;
    return RS_OK;
}

rs_status rs_profile_read(rs_ctx* c, double* total_ms, int* launches) {
    if (!c || !total_ms || !launches) return fail(RS_EINVAL, "null argument");
    double sum = 0.0;
    for (int i = 0; i < c->prof_count; ++i) {
        RS_HIP(hipEventSynchronize(c->prof_events[2 * i + 1]));
        float ms = 0.0f;
        RS_HIP(hipEventElapsedTime(&ms, c->prof_events[2 * i], c->prof_events[2 * i + 1]));
        sum += ms;
    }
    *total_ms = sum;
    *launches = c->prof_count;
    c->prof_count = 0;
    return RS_OK;
}

size_t rs_workspace_bytes(const rs_ctx* c, int max_tokens, int max_requests) {
    if (!c || max_tokens <= 0 || max_requests <= 0) return 0;
    return ws_layout(c, max_tokens, max_requests).total;
}

size_t rs_workspace_bytes_fp8kv(const rs_ctx* c, int max_tokens, int max_requests, size_t max_visible_tokens) {
    if (!c || max_tokens <= 0 || max_requests <= 0) return 0;
    // every request's share is rounded up to whole 64-token blocks
    return ws_layout(c, max_tokens, max_requests).total + fp8_expansion_bytes(c, (long)max_visible_tokens + 63L * max_requests);
}

rs_status rs_prefill_chunk(rs_ctx* ctx, const rs_layer_weights* packed, int layer, rs_kv* kv, const void* x, int T, void* y,
                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!kv) return fail(RS_EINVAL, "kv is null");
    if (T < 0) return fail(RS_EINVAL, "T = %d is negative", T);
    rs_kv* kvs[1] = {kv};
    int lens[1] = {T};
    return prefill_impl(ctx, packed, layer, kvs, lens, 1, x, y, workspace, workspace_bytes, stream);
}

size_t rs_static_workspace_bytes(void) { return RS_STATIC_WORKSPACE_BYTES; }

rs_status rs_prefill_chunk_static(rs_ctx* ctx, const rs_layer_weights* packed, int layer, rs_kv* kv, const void* x, int T, void* y,
                                  void* stream) {
    if (!ctx) return fail(RS_EINVAL, "ctx is null");
    if (!kv) return fail(RS_EINVAL, "kv is null");
    if (T < 0) return fail(RS_EINVAL, "T = %d is negative", T);
    if (ctx->has_device) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
            return fail(RS_ESTATE, "the current GPU (%d) is not the one the context was created on (%d)", dev, ctx->device);
    }
    // (a host-only context has no array to point at; every check before the missing device still runs, on a stand-in address)
    void* ws = ctx->has_device ? ctx->static_ws : reinterpret_cast<void*>(uintptr_t{256});
    rs_kv* kvs[1] = {kv};
    int lens[1] = {T};
    const rs_status s = prefill_impl(ctx, packed, layer, kvs, lens, 1, x, y, ws, RS_STATIC_WORKSPACE_BYTES, stream);
    if (s == RS_EWORKSPACE) {
        const std::string why = g_last_error;
        return fail(RS_EWORKSPACE, "%s: beyond the static workspace of rs_prefill_chunk_static (use rs_prefill_chunk with a workspace of the caller's)",
                    why.c_str());
    }
    return s;
}

rs_status rs_prefill_batch(rs_ctx* ctx, const rs_layer_weights* packed, int layer, rs_kv* const* kvs, const int* chunk_lens, int R,
                           const void* x, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_impl(ctx, packed, layer, kvs, chunk_lens, R, x, y, workspace, workspace_bytes, stream);
}

rs_status rs_ctx_set_mrope_sections(rs_ctx* c, int temporal, int height, int width) {
    if (!c) return fail(RS_EINVAL, "ctx is null");
    if (temporal < 0 || height < 0 || width < 0 || temporal + height + width != c->cfg.head_dim / 2)
        return fail(RS_EINVAL, "sections %d + %d + %d must be non-negative and sum to head_dim / 2 = %d", temporal, height, width,
                    c->cfg.head_dim / 2);
    if (temporal % 4 || height % 4 || width % 4) return fail(RS_EINVAL, "each section must be a multiple of 4 rotary pairs");
    c->mrope_b0 = temporal;
    c->mrope_b1 = temporal + height;
    return RS_OK;
}

rs_status rs_prefill_batch_mrope(rs_ctx* ctx, const rs_layer_weights* packed, int layer, rs_kv* const* kvs, const int* chunk_lens,
                                 int R, const int* positions, const void* x, void* y, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    if (!positions) return fail(RS_EINVAL, "positions is null");
    return prefill_impl(ctx, packed, layer, kvs, chunk_lens, R, x, y, workspace, workspace_bytes, stream, positions);
}

static rs_status model_batch(rs_ctx* ctx, const rs_layer_weights* packed_layers, int n_layers, rs_kv* const* kvs, const int* chunk_lens,
                             int R, const int* positions3, const void* x, void* y, void* workspace, size_t workspace_bytes,
                             void* stream) {
    if (!packed_layers) return fail(RS_EINVAL, "packed_layers is null");
    if (n_layers <= 0) return fail(RS_EINVAL, "n_layers = %d must be positive", n_layers);
    int T = 0;
    PoolNeed need;
    for (int l = 0; l < n_layers; ++l) {  // all checks first: a failing call leaves every cache untouched
        const rs_status s = prefill_check(ctx, &packed_layers[l], l, kvs, chunk_lens, R, x, y, workspace, workspace_bytes, &T,
                                          positions3, &need);
        if (s != RS_OK) return s;
    }
    {
        const rs_status s = check_need(need);  // paged caches: the pages of all layers together must be there
        if (s != RS_OK) return s;
    }
    if (T > 0 && !ctx->has_device) return fail(RS_EHIP, "no HIP device: the context was created on a host without a GPU");
    if (T == 0) return RS_OK;
    // Layer 0 reads x; later layers work on y in place.  Between two layers the split-K sum of the down projection, the
    // pass that takes the next layer's norm factors and the copy into its GEMMs' operand layout are one kernel (see
    // rms_and_fragment_major_kernel<true>): the bits are those of the layers called one by one.
    PendingReduce pending;
    for (int l = 0; l < n_layers; ++l) {
        PendingReduce next;
        const rs_status s = prefill_enqueue(ctx, &packed_layers[l], l, kvs, chunk_lens, R, T, l == 0 ? x : y, y, workspace, stream,
                                            positions3, l > 0 ? &pending : nullptr, l + 1 < n_layers ? &next : nullptr);
        if (s != RS_OK) return s;
        pending = next;
    }
    return RS_OK;
}

rs_status rs_prefill_model_batch(rs_ctx* ctx, const rs_layer_weights* packed_layers, int n_layers, rs_kv* const* kvs,
                                 const int* chunk_lens, int R, const void* x, void* y, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    return model_batch(ctx, packed_layers, n_layers, kvs, chunk_lens, R, nullptr, x, y, workspace, workspace_bytes, stream);
}

rs_status rs_prefill_model_batch_mrope(rs_ctx* ctx, const rs_layer_weights* packed_layers, int n_layers, rs_kv* const* kvs,
                                       const int* chunk_lens, int R, const int* positions, const void* x, void* y, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    if (!positions) return fail(RS_EINVAL, "positions is null");
    return model_batch(ctx, packed_layers, n_layers, kvs, chunk_lens, R, positions, x, y, workspace, workspace_bytes, stream);
}

size_t rs_lm_head_workspace_bytes(const rs_ctx* c, int n_rows) {
    if (!c || n_rows <= 0) return 0;
    return align_up((size_t)n_rows * c->cfg.hidden * 4, 256);
}

rs_status rs_lm_head(rs_ctx* c, const void* final_norm_gain, const void* w_lm, int vocab, const void* x, int n_rows, void* logits,
                     void* workspace, size_t workspace_bytes, void* stream) {
    if (!c) return fail(RS_EINVAL, "ctx is null");
    if (n_rows < 0) return fail(RS_EINVAL, "n_rows = %d is negative", n_rows);
    if (vocab <= 0) return fail(RS_EINVAL, "vocab = %d must be positive", vocab);
    if (n_rows == 0) return RS_OK;
    if (!final_norm_gain || !w_lm || !x || !logits || !workspace) return fail(RS_EINVAL, "null argument");
    if (!aligned(final_norm_gain, 16) || !aligned(w_lm, 16) || !aligned(x, 16) || !aligned(logits, 4) || !aligned(workspace, 256))
        return fail(RS_EINVAL, "misaligned argument");
    if (workspace_bytes < rs_lm_head_workspace_bytes(c, n_rows))
        return fail(RS_EWORKSPACE, "workspace has %zu bytes, this call needs %zu", workspace_bytes, rs_lm_head_workspace_bytes(c, n_rows));
    // the kernel keeps its group of normalised rows (fp32) in LDS: as many rows per launch, up to LM_ROWS, as 160 KB hold
    constexpr size_t LDS_BYTES = 160 * 1024;
    const int H = c->cfg.hidden;
    if ((size_t)H * 4 > LDS_BYTES) return fail(RS_EINVAL, "hidden = %d: one fp32 row does not fit the %zu bytes of LDS the head kernel stages it in", H, LDS_BYTES);
    if (!c->has_device) return fail(RS_EHIP, "no HIP device");
    if (c->lm_rows == 0) {  // first use on this context: opt in to the LDS size once
        const int rows = (int)std::min<size_t>(LM_ROWS, LDS_BYTES / ((size_t)H * 4));
        RS_HIP(hipFuncSetAttribute((const void*)lm_head_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, rows * H * 4));
        c->lm_rows = rows;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    float* h = reinterpret_cast<float*>(workspace);
    hipLaunchKernelGGL(final_norm_kernel, dim3((n_rows + 3) / 4), dim3(256), 0, st, (const bf16*)x, (const bf16*)final_norm_gain, h,
                       n_rows, H, c->cfg.rms_eps);
    RS_HIP(hipGetLastError());
    const int blocks = std::min(4 * c->n_cu, (vocab + 4 * LM_VGROUP - 1) / (4 * LM_VGROUP));
    for (int r0 = 0; r0 < n_rows; r0 += c->lm_rows) {  // the vocabulary matrix is streamed once per group of rows
        const int R = std::min(c->lm_rows, n_rows - r0);
        hipLaunchKernelGGL(lm_head_kernel, dim3(blocks), dim3(256), (size_t)R * H * 4, st, (const bf16*)w_lm, (const float*)(h + (size_t)r0 * H),
                           reinterpret_cast<float*>(logits) + (size_t)r0 * vocab, R, vocab, H);
        RS_HIP(hipGetLastError());
    }
    return RS_OK;
}

}  // extern "C"
