// Chunk-vs-cache causal GQA attention for gfx950 (flash-style, one pass over the keys, online softmax).
//
// Work item = (request, KV head, block of 128 query rows).  The g = Hq/Hkv query heads that share a KV head are
// stacked into the row dimension: row r of a request's chunk means (token r / g, head r % g), so each K / V tile
// is fetched once per KV head rather than once per query head.  A 256-thread workgroup (4 wavefronts x 32 query
// rows) walks the request's cache in tiles of 64 keys.
//
// The kernel computes transposed products so that every per-query quantity lives in one lane:
//   S^T[key, query] = K[key, :] . Q[query, :]      MFMA "A" = K rows from LDS, "B" = Q rows held in registers
//   O^T[d,   query] = sum_key V^T[d, key] P^T[key, query]    "A" = V^T rows from LDS, "B" = P^T from the S^T registers
// With v_mfma_f32_32x32x16_bf16 a lane's accumulator column is one query (lane & 31); the two half-waves hold
// different keys (or different d) of that query.  The running max therefore needs a single cross-half exchange per
// tile and everything else of the online softmax is lane-local.  The MFMA row -> key assignment swaps two index
// bits so that the 8 probabilities a lane must feed to one k-step of the second product are 8 consecutive keys
// sitting in 8 consecutive accumulator registers (no data movement between the two products).
//
// Cache layout (private to the library): K is [Hkv][capacity][d]; V is stored transposed in blocks of 64 tokens,
// [Hkv][capacity/64][d][64], so that a V^T tile is one contiguous 64*d*2-byte run with the key index innermost,
// which is what the MFMA A operand needs.  A paged cache keeps the same 64-token tiles, gathered per page instead of per
// plane (see KVHeadTiles).  Positions >= len inside the last V block hold zeros (the append and import kernels
// maintain this), so masked probabilities (exact zeros) never meet NaN bit patterns.
#pragma once
#include "common.h"

struct ReqDesc {
    int row0;       // first row of this request in the packed [sum T, ...] activations
    int T;          // rows this call
    int P;          // tokens already cached before this call
    int cap;        // capacity (tokens, multiple of 64) of this request's cache (contiguous caches)
    bf16* kcache;   // contiguous: this layer's K [Hkv][cap][d];  paged: the pool's first page
    bf16* vtcache;  // contiguous: this layer's V^T [Hkv][cap/64][d][64];  paged: unused
    const int* pages;  // paged: pages[b] = pool page that holds this layer's 64-token block b;  contiguous: null
    int hkv;           // KV heads (a page is [Hkv] K tiles followed by [Hkv] V^T tiles)
    int pad_;
};

// Where the 64-token tiles of one KV head live.  A tile is K rows [64][d] or V^T [d][64], either one contiguous run of
// 64*D*2 bytes, at  base + index * stride:  in a contiguous cache both planes are arrays of tiles [kvh][block], so the
// index is the block and the stride one tile; in a paged cache the index is the block's page (looked up in the request's
// table, a uniform load) and the stride one page, which holds the K tiles of all heads followed by their V^T tiles.
// Set up once per workgroup, so that a tile's address costs one multiply-add in the loop whatever the kind of cache.
struct KVHeadTiles {
    char* k_base;
    char* v_base;
    uint32_t stride;
    const int* pages;
    // MAY_PAGE = false is for kernels launched only when every cache of the call is contiguous: no lookup, and nothing
    // in the loop that the compiler cannot see to be uniform (the software-pipelined attention kernel is about 3 % slower
    // with the lookup in its loop).
    // The index of a block: may be called long before the address is needed (the lookup's latency then passes unseen).
    template <bool MAY_PAGE = true>
    __device__ __forceinline__ int index_of(int block) const {
        if constexpr (!MAY_PAGE) return block;
        // (a load through the global address space: a generic pointer gives a flat load, which counts on the LDS counter
        //  as well, and every wait for an LDS fragment while it is in flight then becomes a wait for all of them)
        typedef const __attribute__((address_space(1))) int* global_ints;
        return pages == nullptr ? block : ((global_ints)pages)[block];
    }
    // (the index is the same for the whole wavefront; saying so here, where the value is used and not where it was
    // loaded, keeps the address in scalar registers, which the buffer resource of an LDS-DMA load needs)
    template <bool MAY_PAGE = true>
    __device__ __forceinline__ char* k_tile(int index) const {
        if constexpr (!MAY_PAGE) return k_base + (size_t)(uint32_t)index * stride;
        return k_base + (size_t)(uint32_t)__builtin_amdgcn_readfirstlane(index) * stride;
    }
    template <bool MAY_PAGE = true>
    __device__ __forceinline__ char* v_tile(int index) const {
        if constexpr (!MAY_PAGE) return v_base + (size_t)(uint32_t)index * stride;
        return v_base + (size_t)(uint32_t)__builtin_amdgcn_readfirstlane(index) * stride;
    }
};
template <int D>
RS_DEVICE KVHeadTiles kv_head_tiles(const ReqDesc& rq, int kvh) {
    constexpr uint32_t TILE = 64u * D * 2u;
    KVHeadTiles t;
    t.pages = rq.pages;
    if (rq.pages == nullptr) {
        const size_t head = (size_t)kvh * (size_t)(rq.cap >> 6) * TILE;
        t.k_base = reinterpret_cast<char*>(rq.kcache) + head;
        t.v_base = reinterpret_cast<char*>(rq.vtcache) + head;
        t.stride = TILE;
    } else {
        t.k_base = reinterpret_cast<char*>(rq.kcache) + (size_t)kvh * TILE;
        t.v_base = reinterpret_cast<char*>(rq.kcache) + (size_t)(rq.hkv + kvh) * TILE;
        t.stride = 2u * (uint32_t)rq.hkv * TILE;
    }
    return t;
}

constexpr int ATT_ROWS = 128;  // stacked query rows per workgroup
constexpr int ATT_KEYS = 64;   // keys per tile

struct AttnItem {
    int req;
    int kvh;
    int qblock;  // block of 128 stacked query rows
    int nkb;     // number of 64-key tiles this block must visit (tiles [0, nkb), or [kb0, nkb) for a part of a split block)
    int kb0;     // first tile of this part (0 unless the block's key range is split)
    int slot;    // -1: the workgroup finishes the block and writes the output; >= 0: it leaves an unnormalised partial
                 // result in this slot of the split buffer (see AttnPartial) for attn_merge_kernel
    int pad0_, pad1_;
};

// Split key ranges.  With few query rows and a long cache there are fewer blocks than compute units (a 256-token chunk
// at the 7B shape gives 56), each walking the whole cache.  The host then cuts a block's tiles into up to ATT_MAX_PARTS consecutive
// parts, one workgroup each; a part leaves  O~ = sum_k 2^((s_k - m) c) v_k  (fp32, unnormalised), its reference maximum m
// and its row sums l in a slot of the split buffer, and attn_merge_kernel combines the parts of a block:
//   M = max_p m_p,  w_p = 2^((m_p - M) c),  out = sum_p w_p O~_p / sum_p w_p l_p.
// A slot holds 128 rows: O~ as [D/4 chunks of 4 floats][128 rows] (the 32 lanes of a store cover 512 contiguous bytes),
// then m[128], then l[128].
constexpr int ATT_MAX_PARTS = 16;
template <int D>
struct AttnPartial {
    static constexpr int CHUNKS = D / 4;
    static constexpr size_t SLOT_FLOATS = (size_t)ATT_ROWS * (D + 2);
};

// The kernel keeps a query's reference maximum until a tile's maximum exceeds it by more than this
// many powers of two (in the exponent's units, i.e. after the 1/sqrt(d) log2 e scaling): probabilities then reach at most
// 2^8 instead of 1, which fp32 sums and bf16's relative rounding do not mind, and the final division by the row sum
// cancels the reference.  Rescaling the accumulated output is thereby confined to a request's first tiles; with an
// exact running maximum some query of a wavefront grows its maximum in almost every tile.
constexpr float ATT_RESCALE_LOG2 = 8.0f;

// ------------------------------------------------------------------------------------------------------------------
// The kernel is software-pipelined across key tiles.  Per key tile a wavefront has two kinds of work: 32 MFMAs (the two
// products) and the online softmax on the vector ALU (per score a scaling, an exponential - v_exp_f32 issues at 1.2 times
// the cost of a v_fma_f32 on this chip, measured -, the running maximum, the row sum and half a bf16 conversion: about
// 600 issue clocks against 1024 of MFMA); run one after the other, the matrix pipe idles a third of the time.  Here the score product of tile kb+1 is issued between the exponentials of tile
// kb, and the running maximum of tile kb+1 is formed behind the MFMAs of the P.V product of tile kb, so each pipe works
// in the shadow of the other.  K therefore runs one tile ahead of V: iteration kb reads K(kb+1) and V(kb) from LDS while
// K(kb+2) and V(kb+1) travel global -> LDS by DMA (buffer_load ... lds: no staging registers) into the buffers that
// iteration kb-1 finished with.  The four buffers are separate LDS objects so that the compiler can tell that the
// fragment reads of an iteration do not touch the buffers being filled; it waits for the DMA at the barrier that ends
// the iteration.  Two workgroups share a compute unit (256 registers per lane each).
template <int D, bool MAY_PAGE>
__global__ __launch_bounds__(256, 2) void attn_prefill_pipelined_kernel(const ReqDesc* __restrict__ reqs,
                                                                        const AttnItem* __restrict__ items,
                                                                        const bf16* __restrict__ qkv, int ld_qkv,
                                                                        bf16* __restrict__ out, int ld_out,
                                                                        int g, float scale_log2e,
                                                                        float* __restrict__ split_buf) {
    constexpr int KSTEPS = D / 16;
    constexpr int DT = D / 32;
    constexpr int K_ROW_BYTES = D * 2;
    constexpr int K_CPR = K_ROW_BYTES / 16;
    constexpr int TILE_BYTES = ATT_KEYS * D * 2;
    constexpr int LOADS = TILE_BYTES / (256 * 16);
    typedef __attribute__((address_space(3))) void* lds_ptr;
    __shared__ __attribute__((aligned(16))) char k_buf0[TILE_BYTES];
    __shared__ __attribute__((aligned(16))) char k_buf1[TILE_BYTES];
    __shared__ __attribute__((aligned(16))) char v_buf0[TILE_BYTES];
    __shared__ __attribute__((aligned(16))) char v_buf1[TILE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    const AttnItem item = items[blockIdx.x];
    const ReqDesc rq = reqs[item.req];
    const int rows_total = rq.T * g;
    const int row = item.qblock * ATT_ROWS + wave * 32 + l32;
    const int row_c = min(row, rows_total - 1);
    const int tok = row_c / g;
    const int head = item.kvh * g + (row_c - tok * g);
    const int qpos = rq.P + tok;
    const int wrow_lo = min(item.qblock * ATT_ROWS + wave * 32, rows_total - 1);
    const int wpos_lo = rq.P + wrow_lo / g;  // every query of this wavefront sees all keys <= wpos_lo

    bf16x8 qf[KSTEPS];
    {
        const bf16* qp = qkv + (size_t)(rq.row0 + tok) * ld_qkv + head * D + half * 8;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
    }

    // ---- tile loader: a tile is a contiguous TILE_BYTES run of this KV head's cache; load instruction i of a wavefront
    //      fills LDS bytes [(i*256 + wave*64)*16, +1 KB) linearly by lane, each lane fetching the 16-byte chunk that
    //      belongs in its (swizzled) place.  Tiles past the item's last one are not fetched.
    const int nkb = item.nkb;
    uint32_t k_src_off[4], v_src_off[4];  // (fixed bound: LOADS <= 4; a template-dependent bound breaks the host-side stub)
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int q = i * 256 + tid;
        {
            const int r = q / K_CPR, p = q % K_CPR;
            const int c = (K_CPR == 16) ? (p ^ (r & 15)) : (p ^ ((r >> 1) & 7));
            k_src_off[i] = (uint32_t)(r * K_ROW_BYTES + c * 16);
        }
        {
            const int r = q >> 3, p = q & 7;
            const int c = p ^ ((r >> 1) & 7);
            v_src_off[i] = (uint32_t)(r * 128 + c * 16);
        }
    }
    // (the page of a tile is looked up one iteration before the tile is fetched: see the iteration)
    const KVHeadTiles tiles = kv_head_tiles<D>(rq, item.kvh);
    auto page_of = [&](int kb) { return kb < nkb ? tiles.template index_of<MAY_PAGE>(kb) : 0; };
    auto fetch_k = [&](char* buf, int kb, int page) {
        if (kb < nkb) {
            const __amdgpu_buffer_rsrc_t rk =
                __builtin_amdgcn_make_buffer_rsrc((void*)tiles.template k_tile<MAY_PAGE>(page), 0, TILE_BYTES, 0x00020000);
#pragma unroll
            for (int i = 0; i < LOADS; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_ptr)(uintptr_t)(uint32_t)(uintptr_t)(buf + (i * 256 + wave * 64) * 16), 16, k_src_off[i],
                                                         0, 0, 0);
        }
    };
    auto fetch_v = [&](char* buf, int kb, int page) {
        if (kb < nkb) {
            const __amdgpu_buffer_rsrc_t rv =
                __builtin_amdgcn_make_buffer_rsrc((void*)tiles.template v_tile<MAY_PAGE>(page), 0, TILE_BYTES, 0x00020000);
#pragma unroll
            for (int i = 0; i < LOADS; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_ptr)(uintptr_t)(uint32_t)(uintptr_t)(buf + (i * 256 + wave * 64) * 16), 16, v_src_off[i],
                                                         0, 0, 0);
        }
    };

    const int pi = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    uint32_t k_row_off[2], k_swz[2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        const int r = mi * 32 + pi;
        k_row_off[mi] = (uint32_t)(r * K_ROW_BYTES);
        k_swz[mi] = (K_CPR == 16) ? (uint32_t)(r & 15) : (uint32_t)((r >> 1) & 7);
    }
    const uint32_t v_swz = (uint32_t)((lane >> 1) & 7);

    f32x16 acc_o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[t][r] = 0.0f;
    float m_run = -INFINITY;  // reference maximum of the raw scores of this lane's query (shared by both half-waves)
    float l_run = 0.0f;       // running sum over THIS half-wave's keys
    float alpha = 1.0f;       // factor the accumulated output still has to be multiplied by before the next P.V
    bool rescale = false;     // some query of this wavefront moved its reference maximum (wave-uniform)

    // raw scores of one tile: register r of s[mi] holds key  key0 + mi*32 + 16*(r>>3) + 8*half + (r&7)
    auto zero_scores = [&](f32x16 (&s)[2]) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[mi][r] = 0.0f;
    };
    auto score_mfma = [&](f32x16 (&s)[2], const char* ks, int kk, int mi) {
        const uint32_t c = ((uint32_t)(kk * 2 + half) ^ k_swz[mi]) * 16u;
        bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + k_row_off[mi] + c);
        s[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[mi], 0, 0, 0);
    };
    // mask and running maximum of one tile's scores; leaves m_run updated and alpha / rescale for the output
    auto tile_max = [&](f32x16 (&s)[2], int key0) {
        if (key0 + ATT_KEYS - 1 > wpos_lo) {  // some query of this wavefront does not see the whole tile
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + mi * 32 + 16 * (r >> 3) + 8 * half + (r & 7);
                    s[mi][r] = (key <= qpos) ? s[mi][r] : -INFINITY;
                }
        }
        float mloc = s[0][0];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int r = 0; r < 16; r += 2) mloc = fmaxf(fmaxf(s[mi][r], s[mi][r + 1]), mloc);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, WAVE));
        // finite from the first tile on: key 0 is visible to every query
        const float m_new = ((mloc - m_run) * scale_log2e > ATT_RESCALE_LOG2) ? mloc : m_run;
        rescale = __builtin_amdgcn_ballot_w64(m_new != m_run) != 0;
        alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
        m_run = m_new;
    };

    // ---- prologue: K(0), V(0), K(1) into LDS; scores and maximum of tile 0
    const int kb0 = item.kb0;       // this workgroup's tiles are [kb0, nkb)
    int pg_v = page_of(kb0 + 1);   // page of block kb + 1 (V is fetched one tile behind K)
    int pg_k = page_of(kb0 + 2);   // page of block kb + 2
    {
        const int pg0 = page_of(kb0);
        fetch_k(k_buf0, kb0, pg0);
        fetch_v(v_buf0, kb0, pg0);
        fetch_k(k_buf1, kb0 + 1, pg_v);
    }
    __syncthreads();
    f32x16 sA[2], sB[2];
    zero_scores(sA);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) score_mfma(sA, k_buf0, kk, mi);
    tile_max(sA, kb0 * ATT_KEYS);
    __syncthreads();  // every wavefront is done with the first K tile: the first iteration may overwrite it

    // one iteration: scur = raw scores of tile kb (masked, maximum known); snext receives those of tile kb+1.
    // k_next holds K(kb+1), v_cur V(kb); k_fill (= K(kb)'s buffer) receives K(kb+2), v_fill (= V(kb-1)'s) V(kb+1).
    auto iteration = [&](int kb, f32x16 (&scur)[2], f32x16 (&snext)[2], const char* k_next, char* k_fill, const char* v_cur,
                         char* v_fill) {
        fetch_k(k_fill, kb + 2, pg_k);
        fetch_v(v_fill, kb + 1, pg_v);
        pg_v = pg_k;
        pg_k = page_of(kb + 3);  // needed in the next iteration: the lookup's latency passes behind this one
        const float mb = m_run * scale_log2e;
        // ---- phase 1: P(kb) = exp2(S(kb) c - m c), its row sum and bf16 form.  Behind each of the 2*KSTEPS score MFMAs of
        //      tile kb+1 go the exponentials of 32 / (2*KSTEPS) scores of tile kb; scheduling fences keep that order, and
        //      each K fragment is read from LDS one group ahead of the MFMA that uses it.
        zero_scores(snext);
        bf16x8 pf[4];
        float psum = 0.0f;
        constexpr int NS = 2 * KSTEPS;   // score MFMAs per tile
        constexpr int PER = 32 / NS;     // scores of tile kb handled behind each of them (2 for d = 128, 4 for d = 64)
        auto k_frag = [&](int step) {
            const int kk = step >> 1, mi = step & 1;
            const uint32_t c = ((uint32_t)(kk * 2 + half) ^ k_swz[mi]) * 16u;
            return *reinterpret_cast<const bf16x8*>(k_next + k_row_off[mi] + c);
        };
        bf16x8 kf = k_frag(0);
#pragma unroll
        for (int step = 0; step < NS; ++step) {
            const bf16x8 kf_next = k_frag(step + 1 < NS ? step + 1 : step);
            __builtin_amdgcn_sched_barrier(0);  // the read goes out first: its latency hides behind this group's work
            snext[step & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[step >> 1], snext[step & 1], 0, 0, 0);
#pragma unroll
            for (int e = 0; e < PER; e += 2) {
                const int idx = step * PER + e, mi = idx >> 4, r = idx & 15;
                // raw v_exp_f32: arguments are <= ATT_RESCALE_LOG2, results below the normal range may flush to zero
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(scur[mi][r], scale_log2e, -mb));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(scur[mi][r + 1], scale_log2e, -mb));
                const bf16x2 pp = {f32_to_bf16(p0), f32_to_bf16(p1)};
                // plain adds: a v_dot2 here would be one instruction instead of two, but the dot instructions do not run
                // beside an MFMA (measured: each one stalls the matrix pipe for its own duration and more)
                psum += p0 + p1;
                pf[mi * 2 + (r >> 3)][r & 7] = pp[0];
                pf[mi * 2 + (r >> 3)][(r & 7) + 1] = pp[1];
            }
            asm volatile("" : "+v"(psum));  // pins this group's vector work here (it would otherwise sink below the MFMAs)
            kf = kf_next;
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- the accumulated output catches up with the maximum of tile kb
        l_run = l_run * alpha + psum;
        if (rescale) {
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[t][r] *= alpha;
        }
        // ---- phase 2: O += V(kb)^T P(kb); behind the MFMAs, the mask and the running maximum of tile kb+1
        const int key1 = (kb + 1) * ATT_KEYS;
        const bool more = kb + 1 < nkb;
        if (more && key1 + ATT_KEYS - 1 > wpos_lo) {  // some query of this wavefront does not see the whole next tile
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key1 + mi * 32 + 16 * (r >> 3) + 8 * half + (r & 7);
                    snext[mi][r] = (key <= qpos) ? snext[mi][r] : -INFINITY;
                }
        }
        auto v_frag = [&](int step) {
            const int ksx = step / DT, t = step % DT;
            const uint32_t c = ((uint32_t)(ksx * 2 + half) ^ v_swz) * 16u;
            return *reinterpret_cast<const bf16x8*>(v_cur + (uint32_t)(t * 32 + l32) * 128u + c);
        };
        constexpr int NV = 4 * DT;       // P.V MFMAs per tile
        constexpr int MPER = 32 / NV;    // scores of tile kb+1 folded into the maximum behind each of them
        float mloc = snext[0][0];
        bf16x8 vf = v_frag(0);
#pragma unroll
        for (int step = 0; step < NV; ++step) {
            const bf16x8 vf_next = v_frag(step + 1 < NV ? step + 1 : step);
            __builtin_amdgcn_sched_barrier(0);
            acc_o[step % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[step / DT], acc_o[step % DT], 0, 0, 0);
#pragma unroll
            for (int e = 0; e < MPER; e += 2) {
                const int idx = step * MPER + e, mi = idx >> 4, r = idx & 15;
                mloc = fmaxf(fmaxf(snext[mi][r], snext[mi][r + 1]), mloc);
            }
            asm volatile("" : "+v"(mloc));
            vf = vf_next;
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) {
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32, WAVE));
            const float m_new = ((mloc - m_run) * scale_log2e > ATT_RESCALE_LOG2) ? mloc : m_run;
            rescale = __builtin_amdgcn_ballot_w64(m_new != m_run) != 0;
            alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
            m_run = m_new;
        }
        __syncthreads();
    };

    int kb = kb0;
    for (; kb + 1 < nkb; kb += 2) {
        iteration(kb, sA, sB, k_buf1, k_buf0, v_buf0, v_buf1);
        iteration(kb + 1, sB, sA, k_buf0, k_buf1, v_buf1, v_buf0);
    }
    if (kb < nkb) iteration(kb, sA, sB, k_buf1, k_buf0, v_buf0, v_buf1);

    const float l_tot = l_run + __shfl_xor(l_run, 32, WAVE);
    if (item.slot >= 0) {
        // a part of a split block: unnormalised output, reference maximum and row sum go to the slot (all 128 rows of the
        // block, clamped duplicates included: the merge kernel decides what is stored)
        float* const slot = split_buf + (size_t)item.slot * AttnPartial<D>::SLOT_FLOATS;
        const int rs = wave * 32 + l32;  // row inside the block
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 o = {acc_o[t][4 * q], acc_o[t][4 * q + 1], acc_o[t][4 * q + 2], acc_o[t][4 * q + 3]};
                // chunk (features 32t + 8q + 4half .. +3) of row rs
                *reinterpret_cast<f32x4*>(slot + ((size_t)(t * 8 + q * 2 + half) * ATT_ROWS + rs) * 4) = o;
            }
        if (half == 0) {
            slot[(size_t)D * ATT_ROWS + rs] = m_run;
            slot[(size_t)(D + 1) * ATT_ROWS + rs] = l_tot;
        }
        return;
    }
    if (row < rows_total) {
        const float inv = 1.0f / l_tot;
        const uint32_t m = (uint32_t)(rq.row0 + tok);
        char* op = reinterpret_cast<char*>(out) + (size_t)(m >> 5) * (size_t)(ld_out >> 4) * 1024 + (m & 31u) * 16u + half * 8;
        const int ks0 = (head * D) >> 4;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(acc_o[t][4 * q + e] * inv);
                *reinterpret_cast<bf16x4*>(op + (size_t)(((ks0 + 2 * t + (q >> 1)) * 2 + (q & 1)) * 512)) = o;
            }
    }
}

// Combines the parts of split blocks (see AttnPartial).  ATT_MERGE_Y workgroups per block (grid y): thread (row, c2) of
// workgroup y handles row `row` of the block and the chunks 2y + c2, 2y + c2 + 2 ATT_MERGE_Y, ... of its D/4 chunks of 4
// features - one or two chunks, so all of a thread's loads are in flight together (one workgroup per block walking its 16
// chunks one after the other took 13 us, more than a short key range saves).  Every workgroup computes the rows' weights.
constexpr int ATT_MERGE_Y = 8;
struct AttnMergeItem {
    int req;
    int kvh;
    int qblock;
    int n_parts;
    int slot0;  // the parts' slots are slot0 .. slot0 + n_parts - 1
    int pad0_, pad1_, pad2_;
};
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(const ReqDesc* __restrict__ reqs, const AttnMergeItem* __restrict__ items,
                                                         const float* __restrict__ split_buf, bf16* __restrict__ out, int ld_out,
                                                         int g, float scale_log2e) {
    const AttnMergeItem item = items[blockIdx.x];
    const ReqDesc rq = reqs[item.req];
    const int rs = threadIdx.x & (ATT_ROWS - 1), c2 = threadIdx.x >> 7;
    const int row = item.qblock * ATT_ROWS + rs;
    if (row >= rq.T * g) return;
    const int tok = row / g;
    const int head = item.kvh * g + (row - tok * g);
    const float* const base = split_buf + (size_t)item.slot0 * AttnPartial<D>::SLOT_FLOATS;
    // (all loads of a round are issued together: absent parts read as m = -inf, l = 0 and get weight 0)
    float mp[ATT_MAX_PARTS], lp[ATT_MAX_PARTS];
#pragma unroll
    for (int p = 0; p < ATT_MAX_PARTS; ++p) {
        mp[p] = -INFINITY;
        lp[p] = 0.0f;
        if (p < item.n_parts) {
            const float* sp = base + p * AttnPartial<D>::SLOT_FLOATS;
            mp[p] = sp[(size_t)D * ATT_ROWS + rs];
            lp[p] = sp[(size_t)(D + 1) * ATT_ROWS + rs];
        }
    }
    float m_all = -INFINITY;
#pragma unroll
    for (int p = 0; p < ATT_MAX_PARTS; ++p) m_all = fmaxf(m_all, mp[p]);
    float l_all = 0.0f;
    float w[ATT_MAX_PARTS];
#pragma unroll
    for (int p = 0; p < ATT_MAX_PARTS; ++p) {
        w[p] = 0.0f;
        if (p < item.n_parts) {
            w[p] = __builtin_amdgcn_exp2f((mp[p] - m_all) * scale_log2e);
            l_all += w[p] * lp[p];
        }
    }
    const float inv = 1.0f / l_all;
    const uint32_t m = (uint32_t)(rq.row0 + tok);
    char* const op = reinterpret_cast<char*>(out) + (size_t)(m >> 5) * (size_t)(ld_out >> 4) * 1024 + (m & 31u) * 16u;
    const int ks0 = (head * D) >> 4;
    static_assert(AttnPartial<D>::CHUNKS % (2 * ATT_MERGE_Y) == 0, "chunks divide among the merge workgroups");
#pragma unroll
    for (int c = 2 * blockIdx.y + c2; c < AttnPartial<D>::CHUNKS; c += 2 * ATT_MERGE_Y) {
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int p = 0; p < ATT_MAX_PARTS; ++p)
            if (p < item.n_parts) {
                const f32x4 o = *reinterpret_cast<const f32x4*>(base + p * AttnPartial<D>::SLOT_FLOATS + ((size_t)c * ATT_ROWS + rs) * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += w[p] * o[e];
            }
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = f32_to_bf16(acc[e] * inv);
        // chunk c = 8t + 2q + half holds features 32t + 8q + 4half .. +3: the same place the unsplit kernel writes
        const int t = c >> 3, q = (c >> 1) & 3, hf = c & 1;
        *reinterpret_cast<bf16x4*>(op + hf * 8 + (size_t)(((ks0 + 2 * t + (q >> 1)) * 2 + (q & 1)) * 512)) = o4;
    }
}
