// HBM-bound helper kernels: RMSNorm row factors and input repack, K / V append (V transposing), weight packing, cache
// export/import.
#pragma once
#include "attention.h"
#include "common.h"

// ---------------------------------------------------------------- layer input: RMSNorm row factor + fragment-major copy
// One pass over x: inv_rms[row] = rsqrt(mean(x[row]^2) + eps) (fp32 sums; the factor is applied inside the next GEMM's
// epilogue), and dst receives x in the GEMMs' token-operand layout: blocks of 32 tokens x 16 features, the two 8-feature
// halves 512 bytes apart, tokens 16 bytes apart (rows of the last block past `rows` are left untouched: they are never
// used).  One workgroup handles 8 tokens: 32 threads read 512 contiguous bytes of one token per step, and the 8 tokens'
// 16-byte chunks of one (k-step, half) land in 128 contiguous bytes (one cache line).
// The first workgroups of the grid copy the call's descriptors (requests, attention work items, cache blocks, row
// positions) from the pinned host buffer the library filled, which the device reads in place, into the workspace: the
// later kernels of the call then find them in device memory, and no copy command sits between two calls (a runtime copy
// of a few tens of KB costs a blit kernel of 13 us plus the gaps around it).
// REDUCE = true is the same pass with the row taken not from x but from the split-K partial planes of the previous
// layer's down projection (the layers of one rs_prefill_model_batch call): the row is
// bf16(resid[m, :] + sum_s partial[s][m][:]), summed and rounded exactly as splitk_reduce_residual_kernel does, stored
// row-major to y (the previous layer's output, this layer's residual input) and fragment-major to dst, and its 1/rms is
// taken from the rounded values in the same order as from x - so a stack of layers run this way leaves the same bits
// as the layers called one by one, without the previous layer's reduction kernel and this layer's pass over its output.
struct ReduceSource {
    const float* partial;   // [splits][rows][H] fp32
    int splits;             // 2..4
    const bf16* resid;      // [rows, H] fragment-major
    bf16* y;                // [rows, H] row-major
};
template <bool REDUCE>
__global__ __launch_bounds__(256) void rms_and_fragment_major_kernel(const bf16* __restrict__ x, bf16* __restrict__ dst,
                                                                     float* __restrict__ inv_rms, int rows, int H, float eps,
                                                                     const uint4* __restrict__ desc_src,
                                                                     uint4* __restrict__ desc_dst, int desc_chunks,
                                                                     ReduceSource red) {
    // (the copying workgroups come first in the grid: their reads cross the host link, several microseconds each, and
    // should be under way while the row blocks stream; launched last they were the tail of the kernel)
    const int desc_blocks = (desc_chunks + 255) >> 8;
    if ((int)blockIdx.x < desc_blocks) {
        const int i = (int)blockIdx.x * 256 + (int)threadIdx.x;
        if (i < desc_chunks) desc_dst[i] = desc_src[i];
        return;
    }
    const int r = threadIdx.x >> 5, c = threadIdx.x & 31;
    const int m = ((int)blockIdx.x - desc_blocks) * 8 + r;
    const int mc = min(m, rows - 1);  // threads of rows past the end follow along (their shuffles are needed) and store nothing
    const size_t frag_row = ((size_t)(mc >> 5) * (H >> 4) * 2 + c) * 512 + (mc & 31) * 16;   // chunk c of row mc, fragment-major
    const char* src = REDUCE ? reinterpret_cast<const char*>(red.resid) + frag_row
                             : reinterpret_cast<const char*>(x + (size_t)mc * H) + c * 16;
    constexpr size_t SRC_STEP = REDUCE ? 512 : 16;   // bytes from one 16-byte chunk of the row to the next in the source
    char* out = reinterpret_cast<char*>(dst) + ((size_t)(m >> 5) * (H >> 4) * 2 + c) * 512 + (m & 31) * 16;
    float ss = 0.0f;
    const int chunks = H >> 3;  // 16-byte chunks per row; a step covers 32 of them (256 features = 16 k-steps x 2 halves)
    constexpr int U = 4;   // chunks in flight per thread (eight measured no faster for either form)
    for (int c0 = 0; c0 < chunks; c0 += U * 32) {
        uint4 v[U];
        f32x4 part[REDUCE ? U : 1][REDUCE ? 4 : 1][2];   // [chunk in flight][plane][half of the 8 features]
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c0 + u * 32 + c < chunks) {
                v[u] = ld_global_16(src + (size_t)(c0 + u * 32) * SRC_STEP);
                if constexpr (REDUCE) {
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp)
                        if (sp < red.splits) {
                            const float* pp = red.partial + ((size_t)sp * rows + mc) * H + (size_t)(c0 + u * 32 + c) * 8;
                            part[u][sp][0] = *reinterpret_cast<const f32x4*>(pp);
                            part[u][sp][1] = *reinterpret_cast<const f32x4*>(pp + 4);
                        }
                }
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c0 + u * 32 + c < chunks) {
                bf16x8 h = as_bf16x8(v[u]);
                if constexpr (REDUCE) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float f = bf16_to_f32(h[e]);
#pragma unroll
                        for (int sp = 0; sp < 4; ++sp)
                            if (sp < red.splits) f += part[u][sp][e >> 2][e & 3];
                        h[e] = f32_to_bf16(f);
                    }
                    if (m < rows) st_global_16(reinterpret_cast<char*>(red.y + (size_t)m * H) + (size_t)(c0 + u * 32 + c) * 16, as_uint4(h));
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float f = bf16_to_f32(h[e]);
                    ss += f * f;
                }
                if (m < rows) st_global_16(out + (size_t)(c0 + u * 32) * 512, as_uint4(h));
            }
    }
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) ss += __shfl_xor(ss, off, WAVE);
    if (c == 0 && m < rows) inv_rms[m] = rsqrtf(ss / (float)H + eps);
}

// ---------------------------------------------------------------- first-token head: final RMSNorm + vocabulary projection
// h[r][k] = x[r][k] * g[k] * rsqrt(mean(x[r]^2) + eps), kept in fp32.  One wavefront per row.
__global__ __launch_bounds__(256) void final_norm_kernel(const bf16* __restrict__ x, const bf16* __restrict__ gain,
                                                         float* __restrict__ h, int rows, int H, float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const bf16* xr = x + (size_t)row * H;
    float ss = 0.0f;
    for (int c = lane; c < H / 8; c += WAVE) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += bf16_to_f32(v[e]) * bf16_to_f32(v[e]);
    }
    ss = wave_sum(ss);
    const float inv = rsqrtf(ss / (float)H + eps);
    for (int c = lane; c < H / 8; c += WAVE) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c * 8);
        const bf16x8 g = *reinterpret_cast<const bf16x8*>(gain + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) h[(size_t)row * H + c * 8 + e] = bf16_to_f32(v[e]) * inv * bf16_to_f32(g[e]);
    }
}

// logits[r][v] = sum_k h[r][k] * w[v][k] for R <= LM_ROWS rows at a time.  HBM-bound on the vocabulary matrix (read once):
// the normalised rows sit in LDS (fp32); each wavefront walks the vocabulary four rows at a time, its 64 lanes covering
// K in contiguous 16-byte chunks (1 KB per load instruction and row), so that one LDS read of the activations serves
// four weight rows; lanes are reduced at the end of the group.
constexpr int LM_ROWS = 4;
constexpr int LM_VGROUP = 4;
__global__ __launch_bounds__(256) void lm_head_kernel(const bf16* __restrict__ w, const float* __restrict__ h,
                                                      float* __restrict__ logits, int R, int vocab, int H) {
    extern __shared__ __attribute__((aligned(16))) float h_lds[];  // [R][H]
    for (int i = threadIdx.x; i < R * H / 4; i += blockDim.x)
        reinterpret_cast<f32x4*>(h_lds)[i] = reinterpret_cast<const f32x4*>(h)[i];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    for (int v0 = (blockIdx.x * 4 + wave) * LM_VGROUP; v0 < vocab; v0 += gridDim.x * 4 * LM_VGROUP) {
        const bf16* wr[LM_VGROUP];
#pragma unroll
        for (int j = 0; j < LM_VGROUP; ++j) wr[j] = w + (size_t)min(v0 + j, vocab - 1) * H;  // rows past the end repeat the last one
        float acc[LM_VGROUP][LM_ROWS];
#pragma unroll
        for (int j = 0; j < LM_VGROUP; ++j)
#pragma unroll
            for (int r = 0; r < LM_ROWS; ++r) acc[j][r] = 0.0f;
        for (int c = lane; c < H / 8; c += WAVE) {
            bf16x8 wv[LM_VGROUP];
#pragma unroll
            for (int j = 0; j < LM_VGROUP; ++j) wv[j] = *reinterpret_cast<const bf16x8*>(wr[j] + c * 8);
#pragma unroll
            for (int r = 0; r < LM_ROWS; ++r)
                if (r < R) {
                    const f32x4 h0 = *reinterpret_cast<const f32x4*>(h_lds + (size_t)r * H + c * 8);
                    const f32x4 h1 = *reinterpret_cast<const f32x4*>(h_lds + (size_t)r * H + c * 8 + 4);
#pragma unroll
                    for (int j = 0; j < LM_VGROUP; ++j)
                        acc[j][r] += bf16_to_f32(wv[j][0]) * h0[0] + bf16_to_f32(wv[j][1]) * h0[1] + bf16_to_f32(wv[j][2]) * h0[2] +
                                     bf16_to_f32(wv[j][3]) * h0[3] + bf16_to_f32(wv[j][4]) * h1[0] + bf16_to_f32(wv[j][5]) * h1[1] +
                                     bf16_to_f32(wv[j][6]) * h1[2] + bf16_to_f32(wv[j][7]) * h1[3];
                }
        }
#pragma unroll
        for (int j = 0; j < LM_VGROUP; ++j)
#pragma unroll
            for (int r = 0; r < LM_ROWS; ++r)
                if (r < R) {
                    const float t = wave_sum(acc[j][r]);
                    if (lane == 0 && v0 + j < vocab) logits[(size_t)r * vocab + v0 + j] = t;
                }
    }
}

// ---------------------------------------------------------------- K / V append
struct KVBlockItem {
    int req;
    int block;  // absolute 64-token block index in the request's cache
};

// One workgroup per (touched 64-token block, KV head).  The rotated k rows are copied from the qkv buffer to the
// request's K cache (256-byte rows, 16-byte vector copies).  The v rows are transposed through LDS and written as
// [d][64] with the token index innermost, 16 bytes (8 tokens) per store.  Tokens before P keep their content; V
// positions at or beyond P+T inside the block are zero-filled.
template <int D>
__global__ __launch_bounds__(256) void append_kv_kernel(const bf16* __restrict__ qkv, int ld_qkv,
                                                        const ReqDesc* __restrict__ reqs,
                                                        const KVBlockItem* __restrict__ blocks, int Hq, int Hkv) {
    __shared__ __attribute__((aligned(16))) bf16 tile[64][D + 8];  // row stride D*2 + 16 bytes: 16-byte aligned, odd in 16-byte units
    const KVBlockItem it = blocks[blockIdx.x];
    const ReqDesc rq = reqs[it.req];
    const int c = blockIdx.y;
    const int tok0 = it.block * 64;
    const int k_col = (Hq + c) * D;
    const int v_col = (Hq + Hkv + c) * D;
    constexpr int CPR = D / 8;  // 16-byte chunks per row
    const KVHeadTiles tiles = kv_head_tiles<D>(rq, c);
    const int tile_index = tiles.index_of(it.block);
    bf16* const k_tile = reinterpret_cast<bf16*>(tiles.k_tile(tile_index));
    for (int idx = threadIdx.x; idx < 64 * CPR; idx += blockDim.x) {
        const int kk = idx / CPR, ch = idx - kk * CPR;
        const int pos = tok0 + kk;
        const bool live = pos >= rq.P && pos < rq.P + rq.T;
        uint4 k = make_uint4(0u, 0u, 0u, 0u), v = make_uint4(0u, 0u, 0u, 0u);
        if (live) {
            const bf16* row = qkv + (size_t)(rq.row0 + pos - rq.P) * ld_qkv + ch * 8;
            k = ld_global_16(row + k_col);
            v = ld_global_16(row + v_col);
            st_global_16(k_tile + (size_t)kk * D + ch * 8, k);
        }
        *reinterpret_cast<uint4*>(&tile[kk][ch * 8]) = v;  // zeros for positions outside [P, P+T)
    }
    __syncthreads();
    bf16* dst = reinterpret_cast<bf16*>(tiles.v_tile(tile_index));
    // thread -> (feature dd, group of 8 tokens): gathers the 8 tokens' values of feature dd and stores them as one chunk
    for (int idx = threadIdx.x; idx < D * 8; idx += blockDim.x) {
        const int dd = idx >> 3, g8 = idx & 7;
        const int t0 = g8 * 8;
        if (tok0 + t0 + 7 < rq.P) continue;  // all 8 tokens are older than this call: keep them
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = tile[t0 + e][dd];
        if (tok0 + t0 >= rq.P) {
            *reinterpret_cast<bf16x8*>(dst + dd * 64 + t0) = o;
        } else {  // the group straddles P: element-wise, older tokens untouched
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tok0 + t0 + e >= rq.P) dst[dd * 64 + t0 + e] = o[e];
        }
    }
}

// ---------------------------------------------------------------- weight packing (one-time)
// dst[prow][k] = bf16(src[srow][k] * gain[k]): the RMSNorm gain is folded into the weight columns of the GEMM that follows
// the norm, and rows are reordered so that what an epilogue combines sits in one 32-row unit (one MFMA tile), in rows t and
// t + 16, which one lane holds:
//   PACK_GATE_UP (p0 = I):  unit u = 16 gate rows 16u..16u+15, then the up rows I + 16u..
//   PACK_QKV_ROPE (p0 = head_dim, p1 = number of q and k rows): unit u of a head = features 16u..16u+15 of the head's
//                 first half, then their rotate-half partners head_dim/2 + 16u..; v rows keep their order
enum PackMode { PACK_IDENTITY = 0, PACK_GATE_UP = 1, PACK_QKV_ROPE = 2 };
__global__ __launch_bounds__(256) void pack_rows_kernel(const bf16* __restrict__ src, const bf16* __restrict__ gain,
                                                        bf16* __restrict__ dst, int K, int mode, int p0, int p1) {
    const int prow = blockIdx.x;
    int srow = prow;
    const int t = prow & 31;
    if (mode == PACK_GATE_UP) {
        const int u = prow >> 5;
        srow = (t < 16) ? (u * 16 + t) : (p0 + u * 16 + (t - 16));
    } else if (mode == PACK_QKV_ROPE && prow < p1) {
        const int head = prow / p0, uh = (prow % p0) >> 5;
        srow = head * p0 + ((t < 16) ? (uh * 16 + t) : (p0 / 2 + uh * 16 + (t - 16)));
    }
    const bf16* s = src + (size_t)srow * K;
    bf16* d = dst + (size_t)prow * K;
    for (int c = threadIdx.x; c < K / 8; c += blockDim.x) {
        bf16x8 v = *reinterpret_cast<const bf16x8*>(s + c * 8);
        bf16x8 g = *reinterpret_cast<const bf16x8*>(gain + c * 8);
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = f32_to_bf16(bf16_to_f32(v[e]) * bf16_to_f32(g[e]));
        *reinterpret_cast<bf16x8*>(d + c * 8) = o;
    }
}

// ---------------------------------------------------------------- cache export / import (canonical [tokens][Hkv][d])
// The cache is described like a request (ReqDesc: contiguous planes, or the pool base for a paged cache).  The page
// numbers of a paged cache travel in the kernel arguments, a window of KV_PAGE_WINDOW blocks per launch starting at
// block `block0`; tokens [t0, t0 + n) are handled, t0 a multiple of 64 inside the window.
constexpr int KV_PAGE_WINDOW = 256;
struct KVPageWindow {
    int page[KV_PAGE_WINDOW];
};

template <int D>
RS_DEVICE bf16* kv_window_tile(const ReqDesc& rq, const KVPageWindow& win, int block0, bool v, int c, int block) {
    constexpr size_t TILE = (size_t)64 * D;  // elements
    if (rq.pages == nullptr)   // (any non-null value marks a paged cache here; the numbers come from the window)
        return (v ? rq.vtcache : rq.kcache) + ((size_t)c * (size_t)(rq.cap >> 6) + (size_t)block) * TILE;
    return rq.kcache + ((size_t)win.page[block - block0] * 2 * rq.hkv + (size_t)(v ? rq.hkv : 0) + (size_t)c) * TILE;
}

template <int D>
__global__ __launch_bounds__(256) void kv_export_kernel(ReqDesc rq, KVPageWindow win, int block0, bf16* __restrict__ k_out,
                                                        bf16* __restrict__ v_out, int t0, int n) {
    const int Hkv = rq.hkv;
    const size_t total = (size_t)n * Hkv * D;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int dd = (int)(i % D);
        const int c = (int)((i / D) % Hkv);
        const int t = t0 + (int)(i / ((size_t)D * Hkv));
        const size_t o = (size_t)t0 * Hkv * D + i;
        k_out[o] = kv_window_tile<D>(rq, win, block0, false, c, t >> 6)[(size_t)(t & 63) * D + dd];
        v_out[o] = kv_window_tile<D>(rq, win, block0, true, c, t >> 6)[(size_t)dd * 64 + (t & 63)];
    }
}

template <int D>
__global__ __launch_bounds__(256) void kv_import_kernel(ReqDesc rq, KVPageWindow win, int block0, const bf16* __restrict__ k_in,
                                                        const bf16* __restrict__ v_in, int t0, int n) {
    const int Hkv = rq.hkv;
    const int n_pad = (n + 63) & ~63;  // the last touched V block is zero-filled beyond t0 + n
    const size_t total = (size_t)n_pad * Hkv * D;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int dd = (int)(i % D);
        const int c = (int)((i / D) % Hkv);
        const int tl = (int)(i / ((size_t)D * Hkv));
        const int t = t0 + tl;
        const bool live = tl < n;
        const size_t o = (size_t)t0 * Hkv * D + i;
        if (live) kv_window_tile<D>(rq, win, block0, false, c, t >> 6)[(size_t)(t & 63) * D + dd] = k_in[o];
        kv_window_tile<D>(rq, win, block0, true, c, t >> 6)[(size_t)dd * 64 + (t & 63)] = live ? v_in[o] : f32_to_bf16(0.0f);
    }
}
