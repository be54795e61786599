// The 8-bit KV cache: one OCP E4M3 byte per element, one scale for the keys and one for the values of a cache.
//
//   stored  code  = e4m3( fl32( x * fl32(1 / scale) ) )      x: the bfloat16 K~ or V element; nearest, ties to even,
//                                                             saturating at +-448, NaN -> 0x7f
//   read    value = bf16( fl32( decode(code) * scale ) )
//
// The cache keeps the tile layout of the bfloat16 one with one byte per element: per KV head, K tiles [64 tokens][d]
// and V^T tiles [d][64 tokens], contiguous per layer or in pages of 64 tokens.  The attention kernels do not read it: before attention, the blocks a call's rows can see
// are expanded to bfloat16 tiles in the call's workspace (one layer's worth, reused by every layer), which the unchanged
// attention kernel then walks.  Expanding costs one pass over the prefix at HBM speed (a few microseconds per 10k
// tokens), far less than converting inside the attention loop, whose limit is LDS bandwidth and issue slots, not HBM.
#pragma once
#include "attention.h"
#include "common.h"
#include "elementwise.h"

typedef __attribute__((ext_vector_type(2))) float f32x2;

struct Fp8CacheDesc {
    uint8_t* kc;   // contiguous: K codes of the layer, [Hkv][cap/64][64][d];  paged: the pool's base
    uint8_t* vc;   // contiguous: V^T codes of the layer, [Hkv][cap/64][d][64];  paged: unused
    const int* pages;  // paged: page number of each 64-token block of this layer (device memory); null for a contiguous cache
    int cap;       // contiguous: capacity in tokens (multiple of 64)
    int xb0;       // number of the request's first block among the blocks the call expands
    int hkv;       // KV heads (a page holds their K tiles, then their V^T tiles)
    int pad_;
    float k_inv, v_inv;      // fl32(1 / scale)
    float k_scale, v_scale;
};

constexpr float E4M3_MAX = 448.0f;

// Two values to two E4M3 bytes (low 16 bits of the result).
RS_DEVICE uint32_t e4m3_pair(float a, float b) {
    const float ca = fminf(fmaxf(a, -E4M3_MAX), E4M3_MAX);
    const float cb = fminf(fmaxf(b, -E4M3_MAX), E4M3_MAX);
    uint32_t r = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false) & 0xffffu;
    if (a != a) r = (r & 0xff00u) | 0x7fu;
    if (b != b) r = (r & 0x00ffu) | 0x7f00u;
    return r;
}

// Eight bfloat16 values times `inv` to eight codes.
RS_DEVICE uint2 e4m3_from_bf16x8(bf16x8 v, float inv) {
    uint2 o;
    o.x = e4m3_pair(bf16_to_f32(v[0]) * inv, bf16_to_f32(v[1]) * inv) |
          (e4m3_pair(bf16_to_f32(v[2]) * inv, bf16_to_f32(v[3]) * inv) << 16);
    o.y = e4m3_pair(bf16_to_f32(v[4]) * inv, bf16_to_f32(v[5]) * inv) |
          (e4m3_pair(bf16_to_f32(v[6]) * inv, bf16_to_f32(v[7]) * inv) << 16);
    return o;
}

// Four codes (one 32-bit word) times `scale` to four bfloat16 values.
RS_DEVICE bf16x4 bf16x4_from_e4m3(uint32_t w, float scale) {
    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    bf16x4 o;
    o[0] = f32_to_bf16(lo[0] * scale);
    o[1] = f32_to_bf16(lo[1] * scale);
    o[2] = f32_to_bf16(hi[0] * scale);
    o[3] = f32_to_bf16(hi[1] * scale);
    return o;
}

RS_DEVICE bf16 bf16_from_e4m3(uint8_t code, float scale) {
    const f32x2 v = __builtin_amdgcn_cvt_pk_f32_fp8((int)code, false);
    return f32_to_bf16(v[0] * scale);
}

RS_DEVICE uint8_t e4m3_from_bf16(bf16 v, float inv) { return (uint8_t)(e4m3_pair(bf16_to_f32(v) * inv, 0.0f) & 0xffu); }

RS_DEVICE size_t fp8_tile_offset(int cap, int c, int block, int D) { return ((size_t)c * (size_t)(cap >> 6) + (size_t)block) * 64 * D; }

// The K (v = false) or V^T (v = true) tile of KV head c and 64-token block `block` of an 8-bit cache.  A page of a paged
// cache holds 64 tokens of one layer: the K tiles of all KV heads, then their V^T tiles, 64 d bytes each.
RS_DEVICE uint8_t* fp8_tile(const Fp8CacheDesc& fc, bool v, int c, int block, int D) {
    if (fc.pages == nullptr) return (v ? fc.vc : fc.kc) + fp8_tile_offset(fc.cap, c, block, D);
    return fc.kc + ((size_t)fc.pages[block] * 2 * fc.hkv + (size_t)(v ? fc.hkv : 0) + (size_t)c) * 64 * D;
}

// ---------------------------------------------------------------- append
// One workgroup per (touched 64-token block, KV head), as in append_kv_kernel: the rotated k rows and the v rows of the
// call are quantised into the request's 8-bit cache.  Tokens before P keep their codes; V codes at or beyond P + T inside
// the block are zero.
template <int D>
__global__ __launch_bounds__(256) void append_kv_fp8_kernel(const bf16* __restrict__ qkv, int ld_qkv,
                                                            const ReqDesc* __restrict__ reqs,
                                                            const Fp8CacheDesc* __restrict__ caches,
                                                            const KVBlockItem* __restrict__ blocks, int Hq, int Hkv) {
    __shared__ __attribute__((aligned(16))) bf16 tile[64][D + 8];
    const KVBlockItem it = blocks[blockIdx.x];
    const ReqDesc rq = reqs[it.req];
    const Fp8CacheDesc fc = caches[it.req];
    const int c = blockIdx.y;
    const int tok0 = it.block * 64;
    const int k_col = (Hq + c) * D;
    const int v_col = (Hq + Hkv + c) * D;
    constexpr int CPR = D / 8;  // chunks of 8 elements per row
    uint8_t* const k_tile = fp8_tile(fc, false, c, it.block, D);
    uint8_t* const v_tile = fp8_tile(fc, true, c, it.block, D);
    for (int idx = threadIdx.x; idx < 64 * CPR; idx += blockDim.x) {
        const int kk = idx / CPR, ch = idx - kk * CPR;
        const int pos = tok0 + kk;
        const bool live = pos >= rq.P && pos < rq.P + rq.T;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (live) {
            const bf16* row = qkv + (size_t)(rq.row0 + pos - rq.P) * ld_qkv + ch * 8;
            const uint4 k = ld_global_16(row + k_col);
            v = ld_global_16(row + v_col);
            *reinterpret_cast<uint2*>(k_tile + (size_t)kk * D + ch * 8) = e4m3_from_bf16x8(as_bf16x8(k), fc.k_inv);
        }
        *reinterpret_cast<uint4*>(&tile[kk][ch * 8]) = v;  // zeros for positions outside [P, P+T)
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < D * 8; idx += blockDim.x) {
        const int dd = idx >> 3, g8 = idx & 7;
        const int t0 = g8 * 8;
        if (tok0 + t0 + 7 < rq.P) continue;  // all 8 tokens are older than this call: keep them
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = tile[t0 + e][dd];
        const uint2 codes = e4m3_from_bf16x8(o, fc.v_inv);
        if (tok0 + t0 >= rq.P) {
            *reinterpret_cast<uint2*>(v_tile + dd * 64 + t0) = codes;
        } else {  // the group straddles P: byte by byte, older tokens untouched
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tok0 + t0 + e >= rq.P) v_tile[dd * 64 + t0 + e] = (uint8_t)(((e < 4 ? codes.x : codes.y) >> (8 * (e & 3))) & 0xffu);
        }
    }
}

// ---------------------------------------------------------------- expansion
// One workgroup per (64-token block a request's rows can see, KV head): the block's K and V^T codes become bfloat16 tiles
// at reqs[r].kcache / .vtcache, which describe a contiguous cache of reqs[r].cap = 64 * ceil((P + T) / 64) tokens in the
// workspace.  Positions at or beyond P + T become zero whatever bytes the cache holds there.
template <int D>
__global__ __launch_bounds__(256) void kv_expand_fp8_kernel(const ReqDesc* __restrict__ reqs,
                                                            const Fp8CacheDesc* __restrict__ caches, int n_reqs) {
    const int b = blockIdx.x;
    int r = 0;
    while (r + 1 < n_reqs && caches[r + 1].xb0 <= b) ++r;
    const ReqDesc rq = reqs[r];
    const Fp8CacheDesc fc = caches[r];
    const int block = b - fc.xb0;
    const int c = blockIdx.y;
    const int tok0 = block * 64;
    const int end = rq.P + rq.T;
    const uint8_t* k_src = fp8_tile(fc, false, c, block, D);
    const uint8_t* v_src = fp8_tile(fc, true, c, block, D);
    bf16* k_dst = rq.kcache + fp8_tile_offset(rq.cap, c, block, D);
    bf16* v_dst = rq.vtcache + fp8_tile_offset(rq.cap, c, block, D);
    constexpr int CPR = D / 16;  // chunks of 16 codes per K row
    for (int idx = threadIdx.x; idx < 64 * CPR; idx += blockDim.x) {
        const int kk = idx / CPR;
        uint4 w = make_uint4(0u, 0u, 0u, 0u);
        if (tok0 + kk < end) w = ld_global_16(k_src + (size_t)idx * 16);
        bf16x4 o[4];
        if (tok0 + kk < end) {
            o[0] = bf16x4_from_e4m3(w.x, fc.k_scale);
            o[1] = bf16x4_from_e4m3(w.y, fc.k_scale);
            o[2] = bf16x4_from_e4m3(w.z, fc.k_scale);
            o[3] = bf16x4_from_e4m3(w.w, fc.k_scale);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) o[j][e] = f32_to_bf16(0.0f);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<bf16x4*>(k_dst + (size_t)idx * 16 + j * 4) = o[j];
    }
    // V^T rows are [64 tokens] long: four chunks of 16 tokens per feature
    for (int idx = threadIdx.x; idx < D * 4; idx += blockDim.x) {
        const int t0 = (idx & 3) * 16;
        const uint4 w = ld_global_16(v_src + (size_t)idx * 16);
        const uint32_t words[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bf16x4 o = bf16x4_from_e4m3(words[j], fc.v_scale);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (tok0 + t0 + j * 4 + e >= end) o[e] = f32_to_bf16(0.0f);
            *reinterpret_cast<bf16x4*>(v_dst + (size_t)idx * 16 + j * 4) = o;
        }
    }
}

// ---------------------------------------------------------------- export / import (canonical [tokens][Hkv][d])
// Tokens [t0, t0 + n) of one layer, t0 a multiple of 64.  The cache is described by an Fp8CacheDesc whose `pages` is only a
// marker here (non-null: paged): the page numbers of blocks [block0, block0 + KV_PAGE_WINDOW) ride in the kernel
// arguments, as for the bfloat16 caches.  With code outputs (inputs) given the bytes travel as they are; otherwise the
// bfloat16 values are produced (consumed) through the read (store) formula above.
template <int D>
RS_DEVICE uint8_t* fp8_window_tile(const Fp8CacheDesc& fc, const KVPageWindow& win, int block0, bool v, int c, int block) {
    if (fc.pages == nullptr) return (v ? fc.vc : fc.kc) + fp8_tile_offset(fc.cap, c, block, D);
    return fc.kc + ((size_t)win.page[block - block0] * 2 * fc.hkv + (size_t)(v ? fc.hkv : 0) + (size_t)c) * 64 * D;
}

template <int D>
__global__ __launch_bounds__(256) void kv_fp8_export_kernel(Fp8CacheDesc fc, KVPageWindow win, int block0, bf16* __restrict__ k_out,
                                                            bf16* __restrict__ v_out, uint8_t* __restrict__ kc_out,
                                                            uint8_t* __restrict__ vc_out, int t0, int n) {
    const int Hkv = fc.hkv;
    const size_t total = (size_t)n * Hkv * D;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int dd = (int)(i % D);
        const int c = (int)((i / D) % Hkv);
        const int t = t0 + (int)(i / ((size_t)D * Hkv));
        const size_t o = (size_t)t0 * Hkv * D + i;
        const uint8_t ck = fp8_window_tile<D>(fc, win, block0, false, c, t >> 6)[(size_t)(t & 63) * D + dd];
        const uint8_t cv = fp8_window_tile<D>(fc, win, block0, true, c, t >> 6)[(size_t)dd * 64 + (t & 63)];
        if (kc_out) {
            kc_out[o] = ck;
            vc_out[o] = cv;
        } else {
            k_out[o] = bf16_from_e4m3(ck, fc.k_scale);
            v_out[o] = bf16_from_e4m3(cv, fc.v_scale);
        }
    }
}

template <int D>
__global__ __launch_bounds__(256) void kv_fp8_import_kernel(Fp8CacheDesc fc, KVPageWindow win, int block0, const bf16* __restrict__ k_in,
                                                            const bf16* __restrict__ v_in, const uint8_t* __restrict__ kc_in,
                                                            const uint8_t* __restrict__ vc_in, int t0, int n) {
    const int Hkv = fc.hkv;
    const int n_pad = (n + 63) & ~63;  // the last touched V block is zero beyond t0 + n
    const size_t total = (size_t)n_pad * Hkv * D;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int dd = (int)(i % D);
        const int c = (int)((i / D) % Hkv);
        const int tl = (int)(i / ((size_t)D * Hkv));
        const int t = t0 + tl;
        const bool live = tl < n;
        const size_t o = (size_t)t0 * Hkv * D + i;
        uint8_t cv = 0;
        if (live) {
            const uint8_t ck = kc_in ? kc_in[o] : e4m3_from_bf16(k_in[o], fc.k_inv);
            cv = vc_in ? vc_in[o] : e4m3_from_bf16(v_in[o], fc.v_inv);
            fp8_window_tile<D>(fc, win, block0, false, c, t >> 6)[(size_t)(t & 63) * D + dd] = ck;
        }
        fp8_window_tile<D>(fc, win, block0, true, c, t >> 6)[(size_t)dd * 64 + (t & 63)] = cv;
    }
}
