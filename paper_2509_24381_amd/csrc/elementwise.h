// HBM-bound helper kernels: RMSNorm, RoPE + K append, V append (transposing), weight packing, cache export/import.
#pragma once
#include "attention.h"
#include "common.h"

// ---------------------------------------------------------------- RMSNorm: one wavefront per row
// out[row] = bf16( x[row] * rsqrt(mean(x^2) + eps) * g ), sums in fp32.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const bf16* __restrict__ x, const bf16* __restrict__ gain,
                                                      bf16* __restrict__ out, int rows, int H, float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const bf16* xr = x + (size_t)row * H;
    bf16* orow = out + (size_t)row * H;
    const int chunks = H / 8;
    float ss = 0.0f;
    for (int c = lane; c < chunks; c += WAVE) {
        bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float f = bf16_to_f32(v[e]);
            ss += f * f;
        }
    }
    ss = wave_sum(ss);
    const float inv = rsqrtf(ss / (float)H + eps);
    for (int c = lane; c < chunks; c += WAVE) {
        bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c * 8);
        bf16x8 gg = *reinterpret_cast<const bf16x8*>(gain + c * 8);
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = f32_to_bf16(bf16_to_f32(v[e]) * inv * bf16_to_f32(gg[e]));
        *reinterpret_cast<bf16x8*>(orow + c * 8) = o;
    }
}

RS_DEVICE int find_request(const ReqDesc* reqs, int R, int row) {
    // last request whose row0 <= row and that has rows (row0 is non-decreasing; empty requests share a row0)
    int lo = 0, hi = R - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (reqs[mid].row0 <= row) lo = mid; else hi = mid - 1;
    }
    while (lo > 0 && reqs[lo].T == 0) --lo;  // unreachable for rows inside a non-empty request, kept for safety
    return lo;
}

// ---------------------------------------------------------------- RoPE (rotate-half) on q and k, K append
// One workgroup per packed row.  q heads are rotated in place inside the qkv buffer; k heads are rotated and
// written to the request's K cache at the row's absolute position.  cs[pos][j] = (cos, sin) of pos * theta^(-2j/d).
template <int D>
__global__ __launch_bounds__(256) void rope_append_k_kernel(bf16* __restrict__ qkv, int ld_qkv,
                                                            const ReqDesc* __restrict__ reqs, int R,
                                                            const float2* __restrict__ cs, int Hq, int Hkv) {
    constexpr int HALF = D / 2;
    const int row = blockIdx.x;
    const ReqDesc rq = reqs[find_request(reqs, R, row)];
    const int pos = rq.P + (row - rq.row0);
    bf16* base = qkv + (size_t)row * ld_qkv;
    const float2* csr = cs + (size_t)pos * HALF;
    const int pairs = (Hq + Hkv) * HALF;
    for (int idx = threadIdx.x; idx < pairs; idx += blockDim.x) {
        const int head = idx / HALF, j = idx - head * HALF;
        const float2 c = csr[j];
        bf16* hp = base + head * D;
        const float lo = bf16_to_f32(hp[j]), hi = bf16_to_f32(hp[j + HALF]);
        const bf16 rlo = f32_to_bf16(lo * c.x - hi * c.y);
        const bf16 rhi = f32_to_bf16(hi * c.x + lo * c.y);
        if (head < Hq) {
            hp[j] = rlo;
            hp[j + HALF] = rhi;
        } else {
            bf16* kp = rq.kcache + ((size_t)(head - Hq) * rq.cap + pos) * D;
            kp[j] = rlo;
            kp[j + HALF] = rhi;
        }
    }
}

// ---------------------------------------------------------------- V append into the transposed, 64-token-blocked cache
struct VBlockItem {
    int req;
    int block;  // absolute 64-token block index in the request's cache
};

// One workgroup per (touched 64-token block, KV head): gathers up to 64 rows of v from the qkv buffer, transposes them
// through LDS and writes [d][64] with the token index innermost.  Tokens before P keep their content; positions at or
// beyond P+T inside the block are zero-filled.
template <int D>
__global__ __launch_bounds__(256) void append_v_kernel(const bf16* __restrict__ qkv, int ld_qkv,
                                                       const ReqDesc* __restrict__ reqs,
                                                       const VBlockItem* __restrict__ blocks, int Hq, int Hkv) {
    __shared__ bf16 tile[64][D + 2];
    const VBlockItem it = blocks[blockIdx.x];
    const ReqDesc rq = reqs[it.req];
    const int c = blockIdx.y;
    const int tok0 = it.block * 64;
    const int v_col = (Hq + Hkv + c) * D;
    for (int idx = threadIdx.x; idx < 64 * (D / 2); idx += blockDim.x) {
        const int kk = idx / (D / 2), dd = (idx - kk * (D / 2)) * 2;
        const int pos = tok0 + kk;
        bf16x2 v = {f32_to_bf16(0.0f), f32_to_bf16(0.0f)};
        if (pos >= rq.P && pos < rq.P + rq.T)
            v = *reinterpret_cast<const bf16x2*>(qkv + (size_t)(rq.row0 + pos - rq.P) * ld_qkv + v_col + dd);
        tile[kk][dd] = v[0];
        tile[kk][dd + 1] = v[1];
    }
    __syncthreads();
    bf16* dst = rq.vtcache + ((size_t)c * (rq.cap / 64) + it.block) * D * 64;
    for (int idx = threadIdx.x; idx < D * 64; idx += blockDim.x) {
        const int dd = idx >> 6, kk = idx & 63;
        if (tok0 + kk >= rq.P) dst[dd * 64 + kk] = tile[kk][dd];
    }
}

// ---------------------------------------------------------------- weight packing (one-time)
// gate/up interleave: packed row (b*64 + r) = gate row (b*32 + r), packed row (b*64 + 32 + r) = up row (b*32 + r).
__global__ __launch_bounds__(256) void pack_gate_up_kernel(const bf16* __restrict__ src, bf16* __restrict__ dst, int I, int H) {
    const int prow = blockIdx.x;  // packed row in [0, 2I)
    const int b = prow >> 6, r = prow & 63;
    const int srow = (r < 32) ? (b * 32 + r) : (I + b * 32 + (r - 32));
    const uint4* s = reinterpret_cast<const uint4*>(src + (size_t)srow * H);
    uint4* d = reinterpret_cast<uint4*>(dst + (size_t)prow * H);
    for (int c = threadIdx.x; c < H / 8; c += blockDim.x) d[c] = s[c];
}

// ---------------------------------------------------------------- cache export / import (canonical [tokens][Hkv][d])
template <int D>
__global__ __launch_bounds__(256) void kv_export_kernel(const bf16* __restrict__ kcache, const bf16* __restrict__ vtcache,
                                                        bf16* __restrict__ k_out, bf16* __restrict__ v_out,
                                                        int n, int Hkv, int cap) {
    const size_t total = (size_t)n * Hkv * D;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int dd = (int)(i % D);
        const int c = (int)((i / D) % Hkv);
        const int t = (int)(i / ((size_t)D * Hkv));
        k_out[i] = kcache[((size_t)c * cap + t) * D + dd];
        v_out[i] = vtcache[(((size_t)c * (cap / 64) + (t >> 6)) * D + dd) * 64 + (t & 63)];
    }
}

template <int D>
__global__ __launch_bounds__(256) void kv_import_kernel(bf16* __restrict__ kcache, bf16* __restrict__ vtcache,
                                                        const bf16* __restrict__ k_in, const bf16* __restrict__ v_in,
                                                        int n, int Hkv, int cap) {
    const int n_pad = (n + 63) & ~63;  // the last touched V block is zero-filled beyond n
    const size_t total = (size_t)n_pad * Hkv * D;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int dd = (int)(i % D);
        const int c = (int)((i / D) % Hkv);
        const int t = (int)(i / ((size_t)D * Hkv));
        const bool live = t < n;
        if (live) kcache[((size_t)c * cap + t) * D + dd] = k_in[i];
        vtcache[(((size_t)c * (cap / 64) + (t >> 6)) * D + dd) * 64 + (t & 63)] = live ? v_in[i] : f32_to_bf16(0.0f);
    }
}
