// HBM-bound helper kernels: RMSNorm row factors, K / V append (V transposing), weight packing, cache export/import.
#pragma once
#include "attention.h"
#include "common.h"

// ---------------------------------------------------------------- RMSNorm row factor: one wavefront per row
// inv_rms[row] = rsqrt(mean(x[row]^2) + eps), sums in fp32.  The factor is applied inside the next GEMM's epilogue.
__global__ __launch_bounds__(256) void row_inv_rms_kernel(const bf16* __restrict__ x, float* __restrict__ inv_rms,
                                                          int rows, int H, float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const bf16* xr = x + (size_t)row * H;
    float ss = 0.0f;
    for (int c = lane; c < H / 8; c += WAVE) {
        bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float f = bf16_to_f32(v[e]);
            ss += f * f;
        }
    }
    ss = wave_sum(ss);
    if (lane == 0) inv_rms[row] = rsqrtf(ss / (float)H + eps);
}

// ---------------------------------------------------------------- row-major -> fragment-major copy of the layer input
// dst holds x in the GEMMs' token-operand layout: blocks of 32 tokens x 16 features, the two 8-feature halves 512 bytes
// apart, tokens 16 bytes apart (rows of the last block past `rows` are left untouched: they are never used).  One
// workgroup moves 32 tokens x 128 features: 8 threads read one token's 256 contiguous bytes, and the 8 tokens of a
// wavefront's 16-byte chunks of one (k-step, half) land in 128 contiguous bytes.
__global__ __launch_bounds__(256) void to_fragment_major_kernel(const bf16* __restrict__ x, bf16* __restrict__ dst, int rows, int H) {
    const int mb = blockIdx.x;
    const int r = threadIdx.x >> 3, c = threadIdx.x & 7;
    const int m = mb * 32 + r;
    if (m >= rows) return;
    const char* src = reinterpret_cast<const char*>(x + (size_t)m * H) + c * 16;
    char* out = reinterpret_cast<char*>(dst) + ((size_t)mb * (H >> 4) * 2 + c) * 512 + r * 16;
    for (int k0 = blockIdx.y * 64; k0 < H; k0 += gridDim.y * 64)  // 64 features = 8 chunks = 4 k-steps x 2 halves
        st_global_16(out + (size_t)(k0 >> 4) * 1024, ld_global_16(src + (size_t)k0 * 2));
}

// inv_rms[m] = rsqrt(sum_u rowss[m][u] / H + eps): closes the per-row sums of squares left by the EPI_RESIDUAL epilogue.
__global__ __launch_bounds__(256) void rowss_finalize_kernel(const float* __restrict__ rowss, int units, int M, int H,
                                                             float eps, float* __restrict__ inv_rms) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    float ss = 0.0f;
    for (int u = lane; u < units; u += WAVE) ss += rowss[(size_t)m * units + u];
    ss = wave_sum(ss);
    if (lane == 0) inv_rms[m] = rsqrtf(ss / (float)H + eps);
}

// ---------------------------------------------------------------- K / V append
struct KVBlockItem {
    int req;
    int block;  // absolute 64-token block index in the request's cache
};

// One workgroup per (touched 64-token block, KV head).  The rotated k rows are copied from the qkv buffer to the
// request's K cache (256-byte rows, 16-byte vector copies).  The v rows are transposed through LDS and written as
// [d][64] with the token index innermost.  Tokens before P keep their content; V positions at or beyond P+T inside
// the block are zero-filled.
template <int D>
__global__ __launch_bounds__(256) void append_kv_kernel(const bf16* __restrict__ qkv, int ld_qkv,
                                                        const ReqDesc* __restrict__ reqs,
                                                        const KVBlockItem* __restrict__ blocks, int Hq, int Hkv) {
    __shared__ bf16 tile[64][D + 2];
    const KVBlockItem it = blocks[blockIdx.x];
    const ReqDesc rq = reqs[it.req];
    const int c = blockIdx.y;
    const int tok0 = it.block * 64;
    const int k_col = (Hq + c) * D;
    const int v_col = (Hq + Hkv + c) * D;
    constexpr int CPR = D / 8;  // 16-byte chunks per row
    for (int idx = threadIdx.x; idx < 64 * CPR; idx += blockDim.x) {
        const int kk = idx / CPR, ch = idx - kk * CPR;
        const int pos = tok0 + kk;
        if (pos >= rq.P && pos < rq.P + rq.T) {
            const uint4 v = ld_global_16(qkv + (size_t)(rq.row0 + pos - rq.P) * ld_qkv + k_col + ch * 8);
            st_global_16(rq.kcache + ((size_t)c * rq.cap + pos) * D + ch * 8, v);
        }
    }
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
