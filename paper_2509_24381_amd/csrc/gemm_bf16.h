// bf16 MFMA GEMM for gfx950:  out[M,N] = epilogue( X[M,K] * W[N,K]^T ),  fp32 accumulation.
//
// Both operands are K-contiguous ("NT" form), which is what v_mfma_f32_32x32x16_bf16 wants: each lane
// feeds 8 consecutive k values of one row.  A 256x256 output tile is owned by one 256-thread workgroup
// (4 wavefronts in a 2x2 grid, 128x128 per wavefront = 4x4 MFMA tiles of 32x32, 256 fp32 accumulators
// per lane).  The weight rows ride on the MFMA "A" side and the token rows on the "B" side, so a lane ends
// up holding one token and runs of 4 consecutive output features: the epilogue (RMSNorm row factor, bias,
// RoPE, residual, SwiGLU) is lane-local and stores 8-byte bf16 groups.  RMSNorm is folded into the GEMMs that
// follow it: its gain is multiplied into the weight columns when the weights are packed and its per-row
// factor 1/rms multiplies the fp32 accumulators, so the normalised activations are never rounded to bf16.
//
// K is walked in slabs of 64.  A slab of either operand is 256 rows x 128 bytes; it is kept in LDS as
// 16-byte chunks with the chunk index XOR-ed by ((row >> 1) & 7), which makes both the linear 16-byte
// stores of the loader and the row-strided 16-byte fragment reads of the MFMA feed bank-conflict free.
// LDS is double buffered (2 x 64 KB of the CU's 160 KB); the next slab travels global -> registers while
// the current one is multiplied, and is parked in the other LDS buffer before the single barrier per slab.
//
// Workgroup ids are dispatched round-robin over the 8 XCDs; the kernel re-maps them so that each XCD owns a
// contiguous range of tile columns (all row tiles of a weight column block run on one XCD, close in time),
// which makes the weight stream single-pass through HBM and lets the XCD's L2 serve the activation re-reads.
#pragma once
#include "common.h"

enum GemmEpilogue {
    EPI_QKV_ROPE = 0,  // out = bf16(rope(acc * row_scale[m] + bias[n])): RMSNorm's per-row factor applied after the product
                       // (its gain is folded into W), rotate-half RoPE at row_pos[m] on the q and k heads
    EPI_RESIDUAL = 1,  // out = bf16(acc + resid[m, n]); optionally per-row sums of squares of the stored values
    EPI_SWIGLU = 2,    // W rows interleaved in 32-row blocks (gate, up, gate, up, ...):
                       // out[m, n/2] = bf16(silu(gate * row_scale[m]) * (up * row_scale[m]))
    EPI_PARTIAL = 3    // split-K: fp32 partial sums to partial[split][m][n]
};

struct GemmArgs {
    const bf16* X;      // [M, K] activations, row stride ldx elements
    const bf16* W;      // [N, K] weights, row stride K
    bf16* out;          // [M, ldo]
    const bf16* bias;   // [N] or null
    const bf16* resid;  // [M, ldr]
    float* partial;     // [splits, M, N]
    const float* row_scale;  // [M] 1/rms of the row (EPI_QKV_ROPE, EPI_SWIGLU)
    const int* row_pos;      // [M] absolute position of the row (EPI_QKV_ROPE)
    const float2* rope_cs;   // [max_pos][head_dim/2] (cos, sin)
    float* rowss;            // EPI_RESIDUAL: [M][N/128] sum of squares of each stored 128-column run, or null
    int rope_cols;           // columns [0, rope_cols) are q and k heads
    int head_dim;
    int ldx, ldo, ldr;
    int M, N, K;
    int tiles_m, tiles_n;
    int k_slabs_per_split;  // K/64 slabs handled by one blockIdx.y
#ifdef RS_GEMM_TIMING
    unsigned long long* dbg;  // development only: per-workgroup cycle counts of the pipeline's wait points
#endif
};

constexpr int GEMM_BM = 256, GEMM_BN = 256, GEMM_BK = 64;
constexpr int GEMM_STAGE_BYTES = GEMM_BM * GEMM_BK * 2;          // one operand, one slab: 32 KB
constexpr int GEMM_LDS_BYTES = 4 * GEMM_STAGE_BYTES;             // 2 operands x 2 buffers

// silu(g) = g / (1 + 2^(-g log2 e)) with the raw v_exp_f32 / v_rcp_f32 instructions (1 ulp each; the result is rounded to bf16)
RS_DEVICE float silu_f32(float g) {
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

// Lane-local epilogue shared by the GEMM kernels.  acc[i][j][r] holds token m = m0 + wm*128 + j*32 + l32 and
// feature n = n0 + wn*128 + i*32 + 8*(r>>2) + 4*half + (r&3).
template <int EPI>
RS_DEVICE void gemm_epilogue(const GemmArgs& a, f32x16 (&acc)[4][4], int m0, int n0, int wm, int wn, int half, int l32,
                             int split) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int m = m0 + wm * 128 + j * 32 + l32;
        if (m >= a.M) continue;
        if constexpr (EPI == EPI_SWIGLU) {
            const float sc = a.row_scale[m];
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = (n0 + wn * 128) / 2 + i2 * 32 + 8 * q + 4 * half;
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = f32_to_bf16(silu_f32(acc[2 * i2][j][4 * q + e] * sc) * (acc[2 * i2 + 1][j][4 * q + e] * sc));
                    *reinterpret_cast<bf16x4*>(a.out + (size_t)m * a.ldo + col) = o;
                }
        } else if constexpr (EPI == EPI_QKV_ROPE) {
            const int nw = n0 + wn * 128;  // this wavefront's 128 features: whole heads of one kind (q, k or v)
            const float sc = a.row_scale[m];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float b[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (a.bias != nullptr) {
                        bf16x4 b4 = *reinterpret_cast<const bf16x4*>(a.bias + nw + i * 32 + 8 * q + 4 * half);
#pragma unroll
                        for (int e = 0; e < 4; ++e) b[e] = bf16_to_f32(b4[e]);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] = acc[i][j][4 * q + e] * sc + b[e];
                }
            if (nw < a.rope_cols) {
                const int hd2 = a.head_dim >> 1;
                const float2* csr = a.rope_cs + (size_t)a.row_pos[m] * hd2;
                if (a.head_dim == 128) {  // one head per wavefront: column c pairs with c + 64 = two MFMA tiles to the right
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float2 c = csr[i * 32 + 8 * q + 4 * half + e];
                                const float lo = acc[i][j][4 * q + e], hi = acc[i + 2][j][4 * q + e];
                                acc[i][j][4 * q + e] = lo * c.x - hi * c.y;
                                acc[i + 2][j][4 * q + e] = hi * c.x + lo * c.y;
                            }
                } else {  // head_dim 64: two heads per wavefront, column c pairs with c + 32 = the next MFMA tile
#pragma unroll
                    for (int i = 0; i < 4; i += 2)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float2 c = csr[8 * q + 4 * half + e];
                                const float lo = acc[i][j][4 * q + e], hi = acc[i + 1][j][4 * q + e];
                                acc[i][j][4 * q + e] = lo * c.x - hi * c.y;
                                acc[i + 1][j][4 * q + e] = hi * c.x + lo * c.y;
                            }
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(acc[i][j][4 * q + e]);
                    *reinterpret_cast<bf16x4*>(a.out + (size_t)m * a.ldo + nw + i * 32 + 8 * q + 4 * half) = o;
                }
        } else {
            float ss = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + wn * 128 + i * 32 + 8 * q + 4 * half;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
                    if constexpr (EPI == EPI_PARTIAL) {
                        f32x4 o = {v[0], v[1], v[2], v[3]};
                        *reinterpret_cast<f32x4*>(a.partial + ((size_t)split * a.M + m) * a.N + n) = o;
                    } else {
                        bf16x4 r4 = *reinterpret_cast<const bf16x4*>(a.resid + (size_t)m * a.ldr + n);
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            o[e] = f32_to_bf16(v[e] + bf16_to_f32(r4[e]));
                            const float st = bf16_to_f32(o[e]);
                            ss += st * st;
                        }
                        *reinterpret_cast<bf16x4*>(a.out + (size_t)m * a.ldo + n) = o;
                    }
                }
            if constexpr (EPI == EPI_RESIDUAL) {
                if (a.rowss != nullptr) {  // the two half-waves hold the two halves of this token's 128-column run
                    ss += __shfl_xor(ss, 32, WAVE);
                    if (half == 0) a.rowss[(size_t)m * (a.N / 128) + (n0 + wn * 128) / 128] = ss;
                }
            }
        }
    }
}

template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_bf16_256x256_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wn = wave & 1;   // which 128-wide half of the tile's features
    const int wm = wave >> 1;  // which 128-row half of the tile's tokens
    const int half = lane >> 5;
    const int l32 = lane & 31;

    // ---- XCD-aware tile assignment
    const int nwg = a.tiles_m * a.tiles_n;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, loc = pid >> 3;
    const int base = nwg >> 3, rem = nwg & 7;
    const int logical = (xcd < rem ? xcd * (base + 1) : rem * (base + 1) + (xcd - rem) * base) + loc;
    const int tm = logical % a.tiles_m;
    const int tn = logical / a.tiles_m;
    const int m0 = tm * GEMM_BM;
    const int n0 = tn * GEMM_BN;

    const int split = blockIdx.y;
    const int slabs_total = a.K / GEMM_BK;
    const int s0 = split * a.k_slabs_per_split;
    const int s1 = min(s0 + a.k_slabs_per_split, slabs_total);

    // ---- loader geometry: thread -> (row within a 32-row group, 16-byte chunk of the 128-byte slab row)
    const int ld_row = tid >> 3;
    const int ld_chunk = (tid & 7) ^ ((tid >> 4) & 7);
    uint32_t x_off[8];  // byte offsets of this thread's 8 rows of X (rows past M are clamped: loaded, never stored)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int r = min(m0 + i * 32 + ld_row, a.M - 1);
        x_off[i] = (uint32_t)r * (uint32_t)a.ldx * 2u + (uint32_t)ld_chunk * 16u;
    }
    const uint32_t w_off0 = (uint32_t)(n0 + ld_row) * (uint32_t)a.K * 2u + (uint32_t)ld_chunk * 16u;
    const uint32_t w_step = 32u * (uint32_t)a.K * 2u;
    const char* Xb = reinterpret_cast<const char*>(a.X);
    const char* Wb = reinterpret_cast<const char*>(a.W);

    // ---- fragment read geometry
    const int swz = (lane >> 1) & 7;
    uint32_t fr_w[4], fr_x[4];  // LDS byte offset of the lane's row in each 32-row MFMA tile (chunk added per k-step)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        fr_w[t] = (uint32_t)(wn * 128 + t * 32 + l32) * 128u;
        fr_x[t] = (uint32_t)(wm * 128 + t * 32 + l32) * 128u;
    }

    f32x16 acc[4][4];  // [feature tile][token tile]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    uint4 rx[8], rw[8];
    auto load_slab = [&](int s) {
        const uint32_t kb = (uint32_t)s * (GEMM_BK * 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) rx[i] = ld_global_16(Xb + (x_off[i] + kb));
#pragma unroll
        for (int i = 0; i < 8; ++i) rw[i] = ld_global_16(Wb + (w_off0 + (uint32_t)i * w_step + kb));
    };
    auto park_slab = [&](int buf) {
        char* xs = smem + buf * (2 * GEMM_STAGE_BYTES);
        char* ws = xs + GEMM_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<uint4*>(xs + i * 4096 + tid * 16) = rx[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<uint4*>(ws + i * 4096 + tid * 16) = rw[i];
    };

    if (s0 < s1) {
        load_slab(s0);
        park_slab(0);
    }
    __syncthreads();

    for (int s = s0; s < s1; ++s) {
        const int buf = (s - s0) & 1;
        const bool more = (s + 1) < s1;
        if (more) load_slab(s + 1);
        const char* xs = smem + buf * (2 * GEMM_STAGE_BYTES);
        const char* ws = xs + GEMM_STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const uint32_t coff = (uint32_t)(((kk * 2 + half) ^ swz) * 16);
            bf16x8 wf[4], xf[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) wf[t] = *reinterpret_cast<const bf16x8*>(ws + fr_w[t] + coff);
#pragma unroll
            for (int t = 0; t < 4; ++t) xf[t] = *reinterpret_cast<const bf16x8*>(xs + fr_x[t] + coff);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
        }
        if (more) park_slab(buf ^ 1);
        __syncthreads();
    }

    gemm_epilogue<EPI>(a, acc, m0, n0, wm, wn, half, l32, split);
}

// ------------------------------------------------------------------------------------------------------------------
// Same tile, deeper pipeline: operand slabs travel global -> LDS directly (buffer_load ... lds, 16 bytes per lane) through
// a ring of 4 stages of K=32, so three stages of loads are in flight while one is multiplied and no VGPRs are tied up
// by data in transit.  Rows past M are outside the buffer resource and read as zeros.
//
// A stage of one operand is 256 rows x 64 bytes; 16-byte chunk c of row r sits at slot c ^ ((r >> 2) & 3) of its row,
// which keeps the 16 rows a quarter-wave reads at once on 16 different 16-byte bank groups.  A load instruction of one
// wavefront fills 1 KB of LDS (16 rows) linearly by lane, so each lane fetches the chunk that belongs in its slot.
//
// The compiler cannot see through LDS written by DMA (it would wait for every outstanding load before any LDS read),
// so the fragment reads are inline ds_read_b128 and the waits are explicit:
//   - loads retire in order; 8 per thread per stage, so "vmcnt(16)" = everything except the two newest stages landed;
// Each wait is tied by register operands to the fragments it guards, so the MFMAs that consume them cannot move above it.
// Per stage: 16 MFMAs on the kk=0 fragments with the kk=1 fragment reads and the loads of stage s+3 interleaved one per
// MFMA, [wait stage s+1, barrier], 16 MFMAs on the kk=1 fragments with the next stage's kk=0 reads behind the first 8.
constexpr int G2_BK = 32, G2_STAGES = 4;
constexpr int G2_OP_BYTES = 256 * G2_BK * 2;       // 16 KB
constexpr int G2_STAGE_BYTES = 2 * G2_OP_BYTES;    // 32 KB
constexpr int G2_LDS_BYTES = G2_STAGES * G2_STAGE_BYTES;

#define RS_DS_READ_B128(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off))
#define RS_DMA_LOAD(rsrc, dstp, voff, soff) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(dstp), 16, voff, soff, 0, 0)

RS_DEVICE void tie_wait_lgkm8(bf16x8 (&w)[4], bf16x8 (&x)[4]) {
    asm volatile("s_waitcnt lgkmcnt(8)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]));
}
RS_DEVICE void tie_wait_lgkm0(bf16x8 (&w)[4], bf16x8 (&x)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]));
}

template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_bf16_dma_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1;
    const int wm = wave >> 1;
    const int half = lane >> 5;
    const int l32 = lane & 31;

    const int nwg = a.tiles_m * a.tiles_n;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, loc = pid >> 3;
    const int base = nwg >> 3, rem = nwg & 7;
    const int logical = (xcd < rem ? xcd * (base + 1) : rem * (base + 1) + (xcd - rem) * base) + loc;
    const int tm = logical % a.tiles_m;
    const int tn = logical / a.tiles_m;
    const int m0 = tm * GEMM_BM;
    const int n0 = tn * GEMM_BN;

    const int split = blockIdx.y;
    const int stages_total = a.K / G2_BK;
    const int st0 = split * a.k_slabs_per_split * 2;                       // a 64-wide slab = 2 stages
    const int ns = min(a.k_slabs_per_split * 2, stages_total - st0);       // stages this workgroup multiplies (>= 1)

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.X, 0, a.M * a.ldx * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.W, 0, a.N * a.K * 2, 0x00020000);

    // loader: instruction i of this wavefront fills LDS rows [i*64 + wave*16, +16) of the operand's stage
    const int ld_r = wave * 16 + (lane >> 2);
    const int ld_c = (lane & 3) ^ ((lane >> 4) & 3);
    uint32_t vx[4], vw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        vx[i] = (uint32_t)(m0 + i * 64 + ld_r) * (uint32_t)a.ldx * 2u + (uint32_t)ld_c * 16u;
        vw[i] = (uint32_t)(n0 + i * 64 + ld_r) * (uint32_t)a.K * 2u + (uint32_t)ld_c * 16u;
    }
    typedef __attribute__((address_space(3))) void* lds_ptr;
    auto issue_stage = [&](int stage, int buf) {
        const int koff = (st0 + stage) * (G2_BK * 2);
        char* dst = smem + buf * G2_STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr)(dst + i * 4096), 16, vx[i], koff, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr)(dst + G2_OP_BYTES + i * 4096), 16, vw[i], koff, 0, 0);
    };

    // fragment addresses (bytes from the start of a stage's X part); kk selects the 16-wide k-step inside the stage
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t sw = (uint32_t)((l32 >> 2) & 3);
    uint32_t ax[2], aw[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const uint32_t slot = ((uint32_t)(kk * 2 + half) ^ sw) * 16u;
        ax[kk] = lds0 + (uint32_t)(wm * 128 + l32) * 64u + slot;
        aw[kk] = lds0 + (uint32_t)G2_OP_BYTES + (uint32_t)(wn * 128 + l32) * 64u + slot;
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 w0[4], x0[4], w1[4], x1[4];
#define RS_READ_FRAGS(wf, xf, kk, bufoff)                                  \
    do {                                                                   \
        const uint32_t aw_ = aw[kk] + (bufoff), ax_ = ax[kk] + (bufoff);   \
        RS_DS_READ_B128(wf[0], aw_, 0);                                    \
        RS_DS_READ_B128(xf[0], ax_, 0);                                    \
        RS_DS_READ_B128(wf[1], aw_, 2048);                                 \
        RS_DS_READ_B128(xf[1], ax_, 2048);                                 \
        RS_DS_READ_B128(wf[2], aw_, 4096);                                 \
        RS_DS_READ_B128(xf[2], ax_, 4096);                                 \
        RS_DS_READ_B128(wf[3], aw_, 6144);                                 \
        RS_DS_READ_B128(xf[3], ax_, 6144);                                 \
    } while (0)

#ifdef RS_GEMM_TIMING
    unsigned long long dbg_vm = 0, dbg_bar = 0, dbg_first = 0, dbg_last = 0, dbg_start;
    asm volatile("s_memtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(dbg_start));
#endif
    issue_stage(0, 0);
    issue_stage(min(1, ns - 1), 1);
    issue_stage(min(2, ns - 1), 2);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");
    RS_READ_FRAGS(w0, x0, 0, 0u);

#define RS_MFMA(wf, xf, i, j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0)
#define RS_FENCE() __builtin_amdgcn_sched_barrier(0)
    for (int s = 0; s < ns; ++s) {
        const uint32_t bufoff = (uint32_t)(s & 3) * G2_STAGE_BYTES;
        const uint32_t nextoff = (uint32_t)((s + 1) & 3) * G2_STAGE_BYTES;
        // ---- first half: 16 MFMAs on the kk=0 fragments; one memory instruction rides behind each MFMA so that its
        //      issue latency (LDS queue, texture-address queue) overlaps the matrix pipe instead of stalling it
        const int koff = (st0 + min(s + 3, ns - 1)) * (G2_BK * 2);
        char* dst = smem + ((s + 3) & 3) * G2_STAGE_BYTES + wave * 1024;
        const uint32_t aw1 = aw[1] + bufoff, ax1 = ax[1] + bufoff;
        tie_wait_lgkm0(w0, x0);
        RS_MFMA(w0, x0, 0, 0); RS_DS_READ_B128(w1[0], aw1, 0);    RS_FENCE();
        RS_MFMA(w0, x0, 0, 1); RS_DS_READ_B128(x1[0], ax1, 0);    RS_FENCE();
        RS_MFMA(w0, x0, 0, 2); RS_DS_READ_B128(w1[1], aw1, 2048); RS_FENCE();
        RS_MFMA(w0, x0, 0, 3); RS_DS_READ_B128(x1[1], ax1, 2048); RS_FENCE();
        RS_MFMA(w0, x0, 1, 0); RS_DS_READ_B128(w1[2], aw1, 4096); RS_FENCE();
        RS_MFMA(w0, x0, 1, 1); RS_DS_READ_B128(x1[2], ax1, 4096); RS_FENCE();
        RS_MFMA(w0, x0, 1, 2); RS_DS_READ_B128(w1[3], aw1, 6144); RS_FENCE();
        RS_MFMA(w0, x0, 1, 3); RS_DS_READ_B128(x1[3], ax1, 6144); RS_FENCE();
        RS_MFMA(w0, x0, 2, 0); RS_DMA_LOAD(rx, dst, vx[0], koff); RS_FENCE();
        RS_MFMA(w0, x0, 2, 1); RS_DMA_LOAD(rx, dst + 4096, vx[1], koff); RS_FENCE();
        RS_MFMA(w0, x0, 2, 2); RS_DMA_LOAD(rx, dst + 8192, vx[2], koff); RS_FENCE();
        RS_MFMA(w0, x0, 2, 3); RS_DMA_LOAD(rx, dst + 12288, vx[3], koff); RS_FENCE();
        RS_MFMA(w0, x0, 3, 0); RS_DMA_LOAD(rw, dst + G2_OP_BYTES, vw[0], koff); RS_FENCE();
        RS_MFMA(w0, x0, 3, 1); RS_DMA_LOAD(rw, dst + G2_OP_BYTES + 4096, vw[1], koff); RS_FENCE();
        RS_MFMA(w0, x0, 3, 2); RS_DMA_LOAD(rw, dst + G2_OP_BYTES + 8192, vw[2], koff); RS_FENCE();
        RS_MFMA(w0, x0, 3, 3); RS_DMA_LOAD(rw, dst + G2_OP_BYTES + 12288, vw[3], koff); RS_FENCE();
        tie_wait_lgkm0(w1, x1);  // every LDS read of this stage has landed before the barrier frees its buffer
#ifdef RS_GEMM_TIMING
        unsigned long long t0_, t1_, t2_;
        asm volatile("s_memtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(t0_));
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        asm volatile("s_memtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(t1_));
        asm volatile("s_barrier" ::: "memory");
        asm volatile("s_memtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(t2_));
        dbg_vm += t1_ - t0_; dbg_bar += t2_ - t1_;
        if (s == 0) dbg_first = t2_;
        dbg_last = t2_;
#else
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
#endif
        RS_FENCE();
        // ---- second half: 16 MFMAs on the kk=1 fragments; the next stage's kk=0 fragments are fetched behind the first 8
        const uint32_t aw0 = aw[0] + nextoff, ax0 = ax[0] + nextoff;
        RS_MFMA(w1, x1, 0, 0); RS_DS_READ_B128(w0[0], aw0, 0);    RS_FENCE();
        RS_MFMA(w1, x1, 0, 1); RS_DS_READ_B128(x0[0], ax0, 0);    RS_FENCE();
        RS_MFMA(w1, x1, 0, 2); RS_DS_READ_B128(x0[1], ax0, 2048); RS_FENCE();
        RS_MFMA(w1, x1, 0, 3); RS_DS_READ_B128(x0[2], ax0, 4096); RS_FENCE();
        RS_MFMA(w1, x1, 1, 0); RS_DS_READ_B128(x0[3], ax0, 6144); RS_FENCE();
        RS_MFMA(w1, x1, 1, 1); RS_DS_READ_B128(w0[1], aw0, 2048); RS_FENCE();
        RS_MFMA(w1, x1, 1, 2); RS_DS_READ_B128(w0[2], aw0, 4096); RS_FENCE();
        RS_MFMA(w1, x1, 1, 3); RS_DS_READ_B128(w0[3], aw0, 6144); RS_FENCE();
        RS_MFMA(w1, x1, 2, 0); RS_MFMA(w1, x1, 2, 1); RS_MFMA(w1, x1, 2, 2); RS_MFMA(w1, x1, 2, 3);
        RS_MFMA(w1, x1, 3, 0); RS_MFMA(w1, x1, 3, 1); RS_MFMA(w1, x1, 3, 2); RS_MFMA(w1, x1, 3, 3);
        RS_FENCE();
    }
#undef RS_MFMA
#undef RS_FENCE
    tie_wait_lgkm0(w0, x0);  // the look-ahead read of the stage after the last one
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef RS_READ_FRAGS
#ifdef RS_GEMM_TIMING
    if (lane == 0) {
        unsigned long long* d = a.dbg + ((size_t)blockIdx.x * 4 + wave) * 4;
        d[0] = dbg_vm; d[1] = dbg_bar; d[2] = dbg_last - dbg_first; d[3] = ns - 1;
    }
#endif

    gemm_epilogue<EPI>(a, acc, m0, n0, wm, wn, half, l32, split);
#ifdef RS_GEMM_TIMING
    if (tid == 0) {
        unsigned long long dbg_end;
        asm volatile("s_waitcnt vmcnt(0)\n s_memtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(dbg_end));
        unsigned long long* d = a.dbg + (size_t)gridDim.x * 16 + (size_t)blockIdx.x * 2;
        d[0] = dbg_start; d[1] = dbg_end;
    }
#endif
}

// Sums split-K partials, adds the residual and rounds once:  out[m,n] = bf16(resid[m,n] + sum_s partial[s][m][n]).
// One wavefront per row; when inv_rms is given it also leaves rsqrt(mean(out[m,:]^2) + eps) of the stored row there.
__global__ __launch_bounds__(256) void splitk_reduce_residual_kernel(const float* __restrict__ partial, int splits,
                                                                     const bf16* __restrict__ resid, int ldr,
                                                                     bf16* __restrict__ out, int ldo, int M, int N,
                                                                     float* __restrict__ inv_rms, float eps) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    float ss = 0.0f;
    for (int n = lane * 4; n < N; n += WAVE * 4) {
        bf16x4 r4 = *reinterpret_cast<const bf16x4*>(resid + (size_t)m * ldr + n);
        float v[4] = {bf16_to_f32(r4[0]), bf16_to_f32(r4[1]), bf16_to_f32(r4[2]), bf16_to_f32(r4[3])};
        for (int s = 0; s < splits; ++s) {
            f32x4 p = *reinterpret_cast<const f32x4*>(partial + ((size_t)s * M + m) * N + n);
            v[0] += p[0]; v[1] += p[1]; v[2] += p[2]; v[3] += p[3];
        }
        bf16x4 o = {f32_to_bf16(v[0]), f32_to_bf16(v[1]), f32_to_bf16(v[2]), f32_to_bf16(v[3])};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float st = bf16_to_f32(o[e]);
            ss += st * st;
        }
        *reinterpret_cast<bf16x4*>(out + (size_t)m * ldo + n) = o;
    }
    if (inv_rms != nullptr) {
        ss = wave_sum(ss);
        if (lane == 0) inv_rms[m] = rsqrtf(ss / (float)N + eps);
    }
}

// inv_rms[m] = rsqrt(sum_b rowss[m][b] / H + eps): closes the per-row sum of squares left by the EPI_RESIDUAL epilogue.
__global__ __launch_bounds__(256) void rowss_finalize_kernel(const float* __restrict__ rowss, int blocks_per_row, int M, int H,
                                                             float eps, float* __restrict__ inv_rms) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    float ss = 0.0f;
    for (int b = 0; b < blocks_per_row; ++b) ss += rowss[(size_t)m * blocks_per_row + b];
    inv_rms[m] = rsqrtf(ss / (float)H + eps);
}
