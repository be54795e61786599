// bf16 MFMA GEMM for gfx950:  out[M,N] = epilogue( X[M,K] * W[N,K]^T ),  fp32 accumulation.
//
// Both operands are K-contiguous ("NT" form), which is what v_mfma_f32_32x32x16_bf16 wants: each lane feeds 8 consecutive
// k values of one row.  The weight rows ride on the MFMA "A" side and the token rows on the "B" side, so a lane ends up
// holding one token and runs of 4 consecutive output features, and every epilogue (RMSNorm row factor, bias, RoPE,
// residual, SwiGLU) is lane-local.  RMSNorm is folded into the GEMMs that follow it: its gain is multiplied into the
// weight columns when the weights are packed and its per-row factor 1/rms multiplies the fp32 accumulators.
//
// Work decomposition ("strips").  The unit of output width is 32 features (one MFMA tile).  A workgroup owns one block of
// 256 token rows and a contiguous range of units, chosen on the host so that every compute unit of the chip gets the same
// number of units (+-1) whatever N is; it walks its range in tiles of up to 8 units (256 x 256 outputs).  Packing puts
// the two members of every RoPE pair, and the gate and up rows of every SwiGLU feature, into the same unit, so a tile may
// start and end at any unit.  The 4 wavefronts of a workgroup are stacked along the token dimension (64 rows each, 2 x NT
// MFMA tiles, up to 256 fp32 accumulators per lane, one wavefront per SIMD).
//
// Operand slabs travel global -> LDS directly (buffer_load ... lds, 16 bytes per lane, no VGPR staging) through a ring of
// 4 stages of K = 32; the load stream runs three stages ahead of the multiply and does not stop at tile boundaries, so
// the next tile's first slabs arrive while the current tile's epilogue runs.  Rows past M fall outside the buffer resource
// and read as zeros.  A stage row is 64 bytes; 16-byte chunk c of row r sits at slot c ^ ((r >> 2) & 3), which keeps both
// the linear 1 KB-per-wavefront DMA fills and the row-strided fragment reads free of bank conflicts.
//
// The compiler cannot see LDS written by DMA (it would wait for every outstanding load before any LDS read), so the
// fragment reads are inline ds_read_b128 and the waits are explicit: loads retire in order and every wavefront issues the
// same number per stage (4 for X, LW for W, the ones beyond the tile's rows aimed outside the buffer), so "vmcnt(8 + LW)"
// in the middle of stage s means stage s+1 has landed.  One memory instruction rides behind each MFMA, pinned with
// scheduling fences, so its issue latency overlaps the matrix pipe.
#pragma once
#include <type_traits>

#include "common.h"

enum GemmEpilogue {
    EPI_QKV_ROPE = 0,  // out = bf16(rope(acc * row_scale[m] + bias[n])): RMSNorm's per-row factor applied after the product
                       // (its gain is folded into W), rotate-half RoPE at row_pos[m] on the q and k heads
    EPI_RESIDUAL = 1,  // out = bf16(acc + resid[m, n])
    EPI_SWIGLU = 2,    // each unit holds 16 gate rows then the 16 up rows of the same features:
                       // out[m, 16 unit + f] = bf16(silu(gate * row_scale[m]) * (up * row_scale[m]))
    EPI_PARTIAL = 3    // split-K: fp32 partial sums to partial[split][m][n]
};

struct GemmArgs {
    const bf16* X;      // [M, K] activations, row stride ldx elements
    const bf16* W;      // [N, K] packed weights, row stride K
    bf16* out;          // [M, ldo]
    const bf16* bias;   // [N] in the original feature order, or null
    const bf16* resid;  // [M, ldr]
    float* partial;     // [splits, M, N]
    const float* row_scale;  // [M] 1/rms of the row (EPI_QKV_ROPE, EPI_SWIGLU)
    const int* row_pos;      // [M] absolute position of the row (EPI_QKV_ROPE)
    const float2* rope_cs;   // [max_pos][head_dim/2] (cos, sin)
    int rope_cols;           // columns [0, rope_cols) are q and k heads (a multiple of head_dim)
    int head_dim;            // 64 or 128
    int ldx, ldo, ldr;
    int M, N, K;
    int tiles_m;             // ceil(M / 256)
    int strips;              // strips per 256-row block; grid.x = tiles_m * strips
    int stages_per_split;    // K/32 stages handled by one blockIdx.y
};

constexpr int GS_BM = 256;
constexpr int GS_BK = 32, GS_STAGES = 4;
constexpr int GS_X_BYTES = GS_BM * GS_BK * 2;        // 16 KB: the token rows of one stage
constexpr int GS_STAGE_BYTES = 2 * GS_X_BYTES;       // + up to 256 weight rows
constexpr int GS_LDS_BYTES = GS_STAGES * GS_STAGE_BYTES;
constexpr int GS_MAX_NT = 8;                         // units per tile

// silu(g) = g / (1 + 2^(-g log2 e)) with the raw v_exp_f32 / v_rcp_f32 instructions (1 ulp each; the result is rounded to bf16)
RS_DEVICE float silu_f32(float g) {
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

template <int I, int N, class F>
RS_DEVICE void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Lane-local epilogue of one tile.  acc[i][j][r] holds token m = m_base + j*32 + l32 and row 8*(r>>2) + 4*half + (r&3) of
// unit unit0 + i.  Per-row inputs and all outputs go through buffer resources sized to M rows, so lanes whose token lies
// past M read zeros and store nothing without any divergent branch (a divergent branch here, inside the tile loop, makes
// the compiler keep the whole pipeline's scalar state in vector registers).
template <int EPI, int NT>
RS_DEVICE void gemm_epilogue(const GemmArgs& a, f32x16 (&acc)[NT][2], int m_base, int unit0, int half, int l32, int split) {
    constexpr int RSRC_FLAGS = 0x00020000;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int m = m_base + j * 32 + l32;
        if constexpr (EPI == EPI_SWIGLU) {
            const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc((void*)a.out, 0, a.M * a.ldo * 2, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_sc = __builtin_amdgcn_make_buffer_rsrc((void*)a.row_scale, 0, a.M * 4, RSRC_FLAGS);
            const float sc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r_sc, m * 4, 0, 0));
            const uint32_t orow = ((uint32_t)m * (uint32_t)a.ldo + 4u * half) * 2u;
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = f32_to_bf16(silu_f32(acc[i][j][4 * q + e] * sc) * (acc[i][j][8 + 4 * q + e] * sc));
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, o), r_out,
                                                          orow + (uint32_t)((unit0 + i) * 16 + 8 * q) * 2u, 0, 0);
                }
        } else if constexpr (EPI == EPI_QKV_ROPE) {
            const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc((void*)a.out, 0, a.M * a.ldo * 2, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_sc = __builtin_amdgcn_make_buffer_rsrc((void*)a.row_scale, 0, a.M * 4, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_pos = __builtin_amdgcn_make_buffer_rsrc((void*)a.row_pos, 0, a.M * 4, RSRC_FLAGS);
            const float sc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r_sc, m * 4, 0, 0));
            const int pos = (int)__builtin_amdgcn_raw_buffer_load_b32(r_pos, m * 4, 0, 0);  // 0 for a row past M
            const int hd2 = a.head_dim >> 1;
            const int uph_shift = (a.head_dim == 128) ? 2 : 1;  // a head is 4 or 2 units
            const float2* csr = a.rope_cs + (size_t)pos * hd2;
            const uint32_t orow = (uint32_t)m * (uint32_t)a.ldo * 2u;
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const int gu = unit0 + i;
                if (gu * 32 < a.rope_cols) {
                    // rows 0..15 of the unit are features f..f+15 of the head's first half, rows 16..31 their partners
                    const int uh = gu & ((1 << uph_shift) - 1);
                    const int fl = (gu >> uph_shift) * a.head_dim + uh * 16 + 4 * half;  // column of this lane's first "low" run
                    const float2* cs = csr + uh * 16 + 4 * half;
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        float bl[4] = {0.0f, 0.0f, 0.0f, 0.0f}, bh[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (a.bias != nullptr) {
                            const bf16x4 b0 = *reinterpret_cast<const bf16x4*>(a.bias + fl + 8 * q);
                            const bf16x4 b1 = *reinterpret_cast<const bf16x4*>(a.bias + fl + hd2 + 8 * q);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                bl[e] = bf16_to_f32(b0[e]);
                                bh[e] = bf16_to_f32(b1[e]);
                            }
                        }
                        bf16x4 ol, oh;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = acc[i][j][4 * q + e] * sc + bl[e];
                            const float hi = acc[i][j][8 + 4 * q + e] * sc + bh[e];
                            const float2 c = cs[8 * q + e];
                            ol[e] = f32_to_bf16(lo * c.x - hi * c.y);
                            oh[e] = f32_to_bf16(hi * c.x + lo * c.y);
                        }
                        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, ol), r_out, orow + (uint32_t)(fl + 8 * q) * 2u, 0, 0);
                        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, oh), r_out, orow + (uint32_t)(fl + hd2 + 8 * q) * 2u, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = gu * 32 + 8 * q + 4 * half;
                        float b[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (a.bias != nullptr) {
                            const bf16x4 b4 = *reinterpret_cast<const bf16x4*>(a.bias + n);
#pragma unroll
                            for (int e = 0; e < 4; ++e) b[e] = bf16_to_f32(b4[e]);
                        }
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(acc[i][j][4 * q + e] * sc + b[e]);
                        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, o), r_out, orow + (uint32_t)n * 2u, 0, 0);
                    }
                }
            }
        } else if constexpr (EPI == EPI_PARTIAL) {
            const __amdgpu_buffer_rsrc_t r_out =
                __builtin_amdgcn_make_buffer_rsrc((void*)(a.partial + (size_t)split * a.M * a.N), 0, a.M * a.N * 4, RSRC_FLAGS);
            const uint32_t orow = (uint32_t)m * (uint32_t)a.N * 4u;
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = (unit0 + i) * 32 + 8 * q + 4 * half;
                    f32x4 o = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), r_out, orow + (uint32_t)n * 4u, 0, 0);
                }
        } else {
            const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc((void*)a.out, 0, a.M * a.ldo * 2, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_res = __builtin_amdgcn_make_buffer_rsrc((void*)a.resid, 0, a.M * a.ldr * 2, RSRC_FLAGS);
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = (unit0 + i) * 32 + 8 * q + 4 * half;
                    const bf16x4 r4 = __builtin_bit_cast(
                        bf16x4, __builtin_amdgcn_raw_buffer_load_b64(r_res, ((uint32_t)m * (uint32_t)a.ldr + (uint32_t)n) * 2u, 0, 0));
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(acc[i][j][4 * q + e] + bf16_to_f32(r4[e]));
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, o), r_out,
                                                          ((uint32_t)m * (uint32_t)a.ldo + (uint32_t)n) * 2u, 0, 0);
                }
        }
    }
}

#define RS_DS_READ_B128(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off))
#define RS_FENCE() __builtin_amdgcn_sched_barrier(0)

// "s_waitcnt lgkmcnt(0)" tied by register operands to the fragments it guards, so the MFMAs that consume them stay below it
template <int NT>
RS_DEVICE void tie_wait_lgkm0(bf16x8 (&w)[NT], bf16x8 (&x)[2]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x[0]), "+v"(x[1]));
#pragma unroll
    for (int i = 0; i < NT; ++i) asm volatile("" : "+v"(w[i]));
}

// waits until at most `stages` whole stages (4 + lw loads each) plus `extra` loads are still in flight
RS_DEVICE void wait_loads_2stages(int lw) {
    switch (lw) {
        case 1: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(14)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
    }
}
RS_DEVICE void wait_loads_1stage_plus_x(int lw) {
    switch (lw) {
        case 1: asm volatile("s_waitcnt vmcnt(9)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(11)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
    }
}

template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_strip_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;
    const int l32 = lane & 31;

    // ---- which strip: workgroup ids are dispatched round-robin over the 8 XCDs; re-map them so that each XCD owns a
    //      contiguous range of strips (all token blocks of a weight range run on one XCD, close in time: the weight stream
    //      crosses the L2 boundary once)
    const int nwg = gridDim.x;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, loc = pid >> 3;
    const int wbase = nwg >> 3, wrem = nwg & 7;
    const int logical = (xcd < wrem ? xcd * (wbase + 1) : wrem * (wbase + 1) + (xcd - wrem) * wbase) + loc;
    const int tm = logical % a.tiles_m;
    const int strip = logical / a.tiles_m;
    const int m0 = tm * GS_BM;

    // ---- the strip's units and its tiles (sizes differ by at most one, larger ones first)
    const int nu = a.N >> 5;
    const int ub = nu / a.strips, ur = nu % a.strips;
    const int u_first = strip * ub + min(strip, ur);
    const int u_count = ub + (strip < ur ? 1 : 0);
    if (u_count == 0) return;  // more strips than units: never launched this way, and uniform for the whole workgroup
    const int ntiles = (u_count + GS_MAX_NT - 1) / GS_MAX_NT;
    const int tb = u_count / ntiles, tr = u_count % ntiles;
    const int lw = (tb + (tr > 0 ? 1 : 0) + 1) >> 1;  // W load instructions per wavefront per stage (64 rows each, workgroup-wide)

    const int split = blockIdx.y;
    const int stages_total = a.K / GS_BK;
    const int st0 = split * a.stages_per_split;
    const int ns = min(a.stages_per_split, stages_total - st0);  // stages per tile (>= 1)
    const uint32_t k0 = (uint32_t)st0 * (GS_BK * 2);

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.X, 0, a.M * a.ldx * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.W, 0, a.N * a.K * 2, 0x00020000);

    // ---- loader geometry: load instruction i of this wavefront fills LDS rows [i*64 + wave*16, +16) of the operand's stage,
    //      each lane fetching the 16-byte chunk that belongs in its slot
    const int ld_r = wave * 16 + (lane >> 2);
    const uint32_t ld_c = (uint32_t)((lane & 3) ^ ((lane >> 4) & 3));
    const uint32_t vx0 = (uint32_t)(m0 + ld_r) * (uint32_t)a.ldx * 2u + ld_c * 16u;  // instruction i: + i * x_step
    const uint32_t vw0 = (uint32_t)ld_r * (uint32_t)a.K * 2u + ld_c * 16u;             // instruction k: + k * w_step
    const uint32_t x_step = 64u * (uint32_t)a.ldx * 2u, w_step = 64u * (uint32_t)a.K * 2u;
    constexpr uint32_t DEAD = 0x80000000u;  // beyond any buffer this kernel is given: reads as zeros, moves no data

    // ---- the load stream (runs ahead of the multiply, across tile boundaries)
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    int d_tile = 0, d_s = 0;
    uint32_t d_slot = 0;              // byte offset of the ring slot being filled
    uint32_t d_koff = k0;             // byte offset of the stage's k range inside a row
    uint32_t d_wsoff = 0;             // byte offset of the tile's first weight row
    uint32_t d_vx = vx0;              // this wavefront's X row offset (DEAD once the stream is past the last tile)
    uint32_t d_vw0, d_vw1, d_vw2, d_vw3;  // W row offset per load instruction (DEAD: no such row in the tile)
    // (written without branches: stores to different variables in the two arms of an "if" get merged by the compiler into
    // one store through a selected address, which keeps that state in scratch memory)
    auto stream_enter_tile = [&]() {
        const bool in_strip = d_tile < ntiles;  // past the strip's last tile the remaining loads of the pipeline move nothing
        const int nt = tb + (d_tile < tr ? 1 : 0);
        const int unit0 = u_first + d_tile * tb + min(d_tile, tr);
        const int live = in_strip ? nt * 32 - wave * 16 : 0;  // load instruction k covers rows k*64 + wave*16 .. of the tile
        d_wsoff = in_strip ? (uint32_t)unit0 * 32u * (uint32_t)a.K * 2u : 0u;
        d_vx = in_strip ? vx0 : DEAD;
        d_vw0 = (0 < live) ? vw0 : DEAD;
        d_vw1 = (64 < live) ? vw0 + w_step : DEAD;
        d_vw2 = (128 < live) ? vw0 + 2 * w_step : DEAD;
        d_vw3 = (192 < live) ? vw0 + 3 * w_step : DEAD;
    };
    auto stream_advance = [&]() {
        d_slot = (d_slot + GS_STAGE_BYTES) & (GS_LDS_BYTES - 1);
        d_koff += GS_BK * 2;
        if (++d_s == ns) {
            d_s = 0;
            d_koff = k0;
            ++d_tile;
            stream_enter_tile();
        }
    };
    // The row part of an address goes into the vector offset, which is what the buffer range check looks at (the scalar
    // offset is excluded from it): rows past M must stay visible to the check.  DEAD + i * x_step stays out of range.
    auto stream_load_x = [&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + d_slot + wave * 1024 + i * 4096);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr)(uintptr_t)dst, 16, d_vx + i * x_step,
                                                 __builtin_amdgcn_readfirstlane(d_koff), 0, 0);
    };
    auto stream_load_w = [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        if (k < lw) {
            const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + d_slot + GS_X_BYTES + wave * 1024 + k * 4096);
            const uint32_t voff = (k == 0) ? d_vw0 : (k == 1) ? d_vw1 : (k == 2) ? d_vw2 : d_vw3;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr)(uintptr_t)dst, 16, voff,
                                                     __builtin_amdgcn_readfirstlane(d_wsoff + d_koff), 0, 0);
        }
    };

    // ---- fragment addresses (bytes from the start of a stage); kk selects the 16-wide k-step inside the stage
    const uint32_t sw = (uint32_t)((l32 >> 2) & 3);
    uint32_t ax[2], aw[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const uint32_t slot = ((uint32_t)(kk * 2 + half) ^ sw) * 16u;
        ax[kk] = lds0 + (uint32_t)(wave * 64 + l32) * 64u + slot;
        aw[kk] = lds0 + (uint32_t)GS_X_BYTES + (uint32_t)l32 * 64u + slot;
    }
    uint32_t c_slot = 0;  // ring slot of the stage being multiplied

    // ---- fill the pipeline: three stages
    stream_enter_tile();
    static_for<0, 3>([&](auto) {
        static_for<0, 4>([&](auto ic) { stream_load_x(ic); });
        static_for<0, 4>([&](auto kc) { stream_load_w(kc); });
        stream_advance();
    });

    auto run_tile = [&](auto ntc, const int unit0) {
        constexpr int NT = decltype(ntc)::value;
        constexpr int SL = 2 * NT;   // MFMAs (= slots for memory instructions) per half stage
        constexpr int LA = NT + 6;   // memory instructions per half stage: NT + 2 fragment reads, 4 loads
        f32x16 acc[NT][2];
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        bf16x8 w0[NT], x0[2], w1[NT], x1[2];

        // fragment read number o of a half stage: x[0], w[0], x[1], w[1], w[2], ...
        auto read_frag = [&](auto oc, bf16x8 (&wf)[NT], bf16x8 (&xf)[2], const uint32_t awv, const uint32_t axv) {
            constexpr int o = decltype(oc)::value;
            if constexpr (o == 0) RS_DS_READ_B128(xf[0], axv, 0);
            else if constexpr (o == 2) RS_DS_READ_B128(xf[1], axv, 2048);
            else if constexpr (o == 1) RS_DS_READ_B128(wf[0], awv, 0);
            else RS_DS_READ_B128(wf[o - 2], awv, (o - 2) * 2048);
        };

        // the tile's first stage has landed (its loads were issued at least two stages of work ago)
        wait_loads_2stages(lw);
        asm volatile("s_barrier" ::: "memory");
        static_for<0, NT + 2>([&](auto oc) { read_frag(oc, w0, x0, aw[0] + c_slot, ax[0] + c_slot); });

        for (int s = 0; s < ns; ++s) {
            const uint32_t n_slot = (c_slot + GS_STAGE_BYTES) & (GS_LDS_BYTES - 1);
            const uint32_t aw1 = aw[1] + c_slot, ax1 = ax[1] + c_slot;
            const uint32_t aw0 = aw[0] + n_slot, ax0 = ax[0] + n_slot;
            tie_wait_lgkm0<NT>(w0, x0);
            // ---- first half: MFMAs on the kk=0 fragments; behind them the kk=1 fragment reads, then the X loads of stage s+3
            static_for<0, SL>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                constexpr int i = q >> 1, j = q & 1;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0[i], x0[j], acc[i][j], 0, 0, 0);
                constexpr int o_lo = (LA <= SL) ? (q < LA ? q : LA) : (q * LA / SL);
                constexpr int o_hi = (LA <= SL) ? (q + 1 < LA ? q + 1 : LA) : ((q + 1) * LA / SL);
                static_for<o_lo, o_hi>([&](auto oc) {
                    constexpr int o = decltype(oc)::value;
                    if constexpr (o < NT + 2) read_frag(oc, w1, x1, aw1, ax1);
                    else stream_load_x(std::integral_constant<int, o - (NT + 2)>{});
                });
                RS_FENCE();
            });
            tie_wait_lgkm0<NT>(w1, x1);  // also: every LDS read of this stage has landed before the barrier frees its slot
            wait_loads_1stage_plus_x(lw);
            asm volatile("s_barrier" ::: "memory");
            RS_FENCE();
            // ---- second half: MFMAs on the kk=1 fragments; behind them the next stage's kk=0 fragment reads, then the W loads
            static_for<0, SL>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                constexpr int i = q >> 1, j = q & 1;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1[i], x1[j], acc[i][j], 0, 0, 0);
                constexpr int o_lo = (LA <= SL) ? (q < LA ? q : LA) : (q * LA / SL);
                constexpr int o_hi = (LA <= SL) ? (q + 1 < LA ? q + 1 : LA) : ((q + 1) * LA / SL);
                static_for<o_lo, o_hi>([&](auto oc) {
                    constexpr int o = decltype(oc)::value;
                    if constexpr (o < NT + 2) read_frag(oc, w0, x0, aw0, ax0);
                    else stream_load_w(std::integral_constant<int, o - (NT + 2)>{});
                });
                RS_FENCE();
            });
            stream_advance();
            c_slot = n_slot;
        }
        tie_wait_lgkm0<NT>(w0, x0);  // the look-ahead read behind the last stage (discarded: the next tile reads its own)
        gemm_epilogue<EPI, NT>(a, acc, m0 + wave * 64, unit0, half, l32, split);
    };

    for (int t = 0; t < ntiles; ++t) {
        const int nt = tb + (t < tr ? 1 : 0);
        const int unit0 = u_first + t * tb + min(t, tr);
        switch (nt) {
            case 1: run_tile(std::integral_constant<int, 1>{}, unit0); break;
            case 2: run_tile(std::integral_constant<int, 2>{}, unit0); break;
            case 3: run_tile(std::integral_constant<int, 3>{}, unit0); break;
            case 4: run_tile(std::integral_constant<int, 4>{}, unit0); break;
            case 5: run_tile(std::integral_constant<int, 5>{}, unit0); break;
            case 6: run_tile(std::integral_constant<int, 6>{}, unit0); break;
            case 7: run_tile(std::integral_constant<int, 7>{}, unit0); break;
            default: run_tile(std::integral_constant<int, 8>{}, unit0); break;
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stream's last (empty) loads still target this workgroup's LDS
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
