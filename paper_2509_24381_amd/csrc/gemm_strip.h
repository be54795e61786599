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
// The weight rows travel global -> LDS directly (buffer_load ... lds, 16 bytes per lane, no VGPR staging) through a ring
// of slots, one step of K = 64 per slot; the load stream runs SLOTS - 1 steps ahead of the multiply and does not stop at
// tile boundaries, so the next tile's first slabs arrive while the current tile's epilogue runs.  A slot row is 128
// bytes; 16-byte chunk c of row r sits at place c ^ ((r >> 1) & 7), which keeps both the linear 1 KB-per-wavefront DMA
// fills and the row-strided fragment reads free of bank conflicts.  The token rows are stored fragment-major and go
// global -> registers, XD steps ahead.  Rows past M fall outside the buffer resource and read as zeros.
//
// The compiler cannot see LDS written by DMA (it would wait for every outstanding load before any LDS read), so the
// fragment reads are inline ds_read_b128 and the wait for the next weight step is explicit: loads retire in order and
// every wavefront issues the same number per step (8 for X, NT for W, the ones beyond the tile's rows aimed outside the
// buffer), so a vmcnt that leaves this step's token loads and the loads of the SLOTS - 3 steps before it in flight means
// the next weight step has landed.  One memory instruction rides behind each MFMA, pinned with scheduling fences, so
// its issue latency overlaps the matrix pipe.
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
    const bf16* X;      // [M, K] activations, fragment-major (frag_offset_bytes with width K), blocks of 32 tokens
    const bf16* W;      // [N, K] packed weights, row stride K
    bf16* out;          // [M, ldo], row-major or (out_frag) fragment-major of width ldo
    const bf16* bias;   // [N] in the original feature order, or null
    const bf16* resid;  // [M, ldr], row-major or (resid_frag) fragment-major of width ldr
    float* rowss;       // EPI_RESIDUAL (output, or null): [parts][M], one sum of squares per row and workgroup column - a strip
                        // (times the wavefronts that split its units) - over the features of the stored row that the column
                        // owns; parts = rowss_parts(...) of this launch.  EPI_SWIGLU (input, or null): the same array as the
                        // residual GEMM in front left it; the row factor is then rsqrt(sum of the parts / K + rms_eps)
                        // instead of row_scale[m]
    int rowss_parts;    // EPI_SWIGLU: number of parts in rowss
    float rms_eps;      // EPI_SWIGLU with rowss
    float* partial;     // [splits, M, N]
    const float* row_scale;  // [M] 1/rms of the row (EPI_QKV_ROPE, EPI_SWIGLU)
    const int* row_pos;      // [M][3] rotary position of the row on the (temporal, height, width) axes (EPI_QKV_ROPE)
    int mrope_b0, mrope_b1;  // rotary pair j uses axis 0 if j < b0, axis 1 if j < b1, else axis 2 (1-D RoPE: b0 = b1 = d/2)
    const float2* rope_cs;   // [max_pos][head_dim/2] (cos, sin)
    int rope_cols;           // columns [0, rope_cols) are q and k heads (a multiple of head_dim)
    int head_dim;            // 64 or 128
    int ldo, ldr;
    int out_frag, resid_frag;
    int M, N, K;
    int tiles_m;             // ceil(M / 256)
    int strips;              // strips per 256-row block; grid.x = tiles_m * strips
    int steps_per_split;     // K/64 steps handled by one blockIdx.y
};

constexpr int GS_BM = 256;
constexpr int GS_BK = 64;                            // K per pipeline step
// The kernel comes in two geometries.  Wide: tiles of up to 8 units, a ring of 4 slots of 32 KB (three steps of weight
// look-ahead), token fragments loaded one step ahead, one workgroup per compute unit with up to 512 registers per lane.
// Narrow, for launches whose strips hold at most 2 units (few token rows spread over the whole chip): a step is then only
// 8 or 16 MFMAs per wavefront, shorter than the memory latency one step of look-ahead would have to cover, so the ring has
// 8 slots of 8 KB (seven steps of weight look-ahead) and the token fragments are loaded three steps ahead (the accumulators
// leave the registers for that).  Both are built for one wavefront per SIMD (OCC = 1: 512 registers per lane); with the
// budget of two per SIMD the narrow kernel spills its token fragments, and two workgroups per compute unit measured no
// faster.
constexpr int GS_MAX_NT = 8;                         // units per tile (wide)
constexpr int GS_SLOTS = 4;
constexpr int GS_NARROW_NT = 2;
constexpr int GS_NARROW_SLOTS = 8;
constexpr int GS_NARROW_XD = 3;                      // steps the token fragments are loaded ahead (narrow)
constexpr int gs_lds_bytes(int max_nt, int slots) { return slots * max_nt * 32 * GS_BK * 2; }
constexpr int GS_LDS_BYTES = gs_lds_bytes(GS_MAX_NT, GS_SLOTS);                    // 128 KB
constexpr int GS_NARROW_LDS_BYTES = gs_lds_bytes(GS_NARROW_NT, GS_NARROW_SLOTS);   // 64 KB

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

// Fragment-major activation layout: a [M, W] bf16 matrix is cut into blocks of 32 tokens x 16 features; inside a block the
// two 8-feature halves are 512 bytes apart and the 32 tokens 16 bytes apart, so that the 64 lanes of a wavefront, each
// holding 8 consecutive features of one token (the MFMA operand layout), read or write one contiguous kilobyte.
// Byte offset of element (m, n); n's low 3 bits select the element inside the 16-byte chunk.
RS_DEVICE uint32_t frag_offset_bytes(uint32_t m, uint32_t n, uint32_t width) {
    return ((((m >> 5) * (width >> 4) + (n >> 4)) * 2u + ((n >> 3) & 1u)) * 32u + (m & 31u)) * 16u + (n & 7u) * 2u;
}

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// The two half-waves of an MFMA result hold alternate runs of 4 features of the same token: lanes 0..31 features
// 8q..8q+3, lanes 32..63 features 8q+4..8q+7.  Given the runs of two neighbouring 8-feature groups (even, odd), one
// v_permlane32_swap per dword hands the lower lanes the whole even group and the upper lanes the whole odd group, so every
// lane stores one complete 16-byte chunk (whole cache lines per store instead of interleaved 8-byte halves).
RS_DEVICE u32x4 pair_runs(bf16x4 even_run, bf16x4 odd_run) {
    const u32x2 a = __builtin_bit_cast(u32x2, even_run), b = __builtin_bit_cast(u32x2, odd_run);
    const u32x2 s0 = __builtin_amdgcn_permlane32_swap(a[0], b[0], false, false);  // upper lanes of a <-> lower lanes of b
    const u32x2 s1 = __builtin_amdgcn_permlane32_swap(a[1], b[1], false, false);
    return u32x4{s0[0], s1[0], s0[1], s1[1]};
}

// Lane-local epilogue of one tile.  acc[i][j][r] holds token m = m_base + j*32 + l32 and row 8*(r>>2) + 4*half + (r&3) of
// unit unit0 + i.  Per-row inputs and all outputs go through buffer resources sized to M rows, so lanes whose token lies
// past M read zeros and store nothing without any divergent branch (a divergent branch here, inside the tile loop, makes
// the compiler keep the whole pipeline's scalar state in vector registers).
// The accumulators live in accumulation registers, which the vector ALU cannot read.  Left alone, the register allocator
// copies all of a token block's tiles (up to 128 registers) into vector registers at the top of the epilogue and spills
// the pipeline's in-flight fragments to scratch memory to make room (about 100 dwords per lane and tile, written and read
// back).  The empty asm statement at the top of each unit's iteration pins that unit's tile in accumulation registers up to
// there, so the copies are made 16 registers at a time and nothing spills.
template <int EPI, int NT, int USTRIDE = 1>
RS_DEVICE void gemm_epilogue(const GemmArgs& a, f32x16 (&acc)[NT][2], int m_base, int unit0, int half, int l32, int split,
                             float (&row_val)[2]) {
    // row_val[j], one value per lane and token block j: EPI_SWIGLU reads the row's factor 1/rms there; EPI_RESIDUAL adds
    // the sum of squares of what it stores of the row (this lane's 16 of each unit's 32 features)
    constexpr int RSRC_FLAGS = 0x00020000;
    const int m_pad = (a.M + 31) & ~31;  // fragment-major buffers hold whole blocks of 32 tokens
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int m = m_base + j * 32 + l32;
        if constexpr (EPI == EPI_SWIGLU) {
            // the output is the next GEMM's token operand: always fragment-major.  Unit u holds features 16u..16u+15 = one
            // k-step of it, q selects the 8-feature half, so the 64 lanes of a store cover 512 contiguous bytes
            const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc((void*)a.out, 0, m_pad * a.ldo * 2, RSRC_FLAGS);
            const float sc = row_val[j];
            const uint32_t oblk = (uint32_t)(m >> 5) * (uint32_t)(a.ldo >> 4) * 1024u + (uint32_t)l32 * 16u + (uint32_t)half * 512u;
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                asm volatile("" : "+a"(acc[i][j]));
                bf16x4 o[2];
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[q][e] = f32_to_bf16(silu_f32(acc[i][j][4 * q + e] * sc) * (acc[i][j][8 + 4 * q + e] * sc));
                // lower lanes: features 16u..16u+7 (first half of the k-step), upper lanes: 16u+8..16u+15 (second half)
                __builtin_amdgcn_raw_buffer_store_b128(pair_runs(o[0], o[1]), r_out, oblk + (uint32_t)(unit0 + i * USTRIDE) * 1024u, 0, 0);
            }
        } else if constexpr (EPI == EPI_QKV_ROPE) {
            const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc((void*)a.out, 0, a.M * a.ldo * 2, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_sc = __builtin_amdgcn_make_buffer_rsrc((void*)a.row_scale, 0, a.M * 4, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_pos = __builtin_amdgcn_make_buffer_rsrc((void*)a.row_pos, 0, a.M * 12, RSRC_FLAGS);
            const float sc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r_sc, m * 4, 0, 0));
            int pos3[3];  // 0 for a row past M
#pragma unroll
            for (int ax = 0; ax < 3; ++ax) pos3[ax] = (int)__builtin_amdgcn_raw_buffer_load_b32(r_pos, m * 12 + ax * 4, 0, 0);
            const int hd2 = a.head_dim >> 1;
            const int uph_shift = (a.head_dim == 128) ? 2 : 1;  // a head is 4 or 2 units
            const uint32_t orow = (uint32_t)m * (uint32_t)a.ldo * 2u;
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                asm volatile("" : "+a"(acc[i][j]));
                const int gu = unit0 + i * USTRIDE;
                if (gu * 32 < a.rope_cols) {
                    // rows 0..15 of the unit are features f..f+15 of the head's first half, rows 16..31 their partners
                    const int uh = gu & ((1 << uph_shift) - 1);
                    const int fl = (gu >> uph_shift) * a.head_dim + uh * 16 + 4 * half;  // column of this lane's first "low" run
                    bf16x4 olq[2], ohq[2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        // rotary pair index of this lane's run, and the axis whose position turns it (section bounds are
                        // multiples of 4, so a run of 4 never straddles one)
                        const int j0 = uh * 16 + 8 * q + 4 * half;
                        const int pos = j0 < a.mrope_b0 ? pos3[0] : (j0 < a.mrope_b1 ? pos3[1] : pos3[2]);
                        const float2* cs = a.rope_cs + (size_t)pos * hd2 + j0;
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
                            const float2 c = cs[e];
                            ol[e] = f32_to_bf16(lo * c.x - hi * c.y);
                            oh[e] = f32_to_bf16(hi * c.x + lo * c.y);
                        }
                        olq[q] = ol;
                        ohq[q] = oh;
                    }
                    // lower lanes store features 0..7 of the unit's 16, upper lanes 8..15, as whole 16-byte chunks
                    const uint32_t col = (uint32_t)((gu >> uph_shift) * a.head_dim + uh * 16 + 8 * half);
                    __builtin_amdgcn_raw_buffer_store_b128(pair_runs(olq[0], olq[1]), r_out, orow + col * 2u, 0, 0);
                    __builtin_amdgcn_raw_buffer_store_b128(pair_runs(ohq[0], ohq[1]), r_out, orow + (col + (uint32_t)hd2) * 2u, 0, 0);
                } else {
                    bf16x4 o[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = gu * 32 + 8 * q + 4 * half;
                        float b[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (a.bias != nullptr) {
                            const bf16x4 b4 = *reinterpret_cast<const bf16x4*>(a.bias + n);
#pragma unroll
                            for (int e = 0; e < 4; ++e) b[e] = bf16_to_f32(b4[e]);
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[q][e] = f32_to_bf16(acc[i][j][4 * q + e] * sc + b[e]);
                    }
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr)
                        __builtin_amdgcn_raw_buffer_store_b128(pair_runs(o[2 * pr], o[2 * pr + 1]), r_out,
                                                               orow + (uint32_t)(gu * 32 + 16 * pr + 8 * half) * 2u, 0, 0);
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
                    const int n = (unit0 + i * USTRIDE) * 32 + 8 * q + 4 * half;
                    f32x4 o = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), r_out, orow + (uint32_t)n * 4u, 0, 0);
                }
        } else {
            // residual input and output are row-major [M, ld] or fragment-major (blocks of 32 tokens, padded to whole blocks)
            const __amdgpu_buffer_rsrc_t r_out =
                __builtin_amdgcn_make_buffer_rsrc((void*)a.out, 0, (a.out_frag ? m_pad : a.M) * a.ldo * 2, RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t r_res =
                __builtin_amdgcn_make_buffer_rsrc((void*)a.resid, 0, (a.resid_frag ? m_pad : a.M) * a.ldr * 2, RSRC_FLAGS);
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                asm volatile("" : "+a"(acc[i][j]));
                float ss = 0.0f;
                bf16x4 o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t n = (uint32_t)((unit0 + i * USTRIDE) * 32 + 8 * q + 4 * half);
                    const uint32_t roff = a.resid_frag ? frag_offset_bytes(m, n, a.ldr) : ((uint32_t)m * (uint32_t)a.ldr + n) * 2u;
                    const bf16x4 r4 = __builtin_bit_cast(bf16x4, __builtin_amdgcn_raw_buffer_load_b64(r_res, roff, 0, 0));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        o[q][e] = f32_to_bf16(acc[i][j][4 * q + e] + bf16_to_f32(r4[e]));
                        const float st = bf16_to_f32(o[q][e]);
                        ss += st * st;
                    }
                }
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {  // lower lanes store the even 8-feature group of the pair, upper lanes the odd one
                    const uint32_t n = (uint32_t)((unit0 + i * USTRIDE) * 32 + 16 * pr + 8 * half);
                    const uint32_t ooff = a.out_frag ? frag_offset_bytes(m, n, a.ldo) : ((uint32_t)m * (uint32_t)a.ldo + n) * 2u;
                    __builtin_amdgcn_raw_buffer_store_b128(pair_runs(o[2 * pr], o[2 * pr + 1]), r_out, ooff, 0, 0);
                }
                row_val[j] += ss;
                asm volatile("" : "+v"(row_val[j]));   // (one unit at a time: keeps the residual loads of later units from being hoisted)
            }
        }
    }
}

#define RS_DS_READ_B128(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off))
#define RS_FENCE() __builtin_amdgcn_sched_barrier(0)

// "s_waitcnt lgkmcnt(0)" tied by register operands to the weight fragments it guards, so the MFMAs that consume them
// stay below it
template <int NT>
RS_DEVICE void tie_wait_lgkm0(bf16x8 (&w)[NT]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w[0]));
#pragma unroll
    for (int i = 1; i < NT; ++i) asm volatile("" : "+v"(w[i]));
}
// WT of the 4 wavefronts are stacked along the tokens (64 rows each: a workgroup owns a block of 64 WT rows); the other
// WU = 4 / WT ways they split the units of a tile between them (wavefront (tw, uw) multiplies units uw, uw + WU, ...), and
// strips and tiles are made of groups of WU units.  WT = 2 serves the narrow launches of short calls: a step then moves
// 16 KB of token fragments and 8 KB of weights through the vector-memory pipe for two units, where 256 rows x one unit
// move 32 + 4 KB for one.
template <int EPI, int MAXNT = GS_MAX_NT, int SLOTS = GS_SLOTS, int OCC = 1, int XD = 1, int WT = 4>
__global__ __launch_bounds__(256, OCC) void gemm_strip_kernel(GemmArgs a) {
    constexpr int WU = 4 / WT;
    constexpr int BM = 64 * WT;
    static_assert(WT == 2 || WT == 4, "wavefronts along the tokens");
    static_assert(MAXNT % WU == 0, "a tile is a whole number of unit groups");
    static_assert(WT == 4 || MAXNT == 2, "wavefronts split units in the narrow geometry only");
    constexpr int XB = XD + 1;   // token-fragment buffers: the step being multiplied and the XD steps in flight behind it
    constexpr int SLOT_BYTES = MAXNT * 32 * GS_BK * 2;   // up to 32 MAXNT weight rows of one step
    constexpr int RING_BYTES = SLOTS * SLOT_BYTES;       // a power of two
    constexpr int AHEAD = SLOTS - 1;                     // steps the weight stream runs ahead of the multiply
    static_assert((RING_BYTES & (RING_BYTES - 1)) == 0 && AHEAD >= 3, "ring geometry");
    static_assert(8 + (AHEAD - 2) * (MAXNT + 8) <= 63, "the wait for the next weight step must fit the vmcnt field");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tw = wave & (WT - 1), uw = wave / WT;   // place along the tokens and among the unit-splitting wavefronts
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
    const int m0 = tm * BM;

    // ---- the strip's units and its tiles (sizes differ by at most one, smaller ones first: the load stream then never
    //      issues fewer loads per step than the waits of the tile being multiplied assume)
    //      (counted in groups of WU units from here to the tile loop)
    const int nu = (a.N >> 5) / WU;
    const int ub = nu / a.strips, ur = nu % a.strips;
    const int u_first = strip * ub + min(strip, ur);
    const int u_count = ub + (strip < ur ? 1 : 0);
    if (u_count == 0) return;  // more strips than groups: never launched this way, and uniform for the whole workgroup
    constexpr int MAXG = MAXNT / WU;
    const int ntiles = (u_count + MAXG - 1) / MAXG;
    const int tb = u_count / ntiles;
    const int n_small = ntiles - u_count % ntiles;  // tiles [0, n_small) have tb units, the rest tb + 1

    const int split = blockIdx.y;
    const int steps_total = a.K / GS_BK;
    const int st0 = split * a.steps_per_split;
    const int ns = min(a.steps_per_split, steps_total - st0);  // K steps per tile (>= 1)
    const uint32_t k0 = (uint32_t)st0 * (GS_BK * 2);         // byte offset of the K range in a weight row
    const uint32_t xk0 = (uint32_t)st0 * 4096u;              // and in a fragment-major token block (4 k-steps of 1 KB)

    // ---- token fragments go global -> registers.  X is stored fragment-major (see frag_offset_bytes): the 16 bytes lane
    //      (l32, half) feeds to k-step ks of token block mb sit at ((mb * K/16 + ks) * 2 + half) * 512 + l32 * 16, so one
    //      load instruction of a wavefront fetches one contiguous kilobyte (8 whole cache lines).  Token blocks past M
    //      fall outside the buffer resource and read as zeros.  These are ordinary loads the compiler can see: it places
    //      the vmcnt wait in front of their first use itself (a hand-placed wait on inline-asm loads would not stop the
    //      register allocator from copying a register whose load is still in flight).
    const uint32_t x_block_bytes = (uint32_t)(a.K >> 4) * 1024u;  // one block of 32 tokens, all of K
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.X, 0, ((a.M + 31) >> 5) * (int)x_block_bytes, 0x00020000);
    const uint32_t xv0 = (uint32_t)((m0 >> 5) + tw * 2) * x_block_bytes + (uint32_t)half * 512u + (uint32_t)l32 * 16u;
    const uint32_t xv1 = xv0 + x_block_bytes;
    uint32_t x_koff = xk0;  // byte offset of the next step to load inside a token block
    int x_s = 0;
    bf16x8 xbuf[XB][2][4];
    auto load_x = [&](auto oc, bf16x8 (&xn)[2][4]) {  // load number o of a step: (j, kk) = (o >> 2, o & 3)
        constexpr int o = decltype(oc)::value;
        const uint32_t voff = ((o >> 2) ? xv1 : xv0) + (uint32_t)((o & 3) * 1024);
        xn[o >> 2][o & 3] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rx, voff, x_koff, 0));
    };
    auto x_advance = [&]() {  // the same rows are walked again for every tile; past the last tile the loads are idle repeats
        x_koff += 4096;
        if (++x_s == ns) {
            x_s = 0;
            x_koff = xk0;
        }
    };

    // ---- weight rows go global -> LDS by DMA: load instruction k of this wavefront fills rows [(wave + 4k)*8, +8) of the
    //      step's slot, each lane fetching the 16-byte chunk that belongs in its (swizzled) place
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.W, 0, a.N * a.K * 2, 0x00020000);
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t ld_c = (uint32_t)((lane & 7) ^ ((((wave & 1) << 2) + (lane >> 4)) & 7));
    const uint32_t vw0 = (uint32_t)(wave * 8 + (lane >> 3)) * (uint32_t)a.K * 2u + ld_c * 16u;
    const uint32_t w_step = 32u * (uint32_t)a.K * 2u;  // instruction k + 1 is 32 rows further
    constexpr uint32_t DEAD = 0x80000000u;  // beyond any buffer this kernel is given: reads as zeros, moves no data
    int d_tile = 0, d_s = 0, d_nt = 0;
    uint32_t d_slot = 0;    // byte offset of the ring slot being filled
    uint32_t d_koff = k0;
    uint32_t d_wsoff = 0;   // byte offset of the tile's first weight row
    uint32_t d_vw = DEAD;
    // (written without branches: stores to different variables in the two arms of an "if" get merged by the compiler into
    // one store through a selected address, which keeps that state in scratch memory)
    auto stream_enter_tile = [&]() {
        const bool in_strip = d_tile < ntiles;  // past the strip's last tile the remaining loads of the pipeline move nothing
        const int unit0 = (u_first + d_tile * tb + max(d_tile - n_small, 0)) * WU;
        d_nt = (tb + (d_tile >= n_small ? 1 : 0)) * WU;
        d_wsoff = in_strip ? (uint32_t)unit0 * 32u * (uint32_t)a.K * 2u : 0u;
        d_vw = in_strip ? vw0 : DEAD;
    };
    auto stream_advance = [&]() {
        d_slot = (d_slot + SLOT_BYTES) & (RING_BYTES - 1);
        d_koff += GS_BK * 2;
        if (__builtin_expect(++d_s == ns, 0)) {
            d_s = 0;
            d_koff = k0;
            ++d_tile;
            stream_enter_tile();
        }
    };
    auto load_w = [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + d_slot + wave * 1024 + k * 4096);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr)(uintptr_t)dst, 16, d_vw + k * w_step,
                                                 __builtin_amdgcn_readfirstlane(d_wsoff + d_koff), 0, 0);
    };

    const bool wave_has_rows = m0 + tw * 64 < a.M;   // (uniform per wavefront)

    // ---- one value per lane and token block j (token m0 + tw*64 + j*32 + l32): the RMSNorm factor of the row for the
    //      SwiGLU epilogue, the running sum of squares of the stored row for the residual epilogue (see gemm_epilogue)
    float row_val[2] = {0.0f, 0.0f};

    // ---- weight fragment addresses inside a slot: row l32 of unit i at i*4096 + l32*128, chunk (2 kk + half) swizzled
    uint32_t aw[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        aw[kk] = lds0 + (uint32_t)uw * 4096u + (uint32_t)l32 * 128u + (((uint32_t)(kk * 2 + half) ^ (uint32_t)((l32 >> 1) & 7)) * 16u);
    uint32_t c_slot = 0;  // ring slot of the step being multiplied

    // ---- fill the pipeline: W(0) .. W(AHEAD - 2), X(0) .. X(XD - 1), W(AHEAD - 1)
    stream_enter_tile();
    auto prologue_w = [&]() {
        static_for<0, MAXNT>([&](auto kc) {
            if (decltype(kc)::value < d_nt) load_w(kc);
        });
        stream_advance();
    };
    static_for<0, AHEAD - 1>([&](auto) { prologue_w(); });
    static_for<0, XD>([&](auto bc) {
        static_for<0, 8>([&](auto oc) { load_x(oc, xbuf[decltype(bc)::value]); });
        x_advance();
    });
    prologue_w();
    if constexpr (EPI == EPI_SWIGLU) {
        // The row factors, behind the pipeline's first loads (and waited for with them).  With rowss the residual GEMM in
        // front left rowss_parts partial sums of squares per row, [part][M]: half 0 of the wavefront adds the even parts,
        // half 1 the odd ones, in ascending order (one fixed order: the result does not depend on anything else).
        int mj[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) mj[j] = min(m0 + tw * 64 + j * 32 + l32, a.M - 1);   // (rows past M: any valid row, nothing is stored)
        if (a.rowss != nullptr) {
            constexpr int B = 16;   // loads in flight per row: a pass covers 2 B parts (32 strips at 2048 rows: one pass)
            for (int p0 = half; p0 < a.rowss_parts; p0 += 2 * B) {
                float v[2][B];
#pragma unroll
                for (int u = 0; u < B; ++u)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int p = p0 + 2 * u;
                        v[j][u] = a.rowss[(size_t)min(p, a.rowss_parts - 1) * a.M + mj[j]];
                        if (p >= a.rowss_parts) v[j][u] = 0.0f;
                    }
#pragma unroll
                for (int u = 0; u < B; ++u)
#pragma unroll
                    for (int j = 0; j < 2; ++j) row_val[j] += v[j][u];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) row_val[j] = a.row_scale[mj[j]];
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (EPI == EPI_SWIGLU) {
        if (a.rowss != nullptr) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float ss = row_val[j] + __shfl_xor(row_val[j], 32, WAVE);
                row_val[j] = rsqrtf(ss / (float)a.K + a.rms_eps);
            }
        }
    }

    auto run_tile = [&](auto ntc, const int unit0) {
        constexpr int NT = decltype(ntc)::value;   // units of the tile (= weight DMA instructions per step and wavefront)
        constexpr int NTW = NT / WU;               // units this wavefront multiplies
        constexpr int SL = 2 * NTW;  // MFMAs (= slots for memory instructions) per k-step
        f32x16 acc[NTW][2];
#pragma unroll
        for (int i = 0; i < NTW; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        bf16x8 wa[NTW], wb[NTW];

        auto read_w = [&](auto ic, bf16x8 (&wf)[NTW], const uint32_t addr) {
            constexpr int i = decltype(ic)::value;
            RS_DS_READ_B128(wf[i], addr, i * WU * 4096);
        };
        // one k-step of 2 NT MFMAs on (wf, xc[.][KK]); memory instruction number o of the phase rides behind MFMA number
        // o (or several per MFMA when there are more instructions than MFMAs): first the NT fragment reads of the next
        // k-step, then the phase's EXTRA loads
        auto phase = [&](auto kkc, bf16x8 (&wf)[NTW], bf16x8 (&xc)[2][4], bf16x8 (&wnext)[NTW], const uint32_t wnext_addr,
                         auto extra_count, auto&& extra) {
            constexpr int KK = decltype(kkc)::value;
            constexpr int LA = NTW + decltype(extra_count)::value;
            static_for<0, SL>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                constexpr int i = q >> 1, j = q & 1;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xc[j][KK], acc[i][j], 0, 0, 0);
                constexpr int o_lo = (LA <= SL) ? (q < LA ? q : LA) : (q * LA / SL);
                constexpr int o_hi = (LA <= SL) ? (q + 1 < LA ? q + 1 : LA) : ((q + 1) * LA / SL);
                static_for<o_lo, o_hi>([&](auto oc) {
                    constexpr int o = decltype(oc)::value;
                    if constexpr (o < NTW) read_w(oc, wnext, wnext_addr);
                    else extra(std::integral_constant<int, o - NTW>{});
                });
                RS_FENCE();
            });
        };
        // one step of K = 64: the token fragments of the next step are loaded into xn behind k-steps 0 and 1; the
        // barrier in the middle publishes the weights of the next step, whose first fragments are read behind k-step 3
        // together with the DMA of the weights three steps ahead
        auto step = [&](bf16x8 (&xc)[2][4], bf16x8 (&xn)[2][4]) {
            const uint32_t n_slot = (c_slot + SLOT_BYTES) & (RING_BYTES - 1);
            tie_wait_lgkm0<NTW>(wa);
            phase(std::integral_constant<int, 0>{}, wa, xc, wb, aw[1] + c_slot, std::integral_constant<int, 4>{},
                  [&](auto ec) { load_x(ec, xn); });
            tie_wait_lgkm0<NTW>(wb);
            phase(std::integral_constant<int, 1>{}, wb, xc, wa, aw[2] + c_slot, std::integral_constant<int, 4>{},
                  [&](auto ec) { load_x(std::integral_constant<int, decltype(ec)::value + 4>{}, xn); });
            x_advance();
            tie_wait_lgkm0<NTW>(wa);  // also: every LDS read of k-steps 0..2 has landed
            // this wavefront's share of the next W step has landed when at most this step's 8 token loads and the loads of
            // the AHEAD - 2 steps before it (NT weight, 8 token) are still in flight
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(8 + (AHEAD - 2) * (NT + 8)) : "memory");
            asm volatile("s_barrier" ::: "memory");
            RS_FENCE();
            constexpr int W_A = (NT + 1) / 2, W_B = NT - W_A;
            phase(std::integral_constant<int, 2>{}, wa, xc, wb, aw[3] + c_slot, std::integral_constant<int, W_A>{},
                  [&](auto ec) { load_w(ec); });
            tie_wait_lgkm0<NTW>(wb);
            // (the stream's bookkeeping - scalar work and a rarely taken branch - rides behind an MFMA in the middle of the
            // phase like a memory instruction: left after the phase's last MFMA it holds up the next step's first one by
            // about 150 clocks, with one wavefront per SIMD and nothing else to issue)
            phase(std::integral_constant<int, 3>{}, wb, xc, wa, aw[0] + n_slot, std::integral_constant<int, W_B + 1>{},
                  [&](auto ec) {
                      if constexpr (decltype(ec)::value < W_B) {
                          load_w(std::integral_constant<int, decltype(ec)::value + W_A>{});
                      } else {
                          if (__builtin_expect(d_nt > NT, 0))   // the stream is in a wider tile: one more group of units
                              static_for<0, WU>([&](auto gc) {
                                  constexpr int k = NT + decltype(gc)::value;
                                  load_w(std::integral_constant<int, k < MAXNT ? k : 0>{});
                              });
                          stream_advance();
                      }
                  });
            c_slot = n_slot;
        };

        // The narrow geometry reads the weight fragments of a whole step one step ahead (all four k-steps of step s + 1
        // behind the MFMAs of the second half of step s, right after the barrier that publishes them): with one or two
        // units a k-step is 2 or 4 MFMAs, too few to cover the LDS latency of a read issued one k-step ahead, and the
        // matrix pipe would wait for its operands four times per step.
        constexpr bool FA = MAXNT == 2;
        static_assert(!FA || XB % 2 == 0, "the two fragment sets alternate step by step");
        bf16x8 wcA[4][NTW], wcB[4][NTW];
        // (inline asm names only its own lambda's parameters: operands taken from an enclosing scope are not captured)
        auto read_frag = [](auto offc, bf16x8& dst, const uint32_t addr) { RS_DS_READ_B128(dst, addr, decltype(offc)::value); };
        auto read_step_frags = [&](bf16x8 (&wf)[4][NTW], const uint32_t slot) {
            static_for<0, 4>([&](auto kc) {
                static_for<0, NTW>([&](auto ic) {
                    constexpr int kk = decltype(kc)::value, i = decltype(ic)::value;
                    read_frag(std::integral_constant<int, i * WU * 4096>{}, wf[kk][i], aw[kk] + slot);
                });
            });
        };
        auto wait_step_frags = [&](bf16x8 (&wf)[4][NTW]) {   // "s_waitcnt lgkmcnt(0)" tied to the fragments it guards
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[0][0]));
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int i = 0; i < NTW; ++i) asm volatile("" : "+v"(wf[kk][i]));
        };
        // 2 NTW MFMAs of k-step KK with `count` memory operations riding behind them
        auto phase_fa = [&](auto kkc, bf16x8 (&wf)[NTW], bf16x8 (&xc)[2][4], auto count, auto&& op) {
            constexpr int KK = decltype(kkc)::value;
            constexpr int LA = decltype(count)::value;
            static_for<0, SL>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                constexpr int i = q >> 1, j = q & 1;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xc[j][KK], acc[i][j], 0, 0, 0);
                constexpr int o_lo = (LA <= SL) ? (q < LA ? q : LA) : (q * LA / SL);
                constexpr int o_hi = (LA <= SL) ? (q + 1 < LA ? q + 1 : LA) : ((q + 1) * LA / SL);
                static_for<o_lo, o_hi>([&](auto oc) { op(oc); });
                RS_FENCE();
            });
        };
        auto step_fa = [&](bf16x8 (&xc)[2][4], bf16x8 (&xn)[2][4], bf16x8 (&wc)[4][NTW], bf16x8 (&wn)[4][NTW]) {
            const uint32_t n_slot = (c_slot + SLOT_BYTES) & (RING_BYTES - 1);
            wait_step_frags(wc);
            phase_fa(std::integral_constant<int, 0>{}, wc[0], xc, std::integral_constant<int, 4>{}, [&](auto ec) { load_x(ec, xn); });
            phase_fa(std::integral_constant<int, 1>{}, wc[1], xc, std::integral_constant<int, 4>{},
                     [&](auto ec) { load_x(std::integral_constant<int, decltype(ec)::value + 4>{}, xn); });
            x_advance();
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(8 + (AHEAD - 2) * (NT + 8)) : "memory");   // (as in step)
            asm volatile("s_barrier" ::: "memory");
            RS_FENCE();
            constexpr int W_A = (NT + 1) / 2, W_B = NT - W_A;
            constexpr int RD = 2 * NTW;   // fragment reads per half: two k-steps of the next step
            phase_fa(std::integral_constant<int, 2>{}, wc[2], xc, std::integral_constant<int, RD + W_A>{}, [&](auto ec) {
                constexpr int e = decltype(ec)::value;
                if constexpr (e < RD) read_frag(std::integral_constant<int, (e % NTW) * WU * 4096>{}, wn[e / NTW][e % NTW], aw[e / NTW] + n_slot);
                else load_w(std::integral_constant<int, e - RD>{});
            });
            phase_fa(std::integral_constant<int, 3>{}, wc[3], xc, std::integral_constant<int, RD + W_B + 1>{}, [&](auto ec) {
                constexpr int e = decltype(ec)::value;
                if constexpr (e < RD) {
                    read_frag(std::integral_constant<int, (e % NTW) * WU * 4096>{}, wn[2 + e / NTW][e % NTW], aw[2 + e / NTW] + n_slot);
                } else if constexpr (e - RD < W_B) {
                    load_w(std::integral_constant<int, e - RD + W_A>{});
                } else {
                    if (__builtin_expect(d_nt > NT, 0))   // the stream is in a wider tile: one more group of units
                        static_for<0, WU>([&](auto gc) {
                            constexpr int k = NT + decltype(gc)::value;
                            load_w(std::integral_constant<int, k < MAXNT ? k : 0>{});
                        });
                    stream_advance();
                }
            });
            c_slot = n_slot;
        };

        // tile start: xbuf[0 .. XD - 1] hold (or are receiving) the tile's first token fragments; its first weight step was
        // published by the previous tile's last barrier (by the prologue for the first tile)
        asm volatile("s_barrier" ::: "memory");
        // A wavefront whose 64 rows all lie past M (a call of few rows, or the ragged end of the last block) only does its
        // share of the weight DMA and meets the others at their barriers: every token load, even one that falls outside
        // the buffer, takes its 16 clocks of the compute unit's one vector-memory pipe (32 KB of token fragments per step
        // and workgroup, whatever the tile's width), and with one or two units per tile that pipe, not the matrix pipe, is
        // what a step waits for.  Its queue then holds weight loads only: the next step's have landed when at most those
        // of the AHEAD - 2 steps behind it are in flight.
        if (!wave_has_rows) {
            for (int s = 0; s < ns; ++s) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"((AHEAD - 2) * NT) : "memory");
                asm volatile("s_barrier" ::: "memory");
                static_for<0, NT>([&](auto kc) { load_w(kc); });
                if (__builtin_expect(d_nt > NT, 0))
                    static_for<0, WU>([&](auto gc) {
                        constexpr int k = NT + decltype(gc)::value;
                        load_w(std::integral_constant<int, k < MAXNT ? k : 0>{});
                    });
                stream_advance();
                c_slot = (c_slot + SLOT_BYTES) & (RING_BYTES - 1);
            }
            return;
        }
        if constexpr (FA) read_step_frags(wcA, c_slot);
        else static_for<0, NTW>([&](auto ic) { read_w(ic, wa, aw[0] + c_slot); });
        // step number s multiplies buffer s mod XB and loads the fragments of step s + XD into the buffer step s - 1 used
        // (narrow geometry: even steps multiply fragment set A and read set B for the next step, odd steps the reverse)
        auto do_step = [&](auto uc) {
            constexpr int u = decltype(uc)::value;
            if constexpr (!FA) step(xbuf[u], xbuf[(u + XD) % XB]);
            else if constexpr (u % 2 == 0) step_fa(xbuf[u], xbuf[(u + XD) % XB], wcA, wcB);
            else step_fa(xbuf[u], xbuf[(u + XD) % XB], wcB, wcA);
        };
        int s = 0;
        for (; s + XB <= ns; s += XB) static_for<0, XB>([&](auto uc) { do_step(uc); });
        // the steps left over, then the fragments in flight move to where the next tile expects them (buffer 0 first)
        static_for<1, XB>([&](auto rc) {
            constexpr int R = decltype(rc)::value;
            if (ns - s == R) {
                static_for<0, R>([&](auto uc) { do_step(uc); });
                bf16x8 moved[XB][2][4];
#pragma unroll
                for (int b = 0; b < XD; ++b)      // (the buffer multiplied last holds nothing that is still needed)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) moved[b][j][kk] = xbuf[(b + R) % XB][j][kk];
#pragma unroll
                for (int b = 0; b < XD; ++b)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) xbuf[b][j][kk] = moved[b][j][kk];
            }
        });
        // the look-ahead read behind the last step (discarded: the next tile reads its own)
        if constexpr (FA) {
            wait_step_frags(wcA);
            wait_step_frags(wcB);
        } else {
            tie_wait_lgkm0<NTW>(wa);
        }
        gemm_epilogue<EPI, NTW, WU>(a, acc, m0 + tw * 64, unit0 + uw, half, l32, split, row_val);
    };

    for (int t = 0; t < ntiles; ++t) {
        const int nt = (tb + (t >= n_small ? 1 : 0)) * WU;
        const int unit0 = (u_first + t * tb + max(t - n_small, 0)) * WU;
        if constexpr (MAXNT == 2 && WU == 2) {
            run_tile(std::integral_constant<int, 2>{}, unit0);   // one group of two units
        } else if constexpr (MAXNT == 2) {
            if (nt == 1) run_tile(std::integral_constant<int, 1>{}, unit0);
            else run_tile(std::integral_constant<int, 2>{}, unit0);
        } else
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
    if constexpr (EPI == EPI_RESIDUAL) {
        // what this workgroup column stored of each row, squared and summed: the two half-waves hold the two halves of a
        // token's features, half 0 stores (rows past M, and a launch that wants no sums, store nothing)
        if (a.rowss != nullptr && wave_has_rows) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float ss = row_val[j] + __shfl_xor(row_val[j], 32, WAVE);
                const int m = m0 + tw * 64 + j * 32 + l32;
                if (half == 0 && m < a.M) a.rowss[(size_t)(strip * WU + uw) * a.M + m] = ss;
            }
        }
    }
}

// Sums split-K partials, adds the residual and rounds once:  out[m,n] = bf16(resid[m,n] + sum_s partial[s][m][n]).
// resid / out are row-major or fragment-major (see frag_offset_bytes); when inv_rms is given it also leaves
// rsqrt(mean(out[m,:]^2) + eps) of the stored row there.  WPR wavefronts share a row: 1 (a workgroup covers 4 rows), or 4
// (one row per workgroup, for calls of few rows, which would otherwise occupy a fraction of the chip).
template <int WPR>
__global__ __launch_bounds__(256) void splitk_reduce_residual_kernel(const float* __restrict__ partial, int splits,
                                                                     const bf16* __restrict__ resid, int ldr, int resid_frag,
                                                                     bf16* __restrict__ out, int ldo, int out_frag, int M, int N,
                                                                     float* __restrict__ inv_rms, float eps) {
    static_assert(WPR == 1 || WPR == 4, "wavefronts per row");
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int m = WPR == 1 ? blockIdx.x * 4 + wave : blockIdx.x;
    const int col = WPR == 1 ? lane : wave * WAVE + lane;   // this lane's place among the WPR * 64 lanes of the row
    constexpr int ROW_LANES = WPR * WAVE;
    if (m >= M) return;  // (uniform for the workgroup when the wavefronts share a row)
    float ss = 0.0f;
    // four column groups per pass: all their loads are issued before the first sum (the kernel is one pass over
    // (4 splits + 4) N bytes per row; what it has to hide is latency)
    constexpr int G = 4;
    for (int n0 = col * 4; n0 < N; n0 += G * ROW_LANES * 4) {
        bf16x4 r4[G];
        f32x4 p[G][4];  // at most 4 planes
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int n = n0 + g * ROW_LANES * 4;
            if (n < N) {
                const size_t roff = resid_frag ? frag_offset_bytes(m, n, ldr) : ((size_t)m * ldr + n) * 2;
                r4[g] = *reinterpret_cast<const bf16x4*>(reinterpret_cast<const char*>(resid) + roff);
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (s < splits) p[g][s] = *reinterpret_cast<const f32x4*>(partial + ((size_t)s * M + m) * N + n);
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int n = n0 + g * ROW_LANES * 4;
            if (n < N) {
                float v[4] = {bf16_to_f32(r4[g][0]), bf16_to_f32(r4[g][1]), bf16_to_f32(r4[g][2]), bf16_to_f32(r4[g][3])};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (s < splits) {
                        v[0] += p[g][s][0]; v[1] += p[g][s][1]; v[2] += p[g][s][2]; v[3] += p[g][s][3];
                    }
                bf16x4 o = {f32_to_bf16(v[0]), f32_to_bf16(v[1]), f32_to_bf16(v[2]), f32_to_bf16(v[3])};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float st = bf16_to_f32(o[e]);
                    ss += st * st;
                }
                const size_t ooff = out_frag ? frag_offset_bytes(m, n, ldo) : ((size_t)m * ldo + n) * 2;
                *reinterpret_cast<bf16x4*>(reinterpret_cast<char*>(out) + ooff) = o;
            }
        }
    }
    if (inv_rms != nullptr) {
        ss = wave_sum(ss);
        if constexpr (WPR == 1) {
            if (lane == 0) inv_rms[m] = rsqrtf(ss / (float)N + eps);
        } else {
            __shared__ float part[WPR];
            if (lane == 0) part[wave] = ss;
            __syncthreads();
            if (threadIdx.x == 0) inv_rms[m] = rsqrtf((part[0] + part[1] + part[2] + part[3]) / (float)N + eps);
        }
    }
}
