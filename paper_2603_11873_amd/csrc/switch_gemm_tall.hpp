// Fused switch, rank-looped form for contractions of 8 or 16 k-steps (16 rank indices each):
// top-2 at the ranks the paper calls typical (64 and 128), four terms at ranks 32 and 64, ...
// Same MFMA arrangement, same arithmetic, same chain of experts and the same bits as
// switch_gemm_overlap_kernel; what differs is the tile: 128 rows x 256 columns, worked as two
// halves of 64 rows that SHARE the column operands.
//
// At these ranks the operands are several times the bytes of the W tile (rank 128 top-2: 128 KB
// of column operands and 32 KB of row operands per 32 KB of W), all of it through the CU's one
// vector L1, which returns data in request order: operand bytes do not only cost L1 cycles, they
// sit in the same queue as the W stream.  Here a wave requests the column operands of its 64
// columns for ALL k-steps once (8 registers per k-step, resident for the life of the workgroup)
// and uses them for both halves, so they cost half as much per W byte; the row operands are
// per half, as before.  W (both halves, 64 KB) goes straight into LDS behind the operands and is
// first looked at by the first half's epilogue.
//   requests: row operands of half 0, column operands, W;   row operands of half 0 into LDS
//   half 0: contraction (meanwhile W lands; row operands of half 1 requested), wait for W,
//           epilogue, store;   half 1: row operands into LDS, contraction, epilogue, store.
// 80 KB of LDS (two workgroups per CU, the same 128 KB of W in flight per CU as four
// workgroups of the 64-row forms).
#pragma once
#include "switch_gemm_overlap.hpp"

namespace adafuse {

constexpr int kTallTileRows = 128;

template <int R, int NT>
constexpr bool tall_supported()
{
    return NT * ((R + 15) / 16) == 8 || NT * ((R + 15) / 16) == 16;
}

template <int R, int NT>
__global__ __launch_bounds__(256) void switch_gemm_tall_kernel(SwitchParams p)
{
    constexpr int NW = 4;
    constexpr int KS = (R + 15) / 16;      // k-steps per expert
    constexpr int RK = R < 16 ? R : 16;    // rank indices of a k-step that exist
    constexpr int SP = NT * KS;            // k-steps per half
    static_assert(SP == 8 || SP == 16, "8 or 16 k-steps");
    constexpr int NS = 8;                  // row-operand pieces resident in LDS
    constexpr int NTHR = 64 * NW;
    constexpr int HR = kGemmTileRows, TC = kGemmWaveCols * NW;  // a half: 64 x 256
    constexpr int WQ = HR * TC / 8 / NTHR;                      // 16-byte pieces of a half per thread
    constexpr int G = KS >= 2 ? 2 : 1;     // k-step pieces fetched with one load
    constexpr int TPK = NTHR / G;
    constexpr int BT = 2048 / TPK;
    using BPiece = typename std::conditional<BT == 16, uint4_t, uint2_t>::type;
    static_assert(BT == 16 || BT == 8, "4 waves");
    static_assert(SP / G + 2 * SP + 2 * WQ <= 63, "outstanding loads");

    __shared__ __align__(16) uint16_t s_b[NS][HR][16];
    __shared__ __align__(16) uint16_t s_w[2 * HR][TC];  // pieces permuted: w_slot

    Terms terms;
    if (!load_terms<NT>(p, terms)) return;
    sort_terms_by_magnitude<NT>(terms);

    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wc = tid >> 6;
    const int n = lane & 31;
    const int h = lane >> 5;
    const int lcol0 = 64 * wc;
    const int rows_left = tile.rows_left, cols_left = tile.cols_left;

    // operand addressing as in switch_gemm_overlap_kernel
    int acol = lcol0 + 8 * (n & 7);
    acol = tile.col0 + (acol < cols_left ? acol : cols_left - 8);
    const uint32_t in_bytes = 2u * (uint32_t)m.in;
    const uint32_t xoff = (uint32_t)(8 * h + (n >> 3)) * in_bytes + 2u * (uint32_t)acol;
    constexpr int BPR = 32 / BT;
    const int bwhich = tid / TPK;
    const int brow_t = (tid % TPK) / BPR, bpart = (tid % TPK) % BPR;
    const uint32_t b_bytes = (uint32_t)(m.out - tile.row0) * R * 2u;
    auto in_use = [&](int step) { return terms.c[step / KS] != 0.0f; };
    auto fetch_b = [&](BPiece &v, int step, int half) {  // the group of pieces of one half that starts at k-step `step`
        const int row = HR * half + brow_t;
        const int brow = row < rows_left ? row : rows_left - 1;
        const uint32_t boff = BT * bpart < 2 * RK ? 2u * (uint32_t)brow * R + 32u * bwhich + (uint32_t)BT * bpart : 0xffffff00u;
        const __amdgpu_buffer_rsrc_t rs =
            make_buffer(m.b_bank + ((size_t)terms.e[step / KS] * m.out + tile.row0) * R, in_use(step) ? b_bytes : 0u);
        if constexpr (BT == 16)
            v = ld_buffer_b128(rs, boff, 32u * (step % KS));
        else
            v = ld_buffer_b64(rs, boff, 32u * (step % KS));
    };
    auto fetch_x = [&](uint4_t (&d)[2], int step) {
        const __amdgpu_buffer_rsrc_t rs = make_buffer(m.a_bank + ((size_t)terms.e[step / KS] * R + 16 * (step % KS)) * m.in,
                                                      in_use(step) ? (uint32_t)RK * in_bytes : 0u);
        d[0] = ld_buffer_b128(rs, xoff, 0u);
        if constexpr (RK > 4)
            d[1] = ld_buffer_b128(rs, xoff, 4u * in_bytes);
        else
            d[1] = uint4_t{0u, 0u, 0u, 0u};
    };
    auto stash_b = [&](const BPiece &v, int slot) {
        *reinterpret_cast<BPiece *>(&s_b[slot + bwhich][brow_t][(BT / 2) * bpart]) = v;
    };

    // ---- requests: row operands of the first half, ALL column operands, then W (both halves)
    BPiece vb[SP / G];
    uint4_t xq[SP][2];
#pragma unroll
    for (int g = 0; g < SP / G; ++g) fetch_b(vb[g], G * g, 0);
#pragma unroll
    for (int s = 0; s < SP; ++s) fetch_x(xq[s], s);
    __builtin_amdgcn_sched_barrier(0);
    {
        const __amdgpu_buffer_rsrc_t rs = make_buffer(tile.w_src, 0xffffffffu);
#pragma unroll
        for (int i = 0; i < 2 * WQ; ++i) {
            const int q = 64 * (wc + NW * i) + lane;
            const int row = q / (TC / 8), pc = (q % (TC / 8)) ^ (row & 31);
            const int cr = row < rows_left ? row : rows_left - 1;
            const int cc = 8 * pc < cols_left ? 8 * pc : cols_left - 8;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t *)(&s_w[0][0] + 512 * (wc + NW * i)), 16,
                                                     (int)(2u * ((uint32_t)cr * (uint32_t)tile.ldw + (uint32_t)cc)), 0, 0, 2 /* non-temporal */);
        }
    }
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int half = 0; half < 2; ++half) {
        // ---- this half's row operands into LDS (every wave is done with the other half's: it has passed
        // the barrier in front of that half's epilogue)
#pragma unroll
        for (int g = 0; g < NS / G; ++g) stash_b(vb[g], G * g);
        lds_barrier();

        float16_t acc[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;
        float c_last = 0.0f;

        // ---- the contraction (first half: while the W tile lands)
#pragma unroll
        for (int s = 0; s < SP; ++s) {
            if (s % KS == 0 && in_use(s)) {  // a new expert: rescale what is accumulated so far
                const float c = terms.c[s / KS];
                if (c_last != 0.0f) {
                    const float ratio = c_last / c;  // |ratio| <= 1
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[rb][cb][v] *= ratio;
                }
                c_last = c;
            }
            uint32_t d[8];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint32_t r[4] = {xq[s][j][0], xq[s][j][1], xq[s][j][2], xq[s][j][3]};
                transpose_lanes_8_16(r);
#pragma unroll
                for (int i = 0; i < 4; ++i) d[4 * j + i] = r[i];
            }
            const uint4_t xe = {__builtin_amdgcn_perm(d[1], d[0], 0x05040100u), __builtin_amdgcn_perm(d[3], d[2], 0x05040100u),
                                __builtin_amdgcn_perm(d[5], d[4], 0x05040100u), __builtin_amdgcn_perm(d[7], d[6], 0x05040100u)};
            const uint4_t xo = {__builtin_amdgcn_perm(d[1], d[0], 0x07060302u), __builtin_amdgcn_perm(d[3], d[2], 0x07060302u),
                                __builtin_amdgcn_perm(d[5], d[4], 0x07060302u), __builtin_amdgcn_perm(d[7], d[6], 0x07060302u)};
            const bf16x8_t x0 = __builtin_bit_cast(bf16x8_t, xe), x1 = __builtin_bit_cast(bf16x8_t, xo);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const uint4_t y = *reinterpret_cast<const uint4_t *>(&s_b[s % NS][32 * rb + n][8 * h]);
                const bf16x8_t yy = __builtin_bit_cast(bf16x8_t, y);
                acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, yy, acc[rb][0], 0, 0, 0);
                acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, yy, acc[rb][1], 0, 0, 0);
            }
            if ((s + 1) % G == 0 && s + 1 - G + NS < SP) {  // the ring turns: group G (s / G) + NS takes the slots of group s / G
                lds_barrier();
                stash_b(vb[s / G + NS / G], (s + 1 - G) % NS);
                if (s + 1 + NS >= SP) lds_barrier();
            }
        }

        if (half == 0) {
            // the registers of the row operands are free: request the second half's (they land behind W)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < SP / G; ++g) fetch_b(vb[g], G * g, 1);
            __builtin_amdgcn_sched_barrier(0);
            // W has to be there now: every wave waits for its own transfers -- everything it requested
            // except the SP / G loads just issued -- and the workgroup meets
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(SP / G) : "memory");
        }
        lds_barrier();
        if (c_last != 0.0f) w_tile_update_grouped<TC>(s_w + HR * half, acc, c_last, lcol0, n, h);
        lds_barrier();
        // write-back of this half: the pieces go out the way they came in
        w_tile_store<TC, NTHR, WQ>(s_w, tile, opaque_copy(tid), HR * half);
    }
}

}  // namespace adafuse
