// Fused switch, rank-looped form for long contractions (8 to 64 k-steps of 16 rank
// indices per tile: top-2 at ranks 64 and 128, four terms at ranks 32 to 128, ...).
// Same tile, same MFMA arrangement, same arithmetic and same write-back as
// switch_gemm_kernel.  Two things differ.
//
// 1. The W tile goes straight into LDS (buffer_load ... lds: no registers, no park
//    step), requested AFTER the operands, and is first looked at by the epilogue:
//      request row operands, column operands, then W (loads return in issue order,
//      so the cache-resident operands are not queued behind the W tile);
//      row operands into LDS; contraction while W lands; wait for W; epilogue.
//    The transfer has to be the buffer form: for it the compiler keeps exact wait
//    counts and knows that accesses to the row-operand array cannot touch the W
//    tile's landing zone, whereas after a global_load_lds it waits for everything
//    before any LDS access.  The barrier that publishes the row operands must not
//    wait for the transfer either, so it is the bare instruction behind a wait for
//    this wave's LDS writes (lds_barrier) instead of __syncthreads(), whose fence
//    drains the transfers.
// 2. The column operand is loaded 16 bytes per lane (8 columns of one rank index) and
//    transposed across lanes in registers, instead of 4 bytes per lane in the layout
//    the MFMA wants.  The vector L1 of a CU delivers 64 B per cycle to 16-byte loads
//    but only 32 B per cycle to 4- and 8-byte loads (measured), and at these ranks the
//    column operands are two to four times the bytes of the W tile.
// The row operands are k-step pieces of 64 x 16 (2 KB each): up to eight are resident
// (48 KB of LDS with the W tile: three workgroups per CU); with 16 k-steps the later
// pieces wait in registers (all requested before W) and take the slot of a consumed
// one behind a barrier.  More than 16 k-steps (up to 64: eight terms of rank 128) run
// as further phases of 16 after the first.  Shorter contractions are faster in
// switch_gemm_kernel: there the W tile is the only thing worth waiting for, and it is
// requested first.
#pragma once
#include "switch_gemm.hpp"

namespace adafuse {

typedef __attribute__((address_space(3))) void lds_void_t;

// This wave's LDS writes are done, then the workgroup meets.  A compiler barrier for
// memory accesses as well, but no wait for outstanding global or global->LDS loads.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// 4 x 4 transpose of 32-bit values across the four lanes {t, t + 8, t + 16, t + 24} of each
// half-wave: lane a of a group ends up with r[i] = what lane i held in r[a].  Lanes 16 apart
// exchange through the row-swap instruction (one instruction swaps a register pair for both
// partners), lanes 8 apart through a rotation by 8 inside their row of 16, written only into
// the 8 lanes that take the partner's value (bank mask).
__device__ __forceinline__ void transpose_lanes_8_16(uint32_t (&r)[4])
{
    typedef __attribute__((ext_vector_type(2))) unsigned int pair_t;
    const pair_t s02 = __builtin_amdgcn_permlane16_swap(r[0], r[2], false, false);
    const pair_t s13 = __builtin_amdgcn_permlane16_swap(r[1], r[3], false, false);
    const uint32_t a0 = s02[0], a2 = s02[1], a1 = s13[0], a3 = s13[1];
    constexpr int kRowRor8 = 0x128;
    r[1] = __builtin_amdgcn_update_dpp(a1, a0, kRowRor8, 0xf, 0x3, false);  // lanes 0..7 of a row: the partner's r[0]
    r[0] = __builtin_amdgcn_update_dpp(a0, a1, kRowRor8, 0xf, 0xc, false);  // lanes 8..15: the partner's r[1]
    r[3] = __builtin_amdgcn_update_dpp(a3, a2, kRowRor8, 0xf, 0x3, false);
    r[2] = __builtin_amdgcn_update_dpp(a2, a3, kRowRor8, 0xf, 0xc, false);
}

// Epilogue for the column assignment of this kernel (see fetch_x there): MFMA column index
// m = 8 g + 4 h + i of a lane stands for the column pair 16 h + 4 i + g of the wave's 64
// columns, so accumulator cb, v = 4 g + i is column 32 h + 8 i + 2 g + cb: per i one
// 16-byte piece of the W tile again.  W' = rn_bf16(W + c * acc), W added last.
template <int TC>
__device__ __forceinline__ void w_tile_update_grouped(uint16_t (*s_w)[TC], const float16_t (&acc)[2][2], float c, int lcol0, int n, int h)
{
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint4_t *slot = w_slot<TC>(s_w, 32 * rb + n, lcol0 / 8 + 4 * h + i);
            const uint4_t wv = *slot;
            uint4_t out;
#pragma unroll
            for (int hh = 0; hh < 4; ++hh)  // one fused multiply-add per element, one rounding to bf16
                out[hh] = pack_bf16_rne(__builtin_fmaf(c, acc[rb][0][4 * hh + i], bf16_lo(wv[hh])),
                                        __builtin_fmaf(c, acc[rb][1][4 * hh + i], bf16_hi(wv[hh])));
            *slot = out;
        }
}

template <int R, int NT, int NW>
__global__ __launch_bounds__(64 * NW) void switch_gemm_overlap_kernel(SwitchParams p)
{
    static_assert(R % 16 == 0 || R == 8 || R == 4, "rank: a multiple of 16, or 4 or 8 (zero padded to one k-step)");
    constexpr int KS = (R + 15) / 16;  // k-steps per expert
    constexpr int RK = R < 16 ? R : 16;  // rank indices of a k-step that exist
    constexpr int STEPS = NT * KS;  // k-steps per tile
    constexpr int SP = STEPS <= 16 ? STEPS : 16;  // k-steps per phase
    constexpr int PH = STEPS / SP;                // phases
    static_assert(STEPS >= 1 && STEPS <= 64 && STEPS % SP == 0, "1 to 16 k-steps, or 32, 48, 64");
    constexpr int NS = SP <= 8 ? SP : 8;  // row-operand pieces resident in LDS; further ones of the phase wait in registers for a slot
    // Column-operand k-steps requested before W (2 loads and 8 registers each): all of
    // them up to 8 k-steps; with 16, as many as leave the kernel at 168 registers (three
    // workgroups per CU: measured, all 16 with two workgroups is 8 % slower).  The rest is
    // requested as slots are consumed and lands behind W.  In all, a wave must stay
    // within the 63 outstanding loads its counter can hold, or the W requests would stall.
    constexpr int XD = SP <= 8 ? SP : (PH >= 4 ? 4 : (PH >= 2 || NT >= 8 ? 6 : 7));
    constexpr int NTHR = 64 * NW;
    constexpr int TR = kGemmTileRows, TC = kGemmWaveCols * NW;
    constexpr int WQ = TR * TC / 8 / NTHR;
    // Row-operand pieces (one k-step: 64 rows x 32 B) are fetched G at a time: two neighbouring
    // k-steps of an expert with one load where an expert has more than one (16 bytes per lane
    // with 4 waves: the L1 delivers twice the bytes per cycle to such loads), else one.
    constexpr int G = KS >= 2 ? 2 : 1;
    constexpr int TPK = NTHR / G;    // threads that share one piece
    constexpr int BT = 2048 / TPK;   // bytes of it per thread
    static_assert(BT == 16 || BT == 8 || BT == 4, "4 or 8 waves");
    using BPiece = typename std::conditional<BT == 16, uint4_t, typename std::conditional<BT == 8, uint2_t, uint32_t>::type>::type;
    static_assert(SP % G == 0, "whole groups");
    static_assert(SP / G + 2 * XD + WQ <= 63, "outstanding loads");

    __shared__ __align__(16) uint16_t s_b[NS][TR][16];
    __shared__ __align__(16) uint16_t s_w[TR][TC];  // pieces permuted: w_slot

    Terms terms;
    if (!load_terms<NT>(p, terms)) return;
    sort_terms_by_magnitude<NT>(terms);  // ascending |c|: every ratio of the accumulator chain has magnitude <= 1

    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wc = tid >> 6;
    const int n = lane & 31;
    const int h = lane >> 5;
    const int lcol0 = 64 * wc;
    const int rows_left = tile.rows_left, cols_left = tile.cols_left;

    // Operand addressing: one descriptor per k-step, one offset register per lane; a
    // k-step of an expert that is not in use gets an empty descriptor (zeros without a
    // memory access), so all of this is straight-line code and the compiler's wait
    // counts are exact.
    // Column operand: 16-byte loads (8 columns of one rank index; twice the bytes per L1
    // cycle of 4-byte loads, and the L1 is what this kernel keeps busiest).  Lane n = t + 8 a
    // (t < 8, a < 4) loads the wave's columns 8 t .. 8 t + 7 at rank indices 8 h + a and
    // 8 h + 4 + a of a k-step; a transpose across a then leaves it with the column pair
    // 4 t + a at the 8 rank indices 8 h .. 8 h + 7, which is what its MFMA operands hold.
    int acol = lcol0 + 8 * (n & 7);
    acol = tile.col0 + (acol < cols_left ? acol : cols_left - 8);
    const uint32_t in_bytes = 2u * (uint32_t)m.in;
    const uint32_t xoff = (uint32_t)(8 * h + (n >> 3)) * in_bytes + 2u * (uint32_t)acol;
    constexpr int BPR = 32 / BT;     // threads per row of a piece
    const int bwhich = tid / TPK;    // which piece of the group this thread works on
    const int brow_t = (tid % TPK) / BPR, bpart = (tid % TPK) % BPR;
    const int brow = brow_t < rows_left ? brow_t : rows_left - 1;
    // the thread's BT bytes of a 32-byte piece row; beyond a padded rank: an offset outside the descriptor, which reads as zero
    const uint32_t boff = BT * bpart < 2 * RK ? 2u * (uint32_t)brow * R + 32u * bwhich + (uint32_t)BT * bpart : 0xffffff00u;
    const uint32_t b_bytes = (uint32_t)(m.out - tile.row0) * R * 2u;
    auto in_use = [&](int step) { return terms.c[step / KS] != 0.0f; };  // unused slots carry coefficient 0
    auto fetch_b = [&](BPiece &v, int step) {  // the group of pieces that starts at k-step `step`
        const __amdgpu_buffer_rsrc_t rs =
            make_buffer(m.b_bank + ((size_t)terms.e[step / KS] * m.out + tile.row0) * R, in_use(step) ? b_bytes : 0u);
        if constexpr (BT == 16)
            v = ld_buffer_b128(rs, boff, 32u * (step % KS));
        else if constexpr (BT == 8)
            v = ld_buffer_b64(rs, boff, 32u * (step % KS));
        else
            v = ld_buffer_b32(rs, boff, 32u * (step % KS));
    };
    auto fetch_x = [&](uint4_t (&d)[2], int step) {
        const __amdgpu_buffer_rsrc_t rs = make_buffer(m.a_bank + ((size_t)terms.e[step / KS] * R + 16 * (step % KS)) * m.in,
                                                      in_use(step) ? (uint32_t)RK * in_bytes : 0u);  // rank indices beyond a padded rank read as zero
        // Zero padding of ranks 4 and 8: the per-lane offset of the upper half (h = 1, 8 rows in) fails
        // the descriptor's range check and reads as zero.  The uniform offset is not part of that
        // check, so at rank 4 the second load (rank indices 4..7 of the lower half: the next
        // expert's rows, or whatever follows the bank) is not issued at all.
        d[0] = ld_buffer_b128(rs, xoff, 0u);
        if constexpr (RK > 4)
            d[1] = ld_buffer_b128(rs, xoff, 4u * in_bytes);
        else
            d[1] = uint4_t{0u, 0u, 0u, 0u};
    };

    auto stash_b = [&](const BPiece &v, int slot) {  // the group goes into slots slot .. slot + G - 1
        *reinterpret_cast<BPiece *>(&s_b[slot + bwhich][brow_t][(BT / 2) * bpart]) = v;
    };

    float16_t acc[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;
    float c_last = 0.0f;

    // The k-steps run in phases of SP (one phase unless the tile takes more than 16): the registers
    // hold one phase's operands.  The W tile is requested in the FIRST phase, behind that phase's
    // operands; the later phases' operands land behind it and are contracted once it is there
    // (requesting W in the last phase instead leaves the workgroup without W traffic for most of
    // its life: 10.4 against 10.1 ms at rank 128 in place).
#pragma unroll
    for (int ph = 0; ph < PH; ++ph) {
        const int s0 = SP * ph;
        // ---- requests: operands first, the W tile last
        BPiece vb[SP / G];
        uint4_t xq[XD][2];
#pragma unroll
        for (int g = 0; g < SP / G; ++g) fetch_b(vb[g], s0 + G * g);
#pragma unroll
        for (int s = 0; s < XD; ++s) fetch_x(xq[s], s0 + s);
        __builtin_amdgcn_sched_barrier(0);
        if (ph == 0) {
            // W: wave w's instruction i fills the 1 KB of LDS that starts at piece slot 64 (w + NW i);
            // lane l delivers slot 64 (w + NW i) + l, i.e. the piece of the row that w_slot puts there.
            // Rows and columns beyond the matrix edge are clamped to valid ones and never stored.
            const __amdgpu_buffer_rsrc_t rs = make_buffer(tile.w_src, 0xffffffffu);
#pragma unroll
            for (int i = 0; i < WQ; ++i) {
                const int q = 64 * (wc + NW * i) + lane;
                const int row = q / (TC / 8), pc = (q % (TC / 8)) ^ (row & 31);
                const int cr = row < rows_left ? row : rows_left - 1;
                const int cc = 8 * pc < cols_left ? 8 * pc : cols_left - 8;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t *)(&s_w[0][0] + 512 * (wc + NW * i)), 16,
                                                         (int)(2u * ((uint32_t)cr * (uint32_t)tile.ldw + (uint32_t)cc)), 0, 0, 2 /* non-temporal */);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- row operands into LDS, visible to the workgroup without waiting for W
        if (ph > 0) lds_barrier();  // every wave is done reading the previous phase's pieces
#pragma unroll
        for (int g = 0; g < NS / G; ++g) stash_b(vb[g], G * g);
        lds_barrier();

        // ---- the contraction (in the first phase: while the W tile lands)
#pragma unroll
        for (int s = 0; s < SP; ++s) {
            const int step = s0 + s;
            if (step % KS == 0 && in_use(step)) {  // a new expert: rescale what is accumulated so far (uniform branch, no loads inside)
                const float c = terms.c[step / KS];
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
                uint32_t r[4] = {xq[s % XD][j][0], xq[s % XD][j][1], xq[s % XD][j][2], xq[s % XD][j][3]};
                transpose_lanes_8_16(r);
#pragma unroll
                for (int i = 0; i < 4; ++i) d[4 * j + i] = r[i];
            }
            const uint4_t xe = {__builtin_amdgcn_perm(d[1], d[0], 0x05040100u), __builtin_amdgcn_perm(d[3], d[2], 0x05040100u),
                                __builtin_amdgcn_perm(d[5], d[4], 0x05040100u), __builtin_amdgcn_perm(d[7], d[6], 0x05040100u)};
            const uint4_t xo = {__builtin_amdgcn_perm(d[1], d[0], 0x07060302u), __builtin_amdgcn_perm(d[3], d[2], 0x07060302u),
                                __builtin_amdgcn_perm(d[5], d[4], 0x07060302u), __builtin_amdgcn_perm(d[7], d[6], 0x07060302u)};
            const bf16x8_t x0 = __builtin_bit_cast(bf16x8_t, xe), x1 = __builtin_bit_cast(bf16x8_t, xo);
            if (s + XD < SP) fetch_x(xq[s % XD], step + XD);  // the slot is consumed: refill it
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const uint4_t y = *reinterpret_cast<const uint4_t *>(&s_b[s % NS][32 * rb + n][8 * h]);
                const bf16x8_t yy = __builtin_bit_cast(bf16x8_t, y);
                acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, yy, acc[rb][0], 0, 0, 0);
                acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, yy, acc[rb][1], 0, 0, 0);
            }
            if ((s + 1) % G == 0 && s + 1 - G + NS < SP) {  // the ring turns: the group G (s / G) + NS takes the slots of group s / G
                lds_barrier();  // every wave is done reading them
                stash_b(vb[s / G + NS / G], (s + 1 - G) % NS);
                // the refill is visible to its readers through the barrier of the next
                // turn, or, when no further slot turns, through this one
                if (s + 1 + NS >= SP) lds_barrier();
            }
        }
    }

    // ---- the W tile has to be there now: every wave waits for its own transfers (the fence of
    // the barrier makes the compiler wait as well; the explicit wait does not depend on that)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (c_last != 0.0f) w_tile_update_grouped<TC>(s_w, acc, c_last, lcol0, n, h);
    __syncthreads();
    w_tile_store<TC, NTHR, WQ>(s_w, tile, opaque_copy(tid));
}

}  // namespace adafuse
