// Fused switch, rank-looped form for contractions of 8 or 16 k-steps (16 rank indices each):
// top-2 at the ranks the paper calls typical (64 and 128), four terms at ranks 32 and 64, ...
// Same MFMA arrangement, same arithmetic, same chain of experts and the same bits as
// switch_gemm_overlap_kernel.  What differs is what a workgroup owns: a vertical chain of NR
// tiles (64 rows x 256 columns each) of one column strip, worked one after the other.
//
// Why.  At these ranks a 64-row tile spends about half of its workgroup's life contracting,
// finishing and storing -- with no W request of its own in flight -- and only two or three such
// workgroups fit a CU: the W bytes in flight per CU, which set the streaming rate, are a third of
// what the low-rank forms keep in flight.  And the column operands (rank 128 top-2: 128 KB per
// 32 KB of W) all go through the CU's one in-order vector L1, in front of the W requests.
// Here
//   * the NEXT tile's W is requested (straight into the other of two LDS slots) before the current
//     tile's contraction starts, and lands while it runs: a workgroup has 32 KB of W in flight
//     nearly all the time;
//   * a wave requests the column operands of its 64 columns for ALL k-steps once (8 registers per
//     k-step, resident for the life of the workgroup) and reuses them for every tile of the chain:
//     their L1 traffic drops by the chain length;
//   * the row operands are per tile, requested one tile ahead into registers and passed through the
//     LDS ring as before.
// Every wave issues the same number of memory operations per tile whatever the edges look like
// (loads clamp, stores beyond the edge are dropped by their descriptor, a tile beyond the end of
// the matrix still goes through the motions), so the point where a tile's W must have landed is
// one fixed count of later operations (s_waitcnt vmcnt(N)).  80 KB of LDS: two workgroups per CU.
#pragma once
#include "switch_gemm_overlap.hpp"

namespace adafuse {

constexpr int kStripTiles = 8;                                // tiles of 64 rows per workgroup
constexpr int kStripRows = kGemmTileRows * kStripTiles;       // rows of the tile table this form walks

template <int R, int NT>
__global__ __launch_bounds__(256) void switch_gemm_strip_kernel(SwitchParams p)
{
    constexpr int NW = 4, NR = kStripTiles;
    constexpr int KS = (R + 15) / 16;      // k-steps per expert
    constexpr int RK = R < 16 ? R : 16;    // rank indices of a k-step that exist
    constexpr int SP = NT * KS;            // k-steps per tile
    static_assert(SP == 8 || SP == 16, "8 or 16 k-steps");
    static_assert(NR % 2 == 0, "the two W slots alternate");
    constexpr int NS = 8;                  // row-operand pieces resident in LDS
    constexpr int NTHR = 64 * NW;
    constexpr int HR = kGemmTileRows, TC = kGemmWaveCols * NW;  // a tile: 64 x 256
    constexpr int WQ = HR * TC / 8 / NTHR;                      // 16-byte pieces of a tile per thread
    constexpr int G = KS >= 2 ? 2 : 1;     // k-step pieces fetched with one load
    constexpr int TPK = NTHR / G;
    constexpr int BT = 2048 / TPK;
    using BPiece = typename std::conditional<BT == 16, uint4_t, uint2_t>::type;
    static_assert(BT == 16 || BT == 8, "4 waves");
    constexpr int NBL = SP / G;            // row-operand loads per thread and tile
    static_assert(NBL + 2 * SP + 2 * WQ <= 63 && 2 * WQ + 2 * NBL <= 63, "outstanding operations");

    __shared__ __align__(16) uint16_t s_b[NS][HR][16];
    __shared__ __align__(16) uint16_t s_w0[HR][TC], s_w1[HR][TC];  // pieces permuted: w_slot

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
    auto fetch_b = [&](BPiece &v, int step, int rt) {  // the group of pieces of tile rt that starts at k-step `step`
        const int row = HR * rt + brow_t;
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
    // W of tile rt straight into an LDS slot: wave w's instruction i fills the KB that starts at piece slot
    // 64 (w + NW i); rows and columns beyond the edge (or a whole tile beyond it) are clamped to valid ones
    const __amdgpu_buffer_rsrc_t w_rs = make_buffer(tile.w_src, 0xffffffffu);
    auto request_w = [&](uint16_t (*slot)[TC], int rt) {
#pragma unroll
        for (int i = 0; i < WQ; ++i) {
            const int q = 64 * (wc + NW * i) + lane;
            const int lrow = q / (TC / 8), pc = (q % (TC / 8)) ^ (lrow & 31);
            const int row = HR * rt + lrow;
            const int cr = row < rows_left ? row : rows_left - 1;
            const int cc = 8 * pc < cols_left ? 8 * pc : cols_left - 8;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_void_t *)(&slot[0][0] + 512 * (wc + NW * i)), 16,
                                                     (int)(2u * ((uint32_t)cr * (uint32_t)tile.ldw + (uint32_t)cc)), 0, 0, 2 /* non-temporal */);
        }
    };

    // ---- requests: row operands of the first tile, ALL column operands, then the first tile's W
    BPiece vb[NBL];
    uint4_t xq[SP][2];
#pragma unroll
    for (int g = 0; g < NBL; ++g) fetch_b(vb[g], G * g, 0);
#pragma unroll
    for (int s = 0; s < SP; ++s) fetch_x(xq[s], s);
    __builtin_amdgcn_sched_barrier(0);
    request_w(s_w0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // One tile of the chain: `cur` holds (or is about to hold) its W, `nxt` takes the next tile's.
    auto one_tile = [&](uint16_t (*cur)[TC], uint16_t (*nxt)[TC], int rt) {
        // this tile's row operands into LDS.  Every wave is past the previous tile's write-back (its reads
        // of `nxt`) when it leaves this barrier, so the next W may land there.
#pragma unroll
        for (int g = 0; g < NS / G; ++g) stash_b(vb[g], G * g);
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
        request_w(nxt, rt + 1);
        __builtin_amdgcn_sched_barrier(0);

        float16_t acc[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;
        float c_last = 0.0f;
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

        // the registers of the row operands are free: request the next tile's
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NBL; ++g) fetch_b(vb[g], G * g, rt + 1);
        __builtin_amdgcn_sched_barrier(0);
        // This tile's W has to be there now.  Operations this wave has issued since it requested it: the first
        // tile -- the next tile's W and row operands; any later tile -- also its own row operands and the
        // previous tile's write-back, which followed its W request inside the previous tile.
        if (rt == 0)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(WQ + NBL) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * WQ + 2 * NBL) : "memory");
        lds_barrier();
        if (c_last != 0.0f) w_tile_update_grouped<TC>(cur, acc, c_last, lcol0, n, h);
        lds_barrier();
        // write-back: the pieces go out the way they came in (rows of the chain beyond the matrix are dropped)
        {
            const int t2 = opaque_copy(tid);
            const __amdgpu_buffer_rsrc_t rs = make_buffer(tile.w_dst, 0xfffffff0u);
#pragma unroll
            for (int i = 0; i < WQ; ++i) {
                const int q = t2 + NTHR * i;
                const int lrow = q / (TC / 8), pc = q % (TC / 8);
                const int row = HR * rt + lrow;
                const uint32_t off = row < rows_left && 8 * pc < cols_left ? 2u * ((uint32_t)row * (uint32_t)tile.ldw + 8u * (uint32_t)pc) : 0xfffffff8u;
                st_buffer_b128_nt(*w_slot<TC>(cur, lrow, pc), rs, off);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    for (int rt = 0; rt < NR; rt += 2) {
        one_tile(s_w0, s_w1, rt);
        one_tile(s_w1, s_w0, rt + 1);
        if (HR * (rt + 2) >= rows_left) break;  // the chain ends inside this workgroup's rows (a ragged matrix edge)
    }
    // the last tile requested a successor that is never used: let it land before the LDS is given back
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace adafuse
