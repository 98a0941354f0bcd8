// Fused switch, rank-looped form: the default from rank 16 on, and the only form
// for the paper's "typical" ranks 64 and 128 (inner dimension 128..256 with
// top-2, twice that in place).  Here the low-rank product is a real contraction,
// so it runs on the wide matrix-core shape v_mfma_f32_32x32x16_bf16, one expert
// after another.
//
// A wave owns a 64 x 64 piece of W (2 x 2 MFMA blocks, 64 fp32 accumulators per
// lane); a workgroup is 4 waves side by side on a 64 x 256 tile.
//   * W through LDS.  The 32x32 result layout gives a lane 16-byte pieces of 32
//     different rows, which streams badly (every access touches 32 cache lines
//     for 1 KB).  So the workgroup moves its W tile with row-contiguous 128-bit
//     accesses (a wave instruction = two whole 512-byte row pieces), parks it in
//     LDS as soon as it lands, each lane updates its pieces there in the result
//     layout, and the tile goes back out the same way.
//   * Row operand (B bank, [out][rank]): one expert's rows of the tile are one
//     contiguous piece of memory; the workgroup fetches it coalesced into LDS,
//     as many experts up front as the LDS budget holds (all of them in the usual
//     cases, so the main loop has no barrier), the rest rolling.  A lane reads
//     its 8 rank indices of a row as one 16-byte LDS read.
//   * Column operand (A bank, [rank][in]): block cb of a wave takes the even
//     (cb=0) / odd (cb=1) columns of its 64, so the operands of both blocks for
//     one rank index are the two halves of ONE aligned 32-bit word: 8 coalesced
//     dword loads per 16 rank indices, packed with byte permutes, kept in a
//     register queue that runs several chunks ahead of the MFMAs.
//   * Result layout with that column assignment: a lane holds, per row block and
//     b = 0..3, the 8 contiguous columns base + 16 b + 8 (lane/32) + 0..7 of row
//     lane%32 -- one 16-byte piece of the W tile each.
// Everything the tile needs is requested at the start (loads return in issue
// order): W, row operands, the first column operands -- or, with four experts'
// operands to queue, the operands first and W last.  All loads are unconditional
// with clamped addresses: a row or column beyond the matrix edge only feeds
// results that are never stored, and loads inside branches make the compiler
// fall back to waiting for every outstanding load.  Operand loads use buffer
// descriptors (one address register per lane for a whole group of loads).
// The W tile sits in LDS unpadded (32 KB), its 16-byte pieces permuted by the
// row number (w_slot), which leaves 8 KB of a four-workgroups-per-CU share of
// LDS for the row operands.
// Two forms, by the number of k-steps (16 rank indices of one expert) a tile
// takes: switch_gemm_kernel<R, NT> below, fully unrolled with every row operand
// resident, up to 7; switch_gemm_overlap_kernel<R, NT> (its own header) from 8
// on, where the contraction is long enough to be worth running while the W tile
// is still on its way.
// Gates stay out of the bf16 operands.  Experts are chained in ONE accumulator,
// in ascending order of |c_j| (sort_terms_by_magnitude):
//   acc = P_0;  acc = acc * (c_0/c_1) + P_1;  ...;  W' = rn_bf16(fma(c_last, acc, W))
// which equals W + sum_j c_j P_j up to fp32 rounding of the ratios.  Every ratio has
// magnitude <= 1, so a tiny or sub-normal gate beside an ordinary one cannot overflow
// it; terms with a zero coefficient are skipped, so no ratio divides by zero.
#pragma once
#include "device_types.hpp"

namespace adafuse {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float float16_t;

constexpr int kGemmTileRows = 64;
constexpr int kGemmWaveCols = 64;  // a workgroup of NW waves covers 64 NW columns

// The W tile in LDS: TR rows of TC bf16 with no padding (32 KB for 64 x 256, which
// leaves 8 KB of a 40 KB share -- four workgroups per CU -- for the operands).  The
// 16-byte pieces of a row are permuted by the row number instead: row-contiguous
// accesses (in and out) stay conflict-free, and the result-layout accesses (one
// piece column over 32 rows) spread over all banks as they would with a padded pitch.
template <int TC>
__device__ __forceinline__ uint4_t *w_slot(uint16_t (*s_w)[TC], int row, int piece)
{
    return reinterpret_cast<uint4_t *>(&s_w[row][8 * (piece ^ (row & 31))]);
}

// ---- the W tile's way in and out, shared by the three kernel forms ------------------
// Request: row-contiguous non-temporal 128-bit loads, thread q takes the pieces
// q, q + NTHR, ...; rows and columns beyond the matrix edge are clamped to valid
// ones (unconditional loads schedule freely) and are never stored.
template <int TC, int NTHR, int WQ>
__device__ __forceinline__ void w_tile_request(uint4_t (&wreg)[WQ], const TileDev &tile, int tid)
{
#pragma unroll
    for (int i = 0; i < WQ; ++i) {
        const int q = tid + NTHR * i;
        const int row = q / (TC / 8), pc = q % (TC / 8);
        const int cr = row < tile.rows_left ? row : tile.rows_left - 1;
        const int cc = 8 * pc < tile.cols_left ? 8 * pc : tile.cols_left - 8;
        wreg[i] = ld_global_nt(reinterpret_cast<const uint4_t *>(tile.w_src + (size_t)cr * tile.ldw + cc));
    }
}
// Park: the same pieces into LDS as they land.
template <int TC, int NTHR, int WQ>
__device__ __forceinline__ void w_tile_park(uint16_t (*s_w)[TC], const uint4_t (&wreg)[WQ], int tid)
{
#pragma unroll
    for (int i = 0; i < WQ; ++i) {
        const int q = tid + NTHR * i;
        *w_slot<TC>(s_w, q / (TC / 8), q % (TC / 8)) = wreg[i];
    }
}
// Epilogue: each lane updates its pieces of the W tile in LDS, in the MFMA result
// layout (row 32 rb + n of the wave's rows; column p of the 16-column group b is
// accumulator cb = p & 1, v = 4 b + p / 2): W' = rn_bf16(W + c * acc), W added last.
template <int TC>
__device__ __forceinline__ void w_tile_update(uint16_t (*s_w)[TC], const float16_t (&acc)[2][2], float c, int lrow0, int lcol0, int n, int h)
{
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            uint4_t *slot = w_slot<TC>(s_w, lrow0 + 32 * rb + n, lcol0 / 8 + 2 * b + h);
            const uint4_t wv = *slot;
            uint4_t out;
#pragma unroll
            for (int hh = 0; hh < 4; ++hh)  // columns 2 hh, 2 hh + 1 of the piece: one fused multiply-add each, one rounding to bf16
                out[hh] = pack_bf16_rne(__builtin_fmaf(c, acc[rb][0][4 * b + hh], bf16_lo(wv[hh])),
                                        __builtin_fmaf(c, acc[rb][1][4 * b + hh], bf16_hi(wv[hh])));
            *slot = out;
        }
}
// The write-back addresses are the ones the tile was parked with.  The kernels derive
// them again from an opaque copy of the thread index: kept alive across the
// contraction they cost registers (a workgroup per CU where the budget is exact) or are
// spilled, and every reload from scratch memory is a full memory round trip at the end
// of the workgroup's life.
__device__ __forceinline__ int opaque_copy(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}
// Write-back: the pieces go out the way they came in.  Every thread issues all of its stores,
// through a buffer descriptor on the tile's origin: a piece beyond the matrix edge is pointed at an
// offset outside the descriptor, where the hardware drops it.  No store sits in a branch (a branch
// per store costs a few percent of the whole launch: the compiler closes each with its own waits).
template <int TC, int NTHR, int WQ>
__device__ __forceinline__ void w_tile_store(uint16_t (*s_w)[TC], const TileDev &tile, int tid, int row_base = 0)
{
    const __amdgpu_buffer_rsrc_t rs = make_buffer(tile.w_dst, 0xfffffff0u);
#pragma unroll
    for (int i = 0; i < WQ; ++i) {
        const int q = tid + NTHR * i;
        const int row = row_base + q / (TC / 8), pc = q % (TC / 8);
        const uint32_t off = row < tile.rows_left && 8 * pc < tile.cols_left ? 2u * ((uint32_t)row * (uint32_t)tile.ldw + 8u * (uint32_t)pc) : 0xfffffff8u;
        st_buffer_b128_nt(*w_slot<TC>(s_w, row, pc), rs, off);
    }
}

template <int R, int NT>
struct GemmPlan {
    static constexpr int KS = (R + 15) / 16;          // k-steps (16 rank indices) per expert
    static constexpr bool kPadded = R < 16;           // one k-step whose rank indices >= R are zero
    static constexpr int KCH = KS >= 2 ? 2 : 1;       // k-steps per column-operand chunk
    static constexpr int NCH = KS / KCH;              // chunks per expert
    static constexpr int TOT = NT * NCH;              // chunks per tile
    // Chunks in flight: at most 64 VGPRs.  Rank 128 takes half of that and one resident B
    // slice (BMAX) to stay under 168 VGPRs and 53 KB of LDS: three workgroups per CU
    // instead of two outweigh the shorter queue there (not so at rank 64).
    static constexpr int QMAX = KCH == 1 ? 8 : (R >= 128 ? 2 : 4);
    static constexpr int QX = TOT < QMAX ? TOT : QMAX;
    static constexpr int RP = R < 8 ? 8 : R;          // rank padded to one 16-byte piece
    // LDS row pitch of a staged B slice (bf16).  One k-step per row (32 bytes) needs no
    // padding: a wave's 64 reads of 16 bytes cover 1 KB contiguously.  Rows of 2 or 4
    // k-steps are not padded either: their 16-byte pieces are permuted by the row number
    // (b_piece), so that the 16 rows a quarter-wave reads at one piece index fall on 16
    // different bank groups.  Rank 128 keeps a 16-byte pad (the permuted addresses cost
    // it the registers that decide its occupancy).
    static constexpr int BP = R <= 16 ? 16 : (R >= 128 ? R + 8 : R);
    static constexpr int PPRB = BP / 8;  // 16-byte pieces per row
    __device__ static __forceinline__ int b_piece(int row, int piece)
    {
        if constexpr (R <= 16 || BP != R)
            return piece;
        else
            return piece ^ ((row * PPRB / 16) & (PPRB - 1));
    }
    // B slices resident in LDS (more cost a workgroup per CU).  A further expert's slice is
    // requested when the contraction of the expert whose slot it takes begins, and stored
    // behind a barrier once that contraction is done.
    static constexpr int BMAX = R <= 16 ? 4 : (R >= 128 ? 1 : 2);
    static constexpr int NB = NT < BMAX ? NT : BMAX;  // B slices resident
    static constexpr int BV = kGemmTileRows * RP / 8;  // 16-byte pieces of one expert's B slice
    static constexpr int BQ(int nthr) { return (BV + nthr - 1) / nthr; }  // ... per thread
    static_assert(NB >= 2 || NT <= 2, "rolling more than one refill needs two resident slices");
};

template <int R, int NT, int NW>
__global__ __launch_bounds__(64 * NW) void switch_gemm_kernel(SwitchParams p)
{
    static_assert(R % 16 == 0 || R == 8 || R == 4, "rank: a multiple of 16, or 4 or 8 (zero padded)");
    using P = GemmPlan<R, NT>;
    constexpr int NTHR = 64 * NW;
    constexpr int KCH = P::KCH, NCH = P::NCH, TOT = P::TOT, QX = P::QX, NB = P::NB;
    constexpr int BP = P::BP, BV = P::BV, BQ = P::BQ(NTHR);
    constexpr int TR = kGemmTileRows, TC = kGemmWaveCols * NW;
    constexpr int WQ = TR * TC / 8 / NTHR;  // 16-byte pieces of the W tile per thread

    __shared__ __align__(16) uint16_t s_b[NB][TR][BP];  // row operands of the resident experts
    __shared__ __align__(16) uint16_t s_w[TR][TC];      // the W tile, on its way in and out (pieces permuted: w_slot)

    Terms terms;
    if (!load_terms<NT>(p, terms)) return;
    sort_terms_by_magnitude<NT>(terms);  // ascending |c|: zero coefficients (unused slots too) first, skipped by value
    auto in_use = [&](int j) { return terms.c[j] != 0.0f; };

    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wc = tid >> 6;   // the wave's 64-column strip
    const int n = lane & 31;   // row inside a 32-row block (MFMA N index)
    const int h = lane >> 5;   // which half of the k-step / of a 16-column group
    const int lcol0 = 64 * wc;
    const int rows_left = tile.rows_left, cols_left = tile.cols_left;

    // ---- request everything.  Loads return in issue order, so operand loads (cache
    // hits) queued behind the W loads (HBM) sit on their return slots until W has
    // landed.  With one or two experts that costs nothing and W should go first;
    // with four experts' operands in the queue it slowed the W loads themselves
    // (measured: 5.8 ms against 4.7 ms per launch on the 8B shape), so there the
    // operands go first and W last.
    constexpr bool kOperandsFirst = NT >= 4;
    uint4_t wreg[WQ];
    if constexpr (!kOperandsFirst) w_tile_request<TC, NTHR>(wreg, tile, tid);

    // Operand loads go through buffer descriptors: base and size of one expert's
    // slice in scalar registers, ONE 32-bit offset register per lane for all loads
    // of a group, the rest of the address uniform.  (Shapes are limited to 2^22
    // in either direction: a slice stays below 2^31 bytes.)
    const uint32_t b_bytes = (uint32_t)(m.out - tile.row0) * R * 2u;  // from the tile's first row to the end of the expert
    // Up to rank 16 a slice is one k-step per row: 64 rows of 32 bytes in LDS, of which the
    // first 2 R hold data.  EVERY thread brings the same number of dwords of that image
    // (dword d = row d / 8, position d % 8), the positions beyond the rank through an offset
    // outside the descriptor, which reads as zero: no load and no store sits in a branch
    // (the compiler ends a conditional block that loads with a wait for all loads, which
    // made the four experts' slices four round trips in a row).  From rank 32 on the
    // 16-byte pieces of a slice divide evenly among the threads.
    using BReg = typename std::conditional<(R <= 16), uint32_t, uint4_t>::type;
    constexpr int BN = R <= 16 ? TR * 8 / NTHR : BQ;  // registers of that type per thread and slice
    static_assert((TR * 8) % NTHR == 0, "the dwords of a one-k-step slice divide evenly among the threads");
    constexpr bool kAllThreads = R <= 16 || BV % NTHR == 0;  // else (rank 32 with 8 waves) the last pieces are guarded
    auto fetch_b = [&](BReg (&v)[BN], int e, bool used) {
        const __amdgpu_buffer_rsrc_t rs = make_buffer(m.b_bank + ((size_t)e * m.out + tile.row0) * R, used ? b_bytes : 0u);
#pragma unroll
        for (int i = 0; i < BN; ++i) {
            const int q = tid + NTHR * i;
            if constexpr (R <= 16) {
                const int row = q / 8, pos = q % 8;
                const int cr = row < rows_left ? row : rows_left - 1;
                v[i] = ld_buffer_b32(rs, 2 * pos < R ? 2u * (uint32_t)cr * R + 4u * pos : 0xffffff00u, 0u);
            } else {
                const int row = q / (R / 8), piece = q % (R / 8);
                const int cr = row < rows_left ? row : rows_left - 1;
                if (kAllThreads || q < BV) v[i] = ld_buffer_b128(rs, 2u * ((uint32_t)cr * R + 8u * piece), 0u);
            }
        }
    };
    auto stash_b = [&](const BReg (&v)[BN], int slot) {
#pragma unroll
        for (int i = 0; i < BN; ++i) {
            const int q = tid + NTHR * i;
            if constexpr (R <= 16) {
                reinterpret_cast<uint32_t *>(&s_b[slot][0][0])[q] = v[i];
            } else {
                const int row = q / (R / 8), piece = q % (R / 8);
                if (kAllThreads || q < BV) *reinterpret_cast<uint4_t *>(&s_b[slot][row][8 * P::b_piece(row, piece)]) = v[i];
            }
        }
    };

    // column operand: the lane's column pair (clamped), 8 rank indices per k-step
    int acol = lcol0 + 2 * n;
    acol = tile.col0 + (acol < cols_left ? acol : cols_left - 2);
    struct XChunk {
        uint32_t d[KCH][8];
    };
    const uint32_t in_bytes = 2u * (uint32_t)m.in;
    const uint32_t xoff = 8u * h * in_bytes + 2u * (uint32_t)acol;  // rank index 8h of a k-step, this lane's columns
    auto fetch_x = [&](XChunk &x, int e, int kc) {
        const __amdgpu_buffer_rsrc_t rs = make_buffer(m.a_bank + (size_t)e * R * m.in, (uint32_t)R * in_bytes);
#pragma unroll
        for (int s2 = 0; s2 < KCH; ++s2)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                // rank index 16 (KCH kc + s2) + 8h + i.  Zero padding of ranks 4 and 8: an index the
                // PER-LANE offset puts beyond the slice (h = 1: 8 rows in) fails the descriptor's range
                // check and reads as zero; the uniform offset is not part of that check, so indices
                // i >= R of the lower half are not loaded at all (rank 4: they would be the next
                // expert's rows, or whatever follows the bank)
                if (R < 8 && i >= R)
                    x.d[s2][i] = 0u;
                else
                    x.d[s2][i] = ld_buffer_b32(rs, xoff, (uint32_t)(16 * (KCH * kc + s2) + i) * in_bytes);
            }
    };

    BReg vb[NB][BN];
#pragma unroll
    for (int j = 0; j < NB; ++j) fetch_b(vb[j], terms.e[j], in_use(j));  // an unused term: empty descriptor, zeros
    XChunk xq[QX];
#pragma unroll
    for (int i = 0; i < QX; ++i)
        if (in_use(i / NCH)) fetch_x(xq[i], terms.e[i / NCH], i % NCH);
    if constexpr (kOperandsFirst) {
        w_tile_request<TC, NTHR>(wreg, tile, tid);
#pragma unroll
        for (int j = 0; j < NB; ++j) stash_b(vb[j], j);
    }

    // W tile and row operands into LDS as they land: the registers are free for the contraction
    w_tile_park<TC, NTHR>(s_w, wreg, tid);
    if constexpr (!kOperandsFirst) {
#pragma unroll
        for (int j = 0; j < NB; ++j) stash_b(vb[j], j);
    }
    __syncthreads();

    float16_t acc[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;

    // ---- the contraction, fully unrolled over experts and chunks (all queue slots static)
    float c_last = 0.0f;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const float c = terms.c[j];
        const bool active = c != 0.0f;  // uniform; a zero coefficient contributes nothing
        BReg vroll[BN];
        if constexpr (NT > NB) {
            if (j + NB < NT) fetch_b(vroll, terms.e[j + NB], in_use(j + NB));  // rolls into this expert's slot below
        }
        if (active && c_last != 0.0f) {
            const float ratio = c_last / c;  // |ratio| <= 1: the terms come in ascending magnitude
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[rb][cb][v] *= ratio;
        }
        if (active) c_last = c;
#pragma unroll
        for (int kc = 0; kc < NCH; ++kc) {
            const int i = j * NCH + kc;  // chunk number; a constant after unrolling
            XChunk &x = xq[i % QX];
            bf16x8_t x0[KCH], x1[KCH];
#pragma unroll
            for (int s2 = 0; s2 < KCH; ++s2) {
                const uint32_t *d = x.d[s2];
                const uint4_t xe = {__builtin_amdgcn_perm(d[1], d[0], 0x05040100u), __builtin_amdgcn_perm(d[3], d[2], 0x05040100u),
                                    __builtin_amdgcn_perm(d[5], d[4], 0x05040100u), __builtin_amdgcn_perm(d[7], d[6], 0x05040100u)};
                const uint4_t xo = {__builtin_amdgcn_perm(d[1], d[0], 0x07060302u), __builtin_amdgcn_perm(d[3], d[2], 0x07060302u),
                                    __builtin_amdgcn_perm(d[5], d[4], 0x07060302u), __builtin_amdgcn_perm(d[7], d[6], 0x07060302u)};
                x0[s2] = __builtin_bit_cast(bf16x8_t, xe);
                x1[s2] = __builtin_bit_cast(bf16x8_t, xo);
            }
            // the slot is consumed: refill it with the chunk QX ahead
            if (i + QX < TOT && in_use((i + QX) / NCH)) fetch_x(x, terms.e[(i + QX) / NCH], (i + QX) % NCH);
            if (active) {
#pragma unroll
                for (int s2 = 0; s2 < KCH; ++s2) {
                    const int ks = kc * KCH + s2;
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) {
                        const uint4_t y = *reinterpret_cast<const uint4_t *>(&s_b[j % NB][32 * rb + n][8 * P::b_piece(32 * rb + n, 2 * ks + h)]);
                        const bf16x8_t yy = __builtin_bit_cast(bf16x8_t, y);
                        acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0[s2], yy, acc[rb][0], 0, 0, 0);
                        acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1[s2], yy, acc[rb][1], 0, 0, 0);
                    }
                }
            }
        }
        if constexpr (NT > NB) {
            if (j + NB < NT) {
                __syncthreads();  // every wave is done reading this expert's slot ...
                stash_b(vroll, j % NB);
                // ... and the refill is complete before expert j + NB reads it: the barrier
                // after expert j + 1 (NB >= 2) orders it, or, for the last refill, this one
                if (j + NB + 1 >= NT) __syncthreads();
            }
        }
    }

    // ---- epilogue: each lane updates its pieces of the W tile in LDS, in the result
    // layout (column p of a group is accumulator cb = p&1, v = 4b + p/2); tile back out.
    // no term, or only zero coefficients: the bits pass through untouched (-0.0 stays -0.0)
    if (c_last != 0.0f) w_tile_update<TC>(s_w, acc, c_last, 0, lcol0, n, h);
    __syncthreads();
    w_tile_store<TC, NTHR, WQ>(s_w, tile, opaque_copy(tid));
}

}  // namespace adafuse
