// Fused switch, matrix-core form.  Per selected expert the low-rank product
// P_j = B_{e_j} A_{e_j} is formed from the unmodified bf16 operands with
// v_mfma_f32_4x4x4_16b_bf16 (fp32 accumulate), then the element update is
// W' = rn_bf16(W + sum_j (s g_j) P_j): one fp32 FMA per expert, W added last, a
// single rounding to bf16.  Gates never touch a bf16 operand, so no operand is
// re-rounded.
//
// Why the 4x4x4, 16-block shape: its result layout gives every lane 4
// consecutive columns of one row, and the 16 blocks sit side by side along the
// row.  Two such results give a lane 8 consecutive bf16 (one 128-bit access), and
// a wave's access covers 4 rows x 256 contiguous bytes -- the layout a streaming
// copy would use.  The wider MFMA shapes put a whole column in a lane and would
// cut every row into 32- or 64-byte pieces.  At inner dimension r <= 16 the
// matrix cores are a small fraction of the time either way.
//
// Mapping (block b = lane/4, li = lane%4, set s = 0/1):
//   src0 lane: A_e[4c..4c+3][col + 8b + 2 li + s]   (column operand, constant per tile -> registers)
//   src1 lane: B_e[row0 + 4g + li][4c..4c+3]        (row operand, from LDS per row group g)
//   result   : lane holds P_s[row0+4g+li][col + 8b + 2i + s], i = 0..3
// Set s takes the even (s=0) or odd (s=1) columns of the lane's 8, so the two
// column operands of one rank index are the two halves of ONE aligned 32-bit
// word of the A bank: a wave fetches them with a fully coalesced dword load
// (256 contiguous bytes) and a byte permute packs four rank indices per operand.
// No transposition through LDS, and no dependence between waves for A.
// A workgroup is 4 waves on one TR x (128 WC) tile: WC waves side by side, each
// on its own 128-column strip, 4/WC stacked; a wave walks its strip 4 rows at a
// time; the wave's whole share of W (TR/4/(4/WC) row groups) is loaded up front.
#pragma once
#include "device_types.hpp"

namespace adafuse {

template <int TR_, int WC_, int D_ = 0>
struct TileShape {
    static constexpr int TR = TR_;        // tile rows
    static constexpr int WC = WC_;        // waves side by side
    static constexpr int WR = 4 / WC_;    // waves stacked
    static constexpr int TC = 128 * WC_;  // tile columns
    static constexpr int NG = TR_ / 4;    // row groups per tile
    static constexpr int NGW = NG / WR;   // row groups per wave
    static constexpr int DW = D_ ? D_ : NGW;  // W loads a wave keeps in flight (default: its whole share)
    static_assert(WC_ == 1 || WC_ == 2 || WC_ == 4, "4 waves per workgroup");
    static_assert(TR_ % (4 * WR) == 0, "rows must split evenly over the stacked waves");
    static_assert(NGW % DW == 0, "window must divide the wave's row groups");
};

template <int R, int NT, class S>
struct MfmaLds {
    static constexpr int KR = R * NT;
    static constexpr int kStride = KR + 4;  // bf16 elements; the 8-byte pad spreads rows over LDS banks
    uint16_t b[S::TR][kStride];             // [row][kappa]  selected B slices
};

template <int R, int NT, class S>
constexpr bool mfma_shape_fits()
{
    return sizeof(MfmaLds<R, NT, S>) <= 64 * 1024;
}

template <int R, int NT, class S>
__global__ __launch_bounds__(256) void switch_mfma_kernel(SwitchParams p)
{
    constexpr int CH = R / 4;  // 4-wide chunks of the rank
    constexpr int TR = S::TR, WR = S::WR, WC = S::WC, NGW = S::NGW, DW = S::DW;
    static_assert(R % 4 == 0 && NT >= 1 && NT <= kMaxTerms, "unsupported shape");

    __shared__ __align__(16) MfmaLds<R, NT, S> lds;

    Terms terms;
    if (!load_terms<NT>(p, terms)) return;

    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int row0 = tile.row0;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wc = wave % WC, wr = wave / WC;
    const int blk = lane >> 2;
    const int li = lane & 3;
    const int lcol = 128 * wc + 8 * blk;           // column inside the tile
    const int col = tile.col0 + lcol;
    const bool col_ok = lcol < tile.cols_left;
    const int ldw = tile.ldw;
    const int rows_left = tile.rows_left;
    // no restrict: in the in-place form both point at the same matrix (a lane reads
    // its elements before it writes them, and no other lane touches them)
    const uint16_t *wsrc = tile.w_src + lcol;
    uint16_t *wdst = tile.w_dst + lcol;

    // ---- issue order.  Loads return in issue order.  With a small inner dimension
    // the wave's whole share of W goes in flight first and the operand fetch runs
    // under that latency.  With a large one (many operand loads, long update per row
    // group) the operands go first, so the update of row group u can start as soon
    // as w[u] arrives while the rest of W is still in flight.
    constexpr bool kWFirst = (NT * R <= 16);
    uint4_t w[DW];
    auto load_w = [&](int u) -> uint4_t {
        const int lrow = 4 * (wr + WR * u) + li;   // row inside the tile
        uint4_t v = {0u, 0u, 0u, 0u};
        if (col_ok && lrow < rows_left)
            v = ld_global_nt(reinterpret_cast<const uint4_t *>(wsrc + (size_t)lrow * ldw));
        return v;
    };
    auto issue_w_loads = [&]() {
#pragma unroll
        for (int i = 0; i < DW; ++i) w[i] = load_w(i);
    };
    if constexpr (kWFirst) issue_w_loads();

    constexpr int BQ = (TR * CH + 255) / 256;  // B items (4 bf16) per thread and expert
    uint2_t vb[NT][BQ];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const uint16_t *bsrc = m.b_bank + ((size_t)terms.e[j] * m.out + row0) * R;
#pragma unroll
        for (int i = 0; i < BQ; ++i) {
            const int q = tid + 256 * i;
            const int row = q / CH, c = q % CH;
            vb[j][i] = uint2_t{0u, 0u};
            if (q < TR * CH && row0 + row < m.out)
                vb[j][i] = ld_global(reinterpret_cast<const uint2_t *>(bsrc + (size_t)row * R + 4 * c));
        }
    }

    // column operands, constant over the tile: one dword = columns (c, c+1) of one rank index
    uint32_t d[NT][R];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const uint16_t *arow = m.a_bank + (size_t)terms.e[j] * R * m.in + col + 2 * li;
#pragma unroll
        for (int i = 0; i < R; ++i)
            d[j][i] = col_ok ? ld_global(reinterpret_cast<const uint32_t *>(arow + (size_t)i * m.in)) : 0u;
    }

    if constexpr (!kWFirst) issue_w_loads();

    // B slices to LDS as [row][kappa]
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < BQ; ++i) {
            const int q = tid + 256 * i;
            const int row = q / CH, c = q % CH;
            if (q < TR * CH) *reinterpret_cast<uint2_t *>(&lds.b[row][j * R + 4 * c]) = vb[j][i];
        }

    // pack the column operands: even column = low halves of four words, odd column = high halves
    short4_t X[NT][CH][2];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint32_t *dd = &d[j][4 * c];
            uint2_t ev = {__builtin_amdgcn_perm(dd[1], dd[0], 0x05040100u), __builtin_amdgcn_perm(dd[3], dd[2], 0x05040100u)};
            uint2_t od = {__builtin_amdgcn_perm(dd[1], dd[0], 0x07060302u), __builtin_amdgcn_perm(dd[3], dd[2], 0x07060302u)};
            X[j][c][0] = __builtin_bit_cast(short4_t, ev);
            X[j][c][1] = __builtin_bit_cast(short4_t, od);
        }
    __syncthreads();

    // Row groups in windows of DW: slot i is consumed, refilled with the load of
    // row group u + DW, and only then stored, so a refill never queues behind the
    // store of its own step and DW loads stay in flight.
    // Row operands of row group g: NT*CH 8-byte LDS reads, issued together and one
    // step ahead when they are few, so their latency is not paid per expert.
    constexpr bool kPrefetchY = (NT * R <= 32);
    short4_t ycur[NT][CH], ynxt[NT][CH];
    auto read_y = [&](short4_t (&y)[NT][CH], int u) {
        const int g = wr + WR * u;
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int c = 0; c < CH; ++c)
                y[j][c] = *reinterpret_cast<const short4_t *>(&lds.b[4 * g + li][j * R + 4 * c]);
    };
    if constexpr (kPrefetchY) read_y(ycur, 0);

    for (int ub = 0; ub < NGW; ub += DW) {
#pragma unroll
        for (int i = 0; i < DW; ++i) {
            const int u = ub + i;
            const int g = wr + WR * u;
            if constexpr (kPrefetchY) {
                if (u + 1 < NGW) read_y(ynxt, u + 1);
            } else {
                read_y(ycur, u);
            }
            __builtin_amdgcn_sched_barrier(0);
            float4_t P[NT][2];
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                P[j][0] = float4_t{0.f, 0.f, 0.f, 0.f};
                P[j][1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    P[j][0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(X[j][c][0], ycur[j][c], P[j][0], 0, 0, 0);
                    P[j][1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(X[j][c][1], ycur[j][c], P[j][1], 0, 0, 0);
                }
            }
            if constexpr (kPrefetchY) {
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int c = 0; c < CH; ++c) ycur[j][c] = ynxt[j][c];
            }
            // the update is summed on its own and W added last: when W + dW cancels,
            // that last add is exact and the error stays relative to dW, not to W
            float acc[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = terms.c[0] * P[0][q & 1][q >> 1];
#pragma unroll
            for (int j = 1; j < NT; ++j)
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] = __builtin_fmaf(terms.c[j], P[j][q & 1][q >> 1], acc[q]);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                acc[2 * h] += bf16_lo(w[i][h]);
                acc[2 * h + 1] += bf16_hi(w[i][h]);
            }
            uint4_t o;
#pragma unroll
            for (int h = 0; h < 4; ++h) o[h] = pack_bf16_rne(acc[2 * h], acc[2 * h + 1]);
            if (NGW > DW && u + DW < NGW) w[i] = load_w(u + DW);
            const int lrow = 4 * g + li;
            if (col_ok && lrow < rows_left)
                st_global_nt(o, reinterpret_cast<uint4_t *>(wdst + (size_t)lrow * ldw));
        }
    }
}

// UNMERGE: W_work <- W_base over the same tile table, access pattern and load
// window, no arithmetic.  Also the practical read+write ceiling the switch is
// measured against.
template <class S>
__global__ __launch_bounds__(256) void switch_copy_kernel(SwitchParams p)
{
    constexpr int WR = S::WR, WC = S::WC, NGW = S::NGW;
    constexpr int DW = S::DW > 4 ? 4 : S::DW;  // 4 loads in flight per lane is enough without arithmetic
    static_assert(NGW % DW == 0, "window must divide the wave's row groups");
    const TileDev tile = p.tiles[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wc = wave % WC, wr = wave / WC;
    const int blk = lane >> 2, li = lane & 3;
    const int lcol = 128 * wc + 8 * blk;
    if (lcol >= tile.cols_left) return;
    const uint16_t *__restrict__ wsrc = tile.w_src + lcol;
    uint16_t *__restrict__ wdst = tile.w_dst + lcol;
    const int ldw = tile.ldw, rows_left = tile.rows_left;
    for (int u0 = 0; u0 < NGW; u0 += DW) {
        uint4_t w[DW];
#pragma unroll
        for (int i = 0; i < DW; ++i) {
            const int lrow = 4 * (wr + WR * (u0 + i)) + li;
            if (lrow < rows_left) w[i] = ld_global_nt(reinterpret_cast<const uint4_t *>(wsrc + (size_t)lrow * ldw));
        }
#pragma unroll
        for (int i = 0; i < DW; ++i) {
            const int lrow = 4 * (wr + WR * (u0 + i)) + li;
            if (lrow < rows_left) st_global_nt(w[i], reinterpret_cast<uint4_t *>(wdst + (size_t)lrow * ldw));
        }
    }
}

}  // namespace adafuse
