// Fused switch, matrix-core form.  Per selected expert the low-rank product
// P_j = B_{e_j} A_{e_j} is formed from the unmodified bf16 operands with
// v_mfma_f32_4x4x4_16b_bf16 (fp32 accumulate), then the element update is
// W' = rn_bf16(W + sum_j (s g_j) P_j): one fp32 FMA per expert, W added last, a
// single rounding to bf16.  Gates never touch a bf16 operand, so no operand is re-rounded.
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
//   src0 lane: A_e[4c..4c+3][col0 + 8b + 4s + li]   (column operand, constant per tile -> registers)
//   src1 lane: B_e[row0 + 4g + li][4c..4c+3]        (row operand, from LDS per row group g)
//   result   : lane holds P[row0+4g+li][col0 + 8b + 4s + 0..3]
// Workgroup = 4 waves on one TR x 128 tile; wave w takes row groups g = w, w+4, ...
// so the workgroup walks 16 consecutive rows at a time.
#pragma once
#include "device_types.hpp"

namespace adafuse {

constexpr int kMfmaTileRows = 256;
constexpr int kMfmaTileCols = 128;

template <int R, int NT>
struct MfmaLds {
    static constexpr int KR = R * NT;
    static constexpr int kStrideA = KR + 4;  // bf16 elements; +8 bytes keeps 8-byte reads of adjacent columns off one bank
    static constexpr int kStrideB = KR + 4;
    uint16_t a[kMfmaTileCols][kStrideA];  // [col][kappa]  transposed A slices
    uint16_t b[kMfmaTileRows][kStrideB];  // [row][kappa]
};

template <int R, int NT, int U>
__global__ __launch_bounds__(256) void switch_mfma_kernel(SwitchParams p)
{
    constexpr int CH = R / 4;  // 4-wide chunks of the rank
    constexpr int TR = kMfmaTileRows, TC = kMfmaTileCols;
    constexpr int NG = TR / 4;  // row groups per tile
    static_assert(R % 4 == 0 && NT >= 1 && NT <= kMaxTerms, "unsupported shape");
    static_assert((NG / 4) % U == 0, "unroll must divide the row groups per wave");

    __shared__ __align__(16) MfmaLds<R, NT> lds;

    Terms terms;
    if (!load_terms<NT>(p, terms)) return;

    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int row0 = (int)(tile.rc & 0xffffu) * TR;
    const int col0 = (int)(tile.rc >> 16) * TC;
    const int tid = threadIdx.x;

    // ---- stage the selected A slices, transposed to [col][kappa]
    for (int q = tid; q < NT * R * (TC / 8); q += 256) {
        const int kappa = q / (TC / 8);
        const int c8 = q % (TC / 8);
        const int j = kappa / R, rho = kappa % R;
        const int col = col0 + c8 * 8;
        uint4_t v = {0u, 0u, 0u, 0u};
        if (col < m.in)
            v = *reinterpret_cast<const uint4_t *>(m.a_bank + ((size_t)terms.e[j] * R + rho) * m.in + col);
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            lds.a[c8 * 8 + 2 * h][kappa] = (uint16_t)(v[h] & 0xffffu);
            lds.a[c8 * 8 + 2 * h + 1][kappa] = (uint16_t)(v[h] >> 16);
        }
    }
    // ---- stage the selected B slices, [row][kappa], 4 bf16 (8 bytes) per item
    for (int q = tid; q < TR * NT * CH; q += 256) {
        const int row = q / (NT * CH);
        const int rem = q % (NT * CH);
        const int j = rem / CH, c = rem % CH;
        uint2_t v = {0u, 0u};
        if (row0 + row < m.out)
            v = *reinterpret_cast<const uint2_t *>(m.b_bank + ((size_t)terms.e[j] * m.out + row0 + row) * R + 4 * c);
        *reinterpret_cast<uint2_t *>(&lds.b[row][j * R + 4 * c]) = v;
    }
    __syncthreads();

    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int blk = lane >> 2;
    const int li = lane & 3;
    const int col = col0 + 8 * blk;
    const bool col_ok = col < m.in;

    // column operands, constant over the tile
    short4_t X[NT][CH][2];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                X[j][c][s] = *reinterpret_cast<const short4_t *>(&lds.a[8 * blk + 4 * s + li][j * R + 4 * c]);

    const uint16_t *__restrict__ wsrc = m.w_base + (size_t)col;
    uint16_t *__restrict__ wdst = m.w_work + (size_t)col;

    for (int g0 = wave; g0 < NG; g0 += 4 * U) {
        uint4_t w[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = row0 + 4 * (g0 + 4 * u) + li;
            ok[u] = col_ok && row < m.out;
            w[u] = uint4_t{0u, 0u, 0u, 0u};
            if (ok[u])
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>(wsrc + (size_t)row * m.ldw));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + 4 * u;
            float4_t P[NT][2];
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                P[j][0] = float4_t{0.f, 0.f, 0.f, 0.f};
                P[j][1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const short4_t y = *reinterpret_cast<const short4_t *>(&lds.b[4 * g + li][j * R + 4 * c]);
                    P[j][0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(X[j][c][0], y, P[j][0], 0, 0, 0);
                    P[j][1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(X[j][c][1], y, P[j][1], 0, 0, 0);
                }
            }
            // the update is summed on its own and W added last: when W + dW cancels,
            // that last add is exact and the error stays relative to dW, not to W
            float acc[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = terms.c[0] * P[0][q >> 2][q & 3];
#pragma unroll
            for (int j = 1; j < NT; ++j)
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] = __builtin_fmaf(terms.c[j], P[j][q >> 2][q & 3], acc[q]);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                acc[2 * h] += bf16_lo(w[u][h]);
                acc[2 * h + 1] += bf16_hi(w[u][h]);
            }
            if (ok[u]) {
                const int row = row0 + 4 * g + li;
                uint4_t o;
#pragma unroll
                for (int h = 0; h < 4; ++h) o[h] = pack_bf16_rne(acc[2 * h], acc[2 * h + 1]);
                __builtin_nontemporal_store(o, reinterpret_cast<uint4_t *>(wdst + (size_t)row * m.ldw));
            }
        }
    }
}

// UNMERGE: W_work <- W_base over the same tile table and access pattern, no
// arithmetic.  Also the practical read+write ceiling the switch is measured against.
template <int U>
__global__ __launch_bounds__(256) void switch_copy_kernel(SwitchParams p)
{
    constexpr int TR = kMfmaTileRows, TC = kMfmaTileCols, NG = TR / 4;
    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int row0 = (int)(tile.rc & 0xffffu) * TR;
    const int col0 = (int)(tile.rc >> 16) * TC;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = lane >> 2, li = lane & 3;
    const int col = col0 + 8 * blk;
    if (col >= m.in) return;
    const uint16_t *__restrict__ wsrc = m.w_base + (size_t)col;
    uint16_t *__restrict__ wdst = m.w_work + (size_t)col;
    for (int g0 = wave; g0 < NG; g0 += 4 * U) {
        uint4_t w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = row0 + 4 * (g0 + 4 * u) + li;
            if (row < m.out)
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>(wsrc + (size_t)row * m.ldw));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = row0 + 4 * (g0 + 4 * u) + li;
            if (row < m.out)
                __builtin_nontemporal_store(w[u], reinterpret_cast<uint4_t *>(wdst + (size_t)row * m.ldw));
        }
    }
}

}  // namespace adafuse
