// Fused switch, vector-ALU form: the rank-(k r) update of Eq.6 accumulated in
// fp32 on the VALU.  Generic in r and k (runtime loops); kept as the baseline
// the matrix-core kernel is measured against.
//
// Workgroup = 256 threads = one 64 x 256 tile of one matrix.  The k selected
// A slices (bf16, [k r][256]) and the k selected B slices with the coefficient
// s*g_j folded in (fp32, [64][k r]) are staged in LDS.  A thread owns 8
// contiguous columns (one 128-bit load/store) of 8 rows; per inner index it
// reads its 8 A values once and one broadcast B value per row.
#pragma once
#include "device_types.hpp"

namespace adafuse {

constexpr int kValuTileRows = 64;
constexpr int kValuTileCols = 256;

__host__ __device__ constexpr size_t valu_lds_bytes(int kr)
{
    return (size_t)kr * kValuTileCols * 2 + (size_t)kValuTileRows * kr * 4;
}

__global__ __launch_bounds__(256) void switch_valu_kernel(SwitchParams p)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ int32_t s_e[kMaxTerms];
    __shared__ float s_c[kMaxTerms];
    {
        // k is a run-time value here, so the term list lives in LDS (indexed at run time)
        Terms terms;
        if (!load_terms<kMaxTerms>(p, terms)) return;
        if (threadIdx.x == 0) {
#pragma unroll
            for (int j = 0; j < kMaxTerms; ++j) {
                s_e[j] = terms.e[j];
                s_c[j] = terms.c[j];
            }
        }
        __syncthreads();
    }

    const TileDev tile = p.tiles[blockIdx.x];
    const MatDev m = p.mats[tile.mat];
    const int row0 = tile.row0;
    const int col0 = tile.col0;
    const int nt = p.inplace ? (p.mode == 2 ? 2 * p.k : p.k) : (p.mode == 1 ? 0 : p.k);
    const int r = p.r;
    const int kr = nt * r;
    const int tid = threadIdx.x;

    uint16_t *sA = reinterpret_cast<uint16_t *>(lds_raw);                              // [kr][256] bf16
    float *sB = reinterpret_cast<float *>(lds_raw + (size_t)kr * kValuTileCols * 2);   // [64][kr] fp32, c folded

    // stage A slices: 128-bit chunks, zero beyond the matrix edge
    for (int q = tid; q < kr * (kValuTileCols / 8); q += 256) {
        const int kappa = q / (kValuTileCols / 8);
        const int c8 = q % (kValuTileCols / 8);
        const int j = kappa / r, rho = kappa % r;
        const int col = col0 + c8 * 8;
        uint4_t v = {0u, 0u, 0u, 0u};
        if (col < m.in)
            v = ld_global(reinterpret_cast<const uint4_t *>(m.a_bank + ((size_t)s_e[j] * r + rho) * m.in + col));
        *reinterpret_cast<uint4_t *>(sA + (size_t)kappa * kValuTileCols + c8 * 8) = v;
    }
    // stage B slices with the coefficient folded in
    for (int q = tid; q < kValuTileRows * kr; q += 256) {
        const int row = q / kr;
        const int kappa = q % kr;
        const int j = kappa / r, rho = kappa % r;
        float v = 0.0f;
        if (row0 + row < m.out)
            v = s_c[j] * bf16_bits_to_f32(ld_global(m.b_bank + ((size_t)s_e[j] * m.out + row0 + row) * r + rho));
        sB[row * kr + kappa] = v;
    }
    __syncthreads();

    const int c8 = tid % 32;
    const int rsub = tid / 32;  // rows rsub, rsub+8, ...
    const int col = col0 + c8 * 8;
    if (col >= m.in) return;

    // the update is summed from zero and W added last: when W + dW cancels, that
    // last add is exact and the error stays relative to dW, not to W
    float acc[8][8];
    uint4_t w[8];
    bool valid[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = row0 + rsub + 8 * i;
        valid[i] = row < m.out;
        w[i] = uint4_t{0u, 0u, 0u, 0u};
        if (valid[i])
            w[i] = ld_global_nt(reinterpret_cast<const uint4_t *>(m.w_base + (size_t)row * m.ldw + col));
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[i][q] = 0.0f;
    }

    for (int kappa = 0; kappa < kr; ++kappa) {
        const uint4_t av = *reinterpret_cast<const uint4_t *>(sA + (size_t)kappa * kValuTileCols + c8 * 8);
        float a[8];
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            a[2 * h] = bf16_lo(av[h]);
            a[2 * h + 1] = bf16_hi(av[h]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float b = sB[(rsub + 8 * i) * kr + kappa];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[i][q] = __builtin_fmaf(b, a[q], acc[i][q]);
        }
    }

#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (!valid[i]) continue;
        const int row = row0 + rsub + 8 * i;
        uint4_t o = w[i];  // nothing selected (un-merge): the bits pass through untouched
        if (kr > 0) {
#pragma unroll
            for (int h = 0; h < 4; ++h)
                o[h] = pack_bf16_rne(bf16_lo(w[i][h]) + acc[i][2 * h], bf16_hi(w[i][h]) + acc[i][2 * h + 1]);
        }
        st_global_nt(o, reinterpret_cast<uint4_t *>(m.w_work + (size_t)row * m.ldw + col));
    }
}

}  // namespace adafuse
