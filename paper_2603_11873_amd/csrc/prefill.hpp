// Prefill: many tokens through ONE adapted matrix, every token with its own routing
// decision (section "Decoding Phase", prefill paragraph: one merged weight cannot serve
// tokens that selected different experts, so the adapters stay un-merged here, Eq.2):
//   Y[t] = W_base x_t + s * sum_j g_{t,j} * B_{e_{t,j}} (A_{e_{t,j}} x_t),   t < T.
// Two kernels, both on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation):
//
//   prefill_down_kernel   one workgroup per (block of 32 tokens, expert).  A workgroup whose
//       expert none of its tokens selected returns at once; the others form
//       Z[rho][t] = sum_i A_e[rho][i] x_t[i] for the whole block (a dense 32-token product:
//       tokens are grouped by position, the expert decides which blocks run), scale the
//       columns of the tokens that selected e by s * g and store them as a pair of bf16
//       planes hi + lo (16 significant bits) in the slot of that (token, selection).
//   prefill_up_kernel     one workgroup per (tile of 32 MB tokens, strip of 32 output rows):
//       the base product over the whole input width, then, for every expert some token of
//       the tile selected, k-steps over the rank with the token's scaled Z (zero for tokens
//       that did not select it) against B_e's rows -- the adapter is just more inner
//       dimension of the same product, so Y is written once, no atomics, same bits every run.
//
// Both split the inner dimension over the four waves of a workgroup (each wave streams its
// share of the rows' k-range straight from global memory into matrix-core operands: a lane
// holds 8 consecutive inner indices of one row, one 16-byte load) and add the four partial
// results in a fixed order through LDS.  W is read once per token tile; X and the banks come
// out of L2.  Operand loads use buffer descriptors with the "beyond the edge" lanes pointed
// outside the descriptor, so ragged T, out, in and padded ranks read as zero, never as
// whatever sits behind the row.
#pragma once
#include "device_types.hpp"

namespace adafuse {

typedef __attribute__((ext_vector_type(8))) __bf16 pf_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float pf_float16_t;

struct PrefillParams {
    const uint16_t *w;       // [out][ldw] base weights
    const uint16_t *a_bank;  // [E][r][in]
    const uint16_t *b_bank;  // [E][out][r]
    const uint16_t *x;       // [T][in]
    const int32_t *idx;      // [T][k]
    const float *gates;      // [T][k]
    float *y;                // [T][out]
    uint16_t *z_hi;          // [T][k][rp]  scaled down-projections, upper bf16 plane
    uint16_t *z_lo;          // [T][k][rp]  ... and the bf16 rounding of what the upper plane left over
    int32_t out, in, ldw, T, E, r, rp, k;
    float scale;
};

constexpr uint32_t kOutside = 0xffffff00u;  // a per-lane offset no descriptor of this library covers: reads as zero

__device__ __forceinline__ pf_bf16x8_t as_operand(uint4_t v) { return __builtin_bit_cast(pf_bf16x8_t, v); }

__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

// Experts selected by any of the tokens [t0, t0 + n_tok) as a bit mask (E <= 64); every wave
// computes it for itself, lane l looking at tokens t0 + l, t0 + l + 64, ...
__device__ __forceinline__ uint64_t experts_in_tile(const PrefillParams &p, int t0, int n_tok, int lane)
{
    uint64_t mine = 0;
    for (int t = t0 + lane; t < t0 + n_tok && t < p.T; t += 64)
        for (int j = 0; j < p.k; ++j) mine |= 1ull << clamp_expert(p.idx[(size_t)t * p.k + j], p.E);
    uint64_t all = 0;
    for (int e = 0; e < p.E; ++e)
        if (__ballot((mine >> e) & 1ull)) all |= 1ull << e;
    return all;
}

// Partial results of waves 1..3 added to wave 0's in that order, through LDS.  NV = accumulator
// vectors (16 floats each) per lane.  Returns with the sum in wave 0's registers.
template <int NV>
__device__ __forceinline__ void reduce_over_waves(pf_float16_t (&acc)[NV], float *s_part, int wave, int lane)
{
    if (wave > 0) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int q = 0; q < 16; ++q) s_part[(((wave - 1) * NV + v) * 16 + q) * 64 + lane] = acc[v][q];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[v][q] += s_part[((w * NV + v) * 16 + q) * 64 + lane];
    }
}

// ---- down projection -------------------------------------------------------------------------
// RB = blocks of 32 rank indices (1 for ranks up to 32, 2 for 64, 4 for 128).
template <int RB>
__global__ __launch_bounds__(256) void prefill_down_kernel(PrefillParams p)
{
    __shared__ float s_part[3 * RB * 16 * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int t0 = 32 * blockIdx.x;
    const int e = blockIdx.y;
    const uint64_t present = experts_in_tile(p, t0, 32, lane);
    if (!((present >> e) & 1ull)) return;  // uniform over the workgroup

    const int t = t0 + n;
    const uint32_t in_bytes = 2u * (uint32_t)p.in;
    const __amdgpu_buffer_rsrc_t xr = make_buffer(p.x, (uint32_t)p.T * in_bytes);  // host side keeps T * in * 2 below 2^31
    const __amdgpu_buffer_rsrc_t ar = make_buffer(p.a_bank + (size_t)e * p.r * p.in, (uint32_t)p.r * in_bytes);
    const uint32_t xrow = t < p.T ? (uint32_t)t * in_bytes : kOutside;

    pf_float16_t acc[RB];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[b][q] = 0.0f;

    // this wave's share of the k-steps (16 inner indices each; the last may be half a step)
    const int steps = (p.in + 15) / 16, per = (steps + 3) / 4;
    const int s_begin = wave * per, s_end = min(steps, s_begin + per);
    for (int s = s_begin; s < s_end; ++s) {
        const uint32_t kb = 2u * (uint32_t)(16 * s + 8 * h);
        const bool k_ok = 16 * s + 8 * h < p.in;
        const uint4_t xv = ld_buffer_b128(xr, k_ok && xrow != kOutside ? xrow + kb : kOutside, 0u);
#pragma unroll
        for (int b = 0; b < RB; ++b) {
            const int rho = 32 * b + n;
            const uint4_t av = ld_buffer_b128(ar, k_ok && rho < p.r ? (uint32_t)rho * in_bytes + kb : kOutside, 0u);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(av), as_operand(xv), acc[b], 0, 0, 0);
        }
    }
    reduce_over_waves<RB>(acc, s_part, wave, lane);
    if (wave != 0 || t >= p.T) return;

    // the lane's token: coefficient of this expert (all selections of it added) and the slot that takes the result
    int first = -1;
    float c = 0.0f;
    for (int j = 0; j < p.k; ++j)
        if (clamp_expert(p.idx[(size_t)t * p.k + j], p.E) == e) {
            if (first < 0) first = j;
            c += p.scale * p.gates[(size_t)t * p.k + j];
        }
    if (first < 0) return;
    for (int j = 0; j < p.k; ++j) {
        if (clamp_expert(p.idx[(size_t)t * p.k + j], p.E) != e) continue;
        const size_t slot = ((size_t)t * p.k + j) * p.rp;
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rho = 32 * b + 8 * q + 4 * h;  // accumulator entries 4 q .. 4 q + 3 are rank indices rho .. rho + 3
                if (rho >= p.rp) continue;
                uint32_t hi[2] = {0u, 0u}, lo[2] = {0u, 0u};
                if (j == first) {  // a repeated selection of the same expert is folded into the first one
                    float zf[4], zr[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) zf[u] = c * acc[b][4 * q + u];
                    hi[0] = pack_bf16_rne(zf[0], zf[1]);
                    hi[1] = pack_bf16_rne(zf[2], zf[3]);
                    zr[0] = zf[0] - bf16_lo(hi[0]);
                    zr[1] = zf[1] - bf16_hi(hi[0]);
                    zr[2] = zf[2] - bf16_lo(hi[1]);
                    zr[3] = zf[3] - bf16_hi(hi[1]);
                    lo[0] = pack_bf16_rne(zr[0], zr[1]);
                    lo[1] = pack_bf16_rne(zr[2], zr[3]);
                }
                *reinterpret_cast<uint2_t *>(p.z_hi + slot + rho) = uint2_t{hi[0], hi[1]};
                *reinterpret_cast<uint2_t *>(p.z_lo + slot + rho) = uint2_t{lo[0], lo[1]};
            }
    }
}

// ---- base product + up projection --------------------------------------------------------------
// MB = blocks of 32 tokens per workgroup.  blockIdx.x enumerates (strip of 32 output rows, token
// tile) so that the token tiles of one strip run on the same XCD (workgroup i runs on XCD i % 8):
// the second and later token tiles find the strip's W rows in that XCD's L2.
template <int MB>
__global__ __launch_bounds__(256) void prefill_up_kernel(PrefillParams p, int m_tiles, int strips)
{
    __shared__ float s_part[3 * MB * 16 * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int xcd = blockIdx.x % 8, q_in_xcd = blockIdx.x / 8;
    const int strip = (q_in_xcd / m_tiles) * 8 + xcd, m_tile = q_in_xcd % m_tiles;
    if (strip >= strips) return;
    const int o0 = 32 * strip, t0 = 32 * MB * m_tile;

    const uint32_t in_bytes = 2u * (uint32_t)p.in;
    const int o = o0 + n;
    const int rows = min(32, p.out - o0);
    const __amdgpu_buffer_rsrc_t wr = make_buffer(p.w + (size_t)o0 * p.ldw, (uint32_t)rows * 2u * (uint32_t)p.ldw);
    const __amdgpu_buffer_rsrc_t xr = make_buffer(p.x, (uint32_t)p.T * in_bytes);
    const uint32_t wrow = o < p.out ? (uint32_t)n * 2u * (uint32_t)p.ldw : kOutside;
    uint32_t xrow[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) xrow[b] = t0 + 32 * b + n < p.T ? (uint32_t)(t0 + 32 * b + n) * in_bytes : kOutside;

    pf_float16_t acc[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[b][q] = 0.0f;

    // ---- the base product: this wave's share of the k-steps, two at a time, the next pair requested
    // before the current one is multiplied
    const int steps = (p.in + 15) / 16, per = (steps + 3) / 4;
    const int s_begin = wave * per, s_end = min(steps, s_begin + per);
    constexpr int U = 2;
    uint4_t wv[2][U], xv[2][U][MB];
    auto request = [&](int buf, int s) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k0 = 16 * (s + u) + 8 * h;
            const bool k_ok = s + u < s_end && k0 < p.in;
            const uint32_t kb = 2u * (uint32_t)k0;
            wv[buf][u] = ld_buffer_b128(wr, k_ok && wrow != kOutside ? wrow + kb : kOutside, 0u);
#pragma unroll
            for (int b = 0; b < MB; ++b)
                xv[buf][u][b] = ld_buffer_b128(xr, k_ok && xrow[b] != kOutside ? xrow[b] + kb : kOutside, 0u);
        }
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int b = 0; b < MB; ++b)
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(wv[buf][u]), as_operand(xv[buf][u][b]), acc[b], 0, 0, 0);
    };
    // (a request beyond the wave's share puts every lane outside its descriptor: zeros, no memory access)
    int s = s_begin;
    if (s < s_end) request(0, s);
    while (s < s_end) {
        request(1, s + U);
        multiply(0);
        s += U;
        if (s >= s_end) break;
        request(0, s + U);
        multiply(1);
        s += U;
    }

    // ---- the adapters: for every expert some token of the tile selected, k-steps over the rank.
    // The experts are dealt to the four waves; a token that did not select the expert contributes a zero operand.
    const uint64_t present = experts_in_tile(p, t0, 32 * MB, lane);
    const uint32_t z_bytes = (uint32_t)p.T * (uint32_t)p.k * (uint32_t)p.rp * 2u;
    const __amdgpu_buffer_rsrc_t zh = make_buffer(p.z_hi, z_bytes), zl = make_buffer(p.z_lo, z_bytes);
    int turn = 0;
    for (int e = 0; e < p.E; ++e) {
        if (!((present >> e) & 1ull)) continue;
        if ((turn++ & 3) != wave) continue;
        // B_e's rows of this strip: 2 r bytes per row
        const __amdgpu_buffer_rsrc_t br = make_buffer(p.b_bank + ((size_t)e * p.out + o0) * p.r, (uint32_t)rows * 2u * (uint32_t)p.r);
        uint32_t zrow[MB];
#pragma unroll
        for (int b = 0; b < MB; ++b) {
            const int t = t0 + 32 * b + n;
            zrow[b] = kOutside;
            if (t < p.T)
                for (int j = p.k - 1; j >= 0; --j)  // the FIRST selection of e holds the (folded) result
                    if (clamp_expert(p.idx[(size_t)t * p.k + j], p.E) == e) zrow[b] = (uint32_t)(t * p.k + j) * (uint32_t)p.rp * 2u;
        }
        for (int s = 0; 16 * s < p.rp; ++s) {
            const int rho = 16 * s + 8 * h;
            uint4_t bv;
            if (p.r >= 8) {
                bv = ld_buffer_b128(br, rho < p.r && o < p.out ? (uint32_t)n * 2u * (uint32_t)p.r + 2u * (uint32_t)rho : kOutside, 0u);
            } else {  // rank 4: a row is 8 bytes, the upper half of the operand stays zero
                const uint2_t b2 = ld_buffer_b64(br, rho < p.r && o < p.out ? (uint32_t)n * 8u : kOutside, 0u);
                bv = uint4_t{b2[0], b2[1], 0u, 0u};
            }
#pragma unroll
            for (int b = 0; b < MB; ++b) {
                const uint32_t off = rho < p.rp && zrow[b] != kOutside ? zrow[b] + 2u * (uint32_t)rho : kOutside;
                const uint4_t hv = ld_buffer_b128(zh, off, 0u), lv = ld_buffer_b128(zl, off, 0u);
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(bv), as_operand(lv), acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(bv), as_operand(hv), acc[b], 0, 0, 0);
            }
        }
    }

    reduce_over_waves<MB>(acc, s_part, wave, lane);
    if (wave != 0) return;
    // accumulator entries 4 q .. 4 q + 3 of block b: token t0 + 32 b + n, output rows o0 + 8 q + 4 h + 0..3
#pragma unroll
    for (int b = 0; b < MB; ++b) {
        const int t = t0 + 32 * b + n;
        if (t >= p.T) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int oo = o0 + 8 * q + 4 * h;
            float *dst = p.y + (size_t)t * p.out + oo;
            if (oo + 3 < p.out && (p.out & 3) == 0) {
                *reinterpret_cast<float4_t *>(dst) = float4_t{acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]};
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (oo + u < p.out) dst[u] = acc[b][4 * q + u];
            }
        }
    }
}

}  // namespace adafuse
