// Token-level pre-gating router (Eq.1's Softmax(TopK(W_g x)), evaluated once per
// token on x^1 and reused by every layer, Eq.2).
//
// One workgroup (4 waves) per token.  Wave w computes the logits of experts
// w, w+4, ..., two at a time: 128-bit bf16 loads of the hidden row and the router
// rows, exact bf16 x bf16 products in fp32, accumulation in fp64 (full rate on this
// chip and free at this size), butterfly reduction across the wave.  The fp32-rounded
// logits go to LDS; thread 0 then takes k rounds of arg-max (strict '>' so the
// lowest index wins a tie) and the softmax.  The whole step is a few KB of
// traffic and is bound by launch latency.
#pragma once
#include "device_types.hpp"

namespace adafuse {

struct PregateParams {
    const uint16_t *hidden;    // [T][d]
    const uint16_t *w_router;  // [E][d]
    int32_t *idx;              // [T][k]
    float *gates;              // [T][k]
    float *logits;             // [T][E] or null
    int32_t T, d, E, k, gate_norm;
};

__global__ __launch_bounds__(256) void pregate_kernel(PregateParams p)
{
    __shared__ float s_logit[kMaxExperts];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const uint16_t *h = p.hidden + (size_t)t * p.d;

    // Two experts of the wave at a time and four 16-byte pieces of each row per lane:
    // twelve loads in flight instead of two, so a 4096-wide router row costs two memory
    // round trips, not eight per expert.  Pieces beyond the row are loaded from its last
    // piece (a valid address; no load sits in a branch) and left out of the sum.
    constexpr int U = 4;
    for (int e0 = wave; e0 < p.E; e0 += 8) {
        const int e1 = e0 + 4;
        const bool two = e1 < p.E;
        const uint16_t *w0 = p.w_router + (size_t)e0 * p.d;
        const uint16_t *w1 = p.w_router + (size_t)(two ? e1 : e0) * p.d;
        double acc0 = 0.0, acc1 = 0.0;
        for (int i0 = lane * 8; i0 < p.d; i0 += 64 * 8 * U) {
            uint4_t hv[U], v0[U], v1[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + 64 * 8 * u;
                const int ic = i < p.d ? i : p.d - 8;
                hv[u] = *reinterpret_cast<const uint4_t *>(h + ic);
                v0[u] = *reinterpret_cast<const uint4_t *>(w0 + ic);
                v1[u] = *reinterpret_cast<const uint4_t *>(w1 + ic);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i0 + 64 * 8 * u < p.d) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // 8-bit x 8-bit significands: the products are exact in fp32
                        acc0 += (double)(bf16_lo(hv[u][q]) * bf16_lo(v0[u][q]));
                        acc0 += (double)(bf16_hi(hv[u][q]) * bf16_hi(v0[u][q]));
                        acc1 += (double)(bf16_lo(hv[u][q]) * bf16_lo(v1[u][q]));
                        acc1 += (double)(bf16_hi(hv[u][q]) * bf16_hi(v1[u][q]));
                    }
                }
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            acc0 += __shfl_xor(acc0, off, 64);
            acc1 += __shfl_xor(acc1, off, 64);
        }
        if (lane == 0) {
            const float l0 = (float)acc0, l1 = (float)acc1;
            s_logit[e0] = l0;
            if (p.logits) p.logits[(size_t)t * p.E + e0] = l0;
            if (two) {
                s_logit[e1] = l1;
                if (p.logits) p.logits[(size_t)t * p.E + e1] = l1;
            }
        }
    }
    __syncthreads();

    if (threadIdx.x == 0) {
        int sel[kMaxTopK];
        uint64_t taken = 0;
        for (int j = 0; j < p.k; ++j) {
            int best = -1;
            float bv = 0.0f;
            for (int e = 0; e < p.E; ++e) {
                if ((taken >> e) & 1ull) continue;
                const float v = s_logit[e];
                if (best < 0 || v > bv) { best = e; bv = v; }
            }
            taken |= 1ull << best;
            sel[j] = best;
        }
        const double mx = (double)s_logit[sel[0]];
        double denom = 0.0;
        if (p.gate_norm == 0) {
            for (int j = 0; j < p.k; ++j) denom += exp((double)s_logit[sel[j]] - mx);
        } else {
            for (int e = 0; e < p.E; ++e) denom += exp((double)s_logit[e] - mx);
        }
        for (int j = 0; j < p.k; ++j) {
            p.idx[(size_t)t * p.k + j] = sel[j];
            p.gates[(size_t)t * p.k + j] = (float)(exp((double)s_logit[sel[j]] - mx) / denom);
        }
    }
}

}  // namespace adafuse
