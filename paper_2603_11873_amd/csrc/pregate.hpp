// Token-level pre-gating router (Eq.1's Softmax(TopK(W_g x)), evaluated once per
// token on x^1 and reused by every layer, Eq.2).
//
// One workgroup (4 waves) per token.  Wave w computes the logits of experts
// w, w+4, ...: 128-bit bf16 loads of the hidden row and the router row, exact
// bf16 x bf16 products in fp32, accumulation in fp64 (full rate on this chip and
// free at this size), butterfly reduction across the wave.  The fp32-rounded
// logits go to LDS; thread 0 then takes k rounds of arg-max (strict '>' so the
// lowest index wins a tie) and the softmax.  The whole step is a few KB of
// traffic and is bound by launch latency.
#pragma once
#include "device_types.hpp"

namespace adafuse {

constexpr int kMaxExperts = 64;
constexpr int kMaxTopK = 8;

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

    for (int e = wave; e < p.E; e += 4) {
        const uint16_t *w = p.w_router + (size_t)e * p.d;
        double acc = 0.0;
        for (int i = lane * 8; i < p.d; i += 64 * 8) {
            const uint4_t hv = *reinterpret_cast<const uint4_t *>(h + i);
            const uint4_t wv = *reinterpret_cast<const uint4_t *>(w + i);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc += (double)(bf16_lo(hv[q]) * bf16_lo(wv[q]));  // 8-bit x 8-bit significands: exact in fp32
                acc += (double)(bf16_hi(hv[q]) * bf16_hi(wv[q]));
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) {
            const float l = (float)acc;
            s_logit[e] = l;
            if (p.logits) p.logits[(size_t)t * p.E + e] = l;
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
