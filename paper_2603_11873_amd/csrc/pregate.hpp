// Token-level pre-gating router (Eq.1's Softmax(TopK(W_g x)), evaluated once per
// token on x^1 and reused by every layer, Eq.2).
//
// One workgroup (4 waves) per token.  Wave w computes the logits of experts
// w, w+4, ..., two at a time: 128-bit bf16 loads of the hidden row and the router
// rows, exact bf16 x bf16 products in fp32, accumulation in fp64 (full rate on this
// chip and free at this size), butterfly reduction across the wave.  The fp32-rounded
// logits go to LDS; wave 0 then holds one expert per lane and takes k rounds of a
// wave-wide arg-max (the lowest index wins a tie) and the softmax.  The whole step
// is a few KB of traffic and is bound by launch latency.
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

    // Selection and softmax on wave 0, one expert per lane (E <= 64).  Round j: the wave's largest
    // remaining logit by a butterfly of (value, index) pairs, the lower index winning a tie; lane j
    // keeps round j's result.  The sums of the softmax are taken in index order (the order a
    // sequential loop would use), so the gates do not depend on how the lanes are combined.
    if (wave != 0) return;
    const bool valid = lane < p.E;
    const float mine = valid ? s_logit[lane] : 0.0f;
    bool taken = !valid;
    int sel = 0;
    float val = 0.0f;
    for (int j = 0; j < p.k; ++j) {
        float bv = mine;
        int be = taken ? 0x7fffffff : lane;   // a lane that is out of the running loses against any that is in
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oe = __shfl_xor(be, off, 64);
            const bool other_in = oe != 0x7fffffff, self_in = be != 0x7fffffff;
            const bool take = other_in && (!self_in || ov > bv || (ov == bv && oe < be));
            bv = take ? ov : bv;
            be = take ? oe : be;
        }
        if (lane == be) taken = true;
        if (lane == j) {
            sel = be;
            val = bv;
        }
    }
    const double mx = (double)__shfl(val, 0, 64);  // the overall maximum is selected first
    const double ex_sel = exp((double)val - mx);   // lanes j < k: the selected logits
    double denom = 0.0;
    if (p.gate_norm == 0) {
        for (int j = 0; j < p.k; ++j) denom += __shfl(ex_sel, j, 64);
    } else {
        const double ex_all = exp((double)mine - mx);
        for (int e = 0; e < p.E; ++e) denom += __shfl(ex_all, e, 64);
    }
    if (lane < p.k) {
        p.idx[(size_t)t * p.k + lane] = sel;
        p.gates[(size_t)t * p.k + lane] = (float)(ex_sel / denom);
    }
}

}  // namespace adafuse
