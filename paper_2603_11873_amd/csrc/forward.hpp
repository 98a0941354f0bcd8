// The step right after the switch, for checking and for context only: one
// linear layer applied to one token,
//   merged backbone (Eq.3):   y = W_work x
//   dynamic adapter (Eq.2):   y = W_base x + s * sum_j g_j B_{e_j} (A_{e_j} x)
// as a decode loop would launch them: one GEMV per matrix, and for the dynamic
// form two more small launches per selected expert (down, then up projection).
// bf16 weights and input, fp32 accumulation and output.
#pragma once
#include "device_types.hpp"

namespace adafuse {

__device__ __forceinline__ float dot8(uint4_t w, uint4_t x, float acc)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        acc = __builtin_fmaf(bf16_lo(w[q]), bf16_lo(x[q]), acc);
        acc = __builtin_fmaf(bf16_hi(w[q]), bf16_hi(x[q]), acc);
    }
    return acc;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// y[row] = sum_i W[row][i] x[i]; one wave per row, 4 rows per workgroup.
__global__ __launch_bounds__(256) void gemv_rows_kernel(const uint16_t *w, int64_t ldw, const uint16_t *x, float *y,
                                                        int rows, int cols)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const uint16_t *wr = w + (size_t)row * ldw;
    float acc0 = 0.f, acc1 = 0.f;
    int i = lane * 8;
    for (; i + 512 < cols; i += 1024) {
        const uint4_t w0 = ld_global_nt(reinterpret_cast<const uint4_t *>(wr + i));
        const uint4_t w1 = ld_global_nt(reinterpret_cast<const uint4_t *>(wr + i + 512));
        acc0 = dot8(w0, ld_global(reinterpret_cast<const uint4_t *>(x + i)), acc0);
        acc1 = dot8(w1, ld_global(reinterpret_cast<const uint4_t *>(x + i + 512)), acc1);
    }
    for (; i < cols; i += 512)
        acc0 = dot8(ld_global_nt(reinterpret_cast<const uint4_t *>(wr + i)), ld_global(reinterpret_cast<const uint4_t *>(x + i)), acc0);
    const float s = wave_sum(acc0 + acc1);
    if (lane == 0) y[row] = s;
}

// LoRA up projection added into y: y[row] += c * sum_rho B[row][rho] z[rho]; one thread per row.
__global__ __launch_bounds__(256) void lora_up_kernel(const uint16_t *b, const float *z, float *y, int rows, int r, float c)
{
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= rows) return;
    const uint16_t *br = b + (size_t)row * r;
    float acc = 0.f;
    for (int rho = 0; rho < r; ++rho) acc = __builtin_fmaf(bf16_bits_to_f32(ld_global(br + rho)), z[rho], acc);
    y[row] += c * acc;
}

}  // namespace adafuse
