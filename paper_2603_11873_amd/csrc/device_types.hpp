// Device-side tables and small bf16 helpers shared by the switch and router kernels.
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "table_types.hpp"

namespace adafuse {

typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(2))) float float2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) unsigned int uint4_t;
typedef __attribute__((ext_vector_type(2))) unsigned int uint2_t;

struct SwitchParams {
    const MatDev *mats;
    const TileDev *tiles;
    const int32_t *idx_prev;
    const float *gates_prev;
    const int32_t *idx_next;
    const float *gates_next;
    int32_t k;
    int32_t E;
    int32_t r;
    int32_t mode;  // adafuse_mode
    float scale;
    int32_t inplace;  // 1: w_work == w_base for every matrix (paper-literal in-place update)
};

// Pointers read out of the matrix table have no known address space, and the
// compiler would fall back to FLAT instructions, which also count against the
// LDS counter (every LDS wait would then drain the W loads in flight).  These
// helpers state that the memory is global.
#define ADAFUSE_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ T ld_global(const T *p)
{
    return *(const ADAFUSE_GLOBAL T *)p;
}
template <class T>
__device__ __forceinline__ T ld_global_nt(const T *p)
{
    return __builtin_nontemporal_load((const ADAFUSE_GLOBAL T *)p);
}
template <class T>
__device__ __forceinline__ void st_global_nt(T v, T *p)
{
    __builtin_nontemporal_store(v, (ADAFUSE_GLOBAL T *)p);
}

// Raw buffer addressing: a uniform descriptor (base and size in scalar registers), a
// 32-bit byte offset per lane and a uniform byte offset per instruction, so a
// group of loads that differ only in the uniform part shares ONE address
// register.  Reads beyond `bytes` return zero.  Word 3 selects a 32-bit data
// format (ignored by untyped loads, but a descriptor must name a valid one).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint32_t ld_buffer_b32(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)lane_off, (int)uniform_off, 0);
}
__device__ __forceinline__ uint2_t ld_buffer_b64(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(uint2_t, __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_off, (int)uniform_off, 0));
}
__device__ __forceinline__ uint4_t ld_buffer_b128(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(uint4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_off, (int)uniform_off, 0));
}

// Store through a buffer descriptor, streaming (non-temporal); an offset beyond the descriptor's size is dropped.
__device__ __forceinline__ void st_buffer_b128_nt(uint4_t v, __amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)lane_off, 0, 2 /* non-temporal */);
}

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Two fp32 -> packed bf16 pair, round-to-nearest-even in hardware (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    float2_t f = {lo, hi};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

// The token's term list (expert, coefficient s*g) read from device memory; every
// lane reads the same addresses.  Terms beyond k get coefficient 0 on expert 0.
// Returns false when the launch has nothing to do for this mode: SWAP with a
// previous decision bit-identical to the next one.
struct Terms {
    int32_t e[kMaxTerms];
    float c[kMaxTerms];
};

template <int NT>
__device__ __forceinline__ bool load_terms(const SwitchParams &p, Terms &t)
{
    const bool have_prev = p.idx_prev != nullptr && p.gates_prev != nullptr;
    if (p.mode == 2 /*SWAP*/ && have_prev) {
        bool same = true;
        for (int j = 0; j < p.k; ++j) {
            same = same && (p.idx_prev[j] == p.idx_next[j]) &&
                   (__float_as_uint(p.gates_prev[j]) == __float_as_uint(p.gates_next[j]));
        }
        if (same) return false;
    }
    // Out of place the update is built from the immutable base, so only the next
    // token's experts enter.  In place (Eq.7-8) the previous token's experts enter
    // first with a negative sign, then the next token's: [-DOWN^{t-1}, DOWN^t].
    const int n_prev = (p.inplace && p.mode != 0 /*MERGE*/) ? p.k : 0;
    const int n_next = (p.mode != 1 /*UNMERGE*/) ? p.k : 0;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        int32_t e = 0;
        float c = 0.0f;
        if (j < n_prev) {
            e = p.idx_prev[j];
            c = -(p.scale * p.gates_prev[j]);
        } else if (j < n_prev + n_next) {
            e = p.idx_next[j - n_prev];
            c = p.scale * p.gates_next[j - n_prev];
        }
        t.e[j] = e < 0 ? 0 : (e >= p.E ? p.E - 1 : e);
        t.c[j] = c;
    }
    // In place, an expert that both tokens selected enters once, with the difference
    // of its two coefficients (zero when the gates are equal too: the kernels skip
    // such terms), so the contraction covers only what changes between the tokens.
    // Indices are compile-time constants after unrolling: the list stays in registers.
    if (n_prev > 0 && n_next > 0) {
#pragma unroll
        for (int a = 0; a < NT; ++a) {
            bool folded = false;
#pragma unroll
            for (int b = 0; b < NT; ++b) {
                const bool hit = !folded && a < n_prev && b >= n_prev && b < n_prev + n_next && t.e[a] == t.e[b];
                if (hit) {
                    t.c[b] += t.c[a];
                    t.c[a] = 0.0f;
                    folded = true;
                }
            }
        }
    }
    return true;
}

// Order the term list by ascending |coefficient| (a fixed odd-even transposition
// network: every index is a compile-time constant, the values are uniform and the
// comparison is on the integer image of |c|, so the whole thing stays in scalar
// registers).  Kernels that chain the experts in one accumulator,
//   acc = P_0;  acc = acc * (c_0 / c_1) + P_1;  ...;  W' = W + c_last * acc,
// then only ever form ratios of magnitude <= 1: a gate that is tiny or sub-normal
// next to the others can no longer drive a ratio to infinity.  Terms with a zero
// coefficient (unused slots included) come first and are skipped by their value.
template <int NT>
__device__ __forceinline__ void sort_terms_by_magnitude(Terms &t)
{
#pragma unroll
    for (int round = 0; round < NT; ++round) {
#pragma unroll
        for (int a = round & 1; a + 1 < NT; a += 2) {
            const uint32_t ma = __float_as_uint(t.c[a]) & 0x7fffffffu, mb = __float_as_uint(t.c[a + 1]) & 0x7fffffffu;
            const bool swap = ma > mb;
            const int32_t ea = t.e[a], eb = t.e[a + 1];
            const float ca = t.c[a], cb = t.c[a + 1];
            t.e[a] = swap ? eb : ea;
            t.e[a + 1] = swap ? ea : eb;
            t.c[a] = swap ? cb : ca;
            t.c[a + 1] = swap ? ca : cb;
        }
    }
}

}  // namespace adafuse
