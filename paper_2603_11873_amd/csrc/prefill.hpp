// Prefill: many tokens through adapted matrices, every token with its own routing decision
// (section "Decoding Phase", prefill paragraph: one merged weight cannot serve tokens that
// selected different experts, so the adapters stay un-merged here, Eq.2):
//   Y[t] = W_base x_t + s * sum_j g_{t,j} * B_{e_{t,j}} (A_{e_{t,j}} x_t),   t < T.
// One matrix-core product kernel (v_mfma_f32_32x32x16_bf16, fp32 accumulation) and small
// element-wise kernels around it, in two forms.
//
// FEW tokens (a launch costs more than streaming a matrix): two launches for a group of matrices
// that share X.
//   1. prefill_gemm_kernel on a batch of products: X W^T for every matrix of the group and
//      U = X A^T for every bank seen as one [E r][in] matrix (ALL experts, dense: the bank is a
//      fraction of W), all cut into the same number of parts of the inner dimension.
//   2. prefill_finish_kernel: the parts summed in order, the adapters added in fp32 on the
//      vector ALU (2 k r flops per output).
// MANY tokens: matrix by matrix.
//   1. prefill_gemm_kernel on the A bank: U = X A^T.
//   2. prefill_gate_kernel: for every (token, selection) the expert's r columns of U times
//      s * g, stored as a pair of bf16 planes hi + lo (16 significant bits), zero padded to
//      a multiple of 8; a repeated selection of an expert is folded into the first.
//   3. prefill_gemm_kernel on W_base: X W^T, and in the same accumulators, for every expert
//      some token of the tile selected, k-steps over the rank with the token's scaled
//      down-projection (zero for tokens that did not select it) against B_e's rows -- the
//      adapter is just more inner dimension of the same product.
//   4. prefill_sum_kernel (only when the inner dimension was split): the parts, in order.
//
// The product kernel: a workgroup (4 waves side by side, 128 tokens x 64 rows each) owns 128 tokens
// x 256 output rows and a range of the inner dimension; chunks of 64 inner indices of both
// operands go straight into LDS (buffer_load ... lds, row-contiguous 128-byte lines: a wave
// instruction moves 8 whole lines) in three stages -- two chunks, 64 KB of the matrix, in flight
// per CU while a third is multiplied -- and each wave reads its operands from there in the
// matrix-core layout (the 16-byte pieces of a line are permuted by the row number, so both the
// line-wise fill and the column-of-pieces reads are conflict-free).  Loading operands straight
// from global memory in the matrix-core layout (one row per lane) was the first version: 32 cache
// lines per wave instruction, four times the address work in the texture path, and 10 x off the
// roofline.  With few tokens a launch has too few tiles to fill the chip, so the inner dimension
// is split across workgroups and the parts are summed in a fixed order afterwards: no atomics,
// the same bits on every run.  Lanes beyond T, the matrix edge or the split's range point
// outside their buffer descriptor and read as zero.
#pragma once
#include "device_types.hpp"

namespace adafuse {

typedef __attribute__((ext_vector_type(8))) __bf16 pf_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float pf_float16_t;
typedef __attribute__((address_space(3))) void pf_lds_void_t;

constexpr int kPfTileTokens = 128;  // tokens per workgroup
constexpr int kPfTileRows = 256;    // output rows per workgroup: 64 per wave
constexpr int kPfChunk = 64;        // inner indices per LDS stage (one 128-byte line per row)
constexpr uint32_t kOutside = 0xffffff00u;  // a per-lane offset no descriptor of this library covers: reads as zero

struct PrefillGemm {
    const uint16_t *m;       // [rows][ld] bf16: W_base, or the A bank as [E r][in]
    const uint16_t *x;       // [T][in] bf16
    float *out;              // [splits][T][rows] fp32 (splits == 1: the result itself)
    int32_t rows, ld, in, T;
    int32_t splits;          // parts of the inner dimension
    int32_t chunks_per_split;
    int32_t m_tiles, strips;
    // adapters (W pass only; b_bank == nullptr: none)
    const uint16_t *b_bank;  // [E][rows][r]
    const int32_t *idx;      // [T][k]
    const uint16_t *z_hi;    // [T][k][rp]
    const uint16_t *z_lo;
    int32_t E, r, rp, k;
};

__device__ __forceinline__ pf_bf16x8_t as_operand(uint4_t v) { return __builtin_bit_cast(pf_bf16x8_t, v); }
__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

// Experts selected by any of the tokens [t0, t0 + n_tok) as a bit mask (E <= 64); every wave
// computes it for itself, lane l looking at tokens t0 + l, t0 + l + 64, ...
__device__ __forceinline__ uint64_t experts_in_tile(const int32_t *idx, int k, int E, int T, int t0, int n_tok, int lane)
{
    uint64_t mine = 0;
    for (int t = t0 + lane; t < t0 + n_tok && t < T; t += 64)
        for (int j = 0; j < k; ++j) mine |= 1ull << clamp_expert(idx[(size_t)t * k + j], E);
    uint64_t all = 0;
    for (int e = 0; e < E; ++e)
        if (__ballot((mine >> e) & 1ull)) all |= 1ull << e;
    return all;
}

// One chunk of both operands into an LDS stage: 128 token lines and 256 matrix lines of 128 bytes.
// Wave w's instruction i fills the KB that starts at line 8 (w + 4 i); lane l delivers piece slot
// l % 8 of line 8 (w + 4 i) + l / 8, and fetches for it the piece (slot ^ line % 8) of that row.
// Always 12 transfers per wave: a line or piece beyond the edge (or a whole chunk beyond the part's
// range) points outside the descriptor, fetches nothing and fills its slot with zeros.
__device__ __forceinline__ void pf_request(uint16_t *sx, uint16_t *sm, __amdgpu_buffer_rsrc_t xr, __amdgpu_buffer_rsrc_t mr,
                                           uint32_t in_bytes, uint32_t ld_bytes, int t0, int T, int rows_here, int k0, int k_end,
                                           int wave, int lane)
{
#pragma unroll
    for (int i = 0; i < kPfTileTokens / 32; ++i) {  // X: 16 KB
        const int line = 8 * (wave + 4 * i) + lane / 8;
        const int k = k0 + 8 * ((lane % 8) ^ (line % 8));
        const uint32_t off = t0 + line < T && k < k_end ? (uint32_t)(t0 + line) * in_bytes + 2u * (uint32_t)k : kOutside;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (pf_lds_void_t *)(sx + 512 * (wave + 4 * i)), 16, (int)off, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kPfTileRows / 32; ++i) {  // matrix: 32 KB
        const int line = 8 * (wave + 4 * i) + lane / 8;
        const int k = k0 + 8 * ((lane % 8) ^ (line % 8));
        const uint32_t off = line < rows_here && k < k_end ? (uint32_t)line * ld_bytes + 2u * (uint32_t)k : kOutside;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(mr, (pf_lds_void_t *)(sm + 512 * (wave + 4 * i)), 16, (int)off, 0, 0, 2 /* streamed once */);
    }
}
constexpr int kPfRequests = kPfTileTokens / 32 + kPfTileRows / 32;  // transfers per wave and chunk

// The wave's 128 tokens x 64 rows of one chunk: four k-steps, operands from LDS in the matrix-core layout.
// The six operand reads of k-step s + 1 are issued before the eight matrix-core instructions of k-step s
// (two register sets, and scheduling groups so that the compiler keeps that order): with one wave per SIMD
// nothing else hides the LDS latency, and reads placed right in front of their use left the matrix cores
// idle for two thirds of the time.
struct PfOperands {
    uint4_t mv[2], xv[4];
};
__device__ __forceinline__ void pf_read(PfOperands &o, const uint16_t *sx, const uint16_t *sm, int s, int wave, int n, int h)
{
    const int piece = 2 * s + h;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int mrow = 64 * wave + 32 * c + n;
        o.mv[c] = *reinterpret_cast<const uint4_t *>(sm + 64 * mrow + 8 * (piece ^ (mrow % 8)));
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int xrow = 32 * b + n;
        o.xv[b] = *reinterpret_cast<const uint4_t *>(sx + 64 * xrow + 8 * (piece ^ (xrow % 8)));
    }
}
__device__ __forceinline__ void pf_mfma(pf_float16_t (&acc)[4][2], const PfOperands &o)
{
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int c = 0; c < 2; ++c)
            acc[b][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(o.xv[b]), as_operand(o.mv[c]), acc[b][c], 0, 0, 0);
}
__device__ __forceinline__ void pf_multiply(pf_float16_t (&acc)[4][2], const uint16_t *sx, const uint16_t *sm, int wave, int n, int h)
{
    constexpr int kDsRead = 0x100, kMfma = 0x008;
    PfOperands o0, o1;
    pf_read(o0, sx, sm, 0, wave, n, h);
    __builtin_amdgcn_sched_group_barrier(kDsRead, 6, 0);
    pf_read(o1, sx, sm, 1, wave, n, h);
    __builtin_amdgcn_sched_group_barrier(kDsRead, 6, 0);
    pf_mfma(acc, o0);
    __builtin_amdgcn_sched_group_barrier(kMfma, 8, 0);
    pf_read(o0, sx, sm, 2, wave, n, h);
    __builtin_amdgcn_sched_group_barrier(kDsRead, 6, 0);
    pf_mfma(acc, o1);
    __builtin_amdgcn_sched_group_barrier(kMfma, 8, 0);
    pf_read(o1, sx, sm, 3, wave, n, h);
    __builtin_amdgcn_sched_group_barrier(kDsRead, 6, 0);
    pf_mfma(acc, o0);
    __builtin_amdgcn_sched_group_barrier(kMfma, 8, 0);
    pf_mfma(acc, o1);
    __builtin_amdgcn_sched_group_barrier(kMfma, 8, 0);
}

// One launch can carry several products over the same X (workgroups [end[i-1], end[i]) run product i):
// with a tile or two of tokens the down-projection through a bank and the base product are independent,
// as are the matrices of a layer that share an input (q, k, v; gate, up), and each alone is too small to
// fill the chip for long.
constexpr int kPfMaxProducts = 8;
struct PrefillBatch {
    PrefillGemm g[kPfMaxProducts];
    int32_t end[kPfMaxProducts];  // running totals of the products' workgroup counts (multiples of 8); unused entries repeat the last
};

__global__ __launch_bounds__(256) void prefill_gemm_kernel(PrefillBatch batch)
{
    // three stages (144 KB: one workgroup per CU, two chunks -- 64 KB of the matrix -- in flight while a
    // third is multiplied), each its own pair of arrays: the compiler then knows that reading one stage
    // does not have to wait for the transfers into the others
    __shared__ __align__(16) uint16_t s_x0[kPfTileTokens * kPfChunk], s_x1[kPfTileTokens * kPfChunk], s_x2[kPfTileTokens * kPfChunk];
    __shared__ __align__(16) uint16_t s_m0[kPfTileRows * kPfChunk], s_m1[kPfTileRows * kPfChunk], s_m2[kPfTileRows * kPfChunk];

    int which = 0;  // uniform: a scan over scalar registers
#pragma unroll
    for (int j = 0; j + 1 < kPfMaxProducts; ++j)
        if ((int)blockIdx.x >= batch.end[j]) which = j + 1;
    const PrefillGemm &p = batch.g[which];
    const int block = (int)blockIdx.x - (which ? batch.end[which - 1] : 0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;
    // workgroup i runs on XCD i % 8: the token tiles of one (strip, part) follow each other on one XCD,
    // so the second and later ones find the matrix lines in that XCD's L2
    const int xcd = block % 8, q = block / 8;
    const int unit = (q / p.m_tiles) * 8 + xcd, m_tile = q % p.m_tiles;
    if (unit >= p.strips * p.splits) return;
    const int strip = unit / p.splits, part = unit % p.splits;
    const int o0 = kPfTileRows * strip, t0 = kPfTileTokens * m_tile;
    const int rows_here = min(kPfTileRows, p.rows - o0);
    const uint32_t in_bytes = 2u * (uint32_t)p.in, ld_bytes = 2u * (uint32_t)p.ld;
    const __amdgpu_buffer_rsrc_t xr = make_buffer(p.x, (uint32_t)p.T * in_bytes);
    const __amdgpu_buffer_rsrc_t mr = make_buffer(p.m + (size_t)o0 * p.ld, (uint32_t)rows_here * ld_bytes);
    const int k_begin = part * p.chunks_per_split * kPfChunk;
    const int k_end = min(p.in, k_begin + p.chunks_per_split * kPfChunk);
    const int n_chunks = (k_end - k_begin + kPfChunk - 1) / kPfChunk;  // >= 1 by construction of the split
    const bool has_rows = 64 * wave < rows_here;                       // a wave whose 64 rows are all beyond the matrix only moves data

    pf_float16_t acc[4][2];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][c][v] = 0.0f;

    // Chunk c lives in stage c % 3.  Before chunk c is multiplied: wait for this wave's part of it (the
    // kPfRequests transfers of chunk c + 1 may stay outstanding), meet -- every wave is then also done reading
    // the stage of chunk c - 1 --, and request chunk c + 2 into that stage.
#define ADAFUSE_PF_STEP(SX, SM, NX, NM, C)                                                                                     \
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kPfRequests) : "memory");                                                        \
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");                                                            \
    pf_request(NX, NM, xr, mr, in_bytes, ld_bytes, t0, p.T, rows_here, k_begin + kPfChunk * ((C) + 2), k_end, wave, lane);     \
    __builtin_amdgcn_sched_barrier(0);                                                                                         \
    if (has_rows) pf_multiply(acc, SX, SM, wave, n, h);                                                                        \
    __builtin_amdgcn_sched_barrier(0);
    pf_request(s_x0, s_m0, xr, mr, in_bytes, ld_bytes, t0, p.T, rows_here, k_begin, k_end, wave, lane);
    pf_request(s_x1, s_m1, xr, mr, in_bytes, ld_bytes, t0, p.T, rows_here, k_begin + kPfChunk, k_end, wave, lane);
    for (int c = 0; c < n_chunks; c += 3) {
        ADAFUSE_PF_STEP(s_x0, s_m0, s_x2, s_m2, c)
        if (c + 1 >= n_chunks) break;
        ADAFUSE_PF_STEP(s_x1, s_m1, s_x0, s_m0, c + 1)
        if (c + 2 >= n_chunks) break;
        ADAFUSE_PF_STEP(s_x2, s_m2, s_x1, s_m1, c + 2)
    }
#undef ADAFUSE_PF_STEP

    // ---- the adapters: for every expert some token of the tile selected, k-steps over the rank; a token
    // that did not select the expert contributes a zero operand.  The experts are dealt to the parts of the
    // inner dimension (expert e goes to part e % splits: the sum of the parts collects them), so no
    // workgroup carries all of them behind its share of the base product.
    // (Operands straight from global memory, one row per lane: a few KB per tile.)
    const int ow = o0 + 64 * wave;
    if (p.b_bank != nullptr && has_rows) {
        // the lane's four tokens: which selection (if any) holds expert e is looked up in registers
        int sel[4][kMaxTopK];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int t = t0 + 32 * b + n;
#pragma unroll
            for (int j = 0; j < kMaxTopK; ++j) sel[b][j] = t < p.T && j < p.k ? clamp_expert(p.idx[(size_t)t * p.k + j], p.E) : -1;
        }
        uint64_t mine = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int j = 0; j < kMaxTopK; ++j)
                if (sel[b][j] >= 0) mine |= 1ull << sel[b][j];
        uint64_t present = 0;
        for (int e = part; e < p.E; e += p.splits)
            if (__ballot((mine >> e) & 1ull)) present |= 1ull << e;
        const uint32_t z_bytes = (uint32_t)p.T * (uint32_t)p.k * (uint32_t)p.rp * 2u;
        const __amdgpu_buffer_rsrc_t zh = make_buffer(p.z_hi, z_bytes), zl = make_buffer(p.z_lo, z_bytes);
        const int brows = min(64, p.rows - ow);
        for (int e = part; e < p.E; e += p.splits) {
            if (!((present >> e) & 1ull)) continue;
            const __amdgpu_buffer_rsrc_t br = make_buffer(p.b_bank + ((size_t)e * p.rows + ow) * p.r, (uint32_t)brows * 2u * (uint32_t)p.r);
            uint32_t zrow[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                zrow[b] = kOutside;
#pragma unroll
                for (int j = kMaxTopK - 1; j >= 0; --j)  // the FIRST selection of e holds the (folded) result
                    if (sel[b][j] == e) zrow[b] = (uint32_t)((t0 + 32 * b + n) * p.k + j) * (uint32_t)p.rp * 2u;
            }
            for (int s = 0; 16 * s < p.rp; ++s) {
                const int rho = 16 * s + 8 * h;
                uint4_t bv[2], hv[4], lv[4];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int row = 32 * c + n;
                    if (p.r >= 8) {
                        bv[c] = ld_buffer_b128(br, rho < p.r && row < brows ? (uint32_t)row * 2u * (uint32_t)p.r + 2u * (uint32_t)rho : kOutside, 0u);
                    } else {  // rank 4: a row is 8 bytes, the upper half of the operand stays zero
                        const uint2_t b2 = ld_buffer_b64(br, rho < p.r && row < brows ? (uint32_t)row * 8u : kOutside, 0u);
                        bv[c] = uint4_t{b2[0], b2[1], 0u, 0u};
                    }
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t off = rho < p.rp && zrow[b] != kOutside ? zrow[b] + 2u * (uint32_t)rho : kOutside;
                    hv[b] = ld_buffer_b128(zh, off, 0u);
                    lv[b] = ld_buffer_b128(zl, off, 0u);
                }
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        acc[b][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(lv[b]), as_operand(bv[c]), acc[b][c], 0, 0, 0);
                        acc[b][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(hv[b]), as_operand(bv[c]), acc[b][c], 0, 0, 0);
                    }
            }
        }
    }
    if (!has_rows) return;

    // The token operand goes first into the matrix core, so a lane holds ONE output row and its 16
    // accumulator entries of block (b, c) are tokens: entry 4 q + u is token t0 + 32 b + 8 q + 4 h + u, row
    // ow + 32 c + n.  A store instruction then writes, per half-wave, 32 consecutive rows of one token: a
    // whole 128-byte line (one token per lane would scatter 16-byte pieces over 64 lines, which the
    // memory side pays for with partial-line writes: measured 8 us of a 20 us launch at 100 tokens).
    float *dst0 = p.out + (size_t)part * p.T * p.rows;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int oo = ow + 32 * c + n;
        if (oo >= p.rows) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + 32 * b + 8 * (v / 4) + 4 * h + v % 4;
                if (t < p.T) __builtin_nontemporal_store(acc[b][c][v], dst0 + (size_t)t * p.rows + oo);
            }
    }
}

constexpr int kPfMaxSplits = 32;  // parts of a split inner dimension

// y[i] = parts[0][i] + parts[1][i] + ... in that order, i < n.  All parts are requested before the first
// addition (a loop of load-then-add would be a chain of memory round trips); unused slots add +0.
__global__ __launch_bounds__(256) void prefill_sum_kernel(const float *parts, float *y, int64_t n, int splits)
{
    const int64_t i = 4 * ((int64_t)blockIdx.x * 256 + threadIdx.x);
    if (i >= n) return;
    if (i + 3 < n && (n & 3) == 0) {
        float4_t v[kPfMaxSplits];
#pragma unroll
        for (int q = 0; q < kPfMaxSplits; ++q)
            v[q] = q < splits ? *reinterpret_cast<const float4_t *>(parts + (size_t)q * n + i) : float4_t{0.f, 0.f, 0.f, 0.f};
        float4_t s = v[0];
#pragma unroll
        for (int q = 1; q < kPfMaxSplits; ++q) s += v[q];
        *reinterpret_cast<float4_t *>(y + i) = s;
    } else {
        for (int64_t j = i; j < n && j < i + 4; ++j) {
            float s = parts[j];
            for (int q = 1; q < splits; ++q) s += parts[(size_t)q * n + j];
            y[j] = s;
        }
    }
}

// Last step of the few-token form: y[t][o] = sum of the base product's parts, in order, plus the
// adapters in fp32 on the vector ALU,
//   sum_j (s g_{t,j}) sum_rho B_{e_{t,j}}[o][rho] * u[t][e_{t,j} r + rho],   u = the bank product's parts summed in order.
// A workgroup takes one token and 1024 output rows (4 per thread); the token's k r scaled
// down-projections are formed once in LDS.  A repeated selection of an expert simply adds twice.
struct PrefillFinish {
    const float *w_parts;  // [splits][T][rows]
    const float *u_parts;  // [splits][T][E r]
    const uint16_t *b_bank;
    const int32_t *idx;
    const float *gates;
    float *y;
    int32_t T, rows, E, r, k, splits;
    float scale;
};

constexpr int kPfMaxGroup = 4;  // matrices that share an input, finished by one launch (grid z)
struct PrefillFinishBatch {
    PrefillFinish f[kPfMaxGroup];
};

// NS: slots for the parts (at least the number of parts; unused slots add +0): registers, and with them how many
// workgroups a CU holds while each walks its chain of dependent loads.  That chain is kept to three round
// trips -- the routing decision (scalar loads); the parts of both products, all requested at once; after
// the barrier the rows of the selected B_e, four 16-byte pieces at a time -- because at a hundred tokens
// this kernel is nothing but latency.
template <int NS>
__global__ __launch_bounds__(256) void prefill_finish_kernel(PrefillFinishBatch batch)
{
    __shared__ float s_z[kMaxTopK * 128];
    const PrefillFinish p = batch.f[blockIdx.z];
    const int t = blockIdx.y;
    const int kr = p.k * p.r;
    const int log_r = __builtin_ctz((unsigned)p.r);  // ranks are powers of two
    const int o0 = 1024 * blockIdx.x + 4 * threadIdx.x;
    const size_t n_y = (size_t)p.T * p.rows, at = (size_t)t * p.rows + o0;
    const bool whole = o0 + 3 < p.rows && (p.rows & 3) == 0;  // four rows, 16-byte aligned in every part and in B_e
    int ex[kMaxTopK];   // the token's decision: uniform, scalar loads
    float cf[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        ex[j] = j < p.k ? clamp_expert(p.idx[(size_t)t * p.k + j], p.E) : 0;
        cf[j] = j < p.k ? p.scale * p.gates[(size_t)t * p.k + j] : 0.0f;
    }
    // the base product's parts: independent of the decision, requested first
    float4_t wv[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        wv[s] = s < p.splits && whole ? *reinterpret_cast<const float4_t *>(p.w_parts + (size_t)s * n_y + at) : float4_t{0.f, 0.f, 0.f, 0.f};
    // the token's k r scaled down-projections, once per workgroup
    const size_t n_u = (size_t)p.T * p.E * p.r;
    for (int q = threadIdx.x; q < kr; q += 256) {
        const int j = q >> log_r, rho = q & (p.r - 1);
        int e = 0;
        float c = 0.0f;
#pragma unroll
        for (int jj = 0; jj < kMaxTopK; ++jj)
            if (jj == j) e = ex[jj], c = cf[jj];
        const size_t ua = ((size_t)t * p.E + e) * p.r + rho;
        float v[NS];  // all parts requested before the first addition; unused slots add +0
#pragma unroll
        for (int s = 0; s < NS; ++s) v[s] = s < p.splits ? p.u_parts[(size_t)s * n_u + ua] : 0.0f;
        float u = v[0];
#pragma unroll
        for (int s = 1; s < NS; ++s) u += v[s];
        s_z[q] = c * u;
    }
    __syncthreads();
    if (o0 >= p.rows) return;
    float acc[4];
    if (whole) {
        float4_t sum = wv[0];
#pragma unroll
        for (int s = 1; s < NS; ++s) sum += wv[s];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = sum[i];
        // the thread's four rows of B_e are 4 r contiguous bf16: r / 2 pieces of 8, element f of them is
        // row f / r, rank index f % r; rank indices of a row are taken in ascending order
        const int pieces = p.r >> 1;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j >= p.k) break;
            const uint4_t *bp = reinterpret_cast<const uint4_t *>(p.b_bank + ((size_t)ex[j] * p.rows + o0) * p.r);
            const float *z = s_z + (j << log_r);
            for (int pc = 0; pc < pieces; pc += 4) {
                uint4_t bv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) bv[u] = pc + u < pieces ? bp[pc + u] : uint4_t{0u, 0u, 0u, 0u};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (pc + u >= pieces) break;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {  // four elements: one row for every rank
                        const int f = 8 * (pc + u) + 4 * half;
                        const int i = f >> log_r, rho = f & (p.r - 1);
                        float a = 0.0f;
#pragma unroll
                        for (int ii = 0; ii < 4; ++ii)  // (one of the four accumulators: a select, not an indexed register)
                            if (ii == i) a = acc[ii];
                        a = __builtin_fmaf(bf16_lo(bv[u][2 * half]), z[rho], a);
                        a = __builtin_fmaf(bf16_hi(bv[u][2 * half]), z[rho + 1], a);
                        a = __builtin_fmaf(bf16_lo(bv[u][2 * half + 1]), z[rho + 2], a);
                        a = __builtin_fmaf(bf16_hi(bv[u][2 * half + 1]), z[rho + 3], a);
#pragma unroll
                        for (int ii = 0; ii < 4; ++ii)
                            if (ii == i) acc[ii] = a;
                    }
                }
            }
        }
        *reinterpret_cast<float4_t *>(p.y + at) = float4_t{acc[0], acc[1], acc[2], acc[3]};
        return;
    }
    // rows at the edge of a matrix whose height is not a multiple of 4: element by element
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (o0 + i >= p.rows) continue;
        float a = p.w_parts[at + i];
        for (int s = 1; s < p.splits; ++s) a += p.w_parts[(size_t)s * n_y + at + i];
        for (int j = 0; j < p.k; ++j) {
            int e = 0;
#pragma unroll
            for (int jj = 0; jj < kMaxTopK; ++jj)
                if (jj == j) e = ex[jj];
            const uint16_t *brow = p.b_bank + ((size_t)e * p.rows + o0 + i) * p.r;
            const float *z = s_z + (j << log_r);
            for (int rho = 0; rho < p.r; ++rho) a = __builtin_fmaf(__uint_as_float((uint32_t)brow[rho] << 16), z[rho], a);
        }
        p.y[at + i] = a;
    }
}

// Scaled down-projection of every (token, selection): z = (s * sum of the gates of all selections of
// that expert by the token) * U[t][e r .. e r + r), U summed over its parts in order, as bf16 hi + lo
// planes of rp >= r values (zero padded).  A repeated selection of an expert: the first slot takes
// the folded value, the others zeros.  One thread per (token, selection, rank index).
struct PrefillGate {
    const float *u;  // [splits][T][E r]
    const int32_t *idx;
    const float *gates;
    uint16_t *z_hi, *z_lo;
    int32_t T, E, r, rp, k, splits;
    float scale;
};

__global__ __launch_bounds__(256) void prefill_gate_kernel(PrefillGate p)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)p.T * p.k * p.rp;
    if (i >= total) return;
    const int rho = (int)(i % p.rp);
    const int j = (int)((i / p.rp) % p.k);
    const int t = (int)(i / ((int64_t)p.rp * p.k));
    const int e = clamp_expert(p.idx[(size_t)t * p.k + j], p.E);
    bool first = true;
    float c = 0.0f;
    for (int jj = 0; jj < p.k; ++jj)
        if (clamp_expert(p.idx[(size_t)t * p.k + jj], p.E) == e) {
            if (jj < j) first = false;
            c += p.scale * p.gates[(size_t)t * p.k + jj];
        }
    float z = 0.0f;
    if (first && rho < p.r) {
        const size_t n = (size_t)p.T * p.E * p.r, at = ((size_t)t * p.E + e) * p.r + rho;
        float v[kPfMaxSplits];  // all parts requested before the first addition; unused slots add +0
#pragma unroll
        for (int q = 0; q < kPfMaxSplits; ++q) v[q] = q < p.splits ? p.u[(size_t)q * n + at] : 0.0f;
        float u = v[0];
#pragma unroll
        for (int q = 1; q < kPfMaxSplits; ++q) u += v[q];
        z = c * u;
    }
    const uint32_t hi = pack_bf16_rne(z, 0.0f) & 0xffffu;
    const uint32_t lo = pack_bf16_rne(z - bf16_lo(hi), 0.0f) & 0xffffu;
    p.z_hi[i] = (uint16_t)hi;
    p.z_lo[i] = (uint16_t)lo;
}

}  // namespace adafuse
