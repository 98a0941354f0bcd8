// Plain structs of the device-side tables and the library's limits.  No HIP types or
// builtins: this header also compiles with an ordinary host compiler, so the host logic
// that builds the tables can be checked on a machine without a GPU.
#pragma once
#include <stdint.h>

namespace adafuse {

constexpr int kMaxTerms = 8;     // experts accumulated per element in one pass
constexpr int kMaxExperts = 64;  // experts per bank, router outputs
constexpr int kMaxTopK = 8;      // experts the router selects per token

// One adapted matrix: the device copy of a caller descriptor (section "SGMM
// Kernel": pointer arrays plus the shape of each segment).
struct MatDev {
    const uint16_t *w_base;
    uint16_t *w_work;
    const uint16_t *a_bank;  // [E][r][in]
    const uint16_t *b_bank;  // [E][out][r]
    int32_t out, in, ldw, pad;
};

// One workgroup's share of the batched update.  The entry carries everything the
// W loads need (tile origin in both buffers, leading dimension, bounds), so they
// can be issued after ONE table read; the matrix table is read alongside, for
// the operand banks only.
struct TileDev {
    const uint16_t *w_src;  // &W_base[row0][col0]
    uint16_t *w_dst;        // &W_work[row0][col0]
    uint32_t mat;
    int32_t row0, col0;
    int32_t ldw;
    int32_t rows_left;      // out - row0
    int32_t cols_left;      // in - col0
};

}  // namespace adafuse
