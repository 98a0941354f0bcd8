// Host-only logic of libadafuse: descriptor validation and the construction of the matrix
// and tile tables one switch launch walks (section "SGMM Kernel": arrays of pointers plus
// the shape of each segment, one launch for all layers).  Pure C++ with no HIP call, so it
// also builds with g++ under the address and undefined-behaviour sanitizers.
#pragma once
#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "adafuse.h"
#include "table_types.hpp"

namespace adafuse {
namespace host {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool rank_supported(int r) { return r == 4 || r == 8 || r == 16 || r == 32 || r == 64 || r == 128; }

inline adafuse_status validate_mats(const adafuse_matrix_desc *mats, int32_t n_mats, int32_t E, int32_t r, int32_t k_max)
{
    if (!mats) return ADAFUSE_ERR_NULL;
    if (n_mats < 1 || n_mats > 65535) return ADAFUSE_ERR_ARG;
    if (E < 1 || E > kMaxExperts) return ADAFUSE_ERR_ARG;
    if (!rank_supported(r)) return ADAFUSE_ERR_ARG;
    if (k_max < 1 || k_max > E || k_max > kMaxTerms) return ADAFUSE_ERR_ARG;
    for (int32_t i = 0; i < n_mats; ++i) {
        const adafuse_matrix_desc &m = mats[i];
        if (!m.w_base || !m.w_work || !m.a_bank || !m.b_bank) return ADAFUSE_ERR_NULL;
        if (m.reserved != 0) return ADAFUSE_ERR_ARG;
        if ((m.w_base == m.w_work) != (mats[0].w_base == mats[0].w_work)) return ADAFUSE_ERR_ARG;  // all in place or none
        if (m.out < 1 || m.in < 8 || (m.in % 8) != 0 || m.ldw < m.in || (m.ldw % 8) != 0) return ADAFUSE_ERR_SHAPE;
        // 32-bit offsets inside a tile (64 rows of ldw) and inside one expert's slice (rank x in, out x rank)
        if (m.out > (1 << 22) || m.in > (1 << 22) || m.ldw > (1 << 24)) return ADAFUSE_ERR_SHAPE;
        if (!aligned16(m.w_base) || !aligned16(m.w_work) || !aligned16(m.a_bank) || !aligned16(m.b_bank))
            return ADAFUSE_ERR_ALIGN;
    }
    if (mats[0].w_base == mats[0].w_work && 2 * k_max > kMaxTerms) return ADAFUSE_ERR_ARG;  // an in-place SWAP carries 2k terms
    return ADAFUSE_OK;
}

// Workgroup i of a launch runs on XCD i % 8.  Reorder tiles [begin, end) so that
// each XCD gets runs of G consecutive tiles instead of every eighth tile.
inline void deal_to_xcds(std::vector<TileDev> &v, size_t begin, size_t end, size_t G)
{
    const size_t n = end - begin;
    if (n == 0 || G == 0) return;
    std::vector<TileDev> sw;
    sw.reserve(n);
    std::vector<char> used(n, 0);
    const size_t slots = ((n + 8 * G - 1) / (8 * G)) * 8 * G;
    for (size_t i = 0; i < slots; ++i) {
        const size_t x = i % 8, q = i / 8;
        const size_t t = ((q / G) * 8 + x) * G + (q % G);
        if (t < n) {
            sw.push_back(v[begin + t]);
            used[t] = 1;
        }
    }
    for (size_t t = 0; t < n; ++t)
        if (!used[t]) sw.push_back(v[begin + t]);
    std::copy(sw.begin(), sw.end(), v.begin() + begin);
}

struct TablePlan {
    int tile_rows = 64, tile_cols = 256;
    size_t inner = 16;              // rank indices of a launch: terms x rank (sizes the column panels)
    size_t panel_bytes = 2u << 20;  // column operands one XCD may cycle through per row block
    int xcd_run = 1;                // 0: plain order; 1: an eighth of the list per XCD; G > 1: runs of G tiles
};

struct Tables {
    std::vector<MatDev> mats;
    std::vector<TileDev> tiles;      // [0, n): whole model; [n, 2n): the same tiles matrix by matrix
    std::vector<int64_t> mat_off;    // per-matrix ranges inside the second section (n_mats + 1 entries)
    int64_t n_tiles = 0, elements = 0;
};

// Tile order: matrix by matrix, row block by row block, column tiles innermost,
// so workgroups that run together read neighbouring column strips of the same
// rows (shared B slice) and the A/B slices of one matrix stay cache-resident
// while that matrix streams through.  Returns false if the launch would need more
// workgroups than a grid can hold.
inline bool build_tile_tables(const std::vector<adafuse_matrix_desc> &descs, const TablePlan &plan, Tables &t)
{
    const int tr = plan.tile_rows, tc = plan.tile_cols;
    // column tiles per panel: the panel's column operands (2 bytes x inner x columns) within panel_bytes
    const int panel_tiles_max = (int)std::max<size_t>(1, plan.panel_bytes / (2 * std::max<size_t>(1, plan.inner)) / (size_t)tc);
    t.mats.assign(descs.size(), MatDev{});
    t.tiles.clear();
    t.mat_off.assign(1, 0);
    t.elements = 0;
    for (size_t i = 0; i < descs.size(); ++i) {
        const adafuse_matrix_desc &m = descs[i];
        t.mats[i] = MatDev{static_cast<const uint16_t *>(m.w_base), static_cast<uint16_t *>(m.w_work),
                           static_cast<const uint16_t *>(m.a_bank), static_cast<const uint16_t *>(m.b_bank),
                           m.out, m.in, m.ldw, 0};
        const int nrt = (m.out + tr - 1) / tr, nct = (m.in + tc - 1) / tc;
        // A wide matrix is walked in column panels: row block by row block inside a panel, so
        // that the column-operand slices of one panel (selected experts x rank x panel columns)
        // stay in an XCD's L2 while its row blocks stream by.  Without panels, rank 128 top-2 on
        // an 11008-wide matrix cycles 5.6 MB of column operands through a 4 MB L2 once per row
        // block (measured: 1.30 x the algorithmic HBM traffic for the whole model).
        const int n_panels = (nct + panel_tiles_max - 1) / panel_tiles_max;
        const int panel_tiles = (nct + n_panels - 1) / n_panels;
        for (int ct0 = 0; ct0 < nct; ct0 += panel_tiles)
            for (int rt = 0; rt < nrt; ++rt)
                for (int ct = ct0; ct < std::min(nct, ct0 + panel_tiles); ++ct) {
                    const int row0 = rt * tr, col0 = ct * tc;
                    const size_t off = (size_t)row0 * m.ldw + col0;
                    t.tiles.push_back(TileDev{t.mats[i].w_base + off, t.mats[i].w_work + off, (uint32_t)i, row0, col0, m.ldw,
                                              m.out - row0, m.in - col0});
                }
        t.elements += (int64_t)m.out * m.in;
        t.mat_off.push_back((int64_t)t.tiles.size());
    }
    if (t.tiles.size() > 0x3fffffffu) return false;
    // second section: the same tiles grouped per matrix, for the one-launch-per-matrix form
    const size_t n = t.tiles.size();
    t.tiles.insert(t.tiles.end(), t.tiles.begin(), t.tiles.begin() + n);
    if (plan.xcd_run >= 1) {
        auto run = [&](size_t count) { return plan.xcd_run == 1 ? (count + 7) / 8 : (size_t)plan.xcd_run; };
        deal_to_xcds(t.tiles, 0, n, run(n));
        for (size_t i = 0; i + 1 < t.mat_off.size(); ++i)
            deal_to_xcds(t.tiles, n + t.mat_off[i], n + t.mat_off[i + 1], run((size_t)(t.mat_off[i + 1] - t.mat_off[i])));
    }
    t.n_tiles = (int64_t)n;
    return true;
}

// Share of the elements that sit in matrices whose row pitch in bytes is not a power of two.
// The 4-wave workgroup moves 512-byte row pieces, the 8-wave one 1 KB pieces; at such pitches
// the longer pieces stream measurably better (Llama-2-13B shapes: 10240 and 27648 bytes).
inline double odd_pitch_share(const std::vector<adafuse_matrix_desc> &descs)
{
    double odd = 0, all = 0;
    for (const adafuse_matrix_desc &m : descs) {
        const uint64_t pitch = 2ull * (uint64_t)m.ldw;
        const double e = (double)m.out * m.in;
        all += e;
        if (pitch & (pitch - 1)) odd += e;
    }
    return all > 0 ? odd / all : 0.0;
}

}  // namespace host
}  // namespace adafuse
