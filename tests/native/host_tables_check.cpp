// CPU-only check of the library's host logic (descriptor validation, tile enumeration, column
// panels, the XCD deal), built by tests/test_host_tables.py with g++ under the address and
// undefined-behaviour sanitizers.  For every model below and every plan, each (matrix, row
// block, column tile) must appear exactly once in the whole-model section and exactly once in
// its matrix's range of the per-matrix section, with consistent origins and bounds.
// Pointers are fabricated addresses: nothing is dereferenced.
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <vector>

#include "host_tables.hpp"

using namespace adafuse;

static int g_fail = 0;
#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            if (g_fail < 20) { std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } \
            ++g_fail;                                     \
        }                                                 \
    } while (0)

struct Shape { int out, in, ldw; };

static std::vector<adafuse_matrix_desc> make_model(const std::vector<Shape> &shapes, int layers, bool inplace)
{
    std::vector<adafuse_matrix_desc> d;
    uintptr_t next = (uintptr_t)1 << 32;
    auto take = [&](size_t bytes) { uintptr_t p = next; next += (bytes + 4095) / 4096 * 4096 + 4096; return reinterpret_cast<void *>(p); };
    for (int l = 0; l < layers; ++l)
        for (const Shape &s : shapes) {
            adafuse_matrix_desc m{};
            m.w_base = take((size_t)s.out * s.ldw * 2);
            m.w_work = inplace ? const_cast<void *>(m.w_base) : take((size_t)s.out * s.ldw * 2);
            m.a_bank = take(64);
            m.b_bank = take(64);
            m.out = s.out; m.in = s.in; m.ldw = s.ldw; m.reserved = 0;
            d.push_back(m);
        }
    return d;
}

static void check_tables(const char *what, const std::vector<adafuse_matrix_desc> &descs, const host::TablePlan &plan)
{
    host::Tables t;
    const bool ok = host::build_tile_tables(descs, plan, t);
    CHECK(ok, "%s: build failed", what);
    if (!ok) return;
    const int tr = plan.tile_rows, tc = plan.tile_cols;
    int64_t expect = 0, elements = 0;
    for (const auto &m : descs) {
        expect += (int64_t)((m.out + tr - 1) / tr) * ((m.in + tc - 1) / tc);
        elements += (int64_t)m.out * m.in;
    }
    CHECK(t.n_tiles == expect, "%s: %lld tiles, expected %lld", what, (long long)t.n_tiles, (long long)expect);
    CHECK(t.elements == elements, "%s: element count", what);
    CHECK((int64_t)t.tiles.size() == 2 * t.n_tiles, "%s: two sections", what);
    CHECK(t.mat_off.size() == descs.size() + 1 && t.mat_off.front() == 0 && t.mat_off.back() == t.n_tiles, "%s: matrix ranges", what);
    CHECK(t.mats.size() == descs.size(), "%s: matrix table", what);
    for (int section = 0; section < 2; ++section) {
        std::vector<uint64_t> keys;
        keys.reserve((size_t)t.n_tiles);
        int64_t covered = 0;
        for (int64_t i = 0; i < t.n_tiles; ++i) {
            const TileDev &e = t.tiles[(size_t)(section * t.n_tiles + i)];
            CHECK(e.mat < descs.size(), "%s: matrix index %u", what, e.mat);
            if (e.mat >= descs.size()) continue;
            const adafuse_matrix_desc &m = descs[e.mat];
            CHECK(e.row0 >= 0 && e.row0 < m.out && e.row0 % tr == 0, "%s: row0 %d", what, e.row0);
            CHECK(e.col0 >= 0 && e.col0 < m.in && e.col0 % tc == 0, "%s: col0 %d", what, e.col0);
            CHECK(e.rows_left == m.out - e.row0 && e.cols_left == m.in - e.col0 && e.ldw == m.ldw, "%s: bounds of tile %lld", what, (long long)i);
            const size_t off = (size_t)e.row0 * m.ldw + e.col0;
            CHECK(e.w_src == static_cast<const uint16_t *>(m.w_base) + off && e.w_dst == static_cast<uint16_t *>(m.w_work) + off,
                  "%s: origin of tile %lld", what, (long long)i);
            keys.push_back(((uint64_t)e.mat << 44) | ((uint64_t)(e.row0 / tr) << 22) | (uint64_t)(e.col0 / tc));
            covered += (int64_t)std::min(tr, e.rows_left) * std::min(tc, e.cols_left);
            if (section == 1) {  // grouped per matrix
                CHECK(i >= t.mat_off[e.mat] && i < t.mat_off[e.mat + 1], "%s: tile %lld outside its matrix's range", what, (long long)i);
            }
        }
        std::sort(keys.begin(), keys.end());
        const size_t distinct = (size_t)(std::unique(keys.begin(), keys.end()) - keys.begin());
        CHECK((int64_t)distinct == expect, "%s: section %d holds %zu distinct tiles of %lld", what, section, distinct, (long long)expect);
        CHECK(covered == elements, "%s: section %d covers %lld of %lld elements", what, section, (long long)covered, (long long)elements);
    }
}

static void check_deal()
{
    // the deal is a permutation for every length and run length, and XCD x (slots x, x + 8, ...) gets whole runs
    for (size_t n : {0u, 1u, 7u, 8u, 9u, 63u, 64u, 65u, 1000u, 4099u})
        for (size_t G : {1u, 2u, 7u, 64u, 513u, 5000u}) {
            std::vector<TileDev> v(n);
            for (size_t i = 0; i < n; ++i) v[i].row0 = (int32_t)i;
            host::deal_to_xcds(v, 0, n, G);
            std::vector<char> seen(n, 0);
            for (size_t i = 0; i < n; ++i) {
                const size_t id = (size_t)v[i].row0;
                CHECK(id < n && !seen[id], "deal n=%zu G=%zu: not a permutation", n, G);
                if (id < n) seen[id] = 1;
            }
            if (n % (8 * G) == 0)  // full rounds: slot i holds tile ((q / G) * 8 + x) * G + q % G, x = i % 8, q = i / 8
                for (size_t i = 0; i < n; ++i) {
                    const size_t x = i % 8, q = i / 8;
                    CHECK((size_t)v[i].row0 == ((q / G) * 8 + x) * G + q % G, "deal n=%zu G=%zu: slot %zu", n, G, i);
                }
        }
}

static void check_validation()
{
    std::vector<adafuse_matrix_desc> d = make_model({{64, 64, 64}}, 1, false);
    CHECK(host::validate_mats(d.data(), 1, 8, 8, 2) == ADAFUSE_OK, "valid descriptor refused");
    CHECK(host::validate_mats(nullptr, 1, 8, 8, 2) == ADAFUSE_ERR_NULL, "null array");
    CHECK(host::validate_mats(d.data(), 0, 8, 8, 2) == ADAFUSE_ERR_ARG, "no matrices");
    CHECK(host::validate_mats(d.data(), 1, 8, 12, 2) == ADAFUSE_ERR_ARG, "rank 12");
    CHECK(host::validate_mats(d.data(), 1, 8, 8, 9) == ADAFUSE_ERR_ARG, "k_max 9");
    auto bad = d; bad[0].in = 60;
    CHECK(host::validate_mats(bad.data(), 1, 8, 8, 2) == ADAFUSE_ERR_SHAPE, "in not a multiple of 8");
    bad = d; bad[0].ldw = 56;
    CHECK(host::validate_mats(bad.data(), 1, 8, 8, 2) == ADAFUSE_ERR_SHAPE, "ldw < in");
    bad = d; bad[0].a_bank = reinterpret_cast<void *>((uintptr_t)bad[0].a_bank + 2);
    CHECK(host::validate_mats(bad.data(), 1, 8, 8, 2) == ADAFUSE_ERR_ALIGN, "misaligned bank");
    bad = d; bad[0].w_work = nullptr;
    CHECK(host::validate_mats(bad.data(), 1, 8, 8, 2) == ADAFUSE_ERR_NULL, "null pointer in descriptor");
    auto two = make_model({{64, 64, 64}, {64, 64, 64}}, 1, false);
    two[1].w_work = const_cast<void *>(two[1].w_base);
    CHECK(host::validate_mats(two.data(), 2, 8, 8, 2) == ADAFUSE_ERR_ARG, "in place and out of place mixed");
    auto inpl = make_model({{64, 64, 64}}, 1, true);
    CHECK(host::validate_mats(inpl.data(), 1, 8, 8, 4) == ADAFUSE_OK, "in place top-4");
    CHECK(host::validate_mats(inpl.data(), 1, 8, 8, 5) == ADAFUSE_ERR_ARG, "in place top-5 needs 10 terms");
    CHECK(host::odd_pitch_share(make_model({{64, 4096, 4096}}, 1, false)) == 0.0, "pitch 8192 is a power of two");
    CHECK(host::odd_pitch_share(make_model({{64, 5120, 5120}}, 1, false)) == 1.0, "pitch 10240 is not");
}

int main()
{
    struct Model { const char *name; std::vector<Shape> shapes; int layers; };
    const std::vector<Model> models = {
        {"ragged", {{1, 8, 8}, {3, 24, 40}, {301, 200, 200}, {257, 136, 144}, {255, 392, 392}, {130, 128, 128}, {70, 264, 272},
                    {66, 120, 120}, {513, 520, 520}, {200, 328, 328}, {129, 136, 144}, {64, 64, 64}, {331, 72, 72}}, 1},
        {"toy", {{256, 256, 256}, {256, 256, 256}, {256, 256, 256}, {256, 256, 256}}, 2},
        {"llama2_7b_attn", {{4096, 4096, 4096}, {4096, 4096, 4096}, {4096, 4096, 4096}, {4096, 4096, 4096}}, 32},
        {"llama2_7b_all", {{4096, 4096, 4096}, {4096, 4096, 4096}, {4096, 4096, 4096}, {4096, 4096, 4096},
                           {11008, 4096, 4096}, {11008, 4096, 4096}, {4096, 11008, 11008}}, 32},
        {"llama3_8b_gqa_all", {{4096, 4096, 4096}, {1024, 4096, 4096}, {1024, 4096, 4096}, {4096, 4096, 4096},
                               {14336, 4096, 4096}, {14336, 4096, 4096}, {4096, 14336, 14336}}, 32},
        {"llama2_13b_all", {{5120, 5120, 5120}, {5120, 5120, 5120}, {5120, 5120, 5120}, {5120, 5120, 5120},
                            {13824, 5120, 5120}, {13824, 5120, 5120}, {5120, 13824, 13824}}, 40},
    };
    const int tile_shapes[][2] = {{64, 256}, {64, 512}, {256, 512}, {128, 512}, {32, 256}, {128, 256}, {16, 512}};
    int plans = 0;
    for (const Model &m : models) {
        const bool big = m.layers > 2;
        for (int inplace = 0; inplace < 2; ++inplace) {
            const auto descs = make_model(m.shapes, m.layers, inplace != 0);
            for (const auto &ts : tile_shapes) {
                if (big && !(ts[0] == 64 && (ts[1] == 256 || ts[1] == 512))) continue;  // full models: the default kernel's two shapes
                for (size_t inner : {8u, 64u, 256u, 1024u})
                    for (size_t panel_kb : {64u, 2048u})
                        for (int run : {0, 1, 7, 512}) {
                            if (big && (inplace || run == 7 || (inner != 64 && inner != 1024) || (run == 512 && panel_kb == 64))) continue;
                            host::TablePlan plan;
                            plan.tile_rows = ts[0]; plan.tile_cols = ts[1]; plan.inner = inner;
                            plan.panel_bytes = panel_kb * 1024; plan.xcd_run = run;
                            char what[160];
                            std::snprintf(what, sizeof what, "%s%s tile %dx%d inner %zu panel %zu KB run %d", m.name, inplace ? " in place" : "",
                                          ts[0], ts[1], inner, panel_kb, run);
                            check_tables(what, descs, plan);
                            ++plans;
                        }
            }
        }
    }
    check_deal();
    check_validation();
    if (g_fail) { std::printf("%d checks failed\n", g_fail); return 1; }
    std::printf("host tables ok: %d table builds\n", plans);
    return 0;
}
