// C-ABI of libadafuse: argument validation, matrix/tile tables, kernel dispatch.
// Declarations and the contract of every entry point are in include/adafuse.h.
#include "adafuse.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <type_traits>
#include <vector>

#include "device_types.hpp"
#include "host_tables.hpp"
#include "forward.hpp"
#include "hbm_probe.hpp"
#include "prefill.hpp"
#include "pregate.hpp"
#include "switch_gemm.hpp"
#include "switch_gemm_overlap.hpp"
#include "switch_gemm_strip.hpp"
#include "switch_mfma.hpp"
#include "switch_valu.hpp"

using namespace adafuse;

// Scratch of adafuse_forward_dynamic_static: the down-projected activations z (k x r floats)
// that adafuse_forward_dynamic takes as a caller workspace.  One copy per GPU, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress: the device
// address is looked up once per context (build_tables, with the context's device current) and
// kept in adafuse_ctx::scratch, which is what the launches pass.
constexpr int kScratchFloats = 1024;  // k * r <= 8 * 128
constexpr int kSinkFloats = 64;       // behind z: the word the read probe keeps its loads alive with
static __device__ __align__(256) float scratch[kScratchFloats + kSinkFloats];

struct adafuse_ctx {
    std::vector<adafuse_matrix_desc> mats;
    int32_t E = 0, r = 0, k_max = 0;
    int32_t kernel = ADAFUSE_KERNEL_VALU;  // kernel in effect, never AUTO
    int32_t tile_rows = 0, tile_cols = 0;
    int32_t mfma_shape = 0;  // tile shape of the 4x4x4 kernel in effect
    int32_t gemm_waves = 4;  // waves per workgroup of the rank-looped kernel in effect: tile 64 x (64 waves)
    bool inplace = false;    // every matrix has w_work == w_base
    // what adafuse_set_option asked for (0 / -1 = the library chooses)
    int32_t opt_waves = 0, opt_form = 0, opt_xcd_run = 1, opt_panel_kb = 2048, opt_mfma_shape = -1;
    int64_t n_tiles = 0, elements = 0;
    int device = -1;
    float *scratch = nullptr;            // this device's copy of the file-scope scratch array
    MatDev *d_mats = nullptr;
    TileDev *d_tiles = nullptr;          // [0, n_tiles): whole model; [n_tiles, 2 n_tiles): matrix by matrix
    TileDev *d_tall = nullptr;           // the whole model in chains of kStripTiles vertically adjacent tiles (the strip form of the rank-looped kernel), or null
    int64_t n_tall = 0;
    std::vector<int64_t> mat_tile_off;   // per-matrix ranges inside the second section (n_mats + 1 entries)
};

namespace {

using host::aligned16;

int terms_bucket(int k) { return k <= 1 ? 1 : (k <= 2 ? 2 : (k <= 4 ? 4 : 8)); }

// The matrix-core kernel is instantiated for ranks that are multiples of 4 and
// an inner dimension (terms x rank) of at most 128.  In place, a SWAP carries
// the previous and the next token's experts: twice k terms.
bool mfma_supported(int r, int max_terms)
{
    if (r != 4 && r != 8 && r != 16 && r != 32 && r != 64) return false;
    return max_terms <= kMaxTerms && terms_bucket(max_terms) * r <= 128;
}

// Tile shapes the matrix-core kernel is built for: rows, waves side by side, row groups in flight.
using Shape0 = TileShape<64, 4>;        // 64 x 512, the wave's 16 row groups all in flight
using Shape1 = TileShape<256, 4, 8>;    // 256 x 512, 64 row groups per wave, 8 in flight
using Shape2 = TileShape<128, 4, 16>;   // 128 x 512, 32 row groups per wave, 16 in flight
using Shape3 = TileShape<32, 2>;        // 32 x 256
using Shape4 = TileShape<128, 2>;       // 128 x 256
using Shape5 = TileShape<16, 4>;        // 16 x 512
constexpr int kNumShapes = 6;

template <class F>
bool with_shape(int shape, F &&f)
{
    switch (shape) {
    case 0: return f(Shape0{});
    case 1: return f(Shape1{});
    case 2: return f(Shape2{});
    case 3: return f(Shape3{});
    case 4: return f(Shape4{});
    case 5: return f(Shape5{});
    default: return false;
    }
}

template <int R, int NT, class S>
bool launch_mfma(const SwitchParams &p, int64_t n_tiles, hipStream_t s)
{
    if constexpr (R * NT <= 128 && mfma_shape_fits<R, NT, S>()) {
        hipLaunchKernelGGL((switch_mfma_kernel<R, NT, S>), dim3((unsigned)n_tiles), dim3(256), 0, s, p);
        return true;
    } else {
        return false;
    }
}

template <int R, class S>
bool launch_mfma_r(const SwitchParams &p, int nt, int64_t n_tiles, hipStream_t s)
{
    switch (nt) {
    case 1: return launch_mfma<R, 1, S>(p, n_tiles, s);
    case 2: return launch_mfma<R, 2, S>(p, n_tiles, s);
    case 4: return launch_mfma<R, 4, S>(p, n_tiles, s);
    case 8: return launch_mfma<R, 8, S>(p, n_tiles, s);
    default: return false;
    }
}

template <class S>
bool launch_mfma_any(const SwitchParams &p, int nt, int64_t n_tiles, hipStream_t s)
{
    switch (p.r) {
    case 4: return launch_mfma_r<4, S>(p, nt, n_tiles, s);
    case 8: return launch_mfma_r<8, S>(p, nt, n_tiles, s);
    case 16: return launch_mfma_r<16, S>(p, nt, n_tiles, s);
    case 32: return launch_mfma_r<32, S>(p, nt, n_tiles, s);
    case 64: return launch_mfma_r<64, S>(p, nt, n_tiles, s);
    default: return false;
    }
}

// Which form of the rank-looped kernel runs (rank, term bucket): the unrolled kernel up to
// 7 k-steps of 16 rank indices per tile, the overlapped one (W straight into LDS,
// contraction meanwhile) from 8 on.  ADAFUSE_OPT_GEMM_FORM forces one: 1 = the unrolled
// form wherever it can take the launch, 3 = the overlapped form for short contractions too.
enum GemmForm { kFormUnrolled, kFormOverlap, kFormStrip };

constexpr bool can_unroll(int r, int nt) { return nt <= 2 || (nt == 4 && r <= 16); }  // every row operand fits beside the W tile
constexpr bool can_overlap(int r, int nt) { return nt * ((r + 15) / 16) <= 64; }
constexpr bool can_strip(int r, int nt) { return nt * ((r + 15) / 16) == 8 || nt * ((r + 15) / 16) == 16; }

// forced: ADAFUSE_OPT_GEMM_FORM (0 = by the length of the contraction); strip_ok: the context holds the
// table of tile chains (4-wave workgroups, whole-model launch).
GemmForm pick_gemm_form(int r, int nt, int forced, bool strip_ok)
{
    const int steps = nt * ((r + 15) / 16);
    if (forced == 4 && strip_ok && can_strip(r, nt)) return kFormStrip;
    if (!can_unroll(r, nt)) return kFormOverlap;
    if (!can_overlap(r, nt)) return kFormUnrolled;
    if (forced == 1) return kFormUnrolled;
    if (forced == 3) return kFormOverlap;
    return steps >= 8 ? kFormOverlap : kFormUnrolled;
}

template <int R, int NT, int NW>
bool launch_gemm_form(const SwitchParams &p, GemmForm form, int64_t n_tiles, hipStream_t s)
{
    static_assert(can_unroll(R, NT) || can_overlap(R, NT), "some form takes every (rank, terms)");
    const dim3 grid((unsigned)n_tiles), block(64 * NW);
    switch (form) {
    case kFormStrip:
        if constexpr (can_strip(R, NT) && NW == 4) {
            hipLaunchKernelGGL((switch_gemm_strip_kernel<R, NT>), grid, block, 0, s, p);
            return true;
        }
        break;
    case kFormOverlap:
        if constexpr (can_overlap(R, NT)) {
            hipLaunchKernelGGL((switch_gemm_overlap_kernel<R, NT, NW>), grid, block, 0, s, p);
            return true;
        }
        break;
    case kFormUnrolled:
        if constexpr (can_unroll(R, NT)) {
            hipLaunchKernelGGL((switch_gemm_kernel<R, NT, NW>), grid, block, 0, s, p);
            return true;
        }
        break;
    }
    return false;
}

template <int R, int NW>
bool launch_gemm_rw(const SwitchParams &p, int nt, GemmForm form, int64_t n_tiles, hipStream_t s)
{
    switch (nt) {
    case 1: return launch_gemm_form<R, 1, NW>(p, form, n_tiles, s);
    case 2: return launch_gemm_form<R, 2, NW>(p, form, n_tiles, s);
    case 4: return launch_gemm_form<R, 4, NW>(p, form, n_tiles, s);
    case 8: return launch_gemm_form<R, 8, NW>(p, form, n_tiles, s);
    default: return false;
    }
}

template <int R>
bool launch_gemm_r(const SwitchParams &p, int nt, int waves, GemmForm form, int64_t n_tiles, hipStream_t s)
{
    return waves == 8 ? launch_gemm_rw<R, 8>(p, nt, form, n_tiles, s) : launch_gemm_rw<R, 4>(p, nt, form, n_tiles, s);
}

// nt = term bucket (1, 2, 4 or 8); waves = 4 or 8 per workgroup (tile 64 x 64 waves)
bool launch_gemm(const SwitchParams &p, int nt, int waves, GemmForm form, int64_t n_tiles, hipStream_t s)
{
    switch (p.r) {
    case 4: return launch_gemm_r<4>(p, nt, waves, form, n_tiles, s);
    case 8: return launch_gemm_r<8>(p, nt, waves, form, n_tiles, s);
    case 16: return launch_gemm_r<16>(p, nt, waves, form, n_tiles, s);
    case 32: return launch_gemm_r<32>(p, nt, waves, form, n_tiles, s);
    case 64: return launch_gemm_r<64>(p, nt, waves, form, n_tiles, s);
    case 128: return launch_gemm_r<128>(p, nt, waves, form, n_tiles, s);
    default: return false;
    }
}

// Does the LDS footprint of (r, terms) fit this tile shape?
bool shape_fits(int shape, int r, int nt)
{
    const size_t kr = (size_t)r * nt;
    return with_shape(shape, [&](auto sh) {
        using S = decltype(sh);
        return (size_t)S::TR * (kr + 4) * 2 <= 64 * 1024;
    });
}

// Tile shape of the 4x4x4 kernel for a context: the one asked for (ADAFUSE_OPT_MFMA_SHAPE) if it
// fits, else the default, else the first shape that fits.
int pick_shape(int r, int n_terms, int asked)
{
    const int nt = terms_bucket(n_terms);
    // measured on the Llama-shaped workloads: 64 x 512 tiles stream best; at inner
    // dimension 64 the per-tile operand fetch wants more rows per wave (256 x 512,
    // 8 row groups in flight)
    const int want = asked >= 0 ? asked : (nt * r >= 64 ? 1 : 0);
    if (want >= 0 && want < kNumShapes && shape_fits(want, r, nt)) return want;
    for (int sh = 0; sh < kNumShapes; ++sh)
        if (shape_fits(sh, r, nt)) return sh;
    return 0;
}

// The rank-looped kernel takes any rank that is a multiple of its MFMA depth (16), and 4 or 8 zero-padded to it.
bool gemm_supported(int r) { return host::rank_supported(r); }

// Kernel for AUTO, as measured on the Llama-shaped workloads: the rank-looped
// 32x32x16 form is the fastest at every rank (80% of the HBM peak against 79% for
// the 4x4x4 form at rank 8, and far ahead once the inner dimension passes 64).
int32_t auto_kernel(int r, int n_terms)
{
    if (gemm_supported(r)) return ADAFUSE_KERNEL_GEMM;
    if (mfma_supported(r, n_terms)) return ADAFUSE_KERNEL_MFMA;
    return ADAFUSE_KERNEL_VALU;
}

// The tables live on the device that was current at adafuse_create; a launch
// from another device would hand the kernels pointers they cannot use.
bool on_ctx_device(const adafuse_ctx *c)
{
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == c->device;
}

// Largest term count a launch of this context can carry.
int max_terms(const adafuse_ctx *c) { return c->inplace ? 2 * c->k_max : c->k_max; }

void free_tables(adafuse_ctx *c)
{
    if (c->d_mats) (void)hipFree(c->d_mats);
    if (c->d_tiles) (void)hipFree(c->d_tiles);
    if (c->d_tall) (void)hipFree(c->d_tall);
    c->d_mats = nullptr;
    c->d_tiles = nullptr;
    c->d_tall = nullptr;
    c->n_tall = 0;
}

// Waves per workgroup of the rank-looped kernel when the caller leaves the choice to the library:
// 8 (1 KB row pieces) where most of the weights sit at row pitches that are not a power of two
// AND every launch of the context runs the unrolled form (the 8-wave overlapped form does not
// fit three workgroups per CU); else 4 (512-byte pieces).  Measured on the Llama-2-13B shapes
// (pitches 10240 and 27648 bytes): 8 waves +2.6 %; on the 7B shapes (8192 and 22016): -1.5 %.
int auto_gemm_waves(const adafuse_ctx *c)
{
    const int nt = terms_bucket(max_terms(c));
    if (pick_gemm_form(c->r, nt, c->opt_form, false) != kFormUnrolled) return 4;
    return host::odd_pitch_share(c->mats) > 0.75 ? 8 : 4;
}

// Builds the tables for `kernel` with the context's options and uploads them.
adafuse_status build_tables(adafuse_ctx *c, int32_t kernel)
{
    // everything is built aside and handed to the context at the end: a failure leaves it as it was
    host::TablePlan plan;
    plan.tile_rows = kValuTileRows;
    plan.tile_cols = kValuTileCols;
    int mfma_shape = c->mfma_shape, gemm_waves = c->gemm_waves;
    if (kernel == ADAFUSE_KERNEL_MFMA) {
        mfma_shape = pick_shape(c->r, max_terms(c), c->opt_mfma_shape);
        with_shape(mfma_shape, [&](auto sh) {
            plan.tile_rows = decltype(sh)::TR;
            plan.tile_cols = decltype(sh)::TC;
            return true;
        });
    } else if (kernel == ADAFUSE_KERNEL_GEMM) {
        gemm_waves = c->opt_waves == 4 || c->opt_waves == 8 ? c->opt_waves : auto_gemm_waves(c);
        plan.tile_rows = kGemmTileRows;
        plan.tile_cols = kGemmWaveCols * gemm_waves;
    }
    plan.inner = (size_t)max_terms(c) * c->r;
    plan.panel_bytes = (size_t)std::max(1, c->opt_panel_kb) * 1024;
    plan.xcd_run = c->opt_xcd_run;
    host::Tables t, tall;
    if (!host::build_tile_tables(c->mats, plan, t)) return ADAFUSE_ERR_SHAPE;
    const bool want_tall = kernel == ADAFUSE_KERNEL_GEMM && gemm_waves == 4;
    if (want_tall) {  // the same walk in chains of kStripTiles tiles
        host::TablePlan tp = plan;
        tp.tile_rows = kStripRows;
        if (!host::build_tile_tables(c->mats, tp, tall)) return ADAFUSE_ERR_SHAPE;
    }

    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return ADAFUSE_ERR_HIP;
    void *scratch_ptr = nullptr;  // each GPU holds its own copy of the array, at its own address
    if (hipGetSymbolAddress(&scratch_ptr, HIP_SYMBOL(scratch)) != hipSuccess || !scratch_ptr) return ADAFUSE_ERR_HIP;
    MatDev *dm = nullptr;
    TileDev *dt = nullptr;
    if (hipMalloc(&dm, t.mats.size() * sizeof(MatDev)) != hipSuccess) return ADAFUSE_ERR_HIP;
    if (hipMalloc(&dt, t.tiles.size() * sizeof(TileDev)) != hipSuccess) {
        (void)hipFree(dm);
        return ADAFUSE_ERR_HIP;
    }
    TileDev *dtall = nullptr;
    if (want_tall && hipMalloc(&dtall, (size_t)tall.n_tiles * sizeof(TileDev)) != hipSuccess) {
        (void)hipFree(dm);
        (void)hipFree(dt);
        return ADAFUSE_ERR_HIP;
    }
    if (hipMemcpy(dm, t.mats.data(), t.mats.size() * sizeof(MatDev), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(dt, t.tiles.data(), t.tiles.size() * sizeof(TileDev), hipMemcpyHostToDevice) != hipSuccess ||
        (want_tall && hipMemcpy(dtall, tall.tiles.data(), (size_t)tall.n_tiles * sizeof(TileDev), hipMemcpyHostToDevice) != hipSuccess)) {
        (void)hipFree(dm);
        (void)hipFree(dt);
        if (dtall) (void)hipFree(dtall);
        return ADAFUSE_ERR_HIP;
    }
    free_tables(c);
    c->d_mats = dm;
    c->d_tiles = dt;
    c->d_tall = dtall;
    c->n_tall = want_tall ? tall.n_tiles : 0;
    c->device = device;
    c->scratch = static_cast<float *>(scratch_ptr);
    c->kernel = kernel;
    c->mfma_shape = mfma_shape;
    c->gemm_waves = gemm_waves;
    c->tile_rows = plan.tile_rows;
    c->tile_cols = plan.tile_cols;
    c->n_tiles = t.n_tiles;
    c->mat_tile_off.swap(t.mat_off);
    c->elements = t.elements;
    return ADAFUSE_OK;
}

}  // namespace

extern "C" {

adafuse_status adafuse_create(const adafuse_matrix_desc *mats, int32_t n_mats, int32_t E, int32_t r, int32_t k_max,
                              adafuse_ctx **ctx)
{
    if (!ctx) return ADAFUSE_ERR_NULL;
    *ctx = nullptr;
    adafuse_status st = host::validate_mats(mats, n_mats, E, r, k_max);
    if (st != ADAFUSE_OK) return st;
    adafuse_ctx *c = new (std::nothrow) adafuse_ctx();
    if (!c) return ADAFUSE_ERR_HIP;
    try {  // the host tables are std::vectors: no exception may cross the C boundary
        c->mats.assign(mats, mats + n_mats);
        c->E = E;
        c->r = r;
        c->k_max = k_max;
        c->inplace = mats[0].w_base == mats[0].w_work;
        st = build_tables(c, auto_kernel(r, max_terms(c)));
    } catch (...) {
        st = ADAFUSE_ERR_HIP;
    }
    if (st != ADAFUSE_OK) {
        free_tables(c);
        delete c;
        return st;
    }
    *ctx = c;
    return ADAFUSE_OK;
}

adafuse_status adafuse_destroy(adafuse_ctx *ctx)
{
    if (!ctx) return ADAFUSE_OK;
    free_tables(ctx);
    delete ctx;
    return ADAFUSE_OK;
}

adafuse_status adafuse_set_option(adafuse_ctx *ctx, int32_t option, int32_t value)
{
    if (!ctx) return ADAFUSE_ERR_NULL;
    int32_t kernel = ctx->kernel;
    adafuse_ctx saved_opts;  // only the option fields are used
    saved_opts.opt_waves = ctx->opt_waves;
    saved_opts.opt_form = ctx->opt_form;
    saved_opts.opt_xcd_run = ctx->opt_xcd_run;
    saved_opts.opt_panel_kb = ctx->opt_panel_kb;
    saved_opts.opt_mfma_shape = ctx->opt_mfma_shape;
    switch (option) {
    case ADAFUSE_OPT_KERNEL:
        kernel = value == ADAFUSE_KERNEL_AUTO ? auto_kernel(ctx->r, max_terms(ctx)) : value;
        if (kernel != ADAFUSE_KERNEL_VALU && kernel != ADAFUSE_KERNEL_MFMA && kernel != ADAFUSE_KERNEL_GEMM)
            return ADAFUSE_ERR_ARG;
        if (kernel == ADAFUSE_KERNEL_MFMA && !mfma_supported(ctx->r, max_terms(ctx))) return ADAFUSE_ERR_ARG;
        if (kernel == ADAFUSE_KERNEL_GEMM && !gemm_supported(ctx->r)) return ADAFUSE_ERR_ARG;
        if (kernel == ctx->kernel) return ADAFUSE_OK;
        break;
    case ADAFUSE_OPT_GEMM_WAVES:
        if (value != 0 && value != 4 && value != 8) return ADAFUSE_ERR_ARG;
        ctx->opt_waves = value;
        break;
    case ADAFUSE_OPT_GEMM_FORM:
        if (value != 0 && value != 1 && value != 3 && value != 4) return ADAFUSE_ERR_ARG;
        ctx->opt_form = value;
        break;
    case ADAFUSE_OPT_XCD_RUN:
        if (value < 0) return ADAFUSE_ERR_ARG;
        ctx->opt_xcd_run = value;
        break;
    case ADAFUSE_OPT_PANEL_KB:
        if (value < 1) return ADAFUSE_ERR_ARG;
        ctx->opt_panel_kb = value;
        break;
    case ADAFUSE_OPT_MFMA_SHAPE:
        if (value < -1 || value >= kNumShapes) return ADAFUSE_ERR_ARG;
        ctx->opt_mfma_shape = value;
        break;
    default: return ADAFUSE_ERR_ARG;
    }
    adafuse_status st = ADAFUSE_ERR_ARG;
    if (on_ctx_device(ctx)) {
        st = ADAFUSE_ERR_HIP;
        if (hipDeviceSynchronize() == hipSuccess) {  // no launch may still read the old table
            try {
                st = build_tables(ctx, kernel);
            } catch (...) {
                st = ADAFUSE_ERR_HIP;
            }
        }
    }
    if (st != ADAFUSE_OK) {  // the context keeps the kernel, tables and options it had
        ctx->opt_waves = saved_opts.opt_waves;
        ctx->opt_form = saved_opts.opt_form;
        ctx->opt_xcd_run = saved_opts.opt_xcd_run;
        ctx->opt_panel_kb = saved_opts.opt_panel_kb;
        ctx->opt_mfma_shape = saved_opts.opt_mfma_shape;
    }
    return st;
}

adafuse_status adafuse_get_info(const adafuse_ctx *ctx, adafuse_info *info)
{
    if (!ctx || !info) return ADAFUSE_ERR_NULL;
    info->n_mats = (int32_t)ctx->mats.size();
    info->E = ctx->E;
    info->r = ctx->r;
    info->k_max = ctx->k_max;
    info->kernel = ctx->kernel;
    info->tile_rows = ctx->tile_rows;
    info->tile_cols = ctx->tile_cols;
    info->reserved = 0;
    info->n_tiles = ctx->n_tiles;
    info->elements = ctx->elements;
    return ADAFUSE_OK;
}

adafuse_status adafuse_pregate(const void *hidden, const void *w_router, int32_t T, int32_t d, int32_t E, int32_t k,
                               int32_t gate_norm, int32_t *idx, float *gates, float *logits, void *hip_stream)
{
    if (!hidden || !w_router || !idx || !gates) return ADAFUSE_ERR_NULL;
    if (T < 0 || E < 1 || E > kMaxExperts || k < 1 || k > E || k > kMaxTopK) return ADAFUSE_ERR_ARG;
    if (gate_norm != ADAFUSE_GATE_SOFTMAX_OVER_TOPK && gate_norm != ADAFUSE_GATE_TOPK_OF_SOFTMAX) return ADAFUSE_ERR_ARG;
    if (d < 8 || (d % 8) != 0) return ADAFUSE_ERR_SHAPE;
    if (!aligned16(hidden) || !aligned16(w_router)) return ADAFUSE_ERR_ALIGN;
    if (T == 0) return ADAFUSE_OK;
    PregateParams p{static_cast<const uint16_t *>(hidden), static_cast<const uint16_t *>(w_router), idx, gates, logits,
                    T, d, E, k, gate_norm};
    hipLaunchKernelGGL(pregate_kernel, dim3((unsigned)T), dim3(256), 0, static_cast<hipStream_t>(hip_stream), p);
    return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
}

namespace {

// Argument checks shared by the two switch entry points, then one launch per
// entry of `ranges` (offset, count) into the tile table.
adafuse_status switch_launches(adafuse_ctx *ctx, const int32_t *idx_prev, const float *gates_prev,
                               const int32_t *idx_next, const float *gates_next, int32_t k, float scale,
                               int32_t mode, void *hip_stream, bool per_matrix)
{
    if (!ctx) return ADAFUSE_ERR_NULL;
    if (mode != ADAFUSE_MERGE && mode != ADAFUSE_UNMERGE && mode != ADAFUSE_SWAP) return ADAFUSE_ERR_ARG;
    const bool need_next = mode != ADAFUSE_UNMERGE;
    const bool need_prev = ctx->inplace && mode != ADAFUSE_MERGE;  // in place, removing a merge is arithmetic
    if (need_next && (!idx_next || !gates_next)) return ADAFUSE_ERR_NULL;
    if (need_prev && (!idx_prev || !gates_prev)) return ADAFUSE_ERR_NULL;
    if ((idx_prev == nullptr) != (gates_prev == nullptr)) return ADAFUSE_ERR_NULL;
    if ((need_next || need_prev) && (k < 1 || k > ctx->k_max)) return ADAFUSE_ERR_ARG;
    if (!on_ctx_device(ctx)) return ADAFUSE_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool copy_only = !ctx->inplace && mode == ADAFUSE_UNMERGE;
    const int n_terms = (need_prev ? k : 0) + (need_next ? k : 0);
    const size_t valu_lds = valu_lds_bytes(n_terms * ctx->r);
    if (ctx->kernel == ADAFUSE_KERNEL_VALU && valu_lds > 64 * 1024) return ADAFUSE_ERR_ARG;  // terms*r too large to stage

    const size_t n_launches = per_matrix ? ctx->mats.size() : 1;
    for (size_t i = 0; i < n_launches; ++i) {
        const int64_t first = per_matrix ? ctx->n_tiles + ctx->mat_tile_off[i] : 0;
        const int64_t count = per_matrix ? ctx->mat_tile_off[i + 1] - ctx->mat_tile_off[i] : ctx->n_tiles;
        if (count == 0) continue;
        SwitchParams p{ctx->d_mats, ctx->d_tiles + first, idx_prev, gates_prev, idx_next, gates_next,
                       copy_only ? 0 : k, ctx->E, ctx->r, mode, scale, ctx->inplace ? 1 : 0};
        if (ctx->kernel == ADAFUSE_KERNEL_MFMA) {
            const bool launched = with_shape(ctx->mfma_shape, [&](auto sh) {
                using S = decltype(sh);
                if (copy_only) {
                    hipLaunchKernelGGL((switch_copy_kernel<S>), dim3((unsigned)count), dim3(256), 0, s, p);
                    return true;
                }
                return launch_mfma_any<S>(p, terms_bucket(n_terms), count, s);
            });
            if (!launched) return ADAFUSE_ERR_ARG;
        } else if (ctx->kernel == ADAFUSE_KERNEL_GEMM) {
            // the copy (nothing selected) runs through the one-term instance of the unrolled form: there is
            // nothing to overlap, and W first, through registers, is the faster copy
            const int nt = terms_bucket(n_terms > 0 ? n_terms : 1);
            GemmForm form = copy_only ? kFormUnrolled : pick_gemm_form(ctx->r, nt, ctx->opt_form, !per_matrix && ctx->d_tall != nullptr);
            if (form == kFormStrip) {  // its own table: the whole model in chains of vertically adjacent tiles
                p.tiles = ctx->d_tall;
                if (!launch_gemm(p, nt, 4, form, ctx->n_tall, s)) return ADAFUSE_ERR_ARG;
            } else if (!launch_gemm(p, nt, ctx->gemm_waves, form, count, s)) {
                return ADAFUSE_ERR_ARG;
            }
        } else {
            hipLaunchKernelGGL(switch_valu_kernel, dim3((unsigned)count), dim3(256), valu_lds, s, p);
        }
    }
    return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
}

}  // namespace

adafuse_status adafuse_fused_switch(adafuse_ctx *ctx, const int32_t *idx_prev, const float *gates_prev,
                                    const int32_t *idx_next, const float *gates_next, int32_t k, float scale,
                                    int32_t mode, void *hip_stream)
{
    return switch_launches(ctx, idx_prev, gates_prev, idx_next, gates_next, k, scale, mode, hip_stream, false);
}

adafuse_status adafuse_switch_per_matrix(adafuse_ctx *ctx, const int32_t *idx_prev, const float *gates_prev,
                                         const int32_t *idx_next, const float *gates_next, int32_t k, float scale,
                                         int32_t mode, void *hip_stream)
{
    return switch_launches(ctx, idx_prev, gates_prev, idx_next, gates_next, k, scale, mode, hip_stream, true);
}

adafuse_status adafuse_forward_merged(adafuse_ctx *ctx, const void *x, float *y, void *hip_stream)
{
    if (!ctx || !x || !y) return ADAFUSE_ERR_NULL;
    if (!aligned16(x)) return ADAFUSE_ERR_ALIGN;
    if (!on_ctx_device(ctx)) return ADAFUSE_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint16_t *xp = static_cast<const uint16_t *>(x);
    for (const adafuse_matrix_desc &m : ctx->mats) {
        hipLaunchKernelGGL(gemv_rows_kernel, dim3((unsigned)((m.out + 3) / 4)), dim3(256), 0, s,
                           static_cast<const uint16_t *>(m.w_work), (int64_t)m.ldw, xp, y, m.out, m.in);
        xp += m.in;
        y += m.out;
    }
    return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
}

namespace {

adafuse_status forward_dynamic_launches(adafuse_ctx *ctx, const int32_t *idx_host, const float *gates_host, int32_t k,
                                        float scale, const void *x, float *y, float *z, void *hip_stream)
{
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint16_t *xp = static_cast<const uint16_t *>(x);
    const int r = ctx->r;
    for (const adafuse_matrix_desc &m : ctx->mats) {
        hipLaunchKernelGGL(gemv_rows_kernel, dim3((unsigned)((m.out + 3) / 4)), dim3(256), 0, s,
                           static_cast<const uint16_t *>(m.w_base), (int64_t)m.ldw, xp, y, m.out, m.in);
        for (int j = 0; j < k; ++j) {
            const uint16_t *a = static_cast<const uint16_t *>(m.a_bank) + (size_t)idx_host[j] * r * m.in;
            const uint16_t *b = static_cast<const uint16_t *>(m.b_bank) + (size_t)idx_host[j] * m.out * r;
            hipLaunchKernelGGL(gemv_rows_kernel, dim3((unsigned)((r + 3) / 4)), dim3(256), 0, s, a, (int64_t)m.in, xp,
                               z + (size_t)j * r, r, m.in);
            hipLaunchKernelGGL(lora_up_kernel, dim3((unsigned)((m.out + 255) / 256)), dim3(256), 0, s, b,
                               z + (size_t)j * r, y, m.out, r, scale * gates_host[j]);
        }
        xp += m.in;
        y += m.out;
    }
    return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
}

adafuse_status forward_dynamic_checks(adafuse_ctx *ctx, const int32_t *idx_host, const float *gates_host, int32_t k,
                                      const void *x, float *y)
{
    if (!ctx || !idx_host || !gates_host || !x || !y) return ADAFUSE_ERR_NULL;
    if (k < 1 || k > ctx->k_max) return ADAFUSE_ERR_ARG;
    for (int j = 0; j < k; ++j)
        if (idx_host[j] < 0 || idx_host[j] >= ctx->E) return ADAFUSE_ERR_ARG;
    if (ctx->inplace) return ADAFUSE_ERR_ARG;  // needs the unmodified base weights
    if (!aligned16(x)) return ADAFUSE_ERR_ALIGN;
    if (!on_ctx_device(ctx)) return ADAFUSE_ERR_ARG;
    return ADAFUSE_OK;
}

}  // namespace

adafuse_status adafuse_forward_dynamic(adafuse_ctx *ctx, const int32_t *idx_host, const float *gates_host, int32_t k,
                                       float scale, const void *x, float *y, float *z, void *hip_stream)
{
    if (!z) return ADAFUSE_ERR_NULL;
    const adafuse_status st = forward_dynamic_checks(ctx, idx_host, gates_host, k, x, y);
    if (st != ADAFUSE_OK) return st;
    return forward_dynamic_launches(ctx, idx_host, gates_host, k, scale, x, y, z, hip_stream);
}

adafuse_status adafuse_forward_dynamic_static(adafuse_ctx *ctx, const int32_t *idx_host, const float *gates_host,
                                              int32_t k, float scale, const void *x, float *y, void *hip_stream)
{
    const adafuse_status st = forward_dynamic_checks(ctx, idx_host, gates_host, k, x, y);
    if (st != ADAFUSE_OK) return st;
    if ((int64_t)k * ctx->r > kScratchFloats) return ADAFUSE_ERR_ARG;  // beyond the built-in scratch
    // every entry of z that a launch reads was written by the launch before it on the same stream:
    // nothing of the previous call's contents is used, nothing has to be cleared
    return forward_dynamic_launches(ctx, idx_host, gates_host, k, scale, x, y, ctx->scratch, hip_stream);
}

namespace {

// How one product of adafuse_prefill is cut: tiles of 128 tokens x 256 rows, and the inner dimension in
// `splits` parts of `chunks_per_split` chunks of 64, so that a launch has at least one workgroup per CU
// (one is resident at a time: 144 KB of LDS).  Every part costs T x rows x 8 bytes of traffic on top.
struct PrefillCut {
    int m_tiles, strips, splits, chunks_per_split;
};

PrefillCut prefill_cut(int T, int rows, int in)
{
    PrefillCut c;
    c.m_tiles = (T + kPfTileTokens - 1) / kPfTileTokens;
    c.strips = (rows + kPfTileRows - 1) / kPfTileRows;
    const int chunks = (in + kPfChunk - 1) / kPfChunk;
    // as many parts as still give at most one workgroup per CU (256): one more workgroup than CUs is a
    // second round for the whole launch; at least two chunks per part
    int want = 256 / (c.m_tiles * c.strips);
    want = std::max(1, std::min(want, std::min(kPfMaxSplits, chunks / 2)));
    c.chunks_per_split = (chunks + want - 1) / want;
    c.splits = (chunks + c.chunks_per_split - 1) / c.chunks_per_split;       // no empty part
    return c;
}

// Two forms.  FEW tokens (at most four token tiles and little adapter work, see below): the bank products and the base products of ALL
// matrices of the group share ONE launch, cut into the same number of parts so that their workgroups
// take equally long, and a second kernel sums the parts and adds the adapters in fp32 -- two launches
// for the group, no bf16 pair, no dependent chain of four small kernels per matrix (at a hundred tokens a
// launch costs more than streaming a 4096 x 4096 matrix).  MANY tokens: matrix by matrix, the adapters
// as further inner dimension of the base product on the matrix cores (bank product, gate kernel, base
// product, sum of the parts if there are any).
constexpr int kPfFewTiles = 4;
// ... and T k r at most this: the second kernel of the few-token form adds the adapters on the vector ALU
// and re-reads the selected B rows for every token, which grows with T k r; measured on the 7B / 8B / 13B
// shapes at ranks 8 to 128, the two forms cross between T k r = 6400 and 12800
constexpr int64_t kPfFewWork = 8192;
inline int prefill_units8(int units) { return ((units + 7) / 8) * 8; }

struct PrefillPlan {
    bool few;
    int n;
    // few-token form: one cut for every product of the group
    int m_tiles, splits, chunks_per_split, bank_strips;
    int strips[kPfMaxGroup];
    uint64_t u_bytes;                 // one bank product's parts (16-byte multiple)
    uint64_t w_bytes[kPfMaxGroup];    // one base product's parts
    // many-token form, per matrix
    PrefillCut down[kPfMaxGroup], up[kPfMaxGroup];
    int rp;
    uint64_t plane;        // bytes of one bf16 plane of the scaled down-projections
    uint64_t parts_bytes;  // fp32 parts (the two passes and all matrices of the group share the space)
    uint64_t total() const
    {
        if (!few) return 2 * plane + parts_bytes;
        uint64_t t = 0;
        for (int i = 0; i < n; ++i) t += u_bytes + w_bytes[i];
        return t;
    }
};

PrefillPlan prefill_plan(const adafuse_ctx *ctx, const int32_t *mats, int n, int T, int k)
{
    PrefillPlan pl{};
    pl.n = n;
    const int bank_rows = ctx->E * ctx->r;
    const int in = ctx->mats[(size_t)mats[0]].in;
    pl.m_tiles = (T + kPfTileTokens - 1) / kPfTileTokens;
    pl.few = pl.m_tiles <= kPfFewTiles && (int64_t)T * k * ctx->r <= kPfFewWork;
    if (pl.few) {
        pl.bank_strips = (bank_rows + kPfTileRows - 1) / kPfTileRows;
        int total_strips = 0;
        for (int i = 0; i < n; ++i) {
            pl.strips[i] = (ctx->mats[(size_t)mats[i]].out + kPfTileRows - 1) / kPfTileRows;
            total_strips += pl.strips[i] + pl.bank_strips;
        }
        const int chunks = (in + kPfChunk - 1) / kPfChunk;
        // as many parts as keep ALL products in one wave of workgroups (one is resident per CU; a single
        // workgroup more is a second round for the launch), counted the way the launch rounds each
        // product's workgroups up to the 8 XCDs
        int want = std::max(1, std::min(256 / (total_strips * pl.m_tiles), std::min(kPfMaxSplits, chunks / 2)));
        for (;; --want) {
            pl.chunks_per_split = (chunks + want - 1) / want;
            pl.splits = (chunks + pl.chunks_per_split - 1) / pl.chunks_per_split;
            int grid = 0;
            for (int i = 0; i < n; ++i)
                grid += (prefill_units8(pl.strips[i] * pl.splits) + prefill_units8(pl.bank_strips * pl.splits)) * pl.m_tiles;
            if (grid <= 256 || want == 1) break;
        }
        pl.u_bytes = ((uint64_t)pl.splits * T * bank_rows * 4u + 15u) & ~15ull;
        for (int i = 0; i < n; ++i)
            pl.w_bytes[i] = ((uint64_t)pl.splits * T * ctx->mats[(size_t)mats[i]].out * 4u + 15u) & ~15ull;
        return pl;
    }
    pl.rp = ctx->r < 8 ? 8 : ctx->r;  // a slot holds whole 16-byte pieces
    pl.plane = ((uint64_t)T * (uint64_t)k * (uint64_t)pl.rp * 2u + 15u) & ~15ull;
    for (int i = 0; i < n; ++i) {
        const adafuse_matrix_desc &m = ctx->mats[(size_t)mats[i]];
        pl.down[i] = prefill_cut(T, bank_rows, m.in);
        pl.up[i] = prefill_cut(T, m.out, m.in);
        const uint64_t down_parts = (uint64_t)pl.down[i].splits * T * bank_rows * 4u;   // U is always a temporary
        const uint64_t up_parts = pl.up[i].splits > 1 ? (uint64_t)pl.up[i].splits * T * m.out * 4u : 0u;
        pl.parts_bytes = std::max(pl.parts_bytes, std::max(down_parts, up_parts));
    }
    return pl;
}

adafuse_status prefill_group_checks(const adafuse_ctx *ctx, const int32_t *mats, int32_t n, int32_t T, int32_t k)
{
    if (!ctx || !mats) return ADAFUSE_ERR_NULL;
    if (n < 1 || n > kPfMaxGroup || T < 0 || k < 1 || k > ctx->k_max) return ADAFUSE_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        if (mats[i] < 0 || mats[i] >= (int32_t)ctx->mats.size()) return ADAFUSE_ERR_ARG;
        if (ctx->mats[(size_t)mats[i]].in != ctx->mats[(size_t)mats[0]].in) return ADAFUSE_ERR_SHAPE;  // one X for all
        for (int j = 0; j < i; ++j)
            if (mats[j] == mats[i]) return ADAFUSE_ERR_ARG;
    }
    return ADAFUSE_OK;
}

}  // namespace

adafuse_status adafuse_prefill_group_workspace_bytes(const adafuse_ctx *ctx, const int32_t *mats, int32_t n, int32_t T,
                                                     int32_t k, size_t *bytes)
{
    if (!bytes) return ADAFUSE_ERR_NULL;
    const adafuse_status st = prefill_group_checks(ctx, mats, n, T, k);
    if (st != ADAFUSE_OK) return st;
    *bytes = T == 0 ? 0 : (size_t)prefill_plan(ctx, mats, n, T, k).total();
    return ADAFUSE_OK;
}

adafuse_status adafuse_prefill_workspace_bytes(const adafuse_ctx *ctx, int32_t mat, int32_t T, int32_t k, size_t *bytes)
{
    return adafuse_prefill_group_workspace_bytes(ctx, &mat, 1, T, k, bytes);
}

adafuse_status adafuse_prefill_group(adafuse_ctx *ctx, const int32_t *mats, int32_t n, const void *x, int32_t T,
                                     const int32_t *idx, const float *gates, int32_t k, float scale, float *const *y,
                                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const adafuse_status st = prefill_group_checks(ctx, mats, n, T, k);
    if (st != ADAFUSE_OK) return st;
    if (ctx->inplace) return ADAFUSE_ERR_ARG;  // needs the unmodified base weights
    if (T == 0) return ADAFUSE_OK;             // no tokens: nothing to read or write
    if (!x || !idx || !gates || !y || !workspace) return ADAFUSE_ERR_NULL;
    if (!aligned16(x) || !aligned16(workspace)) return ADAFUSE_ERR_ALIGN;
    for (int i = 0; i < n; ++i) {
        if (!y[i]) return ADAFUSE_ERR_NULL;
        if (!aligned16(y[i])) return ADAFUSE_ERR_ALIGN;
    }
    const PrefillPlan pl = prefill_plan(ctx, mats, n, T, k);
    if (workspace_bytes < pl.total()) return ADAFUSE_ERR_ARG;
    const int in = ctx->mats[(size_t)mats[0]].in;
    // the kernels address X and the workspace planes through 32-bit descriptors and offsets
    if ((uint64_t)T * (uint64_t)in * 2u >= (1ull << 31) || pl.plane >= (1ull << 31)) return ADAFUSE_ERR_SHAPE;
    if (!on_ctx_device(ctx)) return ADAFUSE_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint16_t *xp = static_cast<const uint16_t *>(x);
    const int bank_rows = ctx->E * ctx->r;
    auto grid_of = [](int strips, int splits, int m_tiles) { return prefill_units8(strips * splits) * m_tiles; };
    auto close_batch = [](PrefillBatch &b, int used) {
        for (int j = used; j < kPfMaxProducts; ++j) b.end[j] = b.end[used - 1];
    };

    if (pl.few) {
        // 1. every X W^T and every U = X A^T (whole bank), in parts, one launch
        PrefillBatch batch{};
        PrefillFinishBatch fin{};
        char *at = static_cast<char *>(workspace);
        int grid = 0;
        for (int i = 0; i < n; ++i) {
            const adafuse_matrix_desc &m = ctx->mats[(size_t)mats[i]];
            float *u_parts = reinterpret_cast<float *>(at);
            float *w_parts = reinterpret_cast<float *>(at + pl.u_bytes);
            at += pl.u_bytes + pl.w_bytes[i];
            batch.g[2 * i] = PrefillGemm{static_cast<const uint16_t *>(m.w_base), xp, w_parts, m.out, m.ldw, m.in, T,
                                         pl.splits, pl.chunks_per_split, pl.m_tiles, pl.strips[i],
                                         nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0};
            grid += grid_of(pl.strips[i], pl.splits, pl.m_tiles);
            batch.end[2 * i] = grid;
            batch.g[2 * i + 1] = PrefillGemm{static_cast<const uint16_t *>(m.a_bank), xp, u_parts, bank_rows, m.in, m.in, T,
                                             pl.splits, pl.chunks_per_split, pl.m_tiles, pl.bank_strips,
                                             nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0};
            grid += grid_of(pl.bank_strips, pl.splits, pl.m_tiles);
            batch.end[2 * i + 1] = grid;
            fin.f[i] = PrefillFinish{w_parts, u_parts, static_cast<const uint16_t *>(m.b_bank), idx, gates, y[i],
                                     T, m.out, ctx->E, ctx->r, k, pl.splits, scale};
        }
        close_batch(batch, 2 * n);
        hipLaunchKernelGGL(prefill_gemm_kernel, dim3((unsigned)grid), dim3(256), 0, s, batch);
        // 2. parts summed, adapters added
        int max_out = 0;
        for (int i = 0; i < n; ++i) max_out = std::max(max_out, ctx->mats[(size_t)mats[i]].out);
        for (int i = n; i < kPfMaxGroup; ++i) fin.f[i] = fin.f[0];
        const dim3 fin_grid((unsigned)((max_out + 1023) / 1024), (unsigned)T, (unsigned)n);
        if (pl.splits <= 2) hipLaunchKernelGGL(prefill_finish_kernel<2>, fin_grid, dim3(256), 0, s, fin);
        else if (pl.splits <= 4) hipLaunchKernelGGL(prefill_finish_kernel<4>, fin_grid, dim3(256), 0, s, fin);
        else if (pl.splits <= 8) hipLaunchKernelGGL(prefill_finish_kernel<8>, fin_grid, dim3(256), 0, s, fin);
        else if (pl.splits <= 16) hipLaunchKernelGGL(prefill_finish_kernel<16>, fin_grid, dim3(256), 0, s, fin);
        else hipLaunchKernelGGL(prefill_finish_kernel<kPfMaxSplits>, fin_grid, dim3(256), 0, s, fin);
        return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
    }

    uint16_t *z_hi = static_cast<uint16_t *>(workspace);
    uint16_t *z_lo = z_hi + pl.plane / 2;
    float *parts = reinterpret_cast<float *>(z_lo + pl.plane / 2);
    for (int i = 0; i < n; ++i) {
        const adafuse_matrix_desc &m = ctx->mats[(size_t)mats[i]];
        const PrefillCut &dc = pl.down[i], &uc = pl.up[i];
        // 1. U = X A^T over the whole bank, in parts
        PrefillBatch down{};
        down.g[0] = PrefillGemm{static_cast<const uint16_t *>(m.a_bank), xp, parts, bank_rows, m.in, m.in, T,
                                dc.splits, dc.chunks_per_split, dc.m_tiles, dc.strips,
                                nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0};
        down.end[0] = grid_of(dc.strips, dc.splits, dc.m_tiles);
        close_batch(down, 1);
        hipLaunchKernelGGL(prefill_gemm_kernel, dim3((unsigned)down.end[0]), dim3(256), 0, s, down);
        // 2. the selected experts' columns, scaled by s g, as bf16 pairs
        PrefillGate gate{parts, idx, gates, z_hi, z_lo, T, ctx->E, ctx->r, pl.rp, k, dc.splits, scale};
        const int64_t n_z = (int64_t)T * k * pl.rp;
        hipLaunchKernelGGL(prefill_gate_kernel, dim3((unsigned)((n_z + 255) / 256)), dim3(256), 0, s, gate);
        // 3. X W^T with the adapters as further inner dimension; 4. its parts summed
        PrefillBatch up{};
        up.g[0] = PrefillGemm{static_cast<const uint16_t *>(m.w_base), xp, uc.splits > 1 ? parts : y[i], m.out, m.ldw, m.in, T,
                              uc.splits, uc.chunks_per_split, uc.m_tiles, uc.strips,
                              static_cast<const uint16_t *>(m.b_bank), idx, z_hi, z_lo, ctx->E, ctx->r, pl.rp, k};
        up.end[0] = grid_of(uc.strips, uc.splits, uc.m_tiles);
        close_batch(up, 1);
        hipLaunchKernelGGL(prefill_gemm_kernel, dim3((unsigned)up.end[0]), dim3(256), 0, s, up);
        if (uc.splits > 1) {
            const int64_t n_y = (int64_t)T * m.out;
            hipLaunchKernelGGL(prefill_sum_kernel, dim3((unsigned)((n_y + 1023) / 1024)), dim3(256), 0, s, parts, y[i], n_y, uc.splits);
        }
    }
    return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
}

adafuse_status adafuse_prefill(adafuse_ctx *ctx, int32_t mat, const void *x, int32_t T, const int32_t *idx,
                               const float *gates, int32_t k, float scale, float *y, void *workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    float *ys[1] = {y};
    if (ctx && !y && T != 0) return ADAFUSE_ERR_NULL;
    return adafuse_prefill_group(ctx, &mat, 1, x, T, idx, gates, k, scale, ys, workspace, workspace_bytes, hip_stream);
}

adafuse_status adafuse_hbm_probe(adafuse_ctx *ctx, int32_t direction, void *hip_stream)
{
    if (!ctx) return ADAFUSE_ERR_NULL;
    if (direction != ADAFUSE_PROBE_READ_BASE && direction != ADAFUSE_PROBE_ZERO_WORK) return ADAFUSE_ERR_ARG;
    if (ctx->inplace && direction == ADAFUSE_PROBE_ZERO_WORK) return ADAFUSE_ERR_ARG;  // would erase the only copy of W
    if (!on_ctx_device(ctx)) return ADAFUSE_ERR_ARG;
    if (ctx->n_tiles == 0) return ADAFUSE_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int pieces = ctx->tile_rows * ctx->tile_cols / 8;
    uint32_t *sink = reinterpret_cast<uint32_t *>(ctx->scratch + kScratchFloats);
    const dim3 grid((unsigned)ctx->n_tiles), block(256);
    auto launch = [&](auto pt) {
        constexpr int PT = decltype(pt)::value;
        if (direction == ADAFUSE_PROBE_ZERO_WORK)
            hipLaunchKernelGGL((hbm_probe_kernel<PT, true>), grid, block, 0, s, ctx->d_tiles, ctx->tile_cols, sink);
        else
            hipLaunchKernelGGL((hbm_probe_kernel<PT, false>), grid, block, 0, s, ctx->d_tiles, ctx->tile_cols, sink);
    };
    if (pieces % 256 != 0) return ADAFUSE_ERR_ARG;
    switch (pieces / 256) {
    case 4: launch(std::integral_constant<int, 4>{}); break;
    case 8: launch(std::integral_constant<int, 8>{}); break;
    case 16: launch(std::integral_constant<int, 16>{}); break;
    case 32: launch(std::integral_constant<int, 32>{}); break;
    default: return ADAFUSE_ERR_ARG;  // a tile shape this aid is not built for
    }
    return hipGetLastError() == hipSuccess ? ADAFUSE_OK : ADAFUSE_ERR_HIP;
}

const char *adafuse_switch_kernel_name(const adafuse_ctx *ctx, int32_t k, int32_t mode)
{
    if (!ctx) return nullptr;
    if (mode != ADAFUSE_MERGE && mode != ADAFUSE_UNMERGE && mode != ADAFUSE_SWAP) return nullptr;
    const bool need_next = mode != ADAFUSE_UNMERGE;
    const bool need_prev = ctx->inplace && mode != ADAFUSE_MERGE;
    if ((need_next || need_prev) && (k < 1 || k > ctx->k_max)) return nullptr;
    const bool copy_only = !ctx->inplace && mode == ADAFUSE_UNMERGE;
    const int n_terms = (need_prev ? k : 0) + (need_next ? k : 0);
    switch (ctx->kernel) {
    case ADAFUSE_KERNEL_MFMA: return copy_only ? "switch_copy_kernel" : "switch_mfma_kernel";
    case ADAFUSE_KERNEL_GEMM:
        if (copy_only) return "switch_gemm_kernel";
        switch (pick_gemm_form(ctx->r, terms_bucket(n_terms), ctx->opt_form, ctx->d_tall != nullptr)) {
        case kFormStrip: return "switch_gemm_strip_kernel";
        case kFormOverlap: return "switch_gemm_overlap_kernel";
        default: return "switch_gemm_kernel";
        }
    default: return "switch_valu_kernel";
    }
}

const char *adafuse_status_string(int32_t status)
{
    switch (status) {
    case ADAFUSE_OK: return "ok";
    case ADAFUSE_ERR_NULL: return "required pointer is NULL";
    case ADAFUSE_ERR_ARG: return "argument out of range";
    case ADAFUSE_ERR_SHAPE: return "unsupported matrix shape";
    case ADAFUSE_ERR_ALIGN: return "pointer or leading dimension misaligned";
    case ADAFUSE_ERR_HIP: return "HIP runtime call failed";
    default: return "unknown status";
    }
}

}  // extern "C"
