/*
 * libadafuse -- the fused adapter switch of AdaFuse on one MI355X (gfx950).
 *
 * Two operations, each one kernel launch on a caller-supplied HIP stream:
 *
 *   adafuse_pregate       token-level pre-gating router G^1(x^1): one linear map,
 *                         top-k and softmax per token, decided once and reused by
 *                         every adapted layer (paper: Eq.1 for the form of G,
 *                         Eq.2 and section "Model Structure" for its single use).
 *   adafuse_fused_switch  for EVERY adapted matrix of the model at once,
 *                         W' = W + s * sum_{j<k} g_j * B_{e_j} A_{e_j}
 *                         (Eq.4-6, merge), with the previous token's merge removed
 *                         in the same pass (Eq.7-8, fused switch), executed as one
 *                         batched launch over a table of matrix pointers and
 *                         shapes (Eq.9 and section "SGMM Kernel").
 *
 * Layout conventions (y = W x, as torch.nn.Linear stores it):
 *   W        bf16 [out][ldw]   row-major, ldw >= in (elements)
 *   A bank   bf16 [E][r][in]   expert e's LoRA_DOWN
 *   B bank   bf16 [E][out][r]  expert e's LoRA_UP
 *   dW = sum_j (s*g_j) * B_{e_j} A_{e_j}     (the paper's "DOWN x UP")
 *
 * Every pointer marked DEVICE must be device memory reachable from the current
 * HIP device; HOST pointers are ordinary host memory.  Nothing here takes or
 * returns a framework type.  All functions return an adafuse_status; none
 * throws, aborts or prints.  Argument checks that need no GPU run before any
 * HIP call, so invalid arguments are reported on a machine without a GPU too.
 *
 * Threads: a context is not locked.  Calls that only enqueue (pregate, the
 * switches, the forward passes, get_info, switch_kernel_name) may run from
 * several host threads at once; adafuse_set_option and adafuse_destroy must not
 * overlap with any other call on the same context.  Two switches on the same
 * context write the same W_work: order them on one stream (or with events)
 * like any other pair of kernels that write the same memory.
 */
#ifndef ADAFUSE_H
#define ADAFUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct adafuse_ctx adafuse_ctx; /* opaque */

typedef enum {
    ADAFUSE_OK = 0,
    ADAFUSE_ERR_NULL = 1,  /* a required pointer is NULL */
    ADAFUSE_ERR_ARG = 2,   /* a scalar argument is out of range */
    ADAFUSE_ERR_SHAPE = 3, /* a matrix shape is unsupported */
    ADAFUSE_ERR_ALIGN = 4, /* a pointer or leading dimension is misaligned */
    ADAFUSE_ERR_HIP = 5    /* a HIP runtime call or a host allocation failed */
} adafuse_status;

typedef enum {
    ADAFUSE_MERGE = 0,   /* add next's experts; prev ignored */
    ADAFUSE_UNMERGE = 1, /* remove prev's experts; next ignored */
    ADAFUSE_SWAP = 2     /* remove prev, add next, in one pass (see adafuse_fused_switch) */
} adafuse_mode;

typedef enum {
    ADAFUSE_GATE_SOFTMAX_OVER_TOPK = 0, /* Eq.1: softmax over the k kept logits; gates sum to 1 */
    ADAFUSE_GATE_TOPK_OF_SOFTMAX = 1    /* "Router Architecture": softmax over all E, keep k */
} adafuse_gate_norm;

typedef enum {
    ADAFUSE_KERNEL_AUTO = 0, /* library's choice for the context's (r, k_max) */
    ADAFUSE_KERNEL_VALU = 1, /* rank-(k r) update on the vector ALU, fp32 */
    ADAFUSE_KERNEL_MFMA = 2, /* per-expert B_e A_e on the matrix cores (4x4x4 blocks; bf16 in, fp32 out) */
    ADAFUSE_KERNEL_GEMM = 3  /* high ranks: 32x32x16 matrix-core blocks with a loop over the rank */
} adafuse_kernel;

/*
 * One adapted linear matrix (one entry of the pointer/shape arrays the SGMM
 * kernel takes, section "SGMM Kernel").  All pointers are DEVICE pointers, 16-byte
 * aligned, owned by the caller and must stay valid while the context lives.
 * w_work is the matrix the model's forward pass reads.
 * Out of place (w_work != w_base, the default way to use the library): w_base is
 * never written and w_work is rebuilt from it on every switch; the two must not
 * overlap.  In place (w_work == w_base, the paper's own formulation: "the addition
 * ... is performed in place"): the one buffer is updated by adding and subtracting
 * low-rank terms, and its bf16 rounding error accumulates from token to token.
 * Either all matrices of a context are in place or none is.  No buffer may
 * overlap a bank.
 */
typedef struct {
    const void *w_base; /* bf16 [out][ldw] */
    void *w_work;       /* bf16 [out][ldw] */
    const void *a_bank; /* bf16 [E][r][in] */
    const void *b_bank; /* bf16 [E][out][r] */
    int32_t out;        /* rows, >= 1 */
    int32_t in;         /* columns, >= 8 and a multiple of 8 */
    int32_t ldw;        /* leading dimension of both W buffers, >= in, multiple of 8 */
    int32_t reserved;   /* must be 0 */
} adafuse_matrix_desc;

typedef struct {
    int32_t n_mats;
    int32_t E, r, k_max;
    int32_t kernel;          /* adafuse_kernel in effect (never AUTO) */
    int32_t tile_rows;       /* rows x cols of W one workgroup handles */
    int32_t tile_cols;
    int32_t reserved;
    int64_t n_tiles;         /* workgroups per switch launch */
    int64_t elements;        /* sum of out*in over all matrices */
} adafuse_info;

/*
 * Build a context for a fixed set of adapted matrices: copies `mats` (HOST array
 * of n_mats descriptors; may be freed afterwards), builds the matrix and tile
 * tables the switch kernel walks and uploads them to the current device.  This
 * is the only call that allocates device memory or synchronises; the tables are
 * a few bytes per tile.  E = experts per bank, r = LoRA rank (4, 8, 16, 32, 64
 * or 128), k_max = largest k any later call will pass (1 <= k_max <= min(E, 8)).
 * In place, k_max <= 4 (a SWAP then carries 2 k_max experts).
 * Errors: NULL mats/ctx or NULL pointer inside a descriptor -> ERR_NULL;
 * n_mats < 1, bad E/r/k_max, reserved != 0, in-place and out-of-place matrices
 * mixed -> ERR_ARG;
 * out < 1, in < 8, in % 8, ldw < in, ldw % 8, out or in > 2^22, ldw > 2^24
 * (the kernels address a tile and an expert's slice with 32-bit offsets)
 * -> ERR_SHAPE; pointer not 16-byte
 * aligned -> ERR_ALIGN; HIP failure -> ERR_HIP (no context is returned).
 */
adafuse_status adafuse_create(const adafuse_matrix_desc *mats, int32_t n_mats,
                              int32_t E, int32_t r, int32_t k_max, adafuse_ctx **ctx);

/* Free the context's tables.  NULL is accepted.  Caller buffers are untouched. */
adafuse_status adafuse_destroy(adafuse_ctx *ctx);

/*
 * Options of a context, all with a default the library chooses by itself.  They exist for
 * measurements (baselines, ablations); a serving caller needs none of them.
 */
typedef enum {
    ADAFUSE_OPT_KERNEL = 0,     /* adafuse_kernel; AUTO = the library's choice for (r, k_max) */
    ADAFUSE_OPT_GEMM_WAVES = 1, /* waves per workgroup of ADAFUSE_KERNEL_GEMM (tile 64 x 64 waves): 4, 8, or 0 =
                                   chosen from the matrices' row pitches */
    ADAFUSE_OPT_GEMM_FORM = 2,  /* form of ADAFUSE_KERNEL_GEMM: 0 = by the length of the contraction, 1 = unrolled,
                                   3 = overlapped with the W fetch, 4 = chains of eight vertically adjacent tiles
                                   per workgroup (column operands resident, next tile's W in flight during the
                                   contraction); each wherever that form can take the launch */
    ADAFUSE_OPT_XCD_RUN = 3,    /* tile order: 0 = plain, 1 = one contiguous eighth of the tile list per XCD
                                   (default), G > 1 = runs of G tiles per XCD */
    ADAFUSE_OPT_PANEL_KB = 4,   /* column-operand budget of a column panel in KiB (default 2048) */
    ADAFUSE_OPT_MFMA_SHAPE = 5  /* tile shape of ADAFUSE_KERNEL_MFMA: 0..5, -1 = the library's choice */
} adafuse_option;

/* Set one option.  Rebuilds the tile table (allocates and synchronises like
 * adafuse_create; the context's device must be current, else ERR_ARG).  Unknown
 * option or value out of range -> ERR_ARG.  On any error the context keeps the
 * kernel, tables and options it had. */
adafuse_status adafuse_set_option(adafuse_ctx *ctx, int32_t option, int32_t value);

/* Fill *info (HOST) with the context's geometry. */
adafuse_status adafuse_get_info(const adafuse_ctx *ctx, adafuse_info *info);

/* Name of the device function that adafuse_fused_switch(ctx, ..., k, ..., mode, ...)
 * would launch (without template arguments, as a kernel trace shows it), for
 * labelling measurements: the form of the default kernel depends on rank and
 * term count.  A static string; NULL for a NULL context or arguments that the
 * switch would refuse. */
const char *adafuse_switch_kernel_name(const adafuse_ctx *ctx, int32_t k, int32_t mode);

/*
 * Measurement aid (not a step of the method): one pass in ONE direction over the
 * same tile table the fused switch walks, one workgroup per tile, 16 bytes per
 * lane.  The two rates bracket what the switch's read-plus-write pass can reach
 * on the device at hand.
 *   ADAFUSE_PROBE_READ_BASE  reads every element of every w_base and discards it
 *   ADAFUSE_PROBE_ZERO_WORK  writes zero bits to every element of every w_work:
 *                            the merged weights are gone, merge again before use;
 *                            ERR_ARG for an in-place context (w_work == w_base)
 * Enqueues one kernel on `hip_stream`; no allocation, no synchronisation.
 * ERR_ARG for an unknown direction or a tile shape the aid is not built for.
 */
typedef enum { ADAFUSE_PROBE_READ_BASE = 0, ADAFUSE_PROBE_ZERO_WORK = 1 } adafuse_probe_direction;
adafuse_status adafuse_hbm_probe(adafuse_ctx *ctx, int32_t direction, void *hip_stream);

/*
 * Pre-gating router for T tokens (Eq.1's G applied to x^1, Eq.2):
 *   logits[t][e] = sum_i hidden[t][i] * w_router[e][i]      (fp32 result)
 *   idx[t][0..k)  = the k largest logits of token t, ordered by (logit
 *                   descending, expert index ascending); ties take the lower index
 *   gates[t][j]   = softmax per gate_norm, fp32
 * hidden   DEVICE bf16 [T][d], w_router DEVICE bf16 [E][d], both 16-byte aligned,
 *          d a multiple of 8; 1 <= E <= 64, 1 <= k <= min(E, 8) (else ERR_ARG);
 *          T >= 0 (T == 0 is a no-op).
 * idx      DEVICE int32 [T][k], gates DEVICE fp32 [T][k], logits DEVICE fp32
 *          [T][E] or NULL.  Outputs are written by the kernel on `hip_stream`
 *          (a hipStream_t, NULL = default stream); the call does not wait.
 * Selection and gates are taken from the fp32 logits the call returns.
 */
adafuse_status adafuse_pregate(const void *hidden, const void *w_router,
                               int32_t T, int32_t d, int32_t E, int32_t k, int32_t gate_norm,
                               int32_t *idx, float *gates, float *logits, void *hip_stream);

/*
 * Fused adapter switch over every matrix of the context, one launch (Eq.8-9).
 *   idx_next/gates_next  DEVICE int32[k] / fp32[k]: the token's experts and gates
 *   idx_prev/gates_prev  DEVICE, same shapes: what the previous call merged
 *   k      1 <= k <= k_max;   scale = LoRA scaling s
 * MERGE   W_work <- rn_bf16(W_base + s * sum_j gates_next[j] B_{idx_next[j]} A_{idx_next[j]}),
 *         fp32 accumulation, one rounding.  prev may be NULL.
 * UNMERGE W_work <- W_base bit-exact.  prev and next may be NULL.
 * SWAP    the fused switch: the result is that of MERGE(next).  Because W_work is
 *         rebuilt from the immutable W_base, the previous token's update is
 *         removed exactly (no bf16 drift) and Eq.8's signed concatenation needs
 *         no arithmetic.  prev, if not NULL, is only compared with next on the
 *         device: when both are bit-identical W_work already holds the result
 *         and the kernel returns without touching it.  `scale` is not part of
 *         that comparison: the caller's contract is that prev is what the last
 *         call merged, with the same scale (after a change of scale, pass
 *         prev = NULL or use MERGE).
 * In place (w_work == w_base; Eq.7-8 as printed), with dW(x) = s * sum_j g_j B_{e_j} A_{e_j}:
 *   MERGE   W <- rn_bf16(W + dW(next));  UNMERGE  W <- rn_bf16(W - dW(prev));
 *   SWAP    W <- rn_bf16(W - dW(prev) + dW(next)), the signed concatenation
 *           [-DOWN^{t-1}, DOWN^t] summed in fp32 and rounded once per call.
 *   An expert listed in both prev and next enters once, with the difference of
 *   its two coefficients (dropped when that is exactly zero).
 *   prev is required for UNMERGE and SWAP; a SWAP with prev bit-identical to next
 *   is an exactly-zero update and returns without touching W.
 * Both entry points only enqueue kernels (no allocation, no memset, no
 * synchronisation), so they may be recorded into a HIP graph.
 * Each W element is read once and written once (2 + 2 bytes); the selected A/B
 * slices are staged in registers and LDS.  Expert indices outside [0,E) in device memory are
 * clamped into range, not detected.  Gates may be any finite fp32 values (negative,
 * tiny or sub-normal ones included): the experts are accumulated in ascending order
 * of |s g_j|, so no intermediate ratio of coefficients can overflow.  The call enqueues on `hip_stream` and
 * returns; no host synchronisation.
 * Errors: NULL ctx or a NULL pointer the mode needs -> ERR_NULL; bad k or mode, or a
 * current device other than the one the context was created on -> ERR_ARG; launch
 * failure -> ERR_HIP.
 */
adafuse_status adafuse_fused_switch(adafuse_ctx *ctx,
                                    const int32_t *idx_prev, const float *gates_prev,
                                    const int32_t *idx_next, const float *gates_next,
                                    int32_t k, float scale, int32_t mode, void *hip_stream);

/*
 * The "simple merge" the paper measures its fused kernel against (section "SGMM
 * Kernel", first paragraph; ablation table): the same update, same arguments,
 * same kernels and same result as adafuse_fused_switch, but merged layer by
 * layer -- one launch per adapted matrix, n_mats launches per call, enqueued in
 * matrix order on `hip_stream`.  Exists to measure what the single batched
 * launch buys; not meant for production use.
 */
adafuse_status adafuse_switch_per_matrix(adafuse_ctx *ctx,
                                         const int32_t *idx_prev, const float *gates_prev,
                                         const int32_t *idx_next, const float *gates_next,
                                         int32_t k, float scale, int32_t mode, void *hip_stream);

/*
 * The step right AFTER the switch, provided for checking and for context, not as
 * a product path: every matrix of the context applied to one token's input, as a
 * decode loop launches it.
 *   adafuse_forward_merged   y_m = W_work,m x_m                      (Eq.3: the merged backbone)
 *   adafuse_forward_dynamic  y_m = W_base,m x_m + s * sum_j g_j B_{e_j}(A_{e_j} x_m)
 *                            (Eq.2 at run time: per matrix one GEMV plus, per
 *                            selected expert, a down- and an up-projection launch
 *                            -- the "four or more additional kernel calls" of a
 *                            dynamic adapter layer)
 * x  DEVICE bf16: the inputs of all matrices, concatenated in matrix order
 *    (in_0 + in_1 + ... elements; each `in` is a multiple of 8, so every piece is
 *    16-byte aligned if x is);  y  DEVICE fp32: the outputs, concatenated
 *    (out_0 + out_1 + ...).  fp32 accumulation.
 * adafuse_forward_dynamic takes the routing decision from HOST arrays idx[k],
 * gates[k] (a dynamic adapter decides on the host which experts to launch) and a
 * DEVICE scratch z of k*r floats owned by the caller; it needs an out-of-place
 * context.  n_mats (merged) or n_mats*(1+2k) (dynamic) launches on `hip_stream`.
 */
adafuse_status adafuse_forward_merged(adafuse_ctx *ctx, const void *x, float *y, void *hip_stream);
adafuse_status adafuse_forward_dynamic(adafuse_ctx *ctx, const int32_t *idx, const float *gates, int32_t k,
                                       float scale, const void *x, float *y, float *z, void *hip_stream);

/*
 * Prefill: T tokens through ONE adapted matrix of the context, every token with its own
 * routing decision (section "Decoding Phase": in the prefill phase the tokens of a prompt
 * select different experts, so no single merged weight serves them and the adapters are
 * applied un-merged, Eq.2 with the pre-gated G^1(x^1) of each token):
 *   y[t] = W_base x[t] + scale * sum_{j<k} gates[t][j] * B_{idx[t][j]} (A_{idx[t][j]} x[t]),   t < T.
 * mat      index of the matrix in the array given to adafuse_create (0 <= mat < n_mats)
 * x        DEVICE bf16 [T][in], contiguous, 16-byte aligned
 * idx      DEVICE int32 [T][k], gates DEVICE fp32 [T][k]: what adafuse_pregate wrote for these
 *          tokens; 1 <= k <= k_max.  Indices outside [0,E) are clamped.  An expert listed
 *          twice for a token counts twice (its gates add).
 * y        DEVICE fp32 [T][out], contiguous, 16-byte aligned; every element is written once
 *          (no accumulation into previous contents, no atomics: the same bits on every run)
 * workspace  DEVICE, 16-byte aligned, at least adafuse_prefill_workspace_bytes() bytes
 *          (workspace_bytes is checked): the fp32 parts of the products whose inner dimension
 *          is split across workgroups (few tokens leave too few tiles to fill the chip) and,
 *          in the many-token form, the scaled down-projections s g A x of every (token,
 *          selection) as two bf16 planes (value and rounding remainder, 16 significant bits).
 *          Owned by the caller; its previous contents do not matter and nothing in it needs
 *          clearing.
 * Arithmetic: bf16 operands on the matrix cores, fp32 accumulation; the parts of a split inner
 * dimension are added in a fixed order: the same bits on every run.
 * Launches on `hip_stream`, no allocation, no synchronisation.  Few tokens (T <= 512 and T * k * r <= 8192): two (the
 * base product and the down-projection through the whole bank share one, cut into the same
 * number of parts; the second sums the parts and adds the up-projections in fp32).
 * Otherwise: three or four (down projection over the whole bank, gating, base product with the
 * up projection as further inner dimension, sum of the parts).  Needs an out-of-place context
 * (the base weights must be unmodified).
 * Errors: NULL pointer -> ERR_NULL; mat, T < 0, k out of range, in-place context, workspace
 * too small, wrong device -> ERR_ARG; misaligned x / y / workspace -> ERR_ALIGN;
 * T * in or T * k * r beyond 2^30 elements -> ERR_SHAPE.  T == 0 is a no-op.
 */
adafuse_status adafuse_prefill(adafuse_ctx *ctx, int32_t mat, const void *x, int32_t T,
                               const int32_t *idx, const float *gates, int32_t k, float scale,
                               float *y, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of workspace adafuse_prefill needs for T tokens with k selections each through matrix
 * `mat` (HOST result in *bytes; 0 for T == 0).  Errors as adafuse_prefill's argument checks. */
adafuse_status adafuse_prefill_workspace_bytes(const adafuse_ctx *ctx, int32_t mat, int32_t T, int32_t k,
                                               size_t *bytes);

/*
 * adafuse_prefill for a GROUP of matrices that take the same input (the q, k and v projections
 * of a layer; gate and up): the same results, y[i] = adafuse_prefill(mats[i]) up to the order
 * of the fp32 sums, with the launches shared.  The method's own argument for one batched
 * launch ("SGMM Kernel": many small launches leave the GPU under-used) holds here as well: at a
 * hundred tokens a launch costs more than streaming a 4096 x 4096 matrix once.  In the
 * few-token form the whole group takes two launches; otherwise the matrices run one after
 * the other as in adafuse_prefill.
 * mats     HOST int32 [n], distinct matrix indices, 1 <= n <= 4, all with the same `in`
 *          (else ERR_SHAPE)
 * y        HOST array of n DEVICE pointers: y[i] fp32 [T][out of mats[i]], 16-byte aligned
 * workspace  at least adafuse_prefill_group_workspace_bytes() bytes
 * Everything else as adafuse_prefill.
 */
adafuse_status adafuse_prefill_group(adafuse_ctx *ctx, const int32_t *mats, int32_t n, const void *x, int32_t T,
                                     const int32_t *idx, const float *gates, int32_t k, float scale,
                                     float *const *y, void *workspace, size_t workspace_bytes, void *hip_stream);
adafuse_status adafuse_prefill_group_workspace_bytes(const adafuse_ctx *ctx, const int32_t *mats, int32_t n,
                                                     int32_t T, int32_t k, size_t *bytes);

/*
 * adafuse_forward_dynamic for callers that cannot allocate device memory or hand over a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same launches and the same result, with the down-projected activations z
 * held in a scratch array built into the library (1024 floats = 4 KB per GPU, resident until
 * the process ends) instead of a caller buffer.  The call allocates nothing and frees nothing.
 * k * r <= 1024, else ERR_ARG (every (k <= 8, r <= 128) a context accepts fits).  All calls on
 * one GPU share that array: two calls that may run at the same time (different streams, or
 * different host threads) race on it and must be ordered by the caller.  Nothing in it has
 * to start at zero; each call overwrites what it reads.  Other errors as
 * adafuse_forward_dynamic.
 */
adafuse_status adafuse_forward_dynamic_static(adafuse_ctx *ctx, const int32_t *idx, const float *gates, int32_t k,
                                              float scale, const void *x, float *y, void *hip_stream);

const char *adafuse_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* ADAFUSE_H */
