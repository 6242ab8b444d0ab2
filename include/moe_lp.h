/*
 * moe_lp.h -- C ABI of the MI355X (gfx950) MoE expert-FFN hot path that layered
 * prefill speeds up: router + top-k, token permutation, grouped SwiGLU FFN,
 * weighted combine, and a layer-group driver for the chunked and the layered
 * prefill schedules.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller unless a
 *     parameter says "host".  Base pointers must be 16-byte aligned; the packed
 *     codes of MOE_W_MXFP4 expert weights must be 32-byte aligned (their scale
 *     bytes 16, like everything else).
 *   - Tensors are dense row-major.  "dtype" elements are bfloat16 (2 bytes) or
 *     float (4 bytes) as chosen in moe_config.dtype.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return; nothing synchronises with the host
 *     except moe_read_counters.
 *   - The library allocates no device memory: all scratch lives in the
 *     workspace handed to moe_create.  Calls on one moe_ctx must not overlap
 *     in time (they share that workspace); use one ctx per concurrent stream.
 *   - Every failure is a return code; argument errors are detected on the host
 *     before anything is launched.  Outputs are fully overwritten on success.
 *   - A zero token count is a legal no-op.
 */
#ifndef MOE_LP_H
#define MOE_LP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque, host memory, owned by the library */

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = 1,      /* a required pointer is NULL */
    MOE_ERR_SHAPE = 2,     /* a size is negative / zero / inconsistent (k > E, T > max_tokens ...) */
    MOE_ERR_DTYPE = 3,     /* unknown moe_dtype */
    MOE_ERR_ALIGN = 4,     /* H or I not a multiple of 8 (64 for MOE_W_MXFP4), a pointer not 16-byte aligned, or
                              MXFP4 code bytes not 32-byte aligned */
    MOE_ERR_WORKSPACE = 5, /* workspace smaller than moe_workspace_bytes says */
    MOE_ERR_SCHEDULE = 6,  /* unknown schedule kind, or chunk <= 0 for a chunked schedule */
    MOE_ERR_DEVICE = 7     /* a HIP runtime call failed (launch error, wrong device ...) */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

/*
 * Format of the expert weights (w_gate_up, w_down).  MOE_W_MXFP4 (the paper's broader validation, Table 7,
 * runs a model with fp4 expert weights) is the published OCP Microscaling format: FP4 E2M1 elements
 * (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), two per byte with the even element in the low nibble, and one
 * E8M0 scale byte (2^(s-127), s in 1..254) per 32 consecutive elements of a row.  It needs dtype ==
 * MOE_BF16 (activations and the router stay bf16) and H, I multiples of 64.  The code tensors (w_gate_up,
 * w_down) must start on a 32-byte boundary: every row is then a whole number of 32-byte pieces from a
 * 32-byte boundary, which is what lets the weight-streaming kernel fetch rows in whole aligned 128-byte
 * lines; a 16-byte aligned pointer is refused with MOE_ERR_ALIGN before anything is launched.  The scale
 * tensors need the general 16-byte alignment.
 */
typedef enum { MOE_W_DTYPE = 0, MOE_W_MXFP4 = 1 } moe_weight_format;

/* Shape of one MoE layer (Table 3 gives E, K and H of the evaluated models). */
typedef struct {
    int32_t H;           /* hidden size, multiple of 8 */
    int32_t E;           /* number of experts, 1..512 */
    int32_t K;           /* experts per token (top-k), 1..min(E,64) */
    int32_t I;           /* expert intermediate size, multiple of 8 */
    int32_t dtype;       /* moe_dtype of activations and weights */
    int32_t renormalize; /* 1: mixing weights of the K selected experts are divided by their sum */
    int32_t residual;    /* 1: moe_group_forward links layers by x <- x + MoE(x); 0: x <- MoE(x) */
    int32_t weight_format; /* moe_weight_format of the expert weights */
    int32_t y_perm_f32;  /* 0: the expert outputs y_perm are held in dtype between the down GEMM and the combine;
                            1: in fp32 (bf16 contexts: one rounding fewer on the output side, for layers whose
                            expert outputs are large against the tolerance; A*H*2 more bytes written and read
                            per layer).  Every y_perm argument below then is a float tensor. */
    int32_t act_split;   /* 1: the intermediate a = silu(g) * u is held as a PAIR of bf16 values, a ~ hi + lo with
                            hi = bf16(a), lo = bf16(a - hi) (about 16 significant bits instead of 8), and the down
                            GEMM multiplies both halves: for layers whose intermediate is so wide (I in the ten
                            thousands) that its bf16 rounding alone exceeds the tolerance.  Doubles the down
                            GEMM's work and the intermediate's bytes.  Needs dtype == MOE_BF16, weight_format ==
                            MOE_W_DTYPE and y_perm_f32 == 1 (MOE_ERR_DTYPE otherwise). */
} moe_config;

/* Weights of one layer (device pointers). */
typedef struct {
    const void *w_router;     /* [E, H]     dtype */
    const float *router_bias; /* [E] fp32 added to the logits, or NULL */
    const void *w_gate_up;    /* [E, 2I, H] dtype; rows [0,I) gate projection, rows [I,2I) up projection */
    const void *w_down;       /* [E, H, I]  dtype */
    /* MOE_W_MXFP4 only (else ignored): w_gate_up is [E, 2I, H/2] bytes, w_down [E, H, I/2] bytes, and */
    const uint8_t *s_gate_up; /* [E, 2I, H/32] scale bytes */
    const uint8_t *s_down;    /* [E, H, I/32]  scale bytes */
} moe_layer;

typedef enum { MOE_SCHED_CHUNKED = 0, MOE_SCHED_LAYERED = 1 } moe_sched_kind;
typedef struct {
    int32_t kind;  /* moe_sched_kind */
    int32_t chunk; /* prefill tokens per iteration; > 0 when kind == MOE_SCHED_CHUNKED, ignored otherwise */
} moe_schedule;

/* Expert-weight traffic model, accumulated by moe_group_forward (Sec. 5.4: a load
 * byte is counted whenever an expert's parameters are brought in for execution). */
typedef struct {
    uint64_t expert_bytes;         /* sum over (iteration, layer) of active experts * bytes of one expert's weights:
                                      3*H*I*sizeof(dtype), or 3*H*I*17/32 for MOE_W_MXFP4 (codes + scales) */
    uint64_t router_bytes;         /* sum over (iteration, layer) of E*H*sizeof(dtype) */
    uint64_t active_experts_total; /* sum over (iteration, layer) of experts with >= 1 token */
    uint64_t tokens_processed;     /* sum over iterations of the batch rows of that iteration */
    uint32_t iterations;
    uint32_t layer_passes;         /* iterations * n_layers */
} moe_counters;

/* Bytes of device workspace a context for batches of up to max_tokens rows needs. Host-only. */
moe_status moe_workspace_bytes(const moe_config *cfg, int64_t max_tokens, size_t *out_bytes);

/* Create a context over a caller-owned device workspace (256-byte aligned, at least
 * moe_workspace_bytes; it must stay alive and untouched until moe_destroy).  The
 * workspace's counter block is cleared on `stream`. */
moe_status moe_create(const moe_config *cfg, int64_t max_tokens, void *workspace, size_t workspace_bytes,
                      void *stream, moe_ctx **out_ctx);
moe_status moe_destroy(moe_ctx *ctx);

/*
 * Router (Sec. 2.4).
 *   logits z[t,e] = sum_h x[t,h]*w_router[e,h] (+ bias[e]), accumulated in fp64;
 *   topk_idx[t,:] = the K experts with the largest logits, ordered by logit descending,
 *                   equal logits by ascending expert index;
 *   topk_w[t,j]   = softmax over all E logits evaluated at the selected experts, divided by
 *                   the sum over the K selected ones when cfg.renormalize.
 * x [T,H] dtype, w_router [E,H] dtype, bias [E] fp32 or NULL -> topk_idx [T,K] int32, topk_w [T,K] fp32.
 * Routing of a token does not depend on which other tokens are in the batch.
 */
moe_status moe_router_topk(moe_ctx *ctx, const void *x, int64_t T, const void *w_router, const float *bias,
                           int32_t *topk_idx, float *topk_w, void *stream);

/*
 * moe_router_topk for callers that cannot allocate device memory and have no workspace to hand over (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no context; the logits
 * live in a static device array of the library (4 MiB per GPU, held until the process ends), so
 * T * cfg->E must not exceed 524288 (MOE_ERR_WORKSPACE otherwise, before anything is launched).  Same
 * arithmetic, same kernels and same results as moe_router_topk with a context of this cfg; H, E, K,
 * dtype and renormalize of cfg are read.  The call allocates nothing, on the host or the device.  All
 * calls on one GPU share the array: calls that overlap in time on one GPU (different streams, or
 * different threads) race; serialise them.
 */
moe_status moe_router_topk_noalloc(const moe_config *cfg, const void *x, int64_t T, const void *w_router,
                                   const float *bias, int32_t *topk_idx, float *topk_w, void *stream);

/*
 * Token permutation (Sec. 3.1: the tokens routed to each expert form that expert's batch).
 * The T*K assignments (t, j) are listed by expert, then token, then slot:
 *   counts [E], offsets [E+1] (exclusive running sum, offsets[E] = T*K),
 *   perm [T*K]: perm[r] = t*K + j is the assignment held by permuted row r,
 *   inv_perm [T*K]: inv_perm[perm[r]] = r,
 *   x_perm [T*K, H] dtype (optional, may be NULL): x_perm[r,:] = x[perm[r] / K, :].
 * topk_idx entries must lie in [0, E).  The order is deterministic (a stable sort).
 */
moe_status moe_permute(moe_ctx *ctx, const void *x, const int32_t *topk_idx, int64_t T,
                       int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                       void *x_perm, void *stream);

/*
 * Grouped expert FFN (Sec. 2.1: FC layers with a SwiGLU non-linearity; Sec. 2.5: each expert's
 * FC runs over the tokens routed to it).  For expert e and rows r in [offsets[e], offsets[e+1]):
 *   g = x_perm[r,:] . w_gate_up[e, 0:I, :]^T,  u = x_perm[r,:] . w_gate_up[e, I:2I, :]^T,
 *   a = g / (1 + exp(-g)) * u   (rounded once to dtype, or to a bf16 pair when cfg.act_split),
 *   y_perm[r,:] = a . w_down[e]^T.
 * x_perm [A,H] dtype, offsets [E+1] int32 (device), A = offsets[E] rows -> y_perm [A,H] dtype (float when
 * cfg.y_perm_f32).
 * Experts with no rows cause no weight reads.  bf16 inputs accumulate in fp32 on the matrix cores.
 */
moe_status moe_grouped_ffn(moe_ctx *ctx, const void *x_perm, const int32_t *offsets, int64_t A,
                           const void *w_gate_up, const void *w_down, void *y_perm, void *stream);

/*
 * The same step for a context created with weight_format == MOE_W_MXFP4 (Table 7: fp4 expert weights):
 * w_gate_up / w_down are the packed codes, s_gate_up / s_down their scale bytes, layouts as in moe_layer.
 * Every weight is widened exactly to bf16 on the fly; arithmetic and outputs as moe_grouped_ffn.
 * MOE_ERR_DTYPE when the context's weight format is not MOE_W_MXFP4 (and moe_grouped_ffn returns it
 * when it is).
 */
moe_status moe_grouped_ffn_mxfp4(moe_ctx *ctx, const void *x_perm, const int32_t *offsets, int64_t A,
                                 const uint8_t *w_gate_up, const uint8_t *s_gate_up, const uint8_t *w_down,
                                 const uint8_t *s_down, void *y_perm, void *stream);

/*
 * Weighted un-permute and combine (Sec. 2.4: a token's output mixes its selected experts):
 *   y[t,:] = sum_{j<K} topk_w[t,j] * y_perm[inv_perm[t*K+j], :]  (+ residual[t,:]),
 * summed in fp32 in slot order and rounded once.  y_perm [A,H] dtype (float when cfg.y_perm_f32);
 * residual [T,H] dtype or NULL; y may alias residual.
 */
moe_status moe_combine(moe_ctx *ctx, const void *y_perm, const int32_t *inv_perm, const float *topk_w,
                       const void *residual, int64_t T, void *y, void *stream);

/*
 * A contiguous layer group over a hybrid batch (Sec. 2.3), under one of the two schedules:
 *   layered (Sec. 4.1-4.2): ONE iteration; rows [x_decode; x_prefill] cross layers 0..n_layers-1 once.
 *   chunked(C) (Sec. 2.3):  ceil(P/C) iterations; iteration c sends [x_decode; x_prefill[cC : min((c+1)C,P)]]
 *                           through all layers, so every chunk re-streams the experts it activates.
 * P = 0 gives exactly one decode-only iteration under either schedule.  Per layer the four steps above
 * run in order, x <- (x +) MoE_l(x), activations held in dtype between layers.  y_decode [D,H] holds the
 * decode rows' result (identical in every iteration), y_prefill [P,H] the prompt rows'.  Inputs are not
 * modified.  layers is a HOST array of n_layers structs of device pointers.  D + P per iteration must
 * not exceed the context's max_tokens.  Counters accumulate until moe_reset_counters.
 */
moe_status moe_group_forward(moe_ctx *ctx, const moe_layer *layers, int32_t n_layers,
                             const void *x_decode, int64_t D, const void *x_prefill, int64_t P,
                             moe_schedule sched, void *y_decode, void *y_prefill, void *stream);

/*
 * Layer-group count for a prompt of prompt_len tokens (Sec. 4.4): N_lg(L) = max(1, ceil(L / granule)),
 * so that the prefill work of one iteration matches a chunk of `granule` tokens (the paper uses 512:
 * 8192 tokens -> 16 groups, 512 tokens -> 1 group); never more groups than layers.  Host arithmetic
 * only.  Returns 0 when prompt_len < 0, n_layers <= 0 or granule <= 0.
 */
int32_t moe_num_layer_groups(int64_t prompt_len, int32_t n_layers, int32_t granule);

/*
 * Cut layers 0..n_layers-1 into n_groups contiguous groups (Sec. 4.1) whose sizes differ by at most
 * one, the larger groups first: group g holds layers first_layer[g] .. first_layer[g+1]-1.
 * first_layer is a HOST array of n_groups + 1 entries.  MOE_ERR_SHAPE unless 1 <= n_groups <= n_layers.
 */
moe_status moe_layer_groups(int32_t n_layers, int32_t n_groups, int32_t *first_layer);

/* How a whole layer stack is scheduled (Sec. 4.1-4.4). */
typedef struct {
    int32_t chunk;    /* prompt tokens admitted per outer pass (Sec. 4.3); 0 = the whole prompt at once */
    int32_t n_groups; /* layer groups; 0 = moe_num_layer_groups(slice length, n_layers, granule) */
    int32_t granule;  /* tokens per iteration the group-count rule aims for; read only when n_groups == 0 */
} moe_stack_schedule;

/*
 * A whole stack of n_layers MoE layers under the one-group-per-iteration rule (Sec. 4.1-4.2), combined
 * with chunking along the tokens (Sec. 4.3).  The prompt is cut into slices of `chunk` tokens; for each
 * slice the stack is cut into G layer groups and G iterations run.  In iteration g every group runs,
 * in layer order, on the decode rows (which start again from x_decode in every iteration, as under
 * moe_group_forward); group g alone also carries the slice's rows, whose state after group g-1 is kept
 * in y_prefill from the iteration before.  After G iterations the slice has crossed every layer once.
 *   chunk = C, n_groups = 1:            chunked prefill over the whole stack (the baseline, Sec. 2.3);
 *   chunk = 0, n_groups = 0:            layered prefill with the group-count rule of Sec. 4.4;
 *   chunk = 8192, n_groups = 16 (e.g.): both at once (Sec. 4.3-4.4).
 * Every schedule computes the same function of (x_decode, x_prefill); they differ in how many times
 * the expert weights are read, which the counters record (iterations = sum of G over the slices,
 * layer_passes = iterations * n_layers, tokens_processed += D + slice length per iteration).
 * y_decode [D,H], y_prefill [P,H]; neither may be the memory of its input (MOE_ERR_SHAPE).  D + slice
 * length must not exceed the context's max_tokens.  Errors as for moe_group_forward; MOE_ERR_SCHEDULE when chunk < 0,
 * n_groups < 0, n_groups > n_layers, or n_groups == 0 with granule <= 0.
 */
moe_status moe_stack_forward(moe_ctx *ctx, const moe_layer *layers, int32_t n_layers,
                             const void *x_decode, int64_t D, const void *x_prefill, int64_t P,
                             moe_stack_schedule sched, void *y_decode, void *y_prefill, void *stream);

/* Copy the counters to host memory `out`; synchronises `stream`. */
moe_status moe_read_counters(moe_ctx *ctx, moe_counters *out, void *stream);
moe_status moe_reset_counters(moe_ctx *ctx, void *stream);

/*
 * Benchmark aid (not part of the method): bracket the launches of selected kernels inside
 * moe_group_forward with HIP events on the caller's stream.  kernel_mask has bit (1 << id) set for
 * every moe_kernel_id to time; 0 switches timing off.  Setting the mask discards earlier records.
 * moe_read_kernel_timing synchronises `stream` and returns the summed duration (milliseconds) and
 * the number of timed launches of one kernel since the mask was set.  (The permutation may be two
 * launches; they are timed as one.)
 */
typedef enum {
    MOE_KERNEL_ROUTER_LOGITS = 0, MOE_KERNEL_TOPK = 1, MOE_KERNEL_PERMUTE = 2,
    MOE_KERNEL_GATE_UP = 3, MOE_KERNEL_DOWN = 4, MOE_KERNEL_COMBINE = 5, MOE_KERNEL_COUNT = 6
} moe_kernel_id;
moe_status moe_kernel_timing(moe_ctx *ctx, uint32_t kernel_mask);
moe_status moe_read_kernel_timing(moe_ctx *ctx, int32_t kernel, double *total_ms, int64_t *launches, void *stream);

/* Name of the gate_up GEMM kernel variant the context would use for a batch of T rows (host string,
 * static storage): lets a benchmark label its roofline line. */
const char *moe_ffn_variant(const moe_ctx *ctx, int64_t T);

/*
 * Test and tuning aid (not part of the method): the grouped GEMMs come in several kernel shapes, all of
 * which compute the same bits for any batch; the library picks one from the mean rows per expert of a
 * launch.  moe_set_ffn_variant pins the shape for every later launch on this context (MOE_FFN_AUTO
 * restores the rule), so that tests can run every shape on every case.  A shape that cannot run the
 * context's weight format or a launch's K (the pipelined bf16 shapes need K % 64 == 0) is ignored for
 * that launch.  MOE_ERR_SHAPE for an unknown id.
 */
typedef enum {
    MOE_FFN_AUTO = 0,
    MOE_FFN_TILE128 = 1,    /* bf16: 128 x 128 register-staged tiles (any K) */
    MOE_FFN_PIPE_SMALL = 2, /* bf16: 64 x 128 tiles, weight streaming */
    MOE_FFN_PIPE_BIG = 3,   /* bf16: up to 256 x 256 tiles, compute bound */
    MOE_FFN_W4_TILE64 = 4,  /* MXFP4: 64-row tiles */
    MOE_FFN_W4_STREAM = 5   /* MXFP4: 32-row weight-streaming tiles */
} moe_ffn_variant_id;
moe_status moe_set_ffn_variant(moe_ctx *ctx, int32_t variant);

const char *moe_status_string(moe_status s);

#ifdef __cplusplus
}
#endif
#endif /* MOE_LP_H */
