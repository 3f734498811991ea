/*
 * libmoe — coalesced Mixture-of-Experts layer for AMD MI355X (gfx950), C ABI.
 *
 * One MoE layer run over a whole batch of T tokens ("coalesced expert execution": the expert
 * stage takes the ordinary batch, m_exp = B, instead of a sequence of micro-batches —
 * paper Section 3.1 Opportunity 1, Section 4.1.1), plus the micro-batched form of the same
 * call for comparison (paper Section 2.3):
 *
 *     y[t] = sum_{s<k} g[t,s] * Expert_{idx[t,s]}(x[t]),
 *     Expert_e(x) = W2_e ( SiLU(W1_e x) (.) W3_e x ),      SiLU(a) = a / (1 + exp(-a)).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers on the context's GPU, owned by the caller,
 *     row-major, densely packed (the one exception: the *_host arguments of
 *     moe_layer_forward_streamed are HOST pointers to page-locked memory). bf16 tensors are
 *     raw 16-bit patterns (moe_bf16). The library never frees a caller pointer and never uses
 *     one after the work that the call enqueued has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Calls enqueue
 *     work and return without synchronising the host; results are ready when the stream is.
 *   - Return value: MOE_OK or a negative moe_status. Arguments are checked on the host, and
 *     whatever a call must allocate is allocated, before anything is enqueued: when a call returns
 *     MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED_SHAPE or MOE_ERR_WORKSPACE nothing has been
 *     launched. MOE_ERR_HIP reports a failed launch or runtime call in the middle of the
 *     sequence: the stages before it are already enqueued and the outputs are undefined.
 *   - T = 0 is legal and a no-op. An expert that receives no row is legal.
 *   - The calls that take `stream` only enqueue kernels (and, for moe_last_routing, device
 *     copies) on it: after one ordinary call of the same kind and shape (the first launch of a
 *     kernel sets its attributes) they may be recorded into a HIP graph and replayed, except
 *     moe_layer_forward_streamed (second stream) and calls made while profiling is armed.
 *   - A context is bound to one device and must be used from one stream at a time: its
 *     workspace is shared by consecutive calls. That device must be the calling thread's
 *     current device when a call that takes `stream` is made (MOE_ERR_INVALID_ARG otherwise).
 *   - Supported shapes: d_model a multiple of 512, d_ff a multiple of 128,
 *     1 <= k <= min(E, 64), E <= 256, 0 <= T <= T_max, T_max * k < 2^31 (row offsets into the
 *     tensors are 64-bit inside the kernels). Anything else is MOE_ERR_UNSUPPORTED_SHAPE.
 *
 * Weight layout (out, in): W1, W3 are [E, d_ff, d_model]; W2 is [E, d_model, d_ff]; the
 * router matrix is [d_model, E] fp32. These are the three d_h x d_e bf16 matrices per expert
 * of the paper's Table 1, row 3.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx;     /* opaque; owns only its own device workspace, events and
                                       (after a streamed call) a copy stream */
typedef uint16_t moe_bf16;          /* raw bfloat16 bits */

typedef struct {
    int32_t T_max;                  /* largest batch (tokens) any call will pass */
    int32_t d_model;                /* paper's d_h */
    int32_t d_ff;                   /* paper's d_e */
    int32_t E;                      /* experts */
    int32_t k;                      /* experts selected per token */
} moe_shape;

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1,       /* null pointer, T out of range, bad micro_tokens ... */
    MOE_ERR_UNSUPPORTED_SHAPE = -2, /* shape outside the supported set listed above */
    MOE_ERR_WORKSPACE = -3,         /* device allocation failed */
    MOE_ERR_HIP = -4                /* a HIP runtime call or launch reported an error */
} moe_status;

/* Stages of the layer, in execution order; indices into moe_profile_end()'s array. */
enum {
    MOE_STAGE_ROUTE = 0,            /* router logits + top-k + gates */
    MOE_STAGE_PERMUTE = 1,          /* histogram, scan, stable scatter */
    MOE_STAGE_GATHER = 2,           /* x -> x_perm row gather */
    MOE_STAGE_GATEUP = 3,           /* grouped GEMM  H = SiLU(Xp W1^T) * (Xp W3^T) */
    MOE_STAGE_DOWN = 4,             /* grouped GEMM  Yp = H W2^T */
    MOE_STAGE_COMBINE = 5,          /* gate-weighted gather-reduce */
    MOE_NUM_STAGES = 6
};

/* Create a context for `shape` on GPU `device_id` (0..63); allocates the workspace (routing
 * tables, x_perm, H and y_perm for T_max tokens) there and leaves the calling thread's current
 * device as it was. Returns MOE_ERR_UNSUPPORTED_SHAPE for shapes outside the supported set,
 * MOE_ERR_WORKSPACE if the device allocation fails. */
int moe_create(moe_ctx** out, const moe_shape* shape, int device_id);

/* Release the context and its workspace. The caller must have drained the stream. */
int moe_destroy(moe_ctx* ctx);

/* Device bytes moe_create() allocates for `shape` (0 for an unsupported shape). */
size_t moe_workspace_bytes(const moe_shape* shape);

/* Static, human-readable name of a status code. */
const char* moe_status_string(int status);

/* Router (paper Section 2.1: each token is routed to the top-k of the experts).
 *   logits[t,e] = sum_i x[t,i] * w_router[i,e]  (+ bias[e]),  in fp32 with a fixed order:
 *   64 partial sums, element i = 512*j + 8*l + v goes to partial l and is added by a fused
 *   multiply-add for j ascending then v ascending; partials combine by the butterfly
 *   p[l] += p[l xor s], s = 32,16,8,4,2,1; bias is added last.
 *   topk_idx[t,s] = expert with the (s+1)-th largest logit (ties -> lower index, NaN last);
 *   topk_w[t,s]   = exp(l_s - l_0) / sum_{s'<k} exp(l_s' - l_0)   (softmax over the selected k).
 * x [T,d_model] bf16; w_router [d_model,E] fp32; bias [E] fp32 or NULL;
 * topk_idx [T,k] int32 out; topk_w [T,k] fp32 out; logits_out [T,E] fp32 out or NULL. */
int moe_route(moe_ctx* ctx, const moe_bf16* x, const float* w_router, const float* bias,
              int32_t T, int32_t* topk_idx, float* topk_w, float* logits_out, void* stream);

/* The same selection and gates from caller-supplied logits [T,E] fp32. */
int moe_route_from_logits(moe_ctx* ctx, const float* logits, int32_t T, int32_t* topk_idx,
                          float* topk_w, void* stream);

/* Group routed rows by expert (the per-expert inputs of paper Section 3.1).
 * Flat id i = t*k + s. counts[e] = number of ids routed to e; offsets = exclusive prefix sum,
 * offsets[E] = T*k; rows of one expert keep ascending id (stable), so the result is unique:
 * perm[p] = i, inv_perm[i] = p. No atomic operation takes part in the ordering.
 * If x and x_perm are both non-NULL, also gathers x_perm[p,:] = x[perm[p] / k, :].
 * topk_idx [T,k] int32 (values in [0,E)); counts [E], offsets [E+1], perm [T*k],
 * inv_perm [T*k] int32 out; x [T,d_model] bf16 or NULL; x_perm [T*k,d_model] bf16 out or NULL.
 * An index outside [0,E) is not detected on the host; such rows are dropped from every group. */
int moe_permute(moe_ctx* ctx, const int32_t* topk_idx, int32_t T, int32_t* counts,
                int32_t* offsets, int32_t* perm, int32_t* inv_perm, const moe_bf16* x,
                moe_bf16* x_perm, void* stream);

/* moe_permute's grouping for callers that cannot allocate device memory or create a context
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no
 * moe_ctx, no allocation of any kind. The segment tables that moe_permute keeps in the context
 * workspace live in a static device array of the library instead (1 MiB per GPU, held until the
 * process ends), so the size is bounded: ceil(T*k / 256) * E <= 65536 (e.g. T*k <= 2,097,152 ids
 * at E = 8, 65,536 ids at E = 256); larger inputs return MOE_ERR_UNSUPPORTED_SHAPE. Same outputs
 * as moe_permute bit for bit (same kernels); no row gather. 1 <= k <= min(E, 64), E <= 256.
 * All calls on one GPU share that GPU's array: two calls whose work overlaps in time on one GPU
 * (different streams, or different threads) race; calls on one stream are ordered and safe.
 * The first call on a device looks up the array's address (no allocation); the calling thread's
 * current device is the one used. */
int moe_permute_static(const int32_t* topk_idx, int32_t T, int32_t k, int32_t E, int32_t* counts,
                       int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* stream);

/* Grouped SwiGLU expert FFN over rows already grouped by expert (the gated feed-forward network
 * of one expert, paper Section 4.1 and Table 1 row 3): for offsets[e] <= p < offsets[e+1],
 *   y_perm[p,:] = W2_e ( SiLU(W1_e x_perm[p,:]) (.) W3_e x_perm[p,:] ).
 * bf16 operands, fp32 accumulation on the matrix cores, the intermediate H and y_perm
 * rounded to bf16 (nearest even). R = number of rows = offsets[E] (R <= T_max*k).
 * x_perm [R,d_model]; offsets [E+1] int32 (device); W1, W3 [E,d_ff,d_model]; W2 [E,d_model,d_ff];
 * y_perm [R,d_model] bf16 out. Per-element accumulation order does not depend on R. */
int moe_expert_ffn(moe_ctx* ctx, const moe_bf16* x_perm, const int32_t* offsets, int32_t R,
                   const moe_bf16* W1, const moe_bf16* W3, const moe_bf16* W2, moe_bf16* y_perm,
                   void* stream);

/* Gate-weighted combine:  y[t,:] = sum_{s<k} topk_w[t,s] * y_perm[inv_perm[t*k+s], :],
 * slots added in order s = 0..k-1 in fp32, rounded once to bf16. A gather: deterministic.
 * y_perm [T*k,d_model] bf16; inv_perm [T*k] int32; topk_w [T,k] fp32; y [T,d_model] bf16 out. */
int moe_combine(moe_ctx* ctx, const moe_bf16* y_perm, const int32_t* inv_perm,
                const float* topk_w, int32_t T, moe_bf16* y, void* stream);

/* The whole layer over the coalesced batch (paper Section 4.1.1: m_exp = B):
 * route -> permute(+gather) -> expert FFN -> combine, intermediates in the context workspace.
 * x [T,d_model]; w_router [d_model,E]; bias [E] or NULL; W1, W3, W2 as above; y [T,d_model] out. */
int moe_layer_forward(moe_ctx* ctx, const moe_bf16* x, const float* w_router, const float* bias,
                      const moe_bf16* W1, const moe_bf16* W3, const moe_bf16* W2, int32_t T,
                      moe_bf16* y, void* stream);

/* The same layer as consecutive micro-batches of `micro_tokens` tokens (the last may be
 * shorter), run one after the other on `stream` through the same expert weights, each with
 * its own routing and permutation (paper Section 2.3, Section 3.1). The output equals
 * moe_layer_forward's bit for bit; only the cost differs. micro_tokens >= 1. */
int moe_layer_forward_microbatched(moe_ctx* ctx, const moe_bf16* x, const float* w_router,
                                   const float* bias, const moe_bf16* W1, const moe_bf16* W3,
                                   const moe_bf16* W2, int32_t T, int32_t micro_tokens,
                                   moe_bf16* y, void* stream);

/* moe_layer_forward with the weights of the last `n_streamed` experts kept in pinned host memory
 * and moved to the GPU while the other experts compute (the expert group that the paper's
 * Section 4.1.1 moves over PCIe: Eq. 7 prices the transfer at D_Y per moved expert over the PCIe
 * bandwidth; the paper's latency model adds that to the computation time, Eq. 3, whereas this
 * call overlaps the two). Experts [0, E - n_streamed) are resident:
 * W1, W3 [E - n_streamed, d_ff, d_model], W2 [E - n_streamed, d_model, d_ff] in device memory
 * (ignored, may be NULL, when n_streamed == E). Experts [E - n_streamed, E) are read from
 * W1_host, W3_host [n_streamed, d_ff, d_model], W2_host [n_streamed, d_model, d_ff]: HOST pointers
 * to page-locked memory (hipHostMalloc or an equivalent allocator; pageable memory makes the
 * copies synchronous), which must stay unchanged until the work enqueued by the call has finished.
 * The first call allocates two device staging slots of 3*d_model*d_ff*2 bytes each, a copy
 * stream and four events, kept until moe_destroy (MOE_ERR_WORKSPACE if the allocation fails).
 * Transfers run on the library's copy stream; all kernels run on `stream`, resident experts
 * first, then each streamed expert as its weights arrive. The output equals moe_layer_forward's
 * bit for bit (same kernels, same accumulation chains). 0 <= n_streamed <= E. Calls on one
 * context must be enqueued from one host thread at a time. */
int moe_layer_forward_streamed(moe_ctx* ctx, const moe_bf16* x, const float* w_router,
                               const float* bias, const moe_bf16* W1, const moe_bf16* W3,
                               const moe_bf16* W2, const moe_bf16* W1_host,
                               const moe_bf16* W3_host, const moe_bf16* W2_host,
                               int32_t n_streamed, int32_t T, moe_bf16* y, void* stream);

/* Copy the routing tables that the last moe_layer_forward call on this context left in the
 * workspace into caller tensors (device-to-device copies enqueued on `stream`); for the
 * micro-batched call they are the tables of its last micro-batch. T is that call's token count.
 * topk_idx [T,k] int32, topk_w [T,k] fp32, counts [E], offsets [E+1], perm [T*k],
 * inv_perm [T*k] int32; any destination may be NULL. */
int moe_last_routing(moe_ctx* ctx, int32_t T, int32_t* topk_idx, float* topk_w, int32_t* counts,
                     int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* stream);

/* Per-stage device timing for measurement. moe_profile_begin() arms up to `max_calls`
 * subsequent moe_layer_forward / moe_layer_forward_microbatched / moe_layer_forward_streamed /
 * moe_expert_ffn calls: each records HIP events on the caller's stream between stages (the
 * two GEMM stages for moe_expert_ffn). moe_profile_end() waits for those events and
 * writes, per stage, the total milliseconds (stage_ms[MOE_NUM_STAGES], host), the number of
 * kernel launches (stage_launches[MOE_NUM_STAGES], host) and the number of layer calls
 * covered (*calls), then disarms. Costs two event records per stage while armed. */
int moe_profile_begin(moe_ctx* ctx, int32_t max_calls);
int moe_profile_end(moe_ctx* ctx, double* stage_ms, int64_t* stage_launches, int32_t* calls);
/* The same, per call instead of summed: per_call_ms[c * MOE_NUM_STAGES + stage] (host, room for
 * capacity_calls calls, zero-filled first) is the time call c spent in that stage (a
 * micro-batched call adds up its micro-batches); calls beyond capacity_calls are dropped from
 * the table but still counted in *calls. For medians and minima over the timed steps (paper
 * Section 5 reports single figures; this library reports mean, median and minimum). */
int moe_profile_end_per_call(moe_ctx* ctx, double* per_call_ms, int32_t capacity_calls,
                             int64_t* stage_launches, int32_t* calls);

/* Roofline estimate of the expert stage, host arithmetic only (no GPU is touched).
 * Paper Table 1, row 3: per expert D_X = 2*rows*d_h and D_Y = 6*d_h*d_e operand bytes and
 * C = 6*rows*d_h*d_e FLOP (bf16); Eq. 5: an operation costs M * max((D_X + D_Y) / BW, C / TF)
 * over its M micro-batches; Eq. 9 applies that form to the whole expert stage of a device.
 * The table's 2BLd_h/E is the uniform-routing average: here every expert has its own count.
 *   rows [micro_batches * E] int32, HOST: rows routed to expert e in micro-batch m at
 *   rows[m*E + e] (coalesced execution: micro_batches = 1); an expert with 0 rows costs nothing.
 *   machine: the rates to price against (peaks, or rates measured on the device).
 * Only d_model, d_ff and E of `shape` are used (any positive values). Returns
 * MOE_ERR_INVALID_ARG for null pointers, negative counts or non-positive rates. */
typedef struct {
    double tflops;                  /* TF_DEV of Eq. 5, in 1e12 FLOP/s */
    double gbytes_per_s;            /* BW_DEV of Eq. 5, in 1e9 byte/s */
} moe_machine;

typedef struct {
    int32_t micro_batches;          /* M */
    int32_t expert_instances;       /* (micro-batch, expert) pairs with at least one row */
    int32_t memory_bound_instances; /* of those, the ones with (D_X + D_Y)/BW > C/TF */
    double flops;                   /* sum of C */
    double operand_bytes;           /* sum of D_X + D_Y */
    double intermediate_bytes;      /* H written and read, outputs written (not in Table 1) */
    double t_stage_s;               /* Eq. 9 per micro-batch: max(sum bytes/BW, sum C/TF), summed */
    double t_per_expert_s;          /* Eq. 5 expert by expert, summed (experts one after another) */
    double t_kernels_s;             /* gate/up and down as two grouped contractions per micro-batch,
                                       each max(bytes/BW, FLOP/TF) with H counted */
    double ridge_rows;              /* rows per expert above which an expert is compute-bound */
} moe_expert_estimate;

int moe_estimate_expert_stage(const moe_shape* shape, const int32_t* rows, int32_t micro_batches,
                              const moe_machine* machine, moe_expert_estimate* out);

/* Roofline estimate of the expert stage when the weights of `n_moved` experts come over PCIe
 * (paper Section 4.1.1): Eq. 7 prices the transfer, T_load = (D_X3 + EXP_M * D_Y3) / BW_PCIe
 * with D_Y3 = 6*d_h*d_e bytes per moved expert and D_X3 = 2*rows*d_h the stage's inputs (left out
 * when inputs_on_device is non-zero); the computation is the Eq. 9 latency of the GPU with every
 * expert computed there (t_stage_s of moe_estimate_expert_stage for one coalesced batch); Eq. 3
 * adds the two, and their maximum is what complete overlap would give. Host arithmetic only.
 * rows: HOST array [E] of routed row counts; 0 <= n_moved <= E; rates > 0. */
typedef struct {
    double moved_bytes;             /* bytes over PCIe */
    double t_load_s;                /* Eq. 7 */
    double t_comp_s;                /* Eq. 9, all experts on the GPU */
    double t_sum_s;                 /* Eq. 3: t_load_s + t_comp_s */
    double t_overlap_s;             /* max(t_load_s, t_comp_s) */
} moe_streamed_estimate;

int moe_estimate_streamed_stage(const moe_shape* shape, const int32_t* rows, int32_t n_moved,
                                const moe_machine* machine, double pcie_gbytes_per_s,
                                int32_t inputs_on_device, moe_streamed_estimate* out);

/* Tuning / testing knob of ONE context (it lasts until changed; set it from the thread that uses
 * the context): force the expert-GEMM tile configuration
 * (0 = large, 1 = medium, 2 = small, 3 = tiny rows-per-expert tile, 4 = the 96-row medium tile) or -1 for the automatic choice by
 * average rows per expert. Adding 16 to any of these makes the medium and small tiles load the
 * weights as ordinary (cached) lines, adding 32 as non-temporal ones; without either the library
 * picks non-temporal loads when about every expert has a single row tile (decode), where each
 * weight byte is used once. Adding 64 makes moe_layer_forward and its micro-batched form write
 * the gathered rows x_perm to the workspace and run the gate/up GEMM on them (the path taken by
 * itself when T*d_model*2 bytes do not fit 32 bits) instead of reading token rows through the
 * permutation. Adding 128 keeps the 256-row tiles of a last round that is less than half full
 * whole (by default each is run as two 128-row halves). Adding 256 / 512 runs the 256-row tiles
 * with eight wavefronts of 128 x 64 outputs / four of 128 x 128 (the default). Every setting produces identical bits (same accumulation chain per
 * output element); only speed differs. Returns MOE_ERR_INVALID_ARG for other values. */
int moe_set_gemm_config(moe_ctx* ctx, int config);

/* Precision of the expert outputs Yp between the down projection and the combine inside
 * moe_layer_forward, moe_layer_forward_microbatched and moe_layer_forward_streamed. The paper
 * fixes 2-byte operands only (Table 1 row 3 counts bf16 weights and inputs); by default Yp is
 * rounded to bf16 like the other intermediate, which is also what moe_expert_ffn and
 * moe_combine exchange. enable != 0: the down projection stores its fp32 accumulators and the
 * combine reads them, so an output element is rounded to bf16 once, after the gate-weighted
 * sum, instead of twice; costs 2*T*k*d_model more bytes written and as many more read per
 * call. Allocates a [T_max*k, d_model] fp32 buffer on the context's device, which must be the
 * calling thread's current device (MOE_ERR_WORKSPACE if the allocation fails); enable == 0
 * frees it again, the caller having drained the stream first. Routing, permutation and the
 * accumulation order are unchanged; outputs of the two settings differ by that one rounding.
 * Not a stream call: do not make it while a stream is being captured. */
int moe_set_expert_output_fp32(moe_ctx* ctx, int enable);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
