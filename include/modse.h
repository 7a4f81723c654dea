/*
 * modse.h - C ABI of the MI355X (gfx950) library for one Mixture-of-Diverse-
 * Size-Experts (MoDSE) FFN layer, arXiv 2409.12210.
 *
 * The layer (Sec. 2 Eq. 1-3 and Sec. 3.1 of the paper):
 *     logits  H(x)_i = (x W_gate)_i (+ logit_bias_i)
 *     gate    G(x)   = Softmax(KeepTopK(H(x), top_k))         (Eq. 2, Eq. 3)
 *     output  y      = sum_i G_i(x) E_i(x)                     (Eq. 1; Sec. 3.1)
 *     expert  E_i(x) = W2_i ( silu(W1_i x) * (W3_i x) ),  W1_i,W3_i in R^{d_ff[i] x d},
 *                      W2_i in R^{d x d_ff[i]}                 (Llama-2 FFN, Sec. 4.1)
 * Each expert has its own hidden width d_ff[i] (Sec. 3.1).  Ties in top-k go to
 * the lower expert index; no token is ever dropped.
 *
 * Conventions for every call
 *  - "HOST" / "DEVICE" says where a pointer must point.  The library allocates
 *    and frees nothing: all buffers, workspace included, belong to the caller.
 *  - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*,
 *    NULL = the default stream).  They never synchronise and never read device
 *    memory from the host.
 *  - All argument checks run before the first enqueue and need no GPU.
 *    Errors are reported through the return code only.
 *  - T == 0 is valid and does nothing (pointers are then not examined).
 *  - NaN/Inf inputs: behaviour unspecified.
 *
 * Layouts (row-major everywhere, element type = desc.dtype unless said):
 *    x, y, dY, dX   [T, d_model]
 *    W_gate         [d_model, n_experts]
 *    W1, W3         one [F, d_model] matrix, F = sum d_ff; expert e owns rows
 *                   foff[e] .. foff[e+1]-1, foff[e] = sum_{e'<e} d_ff[e']
 *    W2             expert e starts at element d_model*foff[e] and is a
 *                   [d_model, d_ff[e]] matrix
 *    dW_gate, dW1, dW3, dW2   float32, same shapes as the weights
 */
#ifndef MODSE_H_
#define MODSE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MODSE_OK = 0,
  MODSE_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad d_ff, ... */
  MODSE_ERR_UNSUPPORTED = 2, /* top_k not in {1,2}, n_experts > 64, unknown dtype */
  MODSE_ERR_WORKSPACE = 3,   /* ws_bytes smaller than modse_workspace_size() */
  MODSE_ERR_HIP = 4          /* a HIP launch failed */
} modse_status;

typedef enum { MODSE_F32 = 0, MODSE_BF16 = 1 } modse_dtype;

/* Layer description.  Plain HOST struct, read during the call only. */
typedef struct {
  int32_t d_model;      /* multiple of 32 */
  int32_t n_experts;    /* N, 1..64 */
  int32_t top_k;        /* 1 or 2, <= N */
  const int32_t* d_ff;  /* HOST array [n_experts]; each > 0 and a multiple of 32;
                           any order, pairs are not assumed (Sec. 3.1 pair
                           constraint is the caller's business) */
  modse_dtype dtype;    /* element type of x, weights, y, dY, dX */
} modse_desc;

/* Routing artefacts, all DEVICE pointers, caller-allocated.  Permuted row r of
 * expert e lies in offsets[e] <= r < offsets[e+1]; inside an expert rows keep
 * ascending token order. */
typedef struct {
  int32_t* topk_idx;       /* [T, top_k] expert ids, slot 0 = largest logit */
  float* topk_w;           /* [T, top_k] gate weights (Eq. 2), sum to 1 per token */
  int32_t* counts;         /* [N] tokens*slots per expert */
  int32_t* offsets;        /* [N+1] exclusive prefix sum of counts */
  int32_t* row_of;         /* [T, top_k] (token, slot) -> permuted row */
  int32_t* src_of;         /* [T*top_k] permuted row -> token*top_k + slot */
  int32_t* near_tie_count; /* [1] tokens with a gap < 1e-6 between two neighbouring
                              logits among their top_k+1 largest */
} modse_routing;

/* Bytes of DEVICE workspace `ws` that a call requires for T tokens.  `which`:
 * MODSE_WS_FWD for modse_route and for modse_layer_fwd without `saved`,
 * MODSE_WS_BWD for modse_layer_bwd, MODSE_WS_FWD_SAVED for modse_layer_fwd
 * with `saved` (the permuted rows, hidden activations and expert outputs then
 * live in `saved`, and the workspace holds routing scratch and tile plans
 * only; a MODSE_WS_FWD workspace also serves that call).  Any other value:
 * MODSE_ERR_INVALID_ARG. */
#define MODSE_WS_FWD 0
#define MODSE_WS_BWD 1
#define MODSE_WS_FWD_SAVED 2
modse_status modse_workspace_size(const modse_desc* desc, int64_t T, int which, size_t* bytes);

/* Bytes of the DEVICE buffer `saved` that carries activations from
 * modse_layer_fwd to modse_layer_bwd (the derivatives of the SwiGLU hidden
 * activation by its two pre-activations W1 x and W3 x, the hidden activations,
 * the expert outputs and the permuted token rows, all in permuted row order).
 * Its layout is private. */
modse_status modse_saved_size(const modse_desc* desc, int64_t T, size_t* bytes);

/* Router only: logits, top-k, gate weights (Eq. 2-3) and the stable permutation
 * by expert.  x [T,d] DEVICE, W_gate [d,N] DEVICE, logit_bias [N] float32
 * DEVICE or NULL.  Fills every field of *out. */
modse_status modse_route(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                         const float* logit_bias, const modse_routing* out, void* ws, size_t ws_bytes,
                         void* hip_stream);

/* modse_route for callers that cannot allocate or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The router's scratch (per-block histograms, near-tie flags) is a device
 * array inside the library, MODSE_ROUTE_STATIC_SCRATCH_BYTES per GPU, held
 * until the process ends; the call allocates and frees nothing.  Same
 * arguments, results and checks as modse_route otherwise.  The need is about
 * T * (4 + (n_experts + 1) / 8) bytes, so the array serves 65536 tokens at
 * any expert count that is a power of two (other counts also keep a padded
 * copy of W_gate there, 2 * d_model * 64 elements at most); a call whose
 * scratch does not fit returns MODSE_ERR_WORKSPACE before anything is
 * launched.  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams) race. */
#define MODSE_ROUTE_STATIC_SCRATCH_BYTES (1u << 20)
modse_status modse_route_static(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                                const float* logit_bias, const modse_routing* out, void* hip_stream);

/* Forward pass of the layer (Eq. 1 with diverse-size experts, Sec. 3.1):
 * route, permute, grouped up-projection with SwiGLU, grouped down-projection,
 * gate-weighted combine.  y [T,d] DEVICE out.  routing_out may be NULL unless
 * a backward pass follows; saved may be NULL unless a backward pass follows. */
modse_status modse_layer_fwd(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                             const float* logit_bias, const void* W1, const void* W3, const void* W2, void* y,
                             const modse_routing* routing_out, void* saved, void* ws, size_t ws_bytes,
                             void* hip_stream);

/* Backward pass (chain rule through Eq. 1-3; logits outside the kept set get
 * zero gradient).  routing and saved are the ones modse_layer_fwd filled for
 * the same inputs.  dY [T,d] DEVICE in.  Outputs: dX [T,d] (desc.dtype),
 * dW_gate [d,N], dW1 [F,d], dW3 [F,d], dW2 (packed like W2), all float32.
 * accumulate = 0 overwrites the weight gradients, 1 adds to them (fp32
 * gradient accumulation); dX is always overwritten. */
modse_status modse_layer_bwd(const modse_desc* desc, int64_t T, const void* x, const void* W_gate, const void* W1,
                             const void* W3, const void* W2, const modse_routing* routing, const void* saved,
                             const void* dY, void* dX, float* dW_gate, float* dW1, float* dW3, float* dW2,
                             int accumulate, void* ws, size_t ws_bytes, void* hip_stream);

/* ---------------------------------------------------------------- optional parts of the gate
 * One struct switches on the two parts of the paper's gate that the plain
 * entry points leave out.  All pointers are DEVICE pointers owned by the
 * caller; the forward call fills the outputs, the backward call reads them.
 *
 * Noise term (second term of H(x) in Sec. 2, with Eq. 4 RMSNorm and Eq. 5
 * Softplus): H(x)_i += gamma * s_i / sqrt(mean_j s_j^2 + eps), s = Softplus(x
 * W_noise), the norm taken over the N per-expert values of one token.  It has
 * no random factor, so it is a function of x.  On when W_noise != NULL; then
 * gamma and noise_pre are required.
 *
 * Auxiliary load-balance loss (Sec. 3.2 Eq. 9-12): p(x) = softmax of H(x) over
 * all N experts, f_i = share of tokens whose largest probability is expert i
 * (ties to the lower index), P_i = mean of p_i, L_a = aux_alpha N sum_i f_i
 * P_i.  On when probs != NULL; then aux_f, aux_P and aux_loss are required. */
typedef struct {
  const void* W_noise; /* [d,N], desc.dtype, or NULL */
  const float* gamma;  /* [1] RMSNorm gain */
  float eps;           /* RMSNorm epsilon, >= 0 */
  float* noise_pre;    /* [T,N] x W_noise: written by forward, read by backward */
  float aux_alpha;     /* alpha of Eq. 9 */
  float* probs;        /* [T,N] p(x): written by forward, read by backward; or NULL */
  float* aux_f;        /* [N] f_i: written by forward, read by backward */
  float* aux_P;        /* [N] P_i */
  float* aux_loss;     /* [1] L_a */
} modse_gate_ext;

/* modse_route / modse_layer_fwd with the optional gate parts; ext == NULL is
 * the plain call.  Same workspace sizes.  An incomplete ext (a switched-on
 * part with a missing pointer, eps < 0) returns MODSE_ERR_INVALID_ARG. */
modse_status modse_route_ext(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                             const float* logit_bias, const modse_gate_ext* ext, const modse_routing* out, void* ws,
                             size_t ws_bytes, void* hip_stream);
modse_status modse_layer_fwd_ext(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                                 const float* logit_bias, const modse_gate_ext* ext, const void* W1, const void* W3,
                                 const void* W2, void* y, const modse_routing* routing_out, void* saved, void* ws,
                                 size_t ws_bytes, void* hip_stream);

/* Backward pass of loss = <dY, y> + aux_grad * L_a through the gate with its
 * optional parts: adds aux_grad * dL_a/dH (f_i held constant, as it is
 * piecewise constant) to the gradient of the logits, and, when the noise term
 * is on, also returns dW_noise [d,N] float32 and dgamma [1] float32 (both
 * follow `accumulate`) and adds the term's share to dX.  ext must hold the
 * buffers the forward call filled. */
modse_status modse_layer_bwd_ext(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                                 const modse_gate_ext* ext, float aux_grad, const void* W1, const void* W3,
                                 const void* W2, const modse_routing* routing, const void* saved, const void* dY,
                                 void* dX, float* dW_gate, float* dW_noise, float* dgamma, float* dW1, float* dW3,
                                 float* dW2, int accumulate, void* ws, size_t ws_bytes, void* hip_stream);

/* Routing statistics in the shape of the paper's Appendix A tables, from
 * routing->topk_idx: slot_counts [top_k,N] int32 DEVICE out (tokens whose j-th
 * choice is expert i); summary [top_k+2] float32 DEVICE out: max/min of each
 * slot's counts, max/min of the per-expert totals, and the average hidden
 * width of the chosen experts (the workload measure of Sec. 4.3).  A ratio
 * whose minimum is 0 reads +inf. */
modse_status modse_routing_stats(const modse_desc* desc, int64_t T, const modse_routing* routing,
                                 int32_t* slot_counts, float* summary, void* hip_stream);

/* Per-stage timing for benchmarks.  When enabled, modse_layer_fwd/bwd record
 * HIP events between their stages on the caller's stream; modse_stage_times
 * waits for the last recorded call and returns milliseconds per stage
 * (HOST array of MODSE_N_STAGES floats; stages not run read 0). */
enum {
  MODSE_STAGE_ROUTE = 0,    /* router GEMM + top-k + gate (+ auxiliary loss) */
  MODSE_STAGE_PERMUTE = 1,  /* histogram, scan over blocks (+ the tile plans of the forward GEMMs), stable row scatter */
  MODSE_STAGE_UP = 2,       /* grouped W1/W3 GEMM + SwiGLU */
  MODSE_STAGE_DOWN = 3,     /* grouped W2 GEMM */
  MODSE_STAGE_COMBINE = 4,  /* gate-weighted unpermute */
  MODSE_STAGE_BWD_PREP = 5, /* dO = g dY, d gate = <dY, O>, tile plans */
  MODSE_STAGE_BWD_DGRAD = 6,/* dH (+SwiGLU backward) and dX_permuted GEMMs */
  MODSE_STAGE_BWD_WGRAD = 7,/* dW1, dW3, dW2 GEMMs */
  MODSE_STAGE_BWD_ROUTER = 8,/* dX gather, d logits, dW_gate */
  MODSE_N_STAGES = 9
};
modse_status modse_stage_timing_enable(int on);
modse_status modse_stage_times(float* ms);

const char* modse_status_string(modse_status s);

#ifdef __cplusplus
}
#endif
#endif /* MODSE_H_ */
