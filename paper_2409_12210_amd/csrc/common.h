// Internal declarations shared by the translation units of libmodse (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "modse.h"

#define MODSE_MAX_EXPERTS 64
#define MODSE_MAX_PROBLEMS (3 * MODSE_MAX_EXPERTS)  // the three weight-gradient GEMMs share one launch
#define MODSE_SKINNY_TOKENS 64           // batches up to this size take the decode-shaped forward GEMMs
#define MODSE_PERMUTE_SMALL_MAX_T 64      // batches up to this size take the fused permute + plan launch
#define MODSE_ROUTE_TOKENS_PER_BLOCK 32  // tokens handled by one block of the router / scatter kernels

typedef __bf16 bf16_t;
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------- element helpers
// 8 consecutive elements -> 8 floats
__device__ inline void load8(const float* p, float v[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ inline void load8(const bf16_t* p, float v[8]) {
  const bf16x8 a = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
__device__ inline void store8(float* p, const float v[8]) {
  f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
  *reinterpret_cast<f32x4*>(p) = a;
  *reinterpret_cast<f32x4*>(p + 4) = b;
}
__device__ inline void store8(bf16_t* p, const float v[8]) {
  bf16x8 a;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (bf16_t)v[i];
  *reinterpret_cast<bf16x8*>(p) = a;
}
__device__ inline void load4(const float* p, float v[4]) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
}
__device__ inline void load4(const bf16_t* p, float v[4]) {
  const bf16x4 a = *reinterpret_cast<const bf16x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = (float)a[i];
}
__device__ inline void store4(float* p, const float v[4]) {
  f32x4 a = {v[0], v[1], v[2], v[3]};
  *reinterpret_cast<f32x4*>(p) = a;
}
__device__ inline void store4(bf16_t* p, const float v[4]) {
  bf16x4 a;
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = (bf16_t)v[i];
  *reinterpret_cast<bf16x4*>(p) = a;
}

// ---------------------------------------------------------------- grouped GEMM
// One problem per expert:  C[M,N] (+)= A B^T (+ A2 B2^T).  How A and B lie in memory is a property of the
// kernel instantiation (GemmLayout); lda / ldb are the row strides of the stored matrices.  The bf16 kernel
// reads a problem with three scalar loads (64 + 32 + 8 bytes), hence the field order and the alignment.
struct alignas(128) GemmProblem {
  const void* A;
  const void* B;
  const void* A2;  // second operand pair of a K-concatenated product (dX = dA W1 + dB W3), or null
  const void* B2;  // second B matrix: W3 of the up-projection (two accumulators) or pair of A2
  void* C;
  void* C2;        // extra outputs of fused epilogues
  void* C3;
  const void* E1;  // extra epilogue inputs
  const void* E2;
  int32_t M, N, K;
  int32_t lda, ldb, ldc;
  int32_t mtiles, ntiles;
  // tile_magic.h: reciprocals that turn the two divisions of the tile decoding into multiplications
  uint32_t magic_group;  // by GROUP_M * ntiles (tiles in a full group of row blocks)
  uint32_t magic_tail;   // by mtiles % GROUP_M (row blocks of the last, shorter group)
};

struct GemmPlan {
  GemmProblem prob[MODSE_MAX_PROBLEMS];
  int32_t tile_start[MODSE_MAX_PROBLEMS + 1];  // prefix sum of mtiles*ntiles in problem order
  int32_t n_prob;
  int32_t pad[2];
};

enum GemmEpilogue {
  EPI_STORE = 0,       // C = acc (element type of the layer)
  EPI_STORE_F32 = 1,   // C = acc or C += acc, float32 (weight gradients)
  EPI_SWIGLU = 2,      // two accumulators a, b: C = h = silu(a)*b; optionally C2 = dh/da, C3 = dh/db
  EPI_SWIGLU_BWD = 3,  // acc = dh; E1 = dh/da, E2 = dh/db (saved by the forward pass): C = da, C2 = db
  EPI_STORE_DUALK = 4, // C = acc over two operand pairs (A,B) and (A2,B2)
};

enum GemmLayout {
  LAYOUT_TN = 0,    // A [M,K], B [N,K]: both K-contiguous (forward GEMMs)
  LAYOUT_B_KN = 2,  // A [M,K], B [K,N]                    (data gradients: weights as they lie)
  LAYOUT_AB_K = 3,  // A [K,M], B [K,N]                    (weight gradients: contraction over tokens)
};

// Host-known description of the layer handed to kernels by value.
struct LayerDims {
  int32_t d, N, k;
  int32_t T;
  int32_t f[MODSE_MAX_EXPERTS];
  int32_t foff[MODSE_MAX_EXPERTS + 1];
  int32_t order[MODSE_MAX_EXPERTS];  // experts by descending width (ties: lower index)
};

struct RoutingPtrs {
  int32_t* topk_idx;
  float* topk_w;
  int32_t* counts;
  int32_t* offsets;
  int32_t* row_of;
  int32_t* src_of;
  int32_t* near_tie_count;
};

// Optional parts of the gate (device pointers; null W_noise = no noise term, null probs = no auxiliary loss).
struct GateExtPtrs {
  const void* W_noise;  // [d, N], layer dtype
  const float* gamma;   // [1]
  float eps;
  float* noise_pre;     // [T, N]  x W_noise
  float alpha;
  float* probs;         // [T, N]  softmax of H(x) over all experts
  float* aux_f;         // [N]
  float* aux_P;         // [N]
  float* aux_loss;      // [1]
};

// ---------------------------------------------------------------- launchers
// route.hip
// Scratch of the routing kernels.  wpad is needed only when n_experts is not one of 2, 4, 8, 16, 32, 64: the
// routers that read the router matrices from memory fetch whole rows with vector loads, so such matrices are
// first copied into rows of padded_experts(N) columns (W_gate, then W_noise).
struct RouteBufs {
  int32_t* blockhist;  // [ceil(T / MODSE_ROUTE_TOKENS_PER_BLOCK), N + 1]
  int32_t* near_flag;  // [T]
  void* wpad;          // route_wpad_bytes()
};
inline int padded_experts(int N) { return N <= 2 ? 2 : N <= 4 ? 4 : N <= 8 ? 8 : N <= 16 ? 16 : N <= 32 ? 32 : 64; }
inline size_t route_wpad_bytes(const LayerDims& L, size_t elem_size) {
  const int NE = padded_experts(L.N);
  return NE == L.N ? 0 : 2 * (size_t)L.d * NE * elem_size;
}
// launch_route = launch_router (logits, top-k, gate) + launch_permute (histogram, scan, stable scatter; Xp may
// be null).
hipError_t launch_router(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const float* bias,
                         const RoutingPtrs& R, const RouteBufs& B, const GateExtPtrs* G, hipStream_t s);
struct FwdPlanArgs;
// plan != null: the scan launch also makes the tile plans of the two forward GEMMs (batches of at most
// MODSE_PERMUTE_SMALL_MAX_T tokens do all of this in one launch)
hipError_t launch_permute(const LayerDims& L, modse_dtype dt, const void* x, const RoutingPtrs& R, const RouteBufs& B,
                          void* Xp, const GateExtPtrs* G, const FwdPlanArgs* plan, hipStream_t s);
hipError_t launch_route(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const float* bias,
                        const RoutingPtrs& R, const RouteBufs& B, void* Xp, const GateExtPtrs* G, hipStream_t s);
hipError_t launch_routing_stats(const LayerDims& L, const int32_t* topk_idx, int32_t* slot_counts, float* summary,
                                hipStream_t s);
hipError_t launch_combine(const LayerDims& L, modse_dtype dt, const void* O, const RoutingPtrs& R, void* y,
                          hipStream_t s);
hipError_t launch_combine_split(const LayerDims& L, modse_dtype dt, const float* Opart, int kchunk, const RoutingPtrs& R,
                                void* y, hipStream_t s);
hipError_t launch_bwd_prep(const LayerDims& L, modse_dtype dt, const void* dY, const void* O, const RoutingPtrs& R,
                           void* dO, float* dg, hipStream_t s);
struct BwdRouterBufs {  // workspace of the router's backward pass
  float* dl;           // [T, N] dense gradient of the logits
  float* du;           // [T, N] gradient of x W_noise
  float* dgamma_part;  // [ceil(T / 256)]
  float* dW_partial;   // [ceil(T / 32), d, N] per-block shares of a router-side weight gradient (32 tokens per block)
};
hipError_t launch_bwd_router(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const void* dXp,
                             const float* dg, const RoutingPtrs& R, const GateExtPtrs* G, float aux_grad,
                             const BwdRouterBufs& B, void* dX, float* dW_gate, float* dW_noise, float* dgamma,
                             int accumulate, hipStream_t s);

// gemm.hip
struct TileShape {
  int32_t bm, bn;
};
TileShape gemm_tile_shape(modse_dtype dt, int epilogue, int64_t T);
// layout < 0: the layout that goes with the epilogue (see gemm.hip); skinny: the plan was made with the
// decode-sized tile shapes of gemm_tile_shape (every problem has M <= MODSE_SKINNY_TOKENS)
hipError_t launch_grouped_gemm(modse_dtype dt, int epilogue, const GemmPlan* plan, int accumulate, int save_pre,
                               int64_t max_tiles, hipStream_t s, int layout = -1, int skinny = 0);

struct FwdPlanArgs {
  const void *Xp, *W1, *W3, *W2;
  void *H, *dHdA, *dHdB, *O;  // dHdA/dHdB (derivatives of h by the two pre-activations) may be null
  // split-K down-projection for decode-sized batches: expert e's K = f_e is cut into chunks of `kchunk`
  // columns; chunk c writes float32 partial sums to Opart[c] ([T*k, d] each), which the combine step adds up.
  float* Opart;
  int32_t kchunk;  // 0 = no split
  GemmPlan *up, *down;
  TileShape up_tile, down_tile;
};

struct BwdPlanArgs {
  const void *Xp, *dO, *H, *dHdA, *dHdB;
  const void *W1, *W3, *W2;
  void *dA, *dB, *dXp;
  float *dW1, *dW3, *dW2;
  GemmPlan *dh, *dx, *wg;  // wg: dW1, dW3 and dW2 of every expert in one problem list
  TileShape dh_tile, dx_tile, wg_tile;
};
hipError_t launch_plan_bwd(const LayerDims& L, modse_dtype dt, const int32_t* counts, const int32_t* offsets,
                           const BwdPlanArgs& a, hipStream_t s);
