// Ragged grouped GEMMs of the MoDSE layer on gfx950: one problem per expert, M = tokens routed to the
// expert (known only on the device), N or K = the expert's own hidden width d_ff[e] (Sec. 3.1 of
// arXiv 2409.12210).  A tiny plan kernel turns the device-side counts into a problem table and a tile
// prefix; persistent GEMM workgroups walk the tile list without any host round trip.
//
// Operand layouts (GemmLayout): every tensor of the layer is used as it lies in memory.  The forward
// GEMMs have both operands K-contiguous; the data-gradient GEMMs read the weights as [K, N]; the
// weight-gradient GEMMs contract over tokens and read both activations as [K, M] and [K, N].
#include "common.h"
#include "gemm_bf16.h"
#include "gemm_bf16_skinny.h"
#include "gemm_plan.h"
#include "gemm_tiles.h"

namespace {
using namespace modse_gemm;

// ------------------------------------------------------------------------------------------------
// float32 path: plain FMA tiles (parity configuration; no throughput claim)
// ------------------------------------------------------------------------------------------------
template <int EPI, int LAYOUT>
__global__ __launch_bounds__(256) void gg_f32_kernel(const GemmPlan* __restrict__ plan, int accumulate,
                                                     int save_pre) {
  constexpr int BM = 64, BN = 64, BK = 16;
  constexpr int NB = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr bool A_T = (LAYOUT & 1) != 0, B_T = (LAYOUT & 2) != 0;
  static_assert(!(B_T && NB == 2), "the two-matrix up-projection reads K-contiguous weights");
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[NB][BK][BN + 4];
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  // K-contiguous operand: thread loads 4 consecutive k of row tid/4; [K, X] operand: 4 consecutive x of K row tid/16
  const int lrow = tid / 4, lk = (tid % 4) * 4;
  const int tk = tid / 16, tx4 = (tid % 16) * 4;
  const int total = plan->tile_start[plan->n_prob];
  for (int tile = first_tile_of_block(); tile < total; tile += gridDim.x) {
    TileCoord tc;
    if (!decode_tile(plan, tile, tc)) break;
    const GemmProblem P = plan->prob[tc.p];
    const int m0 = tc.mt * BM, n0 = tc.nt * BN;
    float acc[NB][4][4];
#pragma unroll
    for (int q = 0; q < NB; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[q][i][j] = 0.f;
    const int arow = min(m0 + lrow, P.M - 1), brow = min(n0 + lrow, P.N - 1);
    const int acol = min(m0 + tx4, P.M - 4), bcol = min(n0 + tx4, P.N - 4);  // M, N are multiples of 4
    const int npass = (EPI == EPI_STORE_DUALK) ? 2 : 1;
    for (int pass = 0; pass < npass; ++pass) {
      const float* A = static_cast<const float*>(pass ? P.A2 : P.A);
      const float* B = static_cast<const float*>(pass ? P.B2 : P.B);
      const float* B2 = static_cast<const float*>(P.B2);
      for (int k0 = 0; k0 < P.K; k0 += BK) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        f32x4 av, bv, b2v = zero;
        if (A_T) av = k0 + tk < P.K ? *reinterpret_cast<const f32x4*>(A + (size_t)(k0 + tk) * P.lda + acol) : zero;
        else av = *reinterpret_cast<const f32x4*>(A + (size_t)arow * P.lda + k0 + lk);  // K % 16 == 0 here
        if (B_T) bv = k0 + tk < P.K ? *reinterpret_cast<const f32x4*>(B + (size_t)(k0 + tk) * P.ldb + bcol) : zero;
        else bv = *reinterpret_cast<const f32x4*>(B + (size_t)brow * P.ldb + k0 + lk);
        if (NB == 2) b2v = *reinterpret_cast<const f32x4*>(B2 + (size_t)brow * P.ldb + k0 + lk);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (A_T) As[tk][tx4 + i] = av[i];
          else As[lk + i][lrow] = av[i];
          if (B_T) Bs[0][tk][tx4 + i] = bv[i];
          else Bs[0][lk + i][lrow] = bv[i];
          if (NB == 2) Bs[NB - 1][lk + i][lrow] = b2v[i];
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
          float a[4], b[NB][4];
#pragma unroll
          for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
          for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) b[q][j] = Bs[q][k][tx * 4 + j];
#pragma unroll
          for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int j = 0; j < 4; ++j) acc[q][i][j] = fmaf(a[i], b[q][j], acc[q][i][j]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i)
      epilogue4<float, EPI>(P, m0 + ty * 4 + i, n0 + tx * 4, acc[0][i], acc[NB - 1][i], accumulate, save_pre);
  }
}

// ------------------------------------------------------------------------------------------------
// plan kernel of the backward GEMMs (single block): device-side counts -> problem tables.  (The forward plans
// are made by the routing stage's scan launch, see gemm_plan.h.)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void plan_bwd_kernel(LayerDims L, int esize, const int32_t* __restrict__ counts,
                                                      const int32_t* __restrict__ offsets, BwdPlanArgs a) {
  __shared__ int s_tiles[MODSE_MAX_PROBLEMS];
  const int i = threadIdx.x;
  const bool on = i < L.N;
  const int e = on ? L.order[i] : 0;
  size_t hoff = 0;
  for (int q = 0; q < e; ++q) hoff += (size_t)counts[q] * L.f[q];
  const int n_e = counts[e], f = L.f[e], d = L.d;
  const size_t es = esize;
  const size_t woff = (size_t)L.foff[e] * d;   // element offset of expert e in W1/W3/W2 and their gradients
  const size_t roff = (size_t)offsets[e] * d;  // element offset of expert e's rows in [T*k, d] tensors
  if (on) {  // dh = dO W2 (W2_e is [d, f]: a [K, N] operand), fused SwiGLU backward -> dA, dB
    GemmProblem P = {};
    P.A = cadd(a.dO, roff * es);
    P.B = cadd(a.W2, woff * es);
    P.C = vadd(a.dA, hoff * es);
    P.C2 = vadd(a.dB, hoff * es);
    P.E1 = cadd(a.dHdA, hoff * es);
    P.E2 = cadd(a.dHdB, hoff * es);
    P.M = n_e; P.N = f; P.K = d;
    P.lda = d; P.ldb = f; P.ldc = f;
    s_tiles[i] = set_tiles(P, a.dh_tile.bm, a.dh_tile.bn);
    a.dh->prob[i] = P;
  }
  finish_plan(a.dh, i, L.N, s_tiles);
  if (on) {  // dXp = dA W1 + dB W3 (W1_e, W3_e are [f, d]: [K, N] operands)
    GemmProblem P = {};
    P.A = cadd(a.dA, hoff * es);
    P.B = cadd(a.W1, woff * es);
    P.A2 = cadd(a.dB, hoff * es);
    P.B2 = cadd(a.W3, woff * es);
    P.C = vadd(a.dXp, roff * es);
    P.M = n_e; P.N = d; P.K = f;
    P.lda = f; P.ldb = d; P.ldc = d;
    s_tiles[i] = set_tiles(P, a.dx_tile.bm, a.dx_tile.bn);
    a.dx->prob[i] = P;
  }
  finish_plan(a.dx, i, L.N, s_tiles);
  // Weight gradients contract over the expert's tokens, so a tile costs n_e K-steps whatever its expert's
  // width: the three GEMMs of one expert are listed together, experts by falling token count.
  if (on) {
    int rank = 0;
    for (int q = 0; q < L.N; ++q) rank += (counts[q] > n_e || (counts[q] == n_e && q < e)) ? 1 : 0;
    for (int which = 0; which < 2; ++which) {  // dW1 = dA^T Xp, dW3 = dB^T Xp
      GemmProblem P = {};
      P.A = cadd(which ? a.dB : a.dA, hoff * es);  // [K = n_e, M = f]
      P.B = cadd(a.Xp, roff * es);                  // [K = n_e, N = d]
      P.C = (which ? a.dW3 : a.dW1) + woff;
      P.M = f; P.N = d; P.K = n_e;
      P.lda = f; P.ldb = d; P.ldc = d;
      s_tiles[3 * rank + which] = set_tiles(P, a.wg_tile.bm, a.wg_tile.bn);
      a.wg->prob[3 * rank + which] = P;
    }
    GemmProblem P = {};  // dW2 = dO^T H
    P.A = cadd(a.dO, roff * es);  // [K = n_e, M = d]
    P.B = cadd(a.H, hoff * es);   // [K = n_e, N = f]
    P.C = a.dW2 + woff;
    P.M = d; P.N = f; P.K = n_e;
    P.lda = d; P.ldb = f; P.ldc = f;
    s_tiles[3 * rank + 2] = set_tiles(P, a.wg_tile.bm, a.wg_tile.bn);
    a.wg->prob[3 * rank + 2] = P;
  }
  finish_plan(a.wg, i, 3 * L.N, s_tiles);
}

int num_cus() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      n = prop.multiProcessorCount;
    if (n <= 0) n = 256;
  }
  return n;
}

template <int BM, int BN, int NB, int WAVES_M, int WAVES_N, int EPI, int LAYOUT>
hipError_t run_bf16(const GemmPlan* plan, int accumulate, int save_pre, int64_t max_tiles, hipStream_t s) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  int64_t grid = num_cus();  // the LDS panels fill a CU: one persistent workgroup per CU
  if (max_tiles < grid) grid = max_tiles;
  if (grid < 1) grid = 1;
  if constexpr (BM == 64) {  // decode-sized batches
    hipLaunchKernelGGL((gg_bf16_skinny_kernel<BM, BN, NB, WAVES_M, WAVES_N, EPI, LAYOUT>), dim3((unsigned)grid), dim3(NT), 0,
                       s, plan, accumulate, save_pre);
  } else {
    hipLaunchKernelGGL((gg_bf16_kernel<BM, BN, NB, WAVES_M, WAVES_N, EPI, LAYOUT>), dim3((unsigned)grid), dim3(NT), 0, s,
                       plan, accumulate, save_pre);
  }
  return hipGetLastError();
}

template <int EPI, int LAYOUT>
hipError_t run_f32(const GemmPlan* plan, int accumulate, int save_pre, int64_t max_tiles, hipStream_t s) {
  int64_t grid = (int64_t)num_cus() * 8;
  if (max_tiles < grid) grid = max_tiles;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL((gg_f32_kernel<EPI, LAYOUT>), dim3((unsigned)grid), dim3(256), 0, s, plan, accumulate, save_pre);
  return hipGetLastError();
}

}  // namespace

// Forward GEMMs of a decode-sized batch (no expert can have more than MODSE_SKINNY_TOKENS rows) use tiles
// 64 rows high and 8 waves wide: 8/9 of what a stage loads is weights instead of half.
TileShape gemm_tile_shape(modse_dtype dt, int epilogue, int64_t T) {
  if (dt == MODSE_F32) return {64, 64};
  const bool skinny = T <= MODSE_SKINNY_TOKENS && (epilogue == EPI_SWIGLU || epilogue == EPI_STORE);
  if (epilogue == EPI_SWIGLU) return skinny ? TileShape{64, 256} : TileShape{256, 128};
  return skinny ? TileShape{64, 512} : TileShape{256, 256};
}

// The epilogue fixes the operand layout: forward GEMMs are K-contiguous on both sides, data gradients read
// the weights as [K, N], weight gradients read both activations token-major.
hipError_t launch_grouped_gemm(modse_dtype dt, int epilogue, const GemmPlan* plan, int accumulate, int save_pre,
                               int64_t max_tiles, hipStream_t s, int layout, int skinny) {
  if (epilogue == EPI_STORE_F32 && layout == LAYOUT_TN) {  // split-K partial sums of a forward GEMM
    if (dt == MODSE_F32) return run_f32<EPI_STORE_F32, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
    if (skinny) return run_bf16<64, 512, 1, 1, 8, EPI_STORE_F32, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
    return run_bf16<256, 256, 1, 4, 2, EPI_STORE_F32, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
  }
  if (dt == MODSE_BF16 && skinny) {
    if (epilogue == EPI_SWIGLU)
      return run_bf16<64, 256, 2, 1, 8, EPI_SWIGLU, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
    if (epilogue == EPI_STORE)
      return run_bf16<64, 512, 1, 1, 8, EPI_STORE, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
  }
  if (dt == MODSE_F32) {
    switch (epilogue) {
      case EPI_STORE: return run_f32<EPI_STORE, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
      case EPI_SWIGLU: return run_f32<EPI_SWIGLU, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
      case EPI_SWIGLU_BWD: return run_f32<EPI_SWIGLU_BWD, LAYOUT_B_KN>(plan, accumulate, save_pre, max_tiles, s);
      case EPI_STORE_DUALK: return run_f32<EPI_STORE_DUALK, LAYOUT_B_KN>(plan, accumulate, save_pre, max_tiles, s);
      case EPI_STORE_F32: return run_f32<EPI_STORE_F32, LAYOUT_AB_K>(plan, accumulate, save_pre, max_tiles, s);
    }
    return hipErrorInvalidValue;
  }
  switch (epilogue) {
    case EPI_STORE:
      return run_bf16<256, 256, 1, 4, 2, EPI_STORE, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
    case EPI_SWIGLU:
      return run_bf16<256, 128, 2, 4, 2, EPI_SWIGLU, LAYOUT_TN>(plan, accumulate, save_pre, max_tiles, s);
    case EPI_SWIGLU_BWD:
      return run_bf16<256, 256, 1, 4, 2, EPI_SWIGLU_BWD, LAYOUT_B_KN>(plan, accumulate, save_pre, max_tiles, s);
    case EPI_STORE_DUALK:
      return run_bf16<256, 256, 1, 4, 2, EPI_STORE_DUALK, LAYOUT_B_KN>(plan, accumulate, save_pre, max_tiles, s);
    case EPI_STORE_F32:
      return run_bf16<256, 256, 1, 4, 2, EPI_STORE_F32, LAYOUT_AB_K>(plan, accumulate, save_pre, max_tiles, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_plan_bwd(const LayerDims& L, modse_dtype dt, const int32_t* counts, const int32_t* offsets,
                           const BwdPlanArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(plan_bwd_kernel, dim3(1), dim3(64), 0, s, L, dt == MODSE_F32 ? 4 : 2, counts, offsets, a);
  return hipGetLastError();
}
