// Router, permutation, combine and the element-wise backward kernels of the MoDSE layer (gfx950).
//
// Router: logits H(x) = x W_gate (+bias), KeepTopK, softmax over the kept logits (Sec. 2 Eq. 2-3 of
// arXiv 2409.12210).  Logits are accumulated in float64: products of bf16 or fp32 inputs are exact in
// float64, so the integer routing decision is taken at the same precision as a float64 reference and
// does not depend on summation order beyond the last bit.
#include "common.h"

namespace {

constexpr int TPB = MODSE_ROUTE_TOKENS_PER_BLOCK;  // tokens per block
constexpr int ROUTE_THREADS = 256;
constexpr int TOK_PER_WAVE = TPB / (ROUTE_THREADS / 64);  // 8

__device__ inline double shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, 64);
  hi = __shfl_xor(hi, mask, 64);
  return __hiloint2double(hi, lo);
}

// Sum each of the V values over the 64 lanes of a wave.  Every halving step sends half of the values to
// the partner lane and keeps the other half, so V values cost V-1 + (6 - log2 V) shuffles.  On return
// lane l (l < V) holds in vals[0] the total of value index bitrev_{log2 V}(l).
template <int V>
struct Log2 {
  static constexpr int value = 1 + Log2<V / 2>::value;
};
template <>
struct Log2<1> {
  static constexpr int value = 0;
};

template <int V>
__device__ inline void wave_sum_values(double (&vals)[V], int lane) {
  constexpr int P = Log2<V>::value;
#pragma unroll
  for (int s = 0; s < P; ++s) {
    const int width = V >> (s + 1), bit = 1 << s;
    const bool upper = (lane & bit) != 0;
#pragma unroll
    for (int i = 0; i < width; ++i) {
      const double keep = upper ? vals[i + width] : vals[i];
      const double send = upper ? vals[i] : vals[i + width];
      vals[i] = keep + shfl_xor_f64(send, bit);
    }
  }
#pragma unroll
  for (int s = P; s < 6; ++s) vals[0] += shfl_xor_f64(vals[0], 1 << s);
}

template <int P>
__device__ inline int bitrev(int v) {
  int r = 0;
#pragma unroll
  for (int i = 0; i < P; ++i) r |= ((v >> i) & 1) << (P - 1 - i);
  return r;
}

// NE consecutive elements -> floats, with the widest aligned vector loads
template <int NE, typename T>
__device__ inline void load_row(const T* p, float* out) {
  if constexpr (NE % 8 == 0) {
#pragma unroll
    for (int e = 0; e < NE; e += 8) load8(p + e, out + e);
  } else if constexpr (NE == 4) {
    load4(p, out);
  } else {
#pragma unroll
    for (int e = 0; e < NE; ++e) out[e] = (float)p[e];
  }
}

// One block routes TPB consecutive tokens.  blockhist[b][0..N-1] = this block's per-expert assignment
// counts, blockhist[b][N] = its near-tie token count.
template <typename T, int NE, int TOK>
__global__ __launch_bounds__(ROUTE_THREADS) void router_kernel(const T* __restrict__ x, const T* __restrict__ Wg,
                                                               const float* __restrict__ bias, int ntok, int d, int N,
                                                               int top_k, int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_w,
                                                               int32_t* __restrict__ blockhist) {
  constexpr int V = NE * TOK;
  __shared__ double s_logit[ROUTE_THREADS / 64][TOK][NE];
  __shared__ int s_hist[MODSE_MAX_EXPERTS + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tok0 = blockIdx.x * TPB + wave * TOK_PER_WAVE;
  if (tid <= N) s_hist[tid] = 0;
  __syncthreads();

  for (int pass = 0; pass < TOK_PER_WAVE / TOK; ++pass) {
    const int tbase = tok0 + pass * TOK;
    double acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0;
    for (int c = lane * 8; c < d; c += 64 * 8) {
      float xv[TOK][8];
#pragma unroll
      for (int tt = 0; tt < TOK; ++tt) {
        const int t = min(tbase + tt, ntok - 1);  // rows past the end repeat the last token; never written
        load8(x + (size_t)t * d + c, xv[tt]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {  // one W_gate row at a time keeps the register footprint small
        double w[NE];
        const T* wrow = Wg + (size_t)(c + i) * N;
        float wf[NE];
        if (N == NE) {
          load_row<NE>(wrow, wf);  // one vector load per W_gate row
        } else {  // columns e >= N repeat the last expert; their sums are never looked at
#pragma unroll
          for (int e = 0; e < NE; ++e) wf[e] = (float)wrow[min(e, N - 1)];
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) w[e] = (double)wf[e];
#pragma unroll
        for (int tt = 0; tt < TOK; ++tt) {
          const double xd = (double)xv[tt][i];
#pragma unroll
          for (int e = 0; e < NE; ++e) acc[tt * NE + e] = fma(xd, w[e], acc[tt * NE + e]);
        }
      }
    }
    wave_sum_values<V>(acc, lane);
    if (lane < V) {
      const int v = bitrev<Log2<V>::value>(lane);
      s_logit[wave][v / NE][v % NE] = acc[0];
    }
    __syncthreads();
    if (lane < TOK && tbase + lane < ntok) {
      const int t = tbase + lane;
      double m1 = -INFINITY, m2 = -INFINITY, m3 = -INFINITY;
      int i1 = 0, i2 = 0;
      for (int e = 0; e < N; ++e) {
        double l = s_logit[wave][lane][e];
        if (bias) l += (double)bias[e];
        if (l > m1) {  // strict comparisons while scanning upward: ties stay with the lower index
          m3 = m2; m2 = m1; i2 = i1; m1 = l; i1 = e;
        } else if (l > m2) {
          m3 = m2; m2 = l; i2 = e;
        } else if (l > m3) {
          m3 = l;
        }
      }
      bool near;
      if (top_k == 2) {
        const double g1 = 1.0 / (1.0 + exp(m2 - m1));  // softmax over the two kept logits
        topk_idx[(size_t)t * 2] = i1;
        topk_idx[(size_t)t * 2 + 1] = i2;
        topk_w[(size_t)t * 2] = (float)g1;
        topk_w[(size_t)t * 2 + 1] = (float)(1.0 - g1);
        atomicAdd(&s_hist[i1], 1);
        atomicAdd(&s_hist[i2], 1);
        near = (m1 - m2 < 1e-6) || (N > 2 && m2 - m3 < 1e-6);
      } else {
        topk_idx[t] = i1;
        topk_w[t] = 1.f;
        atomicAdd(&s_hist[i1], 1);
        near = (N > 1 && m1 - m2 < 1e-6);
      }
      if (near) atomicAdd(&s_hist[N], 1);
    }
    __syncthreads();
  }
  if (tid <= N) blockhist[(size_t)blockIdx.x * (N + 1) + tid] = s_hist[tid];
}

// Single block.  Turns blockhist[b][e] into the exclusive prefix over blocks (in place) and writes
// counts, offsets and the near-tie total.  Each thread owns a contiguous run of blocks; the 256 run totals
// of one expert are scanned by the first wave.
__global__ __launch_bounds__(256) void route_scan_kernel(int32_t* __restrict__ blockhist, int nb, int N,
                                                         int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ near_tie_count) {
  __shared__ int s_part[256];
  __shared__ int s_total[MODSE_MAX_EXPERTS + 1];
  const int tid = threadIdx.x;
  const int per = (nb + 255) / 256;
  const int b0 = min(tid * per, nb), b1 = min(b0 + per, nb);
  const int W = N + 1;
  for (int e = 0; e < W; ++e) {
    int sum = 0;
    for (int b = b0; b < b1; ++b) sum += blockhist[(size_t)b * W + e];
    s_part[tid] = sum;
    __syncthreads();
    if (tid < 64) {
      int v[4], local = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = s_part[tid * 4 + i];
        local += v[i];
      }
      int incl = local;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if (tid >= o) incl += up;
      }
      int run = incl - local;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s_part[tid * 4 + i] = run;
        run += v[i];
      }
      if (tid == 63) s_total[e] = incl;
    }
    __syncthreads();
    if (e < N) {
      int run = s_part[tid];
      for (int b = b0; b < b1; ++b) {
        const int v = blockhist[(size_t)b * W + e];
        blockhist[(size_t)b * W + e] = run;
        run += v;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < N; ++e) {
      counts[e] = s_total[e];
      offsets[e] = run;
      run += s_total[e];
    }
    offsets[N] = run;
    near_tie_count[0] = s_total[N];
  }
}

// Stable scatter: permuted row = offsets[e] + (assignments to e in earlier blocks) + (earlier tokens of this
// block routed to e).  Also copies the token rows into expert-contiguous order when Xp is given.
template <typename T>
__global__ __launch_bounds__(ROUTE_THREADS) void scatter_kernel(const T* __restrict__ x, int ntok, int d, int N,
                                                                int top_k, const int32_t* __restrict__ topk_idx,
                                                                const int32_t* __restrict__ offsets,
                                                                const int32_t* __restrict__ blockbase,
                                                                int32_t* __restrict__ row_of,
                                                                int32_t* __restrict__ src_of, T* __restrict__ Xp) {
  __shared__ int s_row[TPB][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * TPB;
  if (wave == 0) {
    const int t = t0 + lane;
    const bool valid = lane < TPB && t < ntok;
    int e0 = -1, e1 = -1;
    if (valid) {
      e0 = topk_idx[(size_t)t * top_k];
      if (top_k == 2) e1 = topk_idx[(size_t)t * top_k + 1];
    }
    int r0 = 0, r1 = 0;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int e = 0; e < N; ++e) {
      const unsigned long long m = __ballot(e0 == e || e1 == e);
      const int rank = __popcll(m & below);
      if (e0 == e) r0 = rank;
      if (e1 == e) r1 = rank;
    }
    if (valid) {
      const int32_t* bb = blockbase + (size_t)blockIdx.x * (N + 1);
      const int row0 = offsets[e0] + bb[e0] + r0;
      row_of[(size_t)t * top_k] = row0;
      src_of[row0] = t * top_k;
      s_row[lane][0] = row0;
      if (top_k == 2) {
        const int row1 = offsets[e1] + bb[e1] + r1;
        row_of[(size_t)t * top_k + 1] = row1;
        src_of[row1] = t * top_k + 1;
        s_row[lane][1] = row1;
      }
    }
  }
  __syncthreads();
  if (Xp == nullptr) return;
  for (int i = 0; i < TOK_PER_WAVE; ++i) {
    const int tl = wave * TOK_PER_WAVE + i;
    const int t = t0 + tl;
    if (t >= ntok) break;
    const int row0 = s_row[tl][0];
    const int row1 = top_k == 2 ? s_row[tl][1] : -1;
    constexpr int VEC = 16 / sizeof(T);
    for (int c = lane * VEC; c < d; c += 64 * VEC) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(x + (size_t)t * d + c);
      *reinterpret_cast<f32x4*>(Xp + (size_t)row0 * d + c) = v;
      if (row1 >= 0) *reinterpret_cast<f32x4*>(Xp + (size_t)row1 * d + c) = v;
    }
  }
}

// Xp[r] = x[src_of[r] / k]   (one wave per permuted row)
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T* __restrict__ x, int nrows, int d, int top_k,
                                                          const int32_t* __restrict__ src_of, T* __restrict__ Xp) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= nrows) return;
  const int lane = threadIdx.x & 63;
  const int t = src_of[r] / top_k;
  constexpr int VEC = 16 / sizeof(T);
  for (int c = lane * VEC; c < d; c += 64 * VEC)
    *reinterpret_cast<f32x4*>(Xp + (size_t)r * d + c) = *reinterpret_cast<const f32x4*>(x + (size_t)t * d + c);
}

// y[t] = sum_j g[t,j] * O[row_of[t,j]]   (Eq. 1 on permuted expert outputs; one wave per token, fp32 math)
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ O, int ntok, int d, int top_k,
                                                      const int32_t* __restrict__ row_of,
                                                      const float* __restrict__ topk_w, T* __restrict__ y) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= ntok) return;
  const int lane = threadIdx.x & 63;
  const int r0 = row_of[(size_t)t * top_k];
  const float g0 = topk_w[(size_t)t * top_k];
  const int r1 = top_k == 2 ? row_of[(size_t)t * top_k + 1] : 0;
  const float g1 = top_k == 2 ? topk_w[(size_t)t * top_k + 1] : 0.f;
  for (int c = lane * 8; c < d; c += 64 * 8) {
    float a[8], b[8], o[8];
    load8(O + (size_t)r0 * d + c, a);
    if (top_k == 2) {
      load8(O + (size_t)r1 * d + c, b);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = g0 * a[i] + g1 * b[i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = g0 * a[i];
    }
    store8(y + (size_t)t * d + c, o);
  }
}

// Backward of the combine: for permuted row r = (token t, slot j):
//   dO[r] = g[t,j] * dY[t]      d g[t,j] = <dY[t], O[r]>
template <typename T>
__global__ __launch_bounds__(256) void bwd_prep_kernel(const T* __restrict__ dY, const T* __restrict__ O, int nrows,
                                                       int d, int top_k, const int32_t* __restrict__ src_of,
                                                       const float* __restrict__ topk_w, T* __restrict__ dO,
                                                       float* __restrict__ dg) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= nrows) return;
  const int lane = threadIdx.x & 63;
  const int s = src_of[r];
  const int t = s / top_k;
  const float g = topk_w[s];
  float dot = 0.f;
  for (int c = lane * 8; c < d; c += 64 * 8) {
    float a[8], o[8], w[8];
    load8(dY + (size_t)t * d + c, a);
    load8(O + (size_t)r * d + c, o);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      dot = fmaf(a[i], o[i], dot);
      w[i] = g * a[i];
    }
    store8(dO + (size_t)r * d + c, w);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
  if (lane == 0) dg[r] = dot;
}

// Backward through the gate and the router for TPB tokens per block:
//   dl_j = g_j (dg_j - sum_m g_m dg_m) on the kept logits, 0 elsewhere  (softmax over KeepTopK)
//   dX[t] = sum_j dXp[row_of[t,j]] + W_gate dl
//   partial[b] = sum_{t in block} x[t] (outer) dl[t]     (reduced over blocks by dwg_reduce_kernel)
template <typename T>
__global__ __launch_bounds__(ROUTE_THREADS) void bwd_router_kernel(
    const T* __restrict__ x, const T* __restrict__ Wg, const T* __restrict__ dXp, const float* __restrict__ dg,
    int ntok, int d, int N, int top_k, const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
    const int32_t* __restrict__ row_of, T* __restrict__ dX, float* __restrict__ partial) {
  __shared__ float s_dl[TPB][MODSE_MAX_EXPERTS];
  __shared__ int s_row[TPB][2];
  __shared__ int s_idx[TPB][2];
  __shared__ float s_dlk[TPB][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * TPB;
  for (int i = tid; i < TPB * MODSE_MAX_EXPERTS; i += ROUTE_THREADS) (&s_dl[0][0])[i] = 0.f;
  __syncthreads();
  if (tid < TPB && t0 + tid < ntok) {
    const int t = t0 + tid;
    float g[2] = {0.f, 0.f}, dgv[2] = {0.f, 0.f};
    float mean = 0.f;
    for (int j = 0; j < top_k; ++j) {
      const int r = row_of[(size_t)t * top_k + j];
      s_row[tid][j] = r;
      s_idx[tid][j] = topk_idx[(size_t)t * top_k + j];
      g[j] = topk_w[(size_t)t * top_k + j];
      dgv[j] = dg[r];
      mean += g[j] * dgv[j];
    }
    for (int j = 0; j < top_k; ++j) {
      const float dl = g[j] * (dgv[j] - mean);
      s_dlk[tid][j] = dl;
      s_dl[tid][s_idx[tid][j]] = dl;
    }
  }
  __syncthreads();
  for (int i = 0; i < TOK_PER_WAVE; ++i) {
    const int tl = wave * TOK_PER_WAVE + i;
    const int t = t0 + tl;
    if (t >= ntok) break;
    const int r0 = s_row[tl][0], e0 = s_idx[tl][0];
    const float dl0 = s_dlk[tl][0];
    const int r1 = top_k == 2 ? s_row[tl][1] : 0, e1 = top_k == 2 ? s_idx[tl][1] : 0;
    const float dl1 = top_k == 2 ? s_dlk[tl][1] : 0.f;
    for (int c = lane * 8; c < d; c += 64 * 8) {
      float a[8], o[8];
      load8(dXp + (size_t)r0 * d + c, a);
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = a[q] + dl0 * (float)Wg[(size_t)(c + q) * N + e0];
      if (top_k == 2) {
        load8(dXp + (size_t)r1 * d + c, a);
#pragma unroll
        for (int q = 0; q < 8; ++q) o[q] += a[q] + dl1 * (float)Wg[(size_t)(c + q) * N + e1];
      }
      store8(dX + (size_t)t * d + c, o);
    }
  }
  const int nt = min(TPB, ntok - t0);
  for (int c = tid; c < d; c += ROUTE_THREADS) {
    float xcol[TPB];
#pragma unroll
    for (int tl = 0; tl < TPB; ++tl) xcol[tl] = tl < nt ? (float)x[(size_t)(t0 + tl) * d + c] : 0.f;
    for (int e = 0; e < N; ++e) {
      float acc = 0.f;
#pragma unroll
      for (int tl = 0; tl < TPB; ++tl) acc = fmaf(xcol[tl], s_dl[tl][e], acc);
      partial[((size_t)blockIdx.x * d + c) * N + e] = acc;
    }
  }
}

// Same as bwd_router_kernel for N <= 8, one pass over the data: a thread owns 8 columns of d for all
// BR_TOK tokens of the block, keeps the 8 x 8 slice of W_gate and of the dW_gate partial in registers, and
// per token reads x and the two dXp rows once (16-byte loads, a full row per block instruction).
constexpr int BR_TOK = 64;
template <typename T>
__global__ __launch_bounds__(ROUTE_THREADS) void bwd_router8_kernel(
    const T* __restrict__ x, const T* __restrict__ Wg, const T* __restrict__ dXp, const float* __restrict__ dg,
    int ntok, int d, int N, int top_k, const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
    const int32_t* __restrict__ row_of, T* __restrict__ dX, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) float s_dl[BR_TOK][8];
  __shared__ int s_row[BR_TOK][2];
  const int tid = threadIdx.x;
  const int t0 = blockIdx.x * BR_TOK;
  for (int i = tid; i < BR_TOK * 8; i += ROUTE_THREADS) (&s_dl[0][0])[i] = 0.f;
  __syncthreads();
  if (tid < BR_TOK && t0 + tid < ntok) {
    const int t = t0 + tid;
    float g[2] = {0.f, 0.f}, dgv[2] = {0.f, 0.f};
    int idx[2] = {0, 0};
    float mean = 0.f;
    for (int j = 0; j < top_k; ++j) {
      const int r = row_of[(size_t)t * top_k + j];
      s_row[tid][j] = r;
      idx[j] = topk_idx[(size_t)t * top_k + j];
      g[j] = topk_w[(size_t)t * top_k + j];
      dgv[j] = dg[r];
      mean += g[j] * dgv[j];
    }
    for (int j = 0; j < top_k; ++j) s_dl[tid][idx[j]] = g[j] * (dgv[j] - mean);
  }
  __syncthreads();
  const int nt = min(BR_TOK, ntok - t0);
  for (int c = tid * 8; c < d; c += ROUTE_THREADS * 8) {
    float wg[8][8], acc[8][8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (N == 8) {
        load8(Wg + (size_t)(c + q) * 8, wg[q]);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) wg[q][e] = e < N ? (float)Wg[(size_t)(c + q) * N + e] : 0.f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;
    }
    for (int tl = 0; tl < nt; ++tl) {
      const int t = t0 + tl;
      float dlv[8], xv[8], a[8], o[8];
      load8(&s_dl[tl][0], dlv);
      load8(x + (size_t)t * d + c, xv);
      load8(dXp + (size_t)s_row[tl][0] * d + c, a);
      if (top_k == 2) {
        float b[8];
        load8(dXp + (size_t)s_row[tl][1] * d + c, b);
#pragma unroll
        for (int q = 0; q < 8; ++q) a[q] += b[q];
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float go = a[q];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          go = fmaf(wg[q][e], dlv[e], go);
          acc[q][e] = fmaf(xv[q], dlv[e], acc[q][e]);
        }
        o[q] = go;
      }
      store8(dX + (size_t)t * d + c, o);
    }
    float* out = partial + ((size_t)blockIdx.x * d + c) * N;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e < N) out[q * N + e] = acc[q][e];
  }
}

// dW_gate[i] (+)= sum_b partial[b][i] in a fixed order (deterministic): 64 outputs per block, the blocks'
// partials are split over the 4 waves and combined through LDS.
__global__ __launch_bounds__(256) void dwg_reduce_kernel(const float* __restrict__ partial, int nb, int n,
                                                         int accumulate, float* __restrict__ dWg) {
  __shared__ float s_part[4][64];
  const int li = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + li;
  float acc = 0.f;
  if (i < n)
    for (int b = part; b < nb; b += 4) acc += partial[(size_t)b * n + i];
  s_part[part][li] = acc;
  __syncthreads();
  if (part == 0 && i < n) {
    const float v = (s_part[0][li] + s_part[1][li]) + (s_part[2][li] + s_part[3][li]);
    dWg[i] = accumulate ? dWg[i] + v : v;
  }
}

template <typename T, int NE, int TOK>
hipError_t run_router(const LayerDims& L, const T* x, const T* Wg, const float* bias, const RoutingPtrs& R,
                      int32_t* blockhist, hipStream_t s) {
  const int nb = (L.T + TPB - 1) / TPB;
  hipLaunchKernelGGL((router_kernel<T, NE, TOK>), dim3(nb), dim3(ROUTE_THREADS), 0, s, x, Wg, bias, L.T, L.d, L.N, L.k,
                     R.topk_idx, R.topk_w, blockhist);
  return hipGetLastError();
}

template <typename T>
hipError_t route_typed(const LayerDims& L, const void* xv, const void* Wgv, const float* bias, const RoutingPtrs& R,
                       int32_t* blockhist, void* Xpv, hipStream_t s) {
  const T* x = static_cast<const T*>(xv);
  const T* Wg = static_cast<const T*>(Wgv);
  hipError_t e;
  if (L.N <= 2) e = run_router<T, 2, 4>(L, x, Wg, bias, R, blockhist, s);
  else if (L.N <= 4) e = run_router<T, 4, 4>(L, x, Wg, bias, R, blockhist, s);
  else if (L.N <= 8) e = run_router<T, 8, 2>(L, x, Wg, bias, R, blockhist, s);
  else if (L.N <= 16) e = run_router<T, 16, 1>(L, x, Wg, bias, R, blockhist, s);
  else if (L.N <= 32) e = run_router<T, 32, 1>(L, x, Wg, bias, R, blockhist, s);
  else e = run_router<T, 64, 1>(L, x, Wg, bias, R, blockhist, s);
  if (e != hipSuccess) return e;
  const int nb = (L.T + TPB - 1) / TPB;
  hipLaunchKernelGGL(route_scan_kernel, dim3(1), dim3(256), 0, s, blockhist, nb, L.N, R.counts, R.offsets,
                     R.near_tie_count);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((scatter_kernel<T>), dim3(nb), dim3(ROUTE_THREADS), 0, s, x, L.T, L.d, L.N, L.k, R.topk_idx,
                     R.offsets, blockhist, R.row_of, R.src_of, static_cast<T*>(Xpv));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_route(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const float* bias,
                        const RoutingPtrs& R, int32_t* blockhist, void* Xp, hipStream_t s) {
  return dt == MODSE_F32 ? route_typed<float>(L, x, W_gate, bias, R, blockhist, Xp, s)
                         : route_typed<bf16_t>(L, x, W_gate, bias, R, blockhist, Xp, s);
}

hipError_t launch_combine(const LayerDims& L, modse_dtype dt, const void* O, const RoutingPtrs& R, void* y,
                          hipStream_t s) {
  const int nb = (L.T + 3) / 4;
  if (dt == MODSE_F32)
    hipLaunchKernelGGL((combine_kernel<float>), dim3(nb), dim3(256), 0, s, static_cast<const float*>(O), L.T, L.d, L.k,
                       R.row_of, R.topk_w, static_cast<float*>(y));
  else
    hipLaunchKernelGGL((combine_kernel<bf16_t>), dim3(nb), dim3(256), 0, s, static_cast<const bf16_t*>(O), L.T, L.d,
                       L.k, R.row_of, R.topk_w, static_cast<bf16_t*>(y));
  return hipGetLastError();
}

hipError_t launch_bwd_prep(const LayerDims& L, modse_dtype dt, const void* dY, const void* O, const RoutingPtrs& R,
                           void* dO, float* dg, hipStream_t s) {
  const int nrows = L.T * L.k;
  const int nb = (nrows + 3) / 4;
  if (dt == MODSE_F32)
    hipLaunchKernelGGL((bwd_prep_kernel<float>), dim3(nb), dim3(256), 0, s, static_cast<const float*>(dY),
                       static_cast<const float*>(O), nrows, L.d, L.k, R.src_of, R.topk_w, static_cast<float*>(dO), dg);
  else
    hipLaunchKernelGGL((bwd_prep_kernel<bf16_t>), dim3(nb), dim3(256), 0, s, static_cast<const bf16_t*>(dY),
                       static_cast<const bf16_t*>(O), nrows, L.d, L.k, R.src_of, R.topk_w, static_cast<bf16_t*>(dO),
                       dg);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const LayerDims& L, modse_dtype dt, const void* x, const RoutingPtrs& R, void* Xp,
                              hipStream_t s) {
  const int nrows = L.T * L.k;
  const int nb = (nrows + 3) / 4;
  if (dt == MODSE_F32)
    hipLaunchKernelGGL((gather_rows_kernel<float>), dim3(nb), dim3(256), 0, s, static_cast<const float*>(x), nrows,
                       L.d, L.k, R.src_of, static_cast<float*>(Xp));
  else
    hipLaunchKernelGGL((gather_rows_kernel<bf16_t>), dim3(nb), dim3(256), 0, s, static_cast<const bf16_t*>(x), nrows,
                       L.d, L.k, R.src_of, static_cast<bf16_t*>(Xp));
  return hipGetLastError();
}

hipError_t launch_bwd_router(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const void* dXp,
                             const float* dg, const RoutingPtrs& R, void* dX, float* dWg_partial, float* dW_gate,
                             int accumulate, hipStream_t s) {
  const bool small_n = L.N <= 8;
  const int nb = small_n ? (L.T + BR_TOK - 1) / BR_TOK : (L.T + TPB - 1) / TPB;
  if (dt == MODSE_F32) {
    auto kern = small_n ? bwd_router8_kernel<float> : bwd_router_kernel<float>;
    hipLaunchKernelGGL(kern, dim3(nb), dim3(ROUTE_THREADS), 0, s, static_cast<const float*>(x),
                       static_cast<const float*>(W_gate), static_cast<const float*>(dXp), dg, L.T, L.d, L.N, L.k,
                       R.topk_idx, R.topk_w, R.row_of, static_cast<float*>(dX), dWg_partial);
  } else {
    auto kern = small_n ? bwd_router8_kernel<bf16_t> : bwd_router_kernel<bf16_t>;
    hipLaunchKernelGGL(kern, dim3(nb), dim3(ROUTE_THREADS), 0, s, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(W_gate), static_cast<const bf16_t*>(dXp), dg, L.T, L.d, L.N, L.k,
                       R.topk_idx, R.topk_w, R.row_of, static_cast<bf16_t*>(dX), dWg_partial);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int n = L.d * L.N;
  hipLaunchKernelGGL(dwg_reduce_kernel, dim3((n + 63) / 64), dim3(256), 0, s, dWg_partial, nb, n, accumulate, dW_gate);
  return hipGetLastError();
}
