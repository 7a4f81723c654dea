// Router, permutation, combine and the element-wise backward kernels of the MoDSE layer (gfx950).
//
// Router: logits H(x) = x W_gate (+bias), KeepTopK, softmax over the kept logits (Sec. 2 Eq. 2-3 of
// arXiv 2409.12210).  Logits are accumulated in float64: products of bf16 or fp32 inputs are exact in
// float64, so the integer routing decision is taken at the same precision as a float64 reference and
// does not depend on summation order beyond the last bit.
#include <algorithm>
#include <climits>

#include "common.h"
#include "gemm_plan.h"

namespace {

constexpr int TPB = MODSE_ROUTE_TOKENS_PER_BLOCK;  // tokens per block
constexpr int ROUTE_THREADS = 256;
constexpr int ROUTER_TOKEN_MAX_T = 4096;  // batches up to this size take router_token_kernel
constexpr int TOK_PER_WAVE = TPB / (ROUTE_THREADS / 64);  // 8
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ inline double shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, 64);
  hi = __shfl_xor(hi, mask, 64);
  return __hiloint2double(hi, lo);
}

// Sum each of the V values over the 64 lanes of a wave.  Every halving step sends half of the values to
// the partner lane and keeps the other half, so V values cost V-1 + (6 - log2 V) shuffles.  On return
// lane l (l < V) holds in vals[0] the total of value index bitrev_{log2 V}(l).  (Template recursion, not
// loops: every index into vals is then a constant and the array stays in registers for any V.)
template <int V>
struct Log2 {
  static constexpr int value = 1 + Log2<V / 2>::value;
};
template <>
struct Log2<1> {
  static constexpr int value = 0;
};

template <int W, int I, int BIT, int V>
__device__ inline void halve_one(double (&vals)[V], bool upper) {
  if constexpr (I < W) {
    const double keep = upper ? vals[I + W] : vals[I];
    const double send = upper ? vals[I] : vals[I + W];
    vals[I] = keep + shfl_xor_f64(send, BIT);
    halve_one<W, I + 1, BIT>(vals, upper);
  }
}
template <int LIVE, int BIT, int V>
__device__ inline void halve_all(double (&vals)[V], int lane) {
  if constexpr (LIVE > 1) {
    halve_one<LIVE / 2, 0, BIT>(vals, (lane & BIT) != 0);
    halve_all<LIVE / 2, BIT * 2>(vals, lane);
  }
}
template <int V>
__device__ inline void wave_sum_values(double (&vals)[V], int lane) {
  halve_all<V, 1>(vals, lane);
#pragma unroll
  for (int s = Log2<V>::value; s < 6; ++s) vals[0] += shfl_xor_f64(vals[0], 1 << s);
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

__device__ inline double softplus_f64(double u) {  // log(1 + exp(u)) without overflow
  return u > 0.0 ? u + log1p(exp(-u)) : log1p(exp(u));
}

// KeepTopK on one token's N logits (Sec. 2 Eq. 3), k <= 2: the two largest and the third largest value.  Strict
// comparisons while scanning upward leave ties with the lower index.  The second pick always differs from the
// first: when no logit besides the first is above -inf (all others masked out by an infinite negative bias) it is
// the lowest other index, as in a stable descending sort.
struct TopPick {
  double m1, m2, m3;
  int i1, i2;
};
__device__ inline TopPick pick_top(const double* logits, int N) {
  TopPick p = {-INFINITY, -INFINITY, -INFINITY, 0, -1};
  for (int e = 0; e < N; ++e) {
    const double l = logits[e];
    if (l > p.m1) {
      p.m3 = p.m2; p.m2 = p.m1; p.i2 = p.i1; p.m1 = l; p.i1 = e;
    } else if (l > p.m2) {
      p.m3 = p.m2; p.m2 = l; p.i2 = e;
    } else if (l > p.m3) {
      p.m3 = l;
    }
  }
  if (p.i2 < 0 || p.i2 == p.i1) p.i2 = p.i1 == 0 ? 1 : 0;
  return p;
}
// Writes token t's expert indices and gate weights (softmax over the kept logits, Eq. 2); returns whether the
// gap that decided the selection is under 1e-6.
__device__ inline bool write_gate(const TopPick& p, int t, int N, int top_k, int32_t* __restrict__ topk_idx,
                                  float* __restrict__ topk_w) {
  if (top_k == 2) {
    const double g1 = 1.0 / (1.0 + exp(p.m2 - p.m1));
    topk_idx[(size_t)t * 2] = p.i1;
    topk_idx[(size_t)t * 2 + 1] = p.i2;
    topk_w[(size_t)t * 2] = (float)g1;
    topk_w[(size_t)t * 2 + 1] = (float)(1.0 - g1);
    return (p.m1 - p.m2 < 1e-6) || (N > 2 && p.m2 - p.m3 < 1e-6);
  }
  topk_idx[t] = p.i1;
  topk_w[t] = 1.f;
  return N > 1 && p.m1 - p.m2 < 1e-6;
}

// ---------------------------------------------------------------- the router's dot products
// Both block-wise routers give lane l of a wave the columns 8l..8l+7 of every 512-column step of the token
// rows: a row is read with one contiguous 1 KiB load per wave and step, and the loads of the next step are
// issued before the arithmetic of the current one.  A wave holds TOK tokens x EC experts of float64 sums at a
// time (at most 32, so that sums, the two sets of row registers and one converted matrix row fit the register
// file without spilling); layers with more experts than EC take the expert columns in chunks.

// eight consecutive elements as loaded, and element i of them as float
template <typename T>
struct Raw8;
template <>
struct Raw8<bf16_t> {
  u32x4 v;
  __device__ void load(const bf16_t* p) { v = *reinterpret_cast<const u32x4*>(p); }
  __device__ float get(int i) const {
    const uint32_t w = v[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
};
template <>
struct Raw8<float> {
  f32x4 a, b;
  __device__ void load(const float* p) {
    a = *reinterpret_cast<const f32x4*>(p);
    b = *reinterpret_cast<const f32x4*>(p + 4);
  }
  __device__ float get(int i) const { return i < 4 ? a[i] : b[i - 4]; }
};

// EC columns, from column e0, of row r of a router matrix in memory whose rows are ldw elements apart (ldw
// is the padded expert count, so a row is a whole number of aligned vectors)
template <typename T, int EC>
struct GlobalRows {
  const T* W;
  int ldw, e0;
  __device__ void fetch(int r, float (&wf)[EC]) const { load_row<EC>(W + (size_t)r * ldw + e0, wf); }
};

// The same from the LDS copy that router_stream_kernel keeps: elements of type W (double when the matrix
// fits that way, else float), NE per row; the eight rows of one lane and step lie together, followed by 16
// bytes of padding, so that the 16 lanes which a 128-bit LDS read serves together fall into different banks.
constexpr int rs_group_bytes(int NE, int elem) { return 8 * NE * elem + 16; }
template <typename W, int NE, int EC>
struct LdsRows {
  const char* base;
  int e0;
  __device__ void fetch(int r, W (&wf)[EC]) const {
    constexpr int PER = 16 / sizeof(W);  // elements per 128-bit read
    typedef W vec_t __attribute__((ext_vector_type(PER)));
    const char* p = base + (r >> 3) * rs_group_bytes(NE, sizeof(W)) + (r & 7) * NE * (int)sizeof(W) + e0 * (int)sizeof(W);
    if constexpr (EC >= PER) {
#pragma unroll
      for (int e = 0; e < EC; e += PER) {
        const vec_t q = *reinterpret_cast<const vec_t*>(p + e * sizeof(W));
#pragma unroll
        for (int j = 0; j < PER; ++j) wf[e + j] = q[j];
      }
    } else {  // two floats
      const f32x2 q = *reinterpret_cast<const f32x2*>(p);
      wf[0] = q.x; wf[1] = q.y;
    }
  }
};

// acc[tt * EC + e] += sum over this lane's columns c of row[tt][c] * W[c][e0 + e], in float64
template <typename T, int TOK, int EC, typename Rows>
__device__ inline void lane_dots(const T* const (&row)[TOK], int d, int lane, const Rows& rows,
                                 double (&acc)[TOK * EC]) {
  const int nstep = (d + 511) >> 9;
  Raw8<T> cur[TOK], nxt[TOK];
  {
    const int c = min(lane * 8, d - 8);
#pragma unroll
    for (int tt = 0; tt < TOK; ++tt) cur[tt].load(row[tt] + c);
  }
  for (int st = 0; st < nstep; ++st) {
    const int c = st * 512 + lane * 8;
    const bool more = st + 1 < nstep;
    if (more) {
      const int cn = min(c + 512, d - 8);
#pragma unroll
      for (int tt = 0; tt < TOK; ++tt) nxt[tt].load(row[tt] + cn);
    }
    if (c < d) {
      float wf[EC];
      rows.fetch(c, wf);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float wn[EC];
        if (i < 7) rows.fetch(c + i + 1, wn);  // the next matrix row is on its way during this row's arithmetic
        double wd[EC];
#pragma unroll
        for (int e = 0; e < EC; ++e) wd[e] = (double)wf[e];
#pragma unroll
        for (int tt = 0; tt < TOK; ++tt) {
          const double xd = (double)cur[tt].get(i);
#pragma unroll
          for (int e = 0; e < EC; ++e) acc[tt * EC + e] = fma(xd, wd[e], acc[tt * EC + e]);
        }
        if (i < 7) {
#pragma unroll
          for (int e = 0; e < EC; ++e) wf[e] = wn[e];
        }
        // keeps the scheduler from fetching and converting all eight rows ahead of the arithmetic, which
        // costs more registers than there are
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (more) {
#pragma unroll
      for (int tt = 0; tt < TOK; ++tt) cur[tt] = nxt[tt];
    }
  }
}

// tokens x expert columns that a wave sums at a time
template <int NE>
struct RouterShape {
  static constexpr int EC = NE < 16 ? NE : 16;
  static constexpr int TOK = 32 / EC < 4 ? 32 / EC : 4;  // (more tokens: their row registers no longer fit)
  static constexpr int V = TOK * EC;
};

// One wave's TOK tokens against all NE expert columns of one matrix: sums[tt][e] (an LDS array of the wave)
template <typename T, int NE, typename MakeRows>
__device__ inline void wave_logits(const T* const (&row)[RouterShape<NE>::TOK], int d, int lane, MakeRows make_rows,
                                   double (*sums)[NE]) {
  using S = RouterShape<NE>;
  constexpr int EC = S::EC, TOK = S::TOK, V = S::V;
#pragma unroll 1
  for (int e0 = 0; e0 < NE; e0 += EC) {
    double acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0;
    lane_dots<T, TOK, EC>(row, d, lane, make_rows(e0), acc);
    wave_sum_values<V>(acc, lane);
    if (lane < V) {
      const int v = bitrev<Log2<V>::value>(lane);
      sums[v / EC][e0 + v % EC] = acc[0];
    }
  }
}

// One block routes TPB consecutive tokens, eight per wave.  blockhist[b][0..N-1] = this block's per-expert
// assignment counts, blockhist[b][N] = its near-tie token count.  Reads the router matrices from memory (through
// the caches) for every TOK tokens: the form for layers whose W_gate does not fit router_stream_kernel's LDS
// area, for small batches with many experts, and for the optional parts of the gate (EXT): the noise term
// RMSNorm(Softplus(x W_n)) of H(x) (Sec. 2 Eq. 4-5; G.W_noise != null), which takes a second pass over the
// token rows with W_n in place of W_gate, and the full-softmax probabilities p(x) that the auxiliary loss needs
// (Sec. 3.2 Eq. 11; G.probs != null).
template <typename T, int NE, bool EXT>
__global__ __launch_bounds__(ROUTE_THREADS, 2) void router_kernel(const T* __restrict__ x, const T* __restrict__ Wg,
                                                              const float* __restrict__ bias, int ntok, int d, int N,
                                                              int top_k, int32_t* __restrict__ topk_idx,
                                                              float* __restrict__ topk_w,
                                                              int32_t* __restrict__ blockhist, GateExtPtrs G) {
  constexpr int TOK = RouterShape<NE>::TOK, EC = RouterShape<NE>::EC;
  constexpr int WAVES = ROUTE_THREADS / 64;
  __shared__ double s_logit[WAVES][TOK][NE];
  __shared__ double s_u[EXT ? WAVES : 1][EXT ? TOK : 1][EXT ? NE : 1];
  __shared__ int s_hist[MODSE_MAX_EXPERTS + 1];
  const T* Wn = EXT ? static_cast<const T*>(G.W_noise) : nullptr;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tok0 = blockIdx.x * TPB + wave * TOK_PER_WAVE;
  if (tid <= N) s_hist[tid] = 0;
  __syncthreads();

  for (int pass = 0; pass < TOK_PER_WAVE / TOK; ++pass) {
    const int tbase = tok0 + pass * TOK;
    const T* row[TOK];
#pragma unroll
    for (int tt = 0; tt < TOK; ++tt)  // rows past the end repeat the last token; never written
      row[tt] = x + (size_t)min(tbase + tt, ntok - 1) * d;
    wave_logits<T, NE>(row, d, lane, [&](int e0) { return GlobalRows<T, EC>{Wg, NE, e0}; }, s_logit[wave]);
    if constexpr (EXT) {
      if (Wn) wave_logits<T, NE>(row, d, lane, [&](int e0) { return GlobalRows<T, EC>{Wn, NE, e0}; }, s_u[wave]);
    }
    __syncthreads();
    if (lane < TOK && tbase + lane < ntok) {
      const int t = tbase + lane;
      if (bias)
        for (int e = 0; e < N; ++e) s_logit[wave][lane][e] += (double)bias[e];
      if constexpr (EXT) {
        if (Wn) {  // H(x)_e += gamma s_e / sqrt(mean_i s_i^2 + eps),  s = softplus(x W_n)
          double ss = 0.0;
          for (int e = 0; e < N; ++e) {
            const double u = s_u[wave][lane][e];
            G.noise_pre[(size_t)t * N + e] = (float)u;
            const double sp = softplus_f64(u);
            s_u[wave][lane][e] = sp;
            ss += sp * sp;
          }
          const double scale = (double)G.gamma[0] / sqrt(ss / N + (double)G.eps);
          for (int e = 0; e < N; ++e) s_logit[wave][lane][e] += scale * s_u[wave][lane][e];
        }
      }
      const TopPick p = pick_top(s_logit[wave][lane], N);
      const bool near = write_gate(p, t, N, top_k, topk_idx, topk_w);
      atomicAdd(&s_hist[p.i1], 1);
      if (top_k == 2) atomicAdd(&s_hist[p.i2], 1);
      if (near) atomicAdd(&s_hist[N], 1);
      if constexpr (EXT) {
        if (G.probs) {  // p(x) = softmax over all N logits
          double den = 0.0;
          for (int e = 0; e < N; ++e) den += exp(s_logit[wave][lane][e] - p.m1);
          for (int e = 0; e < N; ++e) G.probs[(size_t)t * N + e] = (float)(exp(s_logit[wave][lane][e] - p.m1) / den);
        }
      }
    }
    __syncthreads();
  }
  if (tid <= N) blockhist[(size_t)blockIdx.x * (N + 1) + tid] = s_hist[tid];
}

// Router for large batches without the optional gate parts.  One 512-thread block per CU copies W_gate into LDS
// once (as float64 when that fits RS_W_BYTES, else as float: both exact) and then walks over groups of 64 tokens
// (two histogram blocks of TPB tokens), eight tokens per wave: the matrix rows then cost an LDS read instead of a
// trip through the vector memory pipeline per TOK tokens, which is what holds router_kernel back.
// A wave's work is a flat sequence of steps (group, pass of TOK tokens, chunk of EC expert columns, 512 columns
// of the token rows); the loads of the step two ahead are issued before the arithmetic of the current step,
// across pass and group boundaries, and the first two steps are under way while W_gate is being copied.
// Sums are float64 FMAs in a fixed order per lane, then wave_sum_values: results do not depend on timing.
constexpr int RS_THREADS = 512, RS_WAVES = RS_THREADS / 64, RS_TOKENS = 64;
constexpr int RS_W_BYTES = 136 * 1024;

template <typename T, int NE, typename W>
__global__ __launch_bounds__(RS_THREADS) void router_stream_kernel(const T* __restrict__ x, const T* __restrict__ Wg,
                                                                  const float* __restrict__ bias, int ntok, int d,
                                                                  int N, int top_k, int32_t* __restrict__ topk_idx,
                                                                  float* __restrict__ topk_w,
                                                                  int32_t* __restrict__ blockhist) {
  using S = RouterShape<NE>;
  constexpr int TOK = S::TOK, EC = S::EC, V = S::V;
  constexpr int NPASS = 8 / TOK, NCHUNK = NE / EC;
  constexpr int GB = rs_group_bytes(NE, sizeof(W));
  constexpr int HW = MODSE_MAX_EXPERTS + 1;
  __shared__ __attribute__((aligned(16))) char s_w[RS_W_BYTES];
  __shared__ double s_logit[RS_WAVES][TOK][NE];
  __shared__ int s_hist[2 * HW];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ngroups = (ntok + RS_TOKENS - 1) / RS_TOKENS;
  const int nhist = (ntok + TPB - 1) / TPB;
  const int nstep = (d + 511) >> 9;

  // the loader runs two steps ahead of the arithmetic
  Raw8<T> cur[TOK], nx1[TOK], nx2[TOK];
  int l_grp = blockIdx.x, l_pass = 0, l_chunk = 0, l_st = 0;
  auto load_next = [&](Raw8<T> (&dst)[TOK]) {
    if (l_grp < ngroups) {
      const int tbase = l_grp * RS_TOKENS + wave * 8 + l_pass * TOK;
      const int c = min(l_st * 512 + lane * 8, d - 8);
#pragma unroll
      for (int tt = 0; tt < TOK; ++tt)  // rows past the end repeat the last token; never written
        dst[tt].load(x + (size_t)min(tbase + tt, ntok - 1) * d + c);
    }
    if (++l_st == nstep) {
      l_st = 0;
      if (++l_chunk == NCHUNK) {
        l_chunk = 0;
        if (++l_pass == NPASS) {
          l_pass = 0;
          l_grp += gridDim.x;
        }
      }
    }
  };
  load_next(cur);
  load_next(nx1);

  for (int r = tid; r < d; r += RS_THREADS) {  // W_gate -> LDS; columns past N read as zero
    float wf[NE];
    if (N == NE) {
      load_row<NE>(Wg + (size_t)r * N, wf);
    } else {
#pragma unroll
      for (int e = 0; e < NE; ++e) wf[e] = e < N ? (float)Wg[(size_t)r * N + e] : 0.f;
    }
    W* dst = reinterpret_cast<W*>(s_w + (r >> 3) * GB + (r & 7) * NE * (int)sizeof(W));
#pragma unroll
    for (int e = 0; e < NE; ++e) dst[e] = (W)wf[e];
  }
  if (tid < 2 * HW) s_hist[tid] = 0;
  __syncthreads();

  for (int grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
    for (int pass = 0; pass < NPASS; ++pass) {
      const int tbase = grp * RS_TOKENS + wave * 8 + pass * TOK;
#pragma unroll 1
      for (int e0 = 0; e0 < NE; e0 += EC) {
        const LdsRows<W, NE, EC> rows = {s_w, e0};
        double acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0;
        for (int st = 0; st < nstep; ++st) {
          load_next(nx2);
          const int c = st * 512 + lane * 8;
          if (c < d) {
            W wf[EC];
            rows.fetch(c, wf);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              W wn[EC];
              if (i < 7) rows.fetch(c + i + 1, wn);  // the next matrix row is on its way during this row's arithmetic
              double wd[EC];
#pragma unroll
              for (int e = 0; e < EC; ++e) wd[e] = (double)wf[e];
#pragma unroll
              for (int tt = 0; tt < TOK; ++tt) {
                const double xd = (double)cur[tt].get(i);
#pragma unroll
                for (int e = 0; e < EC; ++e) acc[tt * EC + e] = fma(xd, wd[e], acc[tt * EC + e]);
              }
              if (i < 7) {
#pragma unroll
                for (int e = 0; e < EC; ++e) wf[e] = wn[e];
              }
              __builtin_amdgcn_sched_barrier(0);  // (see lane_dots)
            }
          }
#pragma unroll
          for (int tt = 0; tt < TOK; ++tt) {
            cur[tt] = nx1[tt];
            nx1[tt] = nx2[tt];
          }
        }
        wave_sum_values<V>(acc, lane);
        if (lane < V) {
          const int v = bitrev<Log2<V>::value>(lane);
          s_logit[wave][v / EC][e0 + v % EC] = acc[0];
        }
      }
      __syncthreads();
      if (lane < TOK && tbase + lane < ntok) {
        const int t = tbase + lane;
        if (bias)
          for (int e = 0; e < N; ++e) s_logit[wave][lane][e] += (double)bias[e];
        const TopPick p = pick_top(s_logit[wave][lane], N);
        const bool near = write_gate(p, t, N, top_k, topk_idx, topk_w);
        int* hist = s_hist + (wave >> 2) * HW;  // waves 0-3 hold the group's first TPB tokens
        atomicAdd(&hist[p.i1], 1);
        if (top_k == 2) atomicAdd(&hist[p.i2], 1);
        if (near) atomicAdd(&hist[N], 1);
      }
      __syncthreads();
    }
    if (tid < 2 * HW) {  // the thread that writes a counter out also clears it for the next group
      const int h = tid / HW, i = tid % HW, b = grp * 2 + h;
      if (i <= N && b < nhist) blockhist[(size_t)b * (N + 1) + i] = s_hist[tid];
      s_hist[tid] = 0;
    }
  }
}

// The same router on the float64 matrix instruction (v_mfma_f64_4x4x4_4b_f64: four independent 4 x 4 x 4 products
// per wave instruction; 64 float64 TFLOP/s measured on this chip against 50 for v_fma_f64 with two resident waves,
// and the conversions and LDS reads no longer compete with the multiply-adds for issue slots).  Operand lane
// 16 k + 4 b + i holds A_b[i][k] (or B_b[k][i]); result lane 16 i + 4 b + j holds D_b[i][j] (checked with a
// one-hot probe).  Here block b, row i is token 4 b + i of a set of 16, column j is expert 4 g + j of expert group g,
// and k runs over the columns of x: one x value per lane and instruction, converted to float64 (exact; the products
// of two bf16 values and their float64 sums are the same as the vector router's up to the order of the additions).
// One 512-thread block per CU keeps W_gate in LDS as float64 and walks over 64-token groups.  Wave w takes the
// columns [w d/8, (w+1) d/8) of all 64 tokens (four sets of 16), so a W value read from LDS serves four matrix
// instructions; a lane loads 16 bytes of a token row (8 columns) at a time, 16 rows x 64 consecutive bytes per wave
// instruction, two steps of 32 columns ahead, across groups.  The eight waves' partial sums meet in LDS and are added
// in a fixed order; then one thread per token does top-k, gate and the block histogram, as in the vector router.
// Needs d % 256 == 0 and the float64 copy of W_gate (d x NE x 8 bytes, NE = 8 or 16) in RM_W_BYTES.
constexpr int RM_THREADS = 512, RM_WAVES = RM_THREADS / 64, RM_TOKENS = 64, RM_SETS = RM_TOKENS / 16;
constexpr int rm_w_bytes(int NE) { return NE <= 8 ? 128 * 1024 : 112 * 1024; }

template <typename T, int NE>
__global__ __launch_bounds__(RM_THREADS) void router_mfma_kernel(const T* __restrict__ x, const T* __restrict__ Wg,
                                                                const float* __restrict__ bias, int ntok, int d, int N,
                                                                int top_k, int32_t* __restrict__ topk_idx,
                                                                float* __restrict__ topk_w,
                                                                int32_t* __restrict__ blockhist) {
  static_assert(NE == 8 || NE == 16, "expert groups of four; rows of 64 or 128 bytes");
  constexpr int EG = NE / 4;  // expert groups
  constexpr int HW = MODSE_MAX_EXPERTS + 1;
  typedef double f64x2 __attribute__((ext_vector_type(2)));
  __shared__ __attribute__((aligned(16))) double s_w[rm_w_bytes(NE) / 8];  // [column][j][g] = W_gate[column][4 g + j]
  __shared__ double s_part[RM_WAVES / 2][RM_TOKENS][NE];
  __shared__ int s_hist[2 * HW];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kq = lane >> 4, blk = (lane >> 2) & 3, ij = lane & 3;
  const int ngroups = (ntok + RM_TOKENS - 1) / RM_TOKENS;
  const int nhist = (ntok + TPB - 1) / TPB;
  const int wcols = d / RM_WAVES, nstep = wcols / 32;
  const int col0 = wave * wcols + kq * 8;  // this lane's first column

  // the loader runs two steps ahead of the arithmetic
  Raw8<T> cur[RM_SETS], nx1[RM_SETS], nx2[RM_SETS];
  int l_grp = blockIdx.x, l_st = 0;
  auto load_next = [&](Raw8<T> (&dst)[RM_SETS]) {
    if (l_grp < ngroups) {
      const int c = col0 + l_st * 32;
#pragma unroll
      for (int q = 0; q < RM_SETS; ++q) {  // rows past the end repeat the last token; never written
        const int t = min(l_grp * RM_TOKENS + q * 16 + blk * 4 + ij, ntok - 1);
        dst[q].load(x + (size_t)t * d + c);
      }
    }
    if (++l_st == nstep) {
      l_st = 0;
      l_grp += gridDim.x;
    }
  };
  load_next(cur);
  load_next(nx1);

  for (int r = tid; r < d; r += RM_THREADS) {  // W_gate -> LDS; columns past N read as zero
    float wf[NE];
    if (N == NE) {
      load_row<NE>(Wg + (size_t)r * N, wf);
    } else {
#pragma unroll
      for (int e = 0; e < NE; ++e) wf[e] = e < N ? (float)Wg[(size_t)r * N + e] : 0.f;
    }
    double* dst = s_w + (size_t)r * NE;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int g = 0; g < EG; ++g) dst[j * EG + g] = (double)wf[4 * g + j];
  }
  if (tid < 2 * HW) s_hist[tid] = 0;
  __syncthreads();

  for (int grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
    double acc[RM_SETS][EG];
#pragma unroll
    for (int q = 0; q < RM_SETS; ++q)
#pragma unroll
      for (int g = 0; g < EG; ++g) acc[q][g] = 0.0;
    for (int st = 0; st < nstep; ++st) {
      load_next(nx2);
      const double* wrow = s_w + (size_t)(col0 + st * 32) * NE + ij * EG;
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        double b[EG];
#pragma unroll
        for (int g2 = 0; g2 < EG / 2; ++g2) {
          const f64x2 v = *reinterpret_cast<const f64x2*>(wrow + m * NE + 2 * g2);
          b[2 * g2] = v[0];
          b[2 * g2 + 1] = v[1];
        }
#pragma unroll
        for (int q = 0; q < RM_SETS; ++q) {
          const double a = (double)cur[q].get(m);
#pragma unroll
          for (int g = 0; g < EG; ++g) acc[q][g] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b[g], acc[q][g], 0, 0, 0);
        }
      }
#pragma unroll
      for (int q = 0; q < RM_SETS; ++q) {
        cur[q] = nx1[q];
        nx1[q] = nx2[q];
      }
    }
    // result lane 16 i + 4 b + j: token 4 b + i of the set, expert 4 g + j.  Waves 4-7 hand their sums to waves
    // 0-3, which add their own and leave four partial sums per logit.
    const int tloc = blk * 4 + kq;
    if (wave >= RM_WAVES / 2) {
#pragma unroll
      for (int q = 0; q < RM_SETS; ++q)
#pragma unroll
        for (int g = 0; g < EG; ++g) s_part[wave - RM_WAVES / 2][q * 16 + tloc][4 * g + ij] = acc[q][g];
    }
    __syncthreads();
    if (wave < RM_WAVES / 2) {
#pragma unroll
      for (int q = 0; q < RM_SETS; ++q)
#pragma unroll
        for (int g = 0; g < EG; ++g) {
          double* p = &s_part[wave][q * 16 + tloc][4 * g + ij];
          *p = acc[q][g] + *p;
        }
    }
    __syncthreads();
    const int tbase = grp * RM_TOKENS;
    if (tid < RM_TOKENS && tbase + tid < ntok) {
      const int t = tbase + tid;
      for (int e = 0; e < N; ++e) {
        double l = (s_part[0][tid][e] + s_part[1][tid][e]) + (s_part[2][tid][e] + s_part[3][tid][e]);
        if (bias) l += (double)bias[e];
        s_part[0][tid][e] = l;
      }
      const TopPick p = pick_top(s_part[0][tid], N);
      const bool near = write_gate(p, t, N, top_k, topk_idx, topk_w);
      int* hist = s_hist + (tid / TPB) * HW;  // the group's first and second TPB tokens
      atomicAdd(&hist[p.i1], 1);
      if (top_k == 2) atomicAdd(&hist[p.i2], 1);
      if (near) atomicAdd(&hist[N], 1);
    }
    __syncthreads();
    if (tid < 2 * HW) {  // the thread that writes a counter out also clears it for the next group
      const int h = tid / HW, i = tid % HW, b = grp * 2 + h;
      if (i <= N && b < nhist) blockhist[(size_t)b * (N + 1) + i] = s_hist[tid];
      s_hist[tid] = 0;
    }
  }
}

// Router without the optional gate parts: one block per G tokens, the 256 threads split the d columns, so
// a token row and the router matrix are read once with 16-byte loads and the whole dot product is one or
// two rounds of memory latency.  Every thread leaves its G x N float64 partial sums in LDS; they are added
// in two fixed-order steps (8 groups of 32 threads, then the 8 group sums), so the result does not depend
// on timing; one thread per token then does top-k and gate.  The block histograms that the permutation
// needs are made by route_hist_kernel from topk_idx and near_flag.
template <typename T, int NE, int G>
__global__ __launch_bounds__(ROUTE_THREADS, 2) void router_token_kernel(const T* __restrict__ x,
                                                                       const T* __restrict__ Wg,
                                                                       const float* __restrict__ bias, int ntok, int d,
                                                                       int N, int top_k,
                                                                       int32_t* __restrict__ topk_idx,
                                                                       float* __restrict__ topk_w,
                                                                       int32_t* __restrict__ near_flag) {
  constexpr int V = G * NE;
  static_assert(V <= 32, "one thread per value and group in the second reduction step");
  __shared__ double s_part[ROUTE_THREADS][V + 1];  // (+1: rows start in different banks)
  __shared__ double s_group[8][V];
  __shared__ double s_logit[G][NE];
  const int tid = threadIdx.x, t0 = blockIdx.x * G;
  double acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = 0.0;
  for (int c = tid * 8; c < d; c += ROUTE_THREADS * 8) {
    float xv[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) load8(x + (size_t)min(t0 + g, ntok - 1) * d + c, xv[g]);  // (clamped rows: never written)
    const GlobalRows<T, NE> rows = {Wg, NE, 0};
    float wf[NE];
    rows.fetch(c, wf);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float wn[NE];
      if (i < 7) rows.fetch(c + i + 1, wn);
#pragma unroll
      for (int e = 0; e < NE; ++e) {
        const double wd = (double)wf[e];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g * NE + e] = fma((double)xv[g][i], wd, acc[g * NE + e]);
      }
      if (i < 7) {
#pragma unroll
        for (int e = 0; e < NE; ++e) wf[e] = wn[e];
      }
      __builtin_amdgcn_sched_barrier(0);  // (see lane_dots)
    }
  }
#pragma unroll
  for (int v = 0; v < V; ++v) s_part[tid][v] = acc[v];
  __syncthreads();
  {
    const int v = tid & 31, grp = tid >> 5;
    if (v < V) {
      double sum = 0.0;
      for (int i = 0; i < 32; ++i) sum += s_part[grp * 32 + i][v];
      s_group[grp][v] = sum;
    }
  }
  __syncthreads();
  if (tid < V) {
    double sum = 0.0;
    for (int q = 0; q < 8; ++q) sum += s_group[q][tid];
    const int e = tid % NE;
    s_logit[tid / NE][e] = sum + ((bias && e < N) ? (double)bias[e] : 0.0);
  }
  __syncthreads();
  if (tid < G && t0 + tid < ntok) {
    const int t = t0 + tid;
    const TopPick p = pick_top(s_logit[tid], N);
    near_flag[t] = write_gate(p, t, N, top_k, topk_idx, topk_w) ? 1 : 0;
  }
}

// blockhist[b][0..N-1] = assignments per expert among the TPB tokens of block b, blockhist[b][N] = its
// near-tie token count (integer atomics in LDS: the result does not depend on their order).
__global__ __launch_bounds__(64) void route_hist_kernel(const int32_t* __restrict__ topk_idx,
                                                        const int32_t* __restrict__ near_flag, int ntok, int N,
                                                        int top_k, int32_t* __restrict__ blockhist) {
  __shared__ int s_hist[MODSE_MAX_EXPERTS + 1];
  const int tid = threadIdx.x;
  for (int i = tid; i <= N; i += 64) s_hist[i] = 0;
  __syncthreads();
  const int t = blockIdx.x * TPB + tid;
  if (tid < TPB && t < ntok) {
    for (int j = 0; j < top_k; ++j) atomicAdd(&s_hist[topk_idx[(size_t)t * top_k + j]], 1);
    if (near_flag[t]) atomicAdd(&s_hist[N], 1);
  }
  __syncthreads();
  for (int i = tid; i <= N; i += 64) blockhist[(size_t)blockIdx.x * (N + 1) + i] = s_hist[i];
}

// Single block.  Turns blockhist[b][e] into the exclusive prefix over blocks (in place), writes counts, offsets
// and the near-tie total and, when a forward pass follows, the tile plans of its two GEMMs (from the counts
// still in LDS: no second launch, no round trip through memory).  Each thread owns a contiguous run of blocks.
// Up to SCAN_EC expert columns are handled at once and a thread's blocks four at a time, so that the loads of
// a step are all in flight together (the launch is a chain of memory latencies and nothing else); the 256 run
// totals of a column are scanned by one wave.
constexpr int SCAN_EC = 16, SCAN_NB = 4;
__global__ __launch_bounds__(256) void route_scan_kernel(int32_t* __restrict__ blockhist, int nb, int N,
                                                         int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ near_tie_count, LayerDims L, int esize,
                                                         FwdPlanArgs plan, int with_plan) {
  __shared__ int s_part[SCAN_EC][256];
  __shared__ int s_total[MODSE_MAX_EXPERTS + 1];
  __shared__ int s_counts[MODSE_MAX_EXPERTS], s_offsets[MODSE_MAX_EXPERTS + 1];
  __shared__ int s_tiles[MODSE_MAX_PROBLEMS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (nb + 255) / 256;
  const int b0 = min(tid * per, nb), b1 = min(b0 + per, nb);
  const int W = N + 1;
  for (int e0 = 0; e0 < W; e0 += SCAN_EC) {
    const int ne = min(SCAN_EC, W - e0);
    int sum[SCAN_EC];
#pragma unroll
    for (int j = 0; j < SCAN_EC; ++j) sum[j] = 0;
    for (int b = b0; b < b1; b += SCAN_NB) {
      int v[SCAN_NB][SCAN_EC];
#pragma unroll
      for (int q = 0; q < SCAN_NB; ++q)
#pragma unroll
        for (int j = 0; j < SCAN_EC; ++j)
          v[q][j] = (b + q < b1 && j < ne) ? blockhist[(size_t)(b + q) * W + e0 + j] : 0;
#pragma unroll
      for (int q = 0; q < SCAN_NB; ++q)
#pragma unroll
        for (int j = 0; j < SCAN_EC; ++j) sum[j] += v[q][j];
    }
#pragma unroll
    for (int j = 0; j < SCAN_EC; ++j) s_part[j][tid] = sum[j];
    __syncthreads();
    for (int j = wave; j < ne; j += 4) {  // exclusive scan of column j's 256 run totals
      int v[4], local = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = s_part[j][lane * 4 + i];
        local += v[i];
      }
      int incl = local;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
      }
      int run = incl - local;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s_part[j][lane * 4 + i] = run;
        run += v[i];
      }
      if (lane == 63) s_total[e0 + j] = incl;
    }
    __syncthreads();
    int run[SCAN_EC];
#pragma unroll
    for (int j = 0; j < SCAN_EC; ++j) run[j] = s_part[j][tid];
    for (int b = b0; b < b1; b += SCAN_NB) {  // (the near-tie column, e == N, keeps its counts)
      int v[SCAN_NB][SCAN_EC];
#pragma unroll
      for (int q = 0; q < SCAN_NB; ++q)
#pragma unroll
        for (int j = 0; j < SCAN_EC; ++j)
          v[q][j] = (b + q < b1 && e0 + j < N) ? blockhist[(size_t)(b + q) * W + e0 + j] : 0;
#pragma unroll
      for (int q = 0; q < SCAN_NB; ++q)
#pragma unroll
        for (int j = 0; j < SCAN_EC; ++j)
          if (b + q < b1 && e0 + j < N) {
            blockhist[(size_t)(b + q) * W + e0 + j] = run[j];
            run[j] += v[q][j];
          }
    }
    __syncthreads();
  }
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < N; ++e) {
      counts[e] = s_counts[e] = s_total[e];
      offsets[e] = s_offsets[e] = run;
      run += s_total[e];
    }
    offsets[N] = s_offsets[N] = run;
    near_tie_count[0] = s_total[N];
  }
  if (with_plan) {
    __syncthreads();
    modse_gemm::plan_fwd_body(L, esize, s_counts, s_offsets, plan, s_tiles);
  }
}

// Auxiliary load-balance loss (Sec. 3.2 Eq. 9-12), single block: f_i = share of tokens whose first choice is
// expert i, P_i = mean of p_i, L_a = alpha N sum_i f_i P_i.  Every thread sums its tokens in ascending
// order and the per-thread sums are added in thread order, so the result does not depend on timing.
__global__ __launch_bounds__(256) void aux_finish_kernel(const float* __restrict__ probs,
                                                         const int32_t* __restrict__ topk_idx, int ntok, int N,
                                                         int top_k, float alpha, float* __restrict__ f_out,
                                                         float* __restrict__ P_out, float* __restrict__ loss) {
  __shared__ float s_p[256];
  __shared__ int s_c[256];
  __shared__ float s_f[MODSE_MAX_EXPERTS], s_P[MODSE_MAX_EXPERTS];
  const int tid = threadIdx.x;
  for (int e = 0; e < N; ++e) {
    float acc = 0.f;
    int cnt = 0;
    for (int t = tid; t < ntok; t += 256) {
      acc += probs[(size_t)t * N + e];
      cnt += topk_idx[(size_t)t * top_k] == e ? 1 : 0;
    }
    s_p[tid] = acc;
    s_c[tid] = cnt;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
      int c = 0;
      for (int i = 0; i < 256; ++i) {
        tot += s_p[i];
        c += s_c[i];
      }
      s_P[e] = tot / (float)ntok;
      s_f[e] = (float)c / (float)ntok;
    }
    __syncthreads();
  }
  if (tid < N) {
    f_out[tid] = s_f[tid];
    P_out[tid] = s_P[tid];
  }
  if (tid == 0) {
    float l = 0.f;
    for (int e = 0; e < N; ++e) l += s_f[e] * s_P[e];
    loss[0] = alpha * (float)N * l;
  }
}

// Routing statistics in the shape of the paper's Appendix A tables, single block: slot_counts[j][i] = tokens
// whose j-th choice is expert i; summary[j] = max/min of row j, summary[k] = max/min of the per-expert
// totals, summary[k+1] = average hidden width of the chosen experts (Sec. 4.3).
__global__ __launch_bounds__(256) void routing_stats_kernel(const int32_t* __restrict__ topk_idx, int ntok, int N,
                                                            int top_k, LayerDims L, int32_t* __restrict__ slot_counts,
                                                            float* __restrict__ summary) {
  __shared__ int s_cnt[2][MODSE_MAX_EXPERTS];
  const int tid = threadIdx.x;
  if (tid < 2 * MODSE_MAX_EXPERTS) (&s_cnt[0][0])[tid] = 0;
  __syncthreads();
  for (int i = tid; i < ntok * top_k; i += 256) atomicAdd(&s_cnt[i % top_k][topk_idx[i]], 1);
  __syncthreads();
  for (int i = tid; i < top_k * N; i += 256) slot_counts[i] = s_cnt[i / N][i % N];
  if (tid == 0) {
    double wsum = 0.0;
    long tot_all = 0;
    int tmax = 0, tmin = INT_MAX;
    for (int e = 0; e < N; ++e) {
      const int tot = s_cnt[0][e] + (top_k == 2 ? s_cnt[1][e] : 0);
      tmax = max(tmax, tot);
      tmin = min(tmin, tot);
      wsum += (double)tot * L.f[e];
      tot_all += tot;
    }
    for (int j = 0; j < top_k; ++j) {
      int mx = 0, mn = INT_MAX;
      for (int e = 0; e < N; ++e) {
        mx = max(mx, s_cnt[j][e]);
        mn = min(mn, s_cnt[j][e]);
      }
      summary[j] = mn > 0 ? (float)mx / (float)mn : INFINITY;
    }
    summary[top_k] = tmin > 0 ? (float)tmax / (float)tmin : INFINITY;
    summary[top_k + 1] = tot_all > 0 ? (float)(wsum / (double)tot_all) : 0.f;
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

// Decode-sized batches (at most 64 tokens): histogram, offsets, stable scatter and, when a forward pass follows,
// the tile plans of its two GEMMs in ONE launch instead of four; at this size every launch gap shows in the
// layer time.  One block per token.  Wave 0 of every block holds one token per lane and ranks all of them with
// one ballot per expert (the same rows as scatter_kernel: tokens of an expert in token order); block 0 also
// writes the routing outputs and the plans; block t copies token t's row to its permuted places.
// Near-tie total: from near_flag (one-block-per-token router) or, when that is null, from the last column of
// the router's block histograms.
template <typename T>
__global__ __launch_bounds__(256) void permute_small_kernel(const T* __restrict__ x, int ntok, int d, int N, int top_k,
                                                            const int32_t* __restrict__ topk_idx,
                                                            const int32_t* __restrict__ near_flag,
                                                            const int32_t* __restrict__ blockhist, RoutingPtrs R,
                                                            T* __restrict__ Xp, LayerDims L, int esize,
                                                            FwdPlanArgs plan, int with_plan) {
  __shared__ int s_row[64][2];
  __shared__ int s_counts[MODSE_MAX_EXPERTS], s_offsets[MODSE_MAX_EXPERTS + 1];
  __shared__ int s_tiles[MODSE_MAX_PROBLEMS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool first = blockIdx.x == 0;
  if (wave == 0) {
    const int t = lane;
    const bool valid = t < ntok;
    int e0 = -1, e1 = -1;
    if (valid) {
      e0 = topk_idx[(size_t)t * top_k];
      if (top_k == 2) e1 = topk_idx[(size_t)t * top_k + 1];
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    int run = 0, row0 = 0, row1 = 0, my_count = 0, my_offset = 0;
    for (int e = 0; e < N; ++e) {
      const unsigned long long m = __ballot(e0 == e || e1 == e);
      const int rank = __popcll(m & below), c = __popcll(m);
      if (e0 == e) row0 = run + rank;
      if (e1 == e) row1 = run + rank;
      if (lane == e) {
        my_count = c;
        my_offset = run;
      }
      run += c;
    }
    if (lane < N) {
      s_counts[lane] = my_count;
      s_offsets[lane] = my_offset;
    }
    if (lane == 0) s_offsets[N] = run;
    if (valid) {
      s_row[t][0] = row0;
      s_row[t][1] = row1;
    }
    if (first) {
      int near;
      if (near_flag) {
        near = __popcll(__ballot(valid && near_flag[t] != 0));
      } else {
        near = 0;
        for (int b = 0; b * TPB < ntok; ++b) near += blockhist[(size_t)b * (N + 1) + N];
      }
      if (lane < N) {
        R.counts[lane] = my_count;
        R.offsets[lane] = my_offset;
      }
      if (lane == 0) {
        R.offsets[N] = run;
        R.near_tie_count[0] = near;
      }
      if (valid) {
        R.row_of[(size_t)t * top_k] = row0;
        R.src_of[row0] = t * top_k;
        if (top_k == 2) {
          R.row_of[(size_t)t * top_k + 1] = row1;
          R.src_of[row1] = t * top_k + 1;
        }
      }
    }
  }
  __syncthreads();
  if (first && with_plan) modse_gemm::plan_fwd_body(L, esize, s_counts, s_offsets, plan, s_tiles);
  if (Xp == nullptr) return;
  const int t = blockIdx.x;
  const int row0 = s_row[t][0];
  const int row1 = top_k == 2 ? s_row[t][1] : -1;
  constexpr int VEC = 16 / sizeof(T);
  for (int c = tid * VEC; c < d; c += 256 * VEC) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(x + (size_t)t * d + c);
    *reinterpret_cast<f32x4*>(Xp + (size_t)row0 * d + c) = v;
    if (row1 >= 0) *reinterpret_cast<f32x4*>(Xp + (size_t)row1 * d + c) = v;
  }
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

// Combine after a split-K down-projection: expert e's output rows are the sum of ceil(f_e / kchunk) float32
// partial slabs Opart[c] ([T*k, d] each), added in ascending c.  One thread per token and 8 columns.
template <typename T>
__global__ __launch_bounds__(256) void combine_split_kernel(const float* __restrict__ Opart, int ntok, int d,
                                                            int top_k, LayerDims L, int kchunk,
                                                            const int32_t* __restrict__ topk_idx,
                                                            const int32_t* __restrict__ row_of,
                                                            const float* __restrict__ topk_w, T* __restrict__ y) {
  const int per_tok = d / 8;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long)ntok * per_tok) return;
  const int t = (int)(i / per_tok), c = (int)(i % per_tok) * 8;
  const size_t slab = (size_t)ntok * top_k * d;
  float o[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) o[q] = 0.f;
  for (int j = 0; j < top_k; ++j) {
    const int e = topk_idx[(size_t)t * top_k + j];
    const float* src = Opart + (size_t)row_of[(size_t)t * top_k + j] * d + c;
    const float g = topk_w[(size_t)t * top_k + j];
    const int nchunk = (L.f[e] + kchunk - 1) / kchunk;
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
#pragma unroll 4
    for (int s = 0; s < nchunk; ++s) {
      float v[8];
      load8(src + s * slab, v);
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] += v[q];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = fmaf(g, acc[q], o[q]);
  }
  store8(y + (size_t)t * d + c, o);
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

// Backward through the gate, one thread per token: the dense gradient of the logits H(x),
//   dl_j = g_j (dg_j - sum_m g_m dg_m) on the kept logits (softmax over KeepTopK), 0 elsewhere,
//   + aux_coef p_i (f_i - sum_m f_m p_m)  when the auxiliary loss is on (Sec. 3.2 Eq. 9-12 with f constant;
//     aux_coef = dLoss/dL_a * alpha N / T),
// and, when the noise term is on (z = gamma s / r, s = softplus(u), r = sqrt(mean s^2 + eps), Sec. 2
// Eq. 4-5), the gradient of u = x W_n and this block's share of d gamma:
//   du_i = gamma (dl_i / r - s_i <s, dl> / (N r^3)) sigmoid(u_i),   dgamma = sum_t <dl, s> / r.
__global__ __launch_bounds__(256) void gate_bwd_kernel(const float* __restrict__ dg, int ntok, int N, int top_k,
                                                       const int32_t* __restrict__ topk_idx,
                                                       const float* __restrict__ topk_w,
                                                       const int32_t* __restrict__ row_of, GateExtPtrs G,
                                                       float aux_coef, float* __restrict__ dl, float* __restrict__ du,
                                                       float* __restrict__ dgamma_part) {
  __shared__ float s_red[256];
  const int tid = threadIdx.x;
  const int t = blockIdx.x * 256 + tid;
  float dgam = 0.f;
  if (t < ntok) {
    float* row = dl + (size_t)t * N;
    if (G.probs && aux_coef != 0.f) {
      const float* p = G.probs + (size_t)t * N;
      float fp = 0.f;
      for (int e = 0; e < N; ++e) fp = fmaf(G.aux_f[e], p[e], fp);
      for (int e = 0; e < N; ++e) row[e] = aux_coef * p[e] * (G.aux_f[e] - fp);
    } else {
      for (int e = 0; e < N; ++e) row[e] = 0.f;
    }
    float g[2] = {0.f, 0.f}, dgv[2] = {0.f, 0.f};
    float mean = 0.f;
    for (int j = 0; j < top_k; ++j) {
      g[j] = topk_w[(size_t)t * top_k + j];
      dgv[j] = dg[row_of[(size_t)t * top_k + j]];
      mean += g[j] * dgv[j];
    }
    for (int j = 0; j < top_k; ++j) row[topk_idx[(size_t)t * top_k + j]] += g[j] * (dgv[j] - mean);
    if (G.W_noise) {
      const float* u = G.noise_pre + (size_t)t * N;
      float ss = 0.f, sd = 0.f;
      for (int e = 0; e < N; ++e) {
        const float sp = u[e] > 15.f ? u[e] : log1pf(__expf(u[e]));
        ss = fmaf(sp, sp, ss);
        sd = fmaf(sp, row[e], sd);
      }
      const float r = sqrtf(ss / (float)N + G.eps), gam = G.gamma[0];
      const float k1 = gam / r, k2 = gam * sd / ((float)N * r * r * r);
      for (int e = 0; e < N; ++e) {
        const float sp = u[e] > 15.f ? u[e] : log1pf(__expf(u[e]));
        du[(size_t)t * N + e] = (k1 * row[e] - k2 * sp) / (1.f + __expf(-u[e]));
      }
      dgam = sd / r;
    }
  }
  if (dgamma_part) {  // fixed-order sum over the block
    s_red[tid] = dgam;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
      for (int i = 0; i < 256; ++i) tot += s_red[i];
      dgamma_part[blockIdx.x] = tot;
    }
  }
}

// Backward through a router-side matrix W [d, ldw] (W_gate with dl, or W_noise with du) for BR_TOK tokens per
// block and up to 8 of its columns [e0, e0 + ne):
//   dX[t]      = (first ? sum_j dXp[row_of[t, j]] : dX[t]) + W[:, e0 : e0+ne] dl[t, e0 : e0+ne]
//   partial[b] = sum_{t in block} x[t] (outer) dl[t, e0 : e0+ne]      (reduced over blocks by dwg_reduce_kernel)
// A thread owns 8 columns of d for all tokens of the block, keeps the 8 x 8 slice of W and of the partial in
// registers, and per token reads x and the dXp rows once (16-byte loads, a full row per block instruction).
constexpr int BR_TOK = 32;
static_assert(BR_TOK == MODSE_ROUTE_TOKENS_PER_BLOCK, "the workspace holds one partial gradient per 32-token block");
template <typename T>
__global__ __launch_bounds__(ROUTE_THREADS) void bwd_gate_rows_kernel(
    const T* __restrict__ x, const T* __restrict__ W, int ldw, int e0, int ne, const T* __restrict__ dXp,
    const float* __restrict__ dl, int ntok, int d, int top_k, const int32_t* __restrict__ row_of, int first,
    T* __restrict__ dX, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) float s_dl[BR_TOK][8];
  __shared__ int s_row[BR_TOK][2];
  const int tid = threadIdx.x;
  const int t0 = blockIdx.x * BR_TOK;
  for (int i = tid; i < BR_TOK * 8; i += ROUTE_THREADS) {
    const int tl = i >> 3, e = i & 7;
    (&s_dl[0][0])[i] = (t0 + tl < ntok && e < ne) ? dl[(size_t)(t0 + tl) * ldw + e0 + e] : 0.f;
  }
  if (first && tid < BR_TOK && t0 + tid < ntok)
    for (int j = 0; j < top_k; ++j) s_row[tid][j] = row_of[(size_t)(t0 + tid) * top_k + j];
  __syncthreads();
  const int nt = min(BR_TOK, ntok - t0);
  for (int c = tid * 8; c < d; c += ROUTE_THREADS * 8) {
    float wg[8][8], acc[8][8];
    if (ldw == 8) {  // whole rows: eight 16-byte loads in flight together
#pragma unroll
      for (int q = 0; q < 8; ++q) load8(W + (size_t)(c + q) * 8, wg[q]);
    } else {  // columns beyond ne repeat the last one and are zeroed afterwards (no branch per element)
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float w = (float)W[(size_t)(c + q) * ldw + e0 + min(e, ne - 1)];
          wg[q][e] = e < ne ? w : 0.f;
        }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;
    // four tokens at a time, all twelve row loads issued before any arithmetic (no branch between them: a
    // missing second row is read from the first one's address and multiplied by zero)
    const float use_b = (first && top_k == 2) ? 1.f : 0.f;
    for (int tl0 = 0; tl0 < nt; tl0 += 4) {
      float xv[4][8], av[4][8], bv[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int tl = min(tl0 + u, nt - 1);
        const int t = t0 + tl;
        const T* pa = first ? dXp + (size_t)s_row[tl][0] * d : dX + (size_t)t * d;
        const T* pb = use_b != 0.f ? dXp + (size_t)s_row[tl][1] * d : pa;
        load8(x + (size_t)t * d + c, xv[u]);
        load8(pa + c, av[u]);
        load8(pb + c, bv[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int tl = tl0 + u;
        if (tl < nt) {
          float dlv[8], o[8];
          load8(&s_dl[tl][0], dlv);
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            float go = fmaf(use_b, bv[u][q], av[u][q]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              go = fmaf(wg[q][e], dlv[e], go);
              acc[q][e] = fmaf(xv[u][q], dlv[e], acc[q][e]);
            }
            o[q] = go;
          }
          store8(dX + (size_t)(t0 + tl) * d + c, o);
        }
      }
    }
    float* out = partial + ((size_t)blockIdx.x * d + c) * ldw + e0;
    if (ldw == 8) {  // the thread's 8 x 8 block is 256 consecutive bytes
#pragma unroll
      for (int q = 0; q < 8; ++q) store8(out + q * 8, acc[q]);
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (e < ne) out[q * ldw + e] = acc[q][e];
    }
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
  if (i < n) {
#pragma unroll 8
    for (int b = part; b < nb; b += 4) acc += partial[(size_t)b * n + i];  // unrolled: several loads in flight
  }
  s_part[part][li] = acc;
  __syncthreads();
  if (part == 0 && i < n) {
    const float v = (s_part[0][li] + s_part[1][li]) + (s_part[2][li] + s_part[3][li]);
    dWg[i] = accumulate ? dWg[i] + v : v;
  }
}

// [d, N] -> [d, NE] with zero columns behind the N real ones
template <typename T>
__global__ __launch_bounds__(256) void pad_rows_kernel(const T* __restrict__ W, int d, int N, int NE,
                                                       T* __restrict__ out) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d * NE) return;
  const int r = i / NE, e = i % NE;
  out[i] = e < N ? W[(size_t)r * N + e] : (T)0.f;
}

template <typename T, int NE>
hipError_t run_router(const LayerDims& L, const T* x, const T* Wg, const float* bias, const RoutingPtrs& R,
                      int32_t* blockhist, const GateExtPtrs* G, hipStream_t s) {
  const int nb = (L.T + TPB - 1) / TPB;
  if (G)
    hipLaunchKernelGGL((router_kernel<T, NE, true>), dim3(nb), dim3(ROUTE_THREADS), 0, s, x, Wg, bias, L.T, L.d, L.N,
                       L.k, R.topk_idx, R.topk_w, blockhist, *G);
  else
    hipLaunchKernelGGL((router_kernel<T, NE, false>), dim3(nb), dim3(ROUTE_THREADS), 0, s, x, Wg, bias, L.T, L.d, L.N,
                       L.k, R.topk_idx, R.topk_w, blockhist, GateExtPtrs{});
  return hipGetLastError();
}

// Which router a layer takes.  Plain gate, small and medium batches: one block per token keeps the chip busy
// where 32-token blocks would leave most CUs idle (measured at d = 2048..4096: 0.04 ms instead of 0.11 ms for 64
// tokens).  Larger plain batches: router_stream_kernel when W_gate fits its LDS area.  Otherwise, and with the
// optional gate parts, router_kernel.
enum RouterKind { ROUTER_TOKEN, ROUTER_STREAM, ROUTER_BLOCK };
RouterKind router_kind(const LayerDims& L, const GateExtPtrs* G) {
  if (G) return ROUTER_BLOCK;
  if (L.N <= 16 && L.T <= ROUTER_TOKEN_MAX_T) return ROUTER_TOKEN;
  if ((size_t)(L.d / 8) * rs_group_bytes(padded_experts(L.N), 4) <= (size_t)RS_W_BYTES && L.T >= 1024) return ROUTER_STREAM;
  return ROUTER_BLOCK;
}

// whether a layer that takes the streaming router can take its matrix-instruction form
bool router_on_mfma(const LayerDims& L) {
  const int NE = L.N <= 8 ? 8 : 16;
  return L.N <= 16 && L.d % 256 == 0 && (size_t)L.d * NE * 8 <= (size_t)rm_w_bytes(NE);
}

// logits, top-k, gate (and, except for ROUTER_TOKEN, the block histograms)
template <typename T>
hipError_t router_typed(const LayerDims& L, const void* xv, const void* Wgv, const float* bias, const RoutingPtrs& R,
                        const RouteBufs& B, const GateExtPtrs* G, hipStream_t s) {
  const T* x = static_cast<const T*>(xv);
  const T* Wg = static_cast<const T*>(Wgv);
  hipError_t e;
  const RouterKind kind = router_kind(L, G);
  const int NE = padded_experts(L.N);
  GateExtPtrs Gp;
  if (G) Gp = *G;
  if (kind != ROUTER_STREAM && NE != L.N) {  // these kernels want matrix rows of NE elements
    T* pad = static_cast<T*>(B.wpad);
    const int nblk = (L.d * NE + 255) / 256;
    hipLaunchKernelGGL((pad_rows_kernel<T>), dim3(nblk), dim3(256), 0, s, Wg, L.d, L.N, NE, pad);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    Wg = pad;
    if (G && G->W_noise) {
      T* pad2 = pad + (size_t)L.d * NE;
      hipLaunchKernelGGL((pad_rows_kernel<T>), dim3(nblk), dim3(256), 0, s, static_cast<const T*>(G->W_noise), L.d,
                         L.N, NE, pad2);
      if ((e = hipGetLastError()) != hipSuccess) return e;
      Gp.W_noise = pad2;
    }
  }
  if (kind == ROUTER_TOKEN) {
    const dim3 grid(L.T), blk(ROUTE_THREADS);
#define MODSE_LAUNCH_TOKEN_ROUTER(NE_)                                                                           \
  hipLaunchKernelGGL((router_token_kernel<T, NE_, 1>), grid, blk, 0, s, x, Wg, bias, L.T, L.d, L.N, L.k, R.topk_idx, \
                     R.topk_w, B.near_flag)
    if (NE == 2) MODSE_LAUNCH_TOKEN_ROUTER(2);
    else if (NE == 4) MODSE_LAUNCH_TOKEN_ROUTER(4);
    else if (NE == 8) MODSE_LAUNCH_TOKEN_ROUTER(8);
    else MODSE_LAUNCH_TOKEN_ROUTER(16);
#undef MODSE_LAUNCH_TOKEN_ROUTER
    e = hipGetLastError();
  } else if (kind == ROUTER_STREAM && router_on_mfma(L)) {
    const int ngroups = (L.T + RM_TOKENS - 1) / RM_TOKENS;
    const dim3 grid(std::min(ngroups, 256)), blk(RM_THREADS);  // one block per CU holds the LDS copy of W_gate
    if (L.N <= 8)
      hipLaunchKernelGGL((router_mfma_kernel<T, 8>), grid, blk, 0, s, x, Wg, bias, L.T, L.d, L.N, L.k, R.topk_idx,
                         R.topk_w, B.blockhist);
    else
      hipLaunchKernelGGL((router_mfma_kernel<T, 16>), grid, blk, 0, s, x, Wg, bias, L.T, L.d, L.N, L.k, R.topk_idx,
                         R.topk_w, B.blockhist);
    e = hipGetLastError();
  } else if (kind == ROUTER_STREAM) {
    const int ngroups = (L.T + RS_TOKENS - 1) / RS_TOKENS;
    const dim3 grid(std::min(ngroups, 256)), blk(RS_THREADS);  // one block per CU holds the LDS copy of W_gate
    const bool w64 = (size_t)(L.d / 8) * rs_group_bytes(NE, 8) <= (size_t)RS_W_BYTES;  // W_gate fits as float64
#define MODSE_LAUNCH_STREAM_ROUTER(NE_)                                                                            \
  do {                                                                                                            \
    if (w64)                                                                                                      \
      hipLaunchKernelGGL((router_stream_kernel<T, NE_, double>), grid, blk, 0, s, x, Wg, bias, L.T, L.d, L.N, L.k, \
                         R.topk_idx, R.topk_w, B.blockhist);                                                      \
    else                                                                                                          \
      hipLaunchKernelGGL((router_stream_kernel<T, NE_, float>), grid, blk, 0, s, x, Wg, bias, L.T, L.d, L.N, L.k,  \
                         R.topk_idx, R.topk_w, B.blockhist);                                                      \
  } while (0)
    switch (NE) {
      case 2: MODSE_LAUNCH_STREAM_ROUTER(2); break;
      case 4: MODSE_LAUNCH_STREAM_ROUTER(4); break;
      case 8: MODSE_LAUNCH_STREAM_ROUTER(8); break;
      case 16: MODSE_LAUNCH_STREAM_ROUTER(16); break;
      case 32: MODSE_LAUNCH_STREAM_ROUTER(32); break;
      default: MODSE_LAUNCH_STREAM_ROUTER(64); break;
    }
#undef MODSE_LAUNCH_STREAM_ROUTER
    e = hipGetLastError();
  } else {
    const GateExtPtrs* g = G ? &Gp : nullptr;
    switch (NE) {
      case 2: e = run_router<T, 2>(L, x, Wg, bias, R, B.blockhist, g, s); break;
      case 4: e = run_router<T, 4>(L, x, Wg, bias, R, B.blockhist, g, s); break;
      case 8: e = run_router<T, 8>(L, x, Wg, bias, R, B.blockhist, g, s); break;
      case 16: e = run_router<T, 16>(L, x, Wg, bias, R, B.blockhist, g, s); break;
      case 32: e = run_router<T, 32>(L, x, Wg, bias, R, B.blockhist, g, s); break;
      default: e = run_router<T, 64>(L, x, Wg, bias, R, B.blockhist, g, s); break;
    }
  }
  if (e != hipSuccess) return e;
  if (G && G->probs) {
    hipLaunchKernelGGL(aux_finish_kernel, dim3(1), dim3(256), 0, s, G->probs, R.topk_idx, L.T, L.N, L.k, G->alpha,
                       G->aux_f, G->aux_P, G->aux_loss);
    e = hipGetLastError();
  }
  return e;
}

// histogram (where the router has not made it), scan over blocks (which also makes the forward tile plans when
// `plan` is given), stable scatter; batches of at most PERMUTE_SMALL_MAX_T tokens: one fused launch for all of it
template <typename T>
hipError_t permute_typed(const LayerDims& L, modse_dtype dt, const void* xv, const RoutingPtrs& R, const RouteBufs& B,
                         void* Xpv, const GateExtPtrs* G, const FwdPlanArgs* plan, hipStream_t s) {
  const T* x = static_cast<const T*>(xv);
  const int nb = (L.T + TPB - 1) / TPB;
  hipError_t e;
  const bool token_router = router_kind(L, G) == ROUTER_TOKEN;
  if (L.T <= MODSE_PERMUTE_SMALL_MAX_T) {
    hipLaunchKernelGGL((permute_small_kernel<T>), dim3(L.T), dim3(256), 0, s, x, L.T, L.d, L.N, L.k, R.topk_idx,
                       token_router ? B.near_flag : nullptr, B.blockhist, R, static_cast<T*>(Xpv), L,
                       dt == MODSE_F32 ? 4 : 2, plan ? *plan : FwdPlanArgs{}, plan ? 1 : 0);
    return hipGetLastError();
  }
  if (token_router) {
    hipLaunchKernelGGL(route_hist_kernel, dim3(nb), dim3(64), 0, s, R.topk_idx, B.near_flag, L.T, L.N, L.k,
                       B.blockhist);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  hipLaunchKernelGGL(route_scan_kernel, dim3(1), dim3(256), 0, s, B.blockhist, nb, L.N, R.counts, R.offsets,
                     R.near_tie_count, L, dt == MODSE_F32 ? 4 : 2, plan ? *plan : FwdPlanArgs{}, plan ? 1 : 0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((scatter_kernel<T>), dim3(nb), dim3(ROUTE_THREADS), 0, s, x, L.T, L.d, L.N, L.k, R.topk_idx,
                     R.offsets, B.blockhist, R.row_of, R.src_of, static_cast<T*>(Xpv));
  return hipGetLastError();
}

// dX and the gradient of one router-side matrix, 8 expert columns per launch
template <typename T>
hipError_t gate_rows_typed(const LayerDims& L, const void* x, const void* W, const void* dXp, const float* dl,
                           const RoutingPtrs& R, int first, void* dX, float* partial, float* dW, int accumulate,
                           hipStream_t s) {
  const int nb = (L.T + BR_TOK - 1) / BR_TOK;
  for (int e0 = 0; e0 < L.N; e0 += 8) {
    hipLaunchKernelGGL((bwd_gate_rows_kernel<T>), dim3(nb), dim3(ROUTE_THREADS), 0, s, static_cast<const T*>(x),
                       static_cast<const T*>(W), L.N, e0, min(8, L.N - e0), static_cast<const T*>(dXp), dl, L.T, L.d,
                       L.k, R.row_of, (first && e0 == 0) ? 1 : 0, static_cast<T*>(dX), partial);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int n = L.d * L.N;
  hipLaunchKernelGGL(dwg_reduce_kernel, dim3((n + 63) / 64), dim3(256), 0, s, partial, nb, n, accumulate, dW);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_router(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const float* bias,
                         const RoutingPtrs& R, const RouteBufs& B, const GateExtPtrs* G, hipStream_t s) {
  return dt == MODSE_F32 ? router_typed<float>(L, x, W_gate, bias, R, B, G, s)
                         : router_typed<bf16_t>(L, x, W_gate, bias, R, B, G, s);
}

hipError_t launch_permute(const LayerDims& L, modse_dtype dt, const void* x, const RoutingPtrs& R, const RouteBufs& B,
                          void* Xp, const GateExtPtrs* G, const FwdPlanArgs* plan, hipStream_t s) {
  return dt == MODSE_F32 ? permute_typed<float>(L, dt, x, R, B, Xp, G, plan, s)
                         : permute_typed<bf16_t>(L, dt, x, R, B, Xp, G, plan, s);
}

hipError_t launch_route(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const float* bias,
                        const RoutingPtrs& R, const RouteBufs& B, void* Xp, const GateExtPtrs* G, hipStream_t s) {
  const hipError_t e = launch_router(L, dt, x, W_gate, bias, R, B, G, s);
  return e != hipSuccess ? e : launch_permute(L, dt, x, R, B, Xp, G, nullptr, s);
}

hipError_t launch_routing_stats(const LayerDims& L, const int32_t* topk_idx, int32_t* slot_counts, float* summary,
                                hipStream_t s) {
  hipLaunchKernelGGL(routing_stats_kernel, dim3(1), dim3(256), 0, s, topk_idx, L.T, L.N, L.k, L, slot_counts, summary);
  return hipGetLastError();
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

hipError_t launch_combine_split(const LayerDims& L, modse_dtype dt, const float* Opart, int kchunk, const RoutingPtrs& R,
                                void* y, hipStream_t s) {
  const int nb = (int)(((long)L.T * (L.d / 8) + 255) / 256);
  if (dt == MODSE_F32)
    hipLaunchKernelGGL((combine_split_kernel<float>), dim3(nb), dim3(256), 0, s, Opart, L.T, L.d, L.k, L, kchunk,
                       R.topk_idx, R.row_of, R.topk_w, static_cast<float*>(y));
  else
    hipLaunchKernelGGL((combine_split_kernel<bf16_t>), dim3(nb), dim3(256), 0, s, Opart, L.T, L.d, L.k, L, kchunk,
                       R.topk_idx, R.row_of, R.topk_w, static_cast<bf16_t*>(y));
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

hipError_t launch_bwd_router(const LayerDims& L, modse_dtype dt, const void* x, const void* W_gate, const void* dXp,
                             const float* dg, const RoutingPtrs& R, const GateExtPtrs* G, float aux_grad,
                             const BwdRouterBufs& B, void* dX, float* dW_gate, float* dW_noise, float* dgamma,
                             int accumulate, hipStream_t s) {
  const GateExtPtrs none = {};
  const GateExtPtrs& g = G ? *G : none;
  const bool noise = g.W_noise != nullptr;
  const float aux_coef = g.probs ? aux_grad * g.alpha * (float)L.N / (float)L.T : 0.f;
  const int nbt = (L.T + 255) / 256;
  hipLaunchKernelGGL(gate_bwd_kernel, dim3(nbt), dim3(256), 0, s, dg, L.T, L.N, L.k, R.topk_idx, R.topk_w, R.row_of, g,
                     aux_coef, B.dl, noise ? B.du : nullptr, noise ? B.dgamma_part : nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = dt == MODSE_F32 ? gate_rows_typed<float>(L, x, W_gate, dXp, B.dl, R, 1, dX, B.dW_partial, dW_gate, accumulate, s)
                      : gate_rows_typed<bf16_t>(L, x, W_gate, dXp, B.dl, R, 1, dX, B.dW_partial, dW_gate, accumulate, s);
  if (e != hipSuccess || !noise) return e;
  e = dt == MODSE_F32
          ? gate_rows_typed<float>(L, x, g.W_noise, nullptr, B.du, R, 0, dX, B.dW_partial, dW_noise, accumulate, s)
          : gate_rows_typed<bf16_t>(L, x, g.W_noise, nullptr, B.du, R, 0, dX, B.dW_partial, dW_noise, accumulate, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(dwg_reduce_kernel, dim3(1), dim3(256), 0, s, B.dgamma_part, nbt, 1, accumulate, dgamma);
  return hipGetLastError();
}
