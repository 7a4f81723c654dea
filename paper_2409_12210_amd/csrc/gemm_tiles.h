// Tile walking and fused epilogues shared by the grouped GEMM kernels (gfx950).
#pragma once
#include "common.h"

namespace modse_gemm {

constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;  // tiles of GROUP_M consecutive row blocks are walked column-first (L2 reuse)

struct TileCoord {
  int p, mt, nt;
};

// Division by a positive divisor d through one multiplication: floor(n / d) == mulhi(n, ceil(2^32 / d))
// whenever n * d < 2^32.  tile_magic returns 0 when the caller's largest n does not satisfy that (the
// decoding then divides).
__host__ __device__ inline uint32_t tile_magic(uint32_t d, uint64_t n_max) {
  if (d <= 1 || n_max * d >= (1ull << 32)) return 0;
  return (uint32_t)(((1ull << 32) + d - 1) / d);
}
__device__ inline uint32_t magic_div(uint32_t n, uint32_t d, uint32_t magic) {
  return magic ? __umulhi(n, magic) : n / d;
}

// Tile `local` of a problem with mtiles x ntiles tiles: tiles are walked in groups of GROUP_M row blocks,
// column-first inside a group.
__device__ inline void decode_local(int local, int mtiles, int ntiles, uint32_t magic_group, uint32_t magic_tail, int& mt,
                                    int& nt) {
  const int per_group = GROUP_M * ntiles;
  const int g = (int)magic_div((uint32_t)local, (uint32_t)per_group, magic_group);
  const int first = g * GROUP_M;
  const int rem = local - g * per_group;
  const int gsz = min(mtiles - first, GROUP_M);
  if (gsz == GROUP_M) {
    nt = rem / GROUP_M;
    mt = first + rem % GROUP_M;
  } else {
    nt = (int)magic_div((uint32_t)rem, (uint32_t)gsz, magic_tail);
    mt = first + rem - nt * gsz;
  }
}

__device__ inline bool decode_tile(const GemmPlan* __restrict__ plan, int tile, TileCoord& tc) {
  const int np = plan->n_prob;
  if (tile >= plan->tile_start[np]) return false;
  int lo = 0, hi = np;  // last p with tile_start[p] <= tile (problems without tiles are stepped over)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (plan->tile_start[mid] <= tile) lo = mid;
    else hi = mid;
  }
  const int p = lo;
  const GemmProblem& P = plan->prob[p];
  tc.p = p;
  decode_local(tile - plan->tile_start[p], P.mtiles, P.ntiles, P.magic_group, P.magic_tail, tc.mt, tc.nt);
  return true;
}

// Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of the tile list so
// that the tiles sharing operand rows meet in the same L2.
__device__ inline int first_tile_of_block() {
  const int G = gridDim.x, b = blockIdx.x;
  return (G % NUM_XCD == 0) ? (b % NUM_XCD) * (G / NUM_XCD) + b / NUM_XCD : b;
}

// Tile of a workgroup in round r: the rounds deal the list out alternately forwards and backwards.  With
// the problems sorted by falling cost per tile this keeps the workgroups' sums close (a plain round-robin
// hands the same workgroups the dearest tile of every round).
__device__ inline int tile_of_round(int first, int r) {
  const int G = gridDim.x;
  return r * G + ((r & 1) ? G - 1 - first : first);
}

__device__ inline float silu_f(float a) { return a / (1.f + __expf(-a)); }

// SwiGLU of the pre-activations a = <W1 row, x>, b = <W3 row, x> with sig = 1 / (1 + exp(-a)):
//   h = silu(a) b,   p = dh/da = b sig (1 + a (1 - sig)),   q = dh/db = silu(a).
// The forward pass saves p and q (not a and b), so the backward epilogue is two multiplications.
__device__ inline void swiglu_terms(float a, float b, float sig, float& h, float& p, float& q) {
  q = a * sig;
  h = q * b;
  p = b * sig * (1.f + a * (1.f - sig));
}

// Epilogue on 4 consecutive columns n..n+3 of row m.  a = first accumulator, b = second (SwiGLU only).
template <typename T, int EPI>
__device__ inline void epilogue4(const GemmProblem& P, int m, int n, const float a[4], const float b[4],
                                 int accumulate, int save_pre) {
  if (m >= P.M || n >= P.N) return;
  const size_t o = (size_t)m * P.ldc + n;
  if constexpr (EPI == EPI_STORE || EPI == EPI_STORE_DUALK) {
    store4(static_cast<T*>(P.C) + o, a);
  } else if constexpr (EPI == EPI_STORE_F32) {
    float* c = static_cast<float*>(P.C) + o;
    float v[4] = {a[0], a[1], a[2], a[3]};
    if (accumulate) {
      float old[4];
      load4(c, old);
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] += old[i];
    }
    store4(c, v);
  } else if constexpr (EPI == EPI_SWIGLU) {
    float h[4], p[4], q[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) swiglu_terms(a[i], b[i], 1.f / (1.f + __expf(-a[i])), h[i], p[i], q[i]);
    store4(static_cast<T*>(P.C) + o, h);
    if (save_pre) {
      store4(static_cast<T*>(P.C2) + o, p);
      store4(static_cast<T*>(P.C3) + o, q);
    }
  } else if constexpr (EPI == EPI_SWIGLU_BWD) {
    float p[4], q[4], da[4], db[4];
    load4(static_cast<const T*>(P.E1) + o, p);
    load4(static_cast<const T*>(P.E2) + o, q);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      da[i] = a[i] * p[i];
      db[i] = a[i] * q[i];
    }
    store4(static_cast<T*>(P.C) + o, da);
    store4(static_cast<T*>(P.C2) + o, db);
  }
}

}  // namespace modse_gemm
