// Device-side tile plans of the grouped GEMMs: the counts that the router leaves on the device become a
// problem table and a tile prefix, without a host round trip.  Included by the GEMM translation unit (plan
// kernels) and by the routing one (the decode-sized fused permute + plan kernel).
#pragma once
#include "common.h"
#include "gemm_tiles.h"

namespace modse_gemm {

// Tile counts and decode constants of a problem (from the fields in registers, before the problem is stored);
// returns its number of tiles.
__device__ inline int set_tiles(GemmProblem& P, int bm, int bn) {
  P.mtiles = (P.M + bm - 1) / bm;
  P.ntiles = (P.N + bn - 1) / bn;
  const int tiles = P.mtiles * P.ntiles;
  P.magic_group = tile_magic((uint32_t)(GROUP_M * P.ntiles), (uint64_t)tiles);
  P.magic_tail = tile_magic((uint32_t)(P.mtiles % GROUP_M), (uint64_t)GROUP_M * P.ntiles);
  return tiles;
}

// Every thread has stored its problems (n in total) and left their tile counts in s_tiles; fills in the tile prefix.
__device__ inline void finish_plan(GemmPlan* plan, int i, int n, int* s_tiles) {
  __syncthreads();
  if (i == 0) {
    int run = 0;
    for (int q = 0; q < n; ++q) {
      plan->tile_start[q] = run;
      run += s_tiles[q];
    }
    plan->tile_start[n] = run;
    plan->n_prob = n;
  }
  __syncthreads();
}

__device__ inline const char* cadd(const void* p, size_t bytes) { return static_cast<const char*>(p) + bytes; }
__device__ inline char* vadd(void* p, size_t bytes) { return p ? static_cast<char*>(p) + bytes : nullptr; }

// Problem tables of the two forward GEMMs.  Every thread of one block calls this (threads beyond the expert count
// only take part in the barriers); s_tiles: MODSE_MAX_PROBLEMS ints of LDS.
__device__ inline void plan_fwd_body(const LayerDims& L, int esize, const int32_t* counts, const int32_t* offsets,
                                     const FwdPlanArgs& a, int* s_tiles) {
  const int i = threadIdx.x;
  const bool on = i < L.N;
  const int e = on ? L.order[i] : 0;
  size_t hoff = 0;  // elements of H before expert e
  for (int q = 0; q < e; ++q) hoff += (size_t)counts[q] * L.f[q];
  const int n_e = counts[e], f = L.f[e], d = L.d;
  const size_t es = esize;
  if (on) {
    GemmProblem P = {};
    P.A = cadd(a.Xp, (size_t)offsets[e] * d * es);
    P.B = cadd(a.W1, (size_t)L.foff[e] * d * es);
    P.B2 = cadd(a.W3, (size_t)L.foff[e] * d * es);
    P.C = vadd(a.H, hoff * es);
    P.C2 = vadd(a.dHdA, hoff * es);
    P.C3 = vadd(a.dHdB, hoff * es);
    P.M = n_e; P.N = f; P.K = d;
    P.lda = d; P.ldb = d; P.ldc = f;
    s_tiles[i] = set_tiles(P, a.up_tile.bm, a.up_tile.bn);
    a.up->prob[i] = P;
  }
  finish_plan(a.up, i, L.N, s_tiles);
  if (a.kchunk > 0) {  // split-K: one problem per (expert, chunk of K), float32 partial sums
    int first = 0;     // problems of the experts listed before this one
    for (int q = 0; q < i && q < L.N; ++q) first += (L.f[L.order[q]] + a.kchunk - 1) / a.kchunk;
    int total = 0;
    for (int q = 0; q < L.N; ++q) total += (L.f[q] + a.kchunk - 1) / a.kchunk;
    if (on) {
      const int nchunk = (f + a.kchunk - 1) / a.kchunk;
      for (int c = 0; c < nchunk; ++c) {
        const int k0 = c * a.kchunk;
        GemmProblem P = {};
        P.A = cadd(a.H, (hoff + k0) * es);
        P.B = cadd(a.W2, ((size_t)L.foff[e] * d + k0) * es);
        P.C = a.Opart + ((size_t)c * L.T * L.k + offsets[e]) * d;
        P.M = n_e; P.N = d; P.K = min(a.kchunk, f - k0);
        P.lda = f; P.ldb = f; P.ldc = d;
        s_tiles[first + c] = set_tiles(P, a.down_tile.bm, a.down_tile.bn);
        a.down->prob[first + c] = P;
      }
    }
    finish_plan(a.down, i, total, s_tiles);
    return;
  }
  if (on) {
    GemmProblem P = {};
    P.A = cadd(a.H, hoff * es);
    P.B = cadd(a.W2, (size_t)L.foff[e] * d * es);
    P.C = vadd(a.O, (size_t)offsets[e] * d * es);
    P.M = n_e; P.N = d; P.K = f;
    P.lda = f; P.ldb = f; P.ldc = d;
    s_tiles[i] = set_tiles(P, a.down_tile.bm, a.down_tile.bn);
    a.down->prob[i] = P;
  }
  finish_plan(a.down, i, L.N, s_tiles);
}

}  // namespace modse_gemm
