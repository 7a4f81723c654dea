// bf16 grouped GEMM for gfx950: MFMA 32x32x16, fp32 accumulate, direct global->LDS loads.
//
// One persistent workgroup of 8 waves (WAVES_M x WAVES_N, two per SIMD) walks the tile list.  A tile is
// BM x BN (x NB matrices B that share A: the up-projection's W1 and W3); K advances 64 elements per step.
//
// LDS: two stages, each (BM + NB*BN) rows of 128 bytes (64 bf16 along K).  The LDS of gfx950 has 64
// banks of 4 bytes and serves a ds_read_b128 sixteen lanes at a time; the 16-byte chunk index of a row
// is XOR-ed with ((row >> 1) & 7), so 16 consecutive rows read at the same K offset cover all 64 banks
// (measured: SQ_LDS_BANK_CONFLICT = 0, 4 LDS cycles per ds_read_b128).  Stages are filled by
// global_load_lds_dwordx4: one wave instruction writes 1 KiB of consecutive LDS (8 rows); which global
// chunk a lane fetches is chosen so that the data lands pre-swizzled.  The loads are issued from inline
// assembly with a scalar base and a 32-bit lane offset, so every vmcnt wait is explicit here.
//
// Pipeline: the loads of stage g+1 are issued in slices between the MFMA groups of stage g (a wave that
// blocks on a full load queue cannot feed the matrix pipe), and the K loop is rotated: the barrier that
// opens stage g+1 and the first fragment reads of that stage sit in front of the last MFMA group of
// stage g.  The issue cursor runs across tile boundaries, so the first stage of the next tile is in
// flight while the epilogue of the current one stores.
//
// The accumulator of v_mfma_f32_32x32x16_bf16 holds, per lane, 4 consecutive rows of the instruction's
// first operand.  The B tile is fed as first operand, so those 4 values are consecutive columns of C.
#pragma once
#include "gemm_bf16_util.h"

namespace modse_gemm {

#ifndef MODSE_DMA_SPREAD
#define MODSE_DMA_SPREAD 2  // the stage loads of a step are issued in this many slices, between the MFMA groups
#endif

template <int BM, int BN, int NB, int WAVES_M, int WAVES_N>
struct SkinnyTile {
  static constexpr int BK = 64;
  static constexpr int NWAVES = WAVES_M * WAVES_N;
  static constexpr int NT = NWAVES * 64;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int MI = WM / 32, NI = WN / 32;
  static constexpr int ROWS = BM + NB * BN;  // LDS rows of one stage
  static constexpr int UA = BM / 8;          // 1 KiB load units (8 rows) of the A tile
  static constexpr int UNITS = ROWS / 8;     // ... of the whole stage
  static constexpr int UPW = UNITS / NWAVES; // units per wave and stage
  static constexpr int STAGE = ROWS * 128;
  static constexpr bool SKINNY = BM == 64;  // decode-sized M: every wave loads one A unit and UPW - 1 B units
  static_assert(UNITS % NWAVES == 0 && (UPW % 2 == 0 || SKINNY), "load units must divide evenly among waves");
  static_assert(MODSE_DMA_SPREAD == 2, "the stage loads go out in two slices");
  static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile must be a multiple of 32");
};

// Walks the K steps of this workgroup's tiles in order.
struct StepCursor {
  const GemmProblem* gp;  // the tile's problem (read field by field: a copy of the struct would live in scratch)
  int tile, round, step, nsteps, nk, K;
  int m0, n0;
  bool valid;
};

// LAYOUT bit 0: A is stored [K, M] (M contiguous) instead of [M, K]; bit 1: B is stored [K, N].  Such an
// operand keeps its memory order in LDS (64 rows of K, 512 bytes each, 32-byte chunk index XOR-ed with
// 2 * (k & 3)) and its MFMA fragments are read with ds_read_b64_tr_b16, which hands lane i of a 16-lane
// group the i-th column of a 4 x 16 block of 16-bit elements: 4 consecutive K for one M (or N).
template <int BM, int BN, int NB, int WAVES_M, int WAVES_N, int EPI, int LAYOUT = 0>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gg_bf16_skinny_kernel(const GemmPlan* __restrict__ plan,
                                                                        int accumulate, int save_pre) {
  using Cfg = SkinnyTile<BM, BN, NB, WAVES_M, WAVES_N>;
  constexpr int BK = Cfg::BK, MI = Cfg::MI, NI = Cfg::NI, UA = Cfg::UA, UPW = Cfg::UPW, STAGE = Cfg::STAGE;
  constexpr int WM = Cfg::WM, WN = Cfg::WN;
  constexpr int SLICE0 = (UPW + 1) / 2;  // units of the first of the two load slices
  constexpr bool SKINNY = Cfg::SKINNY;
  constexpr bool A_T = (LAYOUT & 1) != 0, B_T = (LAYOUT & 2) != 0;
  static_assert(!SKINNY || (!A_T && !B_T && UA == Cfg::NWAVES && WAVES_M == 1), "skinny tiles: forward layouts, one A unit per wave");
  static_assert(!(A_T && BM != 256) && !(B_T && (BN != 256 || NB != 1)), "transposed operands use 256-wide tiles");
  static_assert(SKINNY || (UA % UPW == 0 && (BN / 8) % UPW == 0), "all load units of a wave must belong to one operand");
  __shared__ __attribute__((aligned(1024))) char stages[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int total = plan->tile_start[plan->n_prob];
  const int first_tile = first_tile_of_block();
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane(lds_address(stages));
  // load unit (8 LDS rows) that this wave's i-th load of a stage fills.  Regular tiles: UPW consecutive units,
  // all of one operand.  Skinny tiles: A unit `wave`, then UPW - 1 consecutive B units.
  auto unit_of = [&](int i) -> int {
    if (SKINNY) return i == 0 ? wave : UA + wave * (UPW - 1) + (i - 1);
    return wave * UPW + i;
  };
  const int first_b_unit = SKINNY ? UA + wave * (UPW - 1) : wave * UPW;  // (meaningful when the wave loads B)
  const int lrow = lane >> 3;  // row inside a load unit
  // element offset of the chunk this lane fetches, for even and odd load units: LDS position (row, p)
  // holds logical chunk p ^ ((row >> 1) & 7), and row = 8 * unit + lrow
  const int lchunk_even = ((lane & 7) ^ (lrow >> 1)) * 8;
  const int lchunk_odd = ((lane & 7) ^ (4 | (lrow >> 1))) * 8;
  // fragment read offsets inside a stage (bytes), without the kk-dependent swizzle term
  const int a_frag = (wm * WM + (lane & 31)) * 128;
  const int b_frag = BM * 128 + (wn * WN + (lane & 31)) * 128;
  const int khalf = lane >> 5, lsw = (lane >> 1) & 7;
  // transposed operands: this lane's row inside a load unit (2 rows of 32 chunks) and its chunk
  const int t_row = lane >> 5, t_chunk = lane & 31;
  const bool loads_a = !SKINNY && wave * UPW < UA;            // wave-uniform: which operand a regular wave loads
  const bool loads_t = loads_a ? A_T : B_T;                   // ... and whether it is a transposed one

  auto open_tile = [&](StepCursor& c) {
    TileCoord tc;
    c.valid = c.tile < total && decode_tile(plan, c.tile, tc);
    if (!c.valid) return;
    c.gp = plan->prob + tc.p;
    c.m0 = tc.mt * BM;
    c.n0 = tc.nt * BN;
    c.step = 0;
    c.K = c.gp->K;
    c.nk = (c.K + BK - 1) / BK;
    c.nsteps = (EPI == EPI_STORE_DUALK) ? 2 * c.nk : c.nk;
  };

  // ---- issue side: runs one K step ahead of the MFMAs, across tile boundaries
  StepCursor ic;
  const char* ibase[2] = {nullptr, nullptr};  // operand this wave loads from, per pass of a dual-K product
  const char* ibase_a = nullptr;              // skinny tiles: the A operand (unit 0 of every wave)
  bool ia_needed = true;                      // ... and whether any of its 8 rows exists (rows >= M are never stored)
  int ikstride = 1;                           // elements between consecutive K of that operand
  uint32_t ioff[UPW];  // byte offset of this lane's chunk per load unit (K offset 0) from the operand base
  // tiles without K steps (an expert that received no token, in a weight-gradient GEMM) take no stage
  auto skip_empty = [&]() {
    while (ic.valid && ic.nsteps == 0) {
      ic.tile = tile_of_round(first_tile, ++ic.round);
      open_tile(ic);
    }
  };
  auto issue_offsets = [&]() {
    const GemmProblem* P = ic.gp;
    {  // operand this wave loads from (wave-uniform)
      const int u = first_b_unit;
      if (SKINNY) ibase_a = static_cast<const char*>(P->A);
      if (!SKINNY && u < UA) {
        ibase[0] = static_cast<const char*>(P->A);
        ibase[1] = static_cast<const char*>(P->A2);
      } else if (NB == 2) {
        ibase[0] = ibase[1] = static_cast<const char*>((u - UA) * 8 >= BN ? P->B2 : P->B);
      } else {
        ibase[0] = static_cast<const char*>(P->B);
        ibase[1] = static_cast<const char*>(P->B2);
      }
    }
    const int PM = P->M, PN = P->N, lda = P->lda, ldb = P->ldb;
    if (SKINNY) ia_needed = __builtin_amdgcn_readfirstlane(ic.m0 + wave * 8 < PM ? 1 : 0) != 0;
    ikstride = loads_t ? (loads_a ? lda : ldb) : 1;
    if (loads_t) {  // unit = K rows 2u, 2u+1; LDS position (k, p) holds 16-byte chunk p ^ (4 * (k & 3))
#pragma unroll
      for (int i = 0; i < UPW; ++i) {
        const int ul = (wave * UPW + i) - (loads_a ? 0 : UA);
        const int k = 2 * ul + t_row;
        const int c16 = t_chunk ^ (4 * (k & 3));
        const int x0 = loads_a ? ic.m0 : ic.n0, X = loads_a ? PM : PN, ld = loads_a ? lda : ldb;
        ioff[i] = (uint32_t)(k * ld + min(x0 + c16 * 8, X - 8)) * 2u;  // columns past the end repeat the last chunk
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
      const int u = unit_of(i);
      const int lchunk = (u & 1) ? lchunk_odd : lchunk_even;  // both operand regions start at an even unit
      if (u < UA) {
        ioff[i] = (uint32_t)(min(ic.m0 + u * 8 + lrow, PM - 1) * lda + lchunk) * 2u;
      } else {
        const int r = ((u - UA) * 8 + lrow) % BN;
        ioff[i] = (uint32_t)(min(ic.n0 + r, PN - 1) * ldb + lchunk) * 2u;
      }
    }
  };
  // issue load units [first, first + count) of the issue cursor's step into stage buffer `buf`
  auto issue_slice = [&](int buf, int first, int count) {
    if (!ic.valid) return;
    const int pass = (EPI == EPI_STORE_DUALK && ic.step >= ic.nk) ? 1 : 0;
    const int k0 = (ic.step - pass * ic.nk) * BK;
    const uint32_t dst = lds_base + buf * STAGE;
    const char* base = ibase[pass] + (size_t)k0 * ikstride * 2;
    if (k0 + BK <= ic.K) {
#pragma unroll
      for (int i = first; i < first + count; ++i) {
        if (SKINNY && i == 0) {  // the activation rows: every tile of the expert reads them again
          if (ia_needed) dma_b128_s(ibase_a + (size_t)k0 * 2, ioff[i], dst + unit_of(i) * 1024);
        } else  // a skinny tile's weights are read once in the whole launch
          dma_b128_s<SKINNY>(base, ioff[i], dst + unit_of(i) * 1024);
      }
    } else if (loads_t) {  // partial last step: K rows beyond K read zeros
#pragma unroll
      for (int i = first; i < first + count; ++i) {
        const int ul = (wave * UPW + i) - (loads_a ? 0 : UA);
        const char* src = base + ioff[i];
        if (k0 + 2 * ul + t_row >= ic.K) src = reinterpret_cast<const char*>(g_zero_chunk);
        dma_b128(src, dst + unit_of(i) * 1024);
      }
    } else {  // last step of a pass when K % 64 != 0: chunks beyond K read zeros
#pragma unroll
      for (int i = first; i < first + count; ++i) {
        if (SKINNY && i == 0 && !ia_needed) continue;
        const char* src = ((SKINNY && i == 0) ? ibase_a + (size_t)k0 * 2 : base) + ioff[i];
        if (k0 + ((unit_of(i) & 1) ? lchunk_odd : lchunk_even) >= ic.K) src = reinterpret_cast<const char*>(g_zero_chunk);
        dma_b128(src, dst + unit_of(i) * 1024);
      }
    }
  };
  auto advance_issue = [&]() {
    if (!ic.valid) return;
    if (++ic.step >= ic.nsteps) {
      ic.tile = tile_of_round(first_tile, ++ic.round);
      open_tile(ic);
      skip_empty();
      if (ic.valid) issue_offsets();
    }
  };

  // ---- compute side
  StepCursor cc;
  cc.tile = first_tile;
  cc.round = 0;
  open_tile(cc);
  if (!cc.valid) return;
  ic = cc;
  skip_empty();
  if (ic.valid) issue_offsets();
  const bool any_stage = ic.valid;
  issue_slice(0, 0, UPW);  // stage of global step 0
  advance_issue();
  // A skinny tile is bound by the weight stream, not by the matrix pipe: its stage loads go out in one piece as
  // early as their buffer is free, straight behind the barrier that retires it (and those of step 1 right here),
  // instead of in slices between the MFMA groups.  (A loader alone in this shape, 64 KiB stages, streams 6.7 TB/s.)
  bool early_next = false;  // SKINNY: the stage of the step after the current one exists (and has been issued)
  if constexpr (SKINNY) {
    early_next = ic.valid;
    issue_slice(1, 0, UPW);
    advance_issue();
  }

  // Fragments are double-buffered in registers: set (kk & 1) feeds the MFMAs of K slice kk while the
  // other set is being read from LDS.
  bf16x8 af[2][MI], bfr[2][NB][NI];
  // Transposed operands.  Lane l = 16 * blk + s reads, for K slice kk and half h, the 8 bytes at
  // K row kk*16 + (blk >> 1)*8 + h*4 + (s >> 2), column x = tile_x + 32*i + (blk & 1)*16 + 4*(s & 3); the
  // instruction returns K rows +0..+3 of column tile_x + 32*i + (blk & 1)*16 + s.
  int tr_a[MI], tr_b[NI];
  {
    const int blk = lane >> 4, sl = lane & 15, kq = sl >> 2;
    const int rowbyte = ((blk >> 1) * 8 + kq) * 512 + (sl & 1) * 8;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int c16 = (wm * WM + i * 32 + (blk & 1) * 16) / 8 + ((sl & 3) >> 1);
      tr_a[i] = rowbyte + ((c16 ^ (4 * kq)) << 4);
    }
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int c16 = (wn * WN + j * 32 + (blk & 1) * 16) / 8 + ((sl & 3) >> 1);
      tr_b[j] = BM * 128 + rowbyte + ((c16 ^ (4 * kq)) << 4);
    }
  }
  auto read_tr = [&](const char* p) -> bf16x8 {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * 512));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  };
  auto load_frags = [&](const char* buf, int kk, int set) {
    const int sw = ((kk * 2 + khalf) ^ lsw) << 4;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      if (A_T) af[set][i] = read_tr(buf + tr_a[i] + kk * 16 * 512);
      else af[set][i] = *reinterpret_cast<const bf16x8*>(buf + a_frag + i * 32 * 128 + sw);
    }
#pragma unroll
    for (int q = 0; q < NB; ++q)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        if (B_T) bfr[set][q][j] = read_tr(buf + tr_b[j] + kk * 16 * 512);
        else bfr[set][q][j] = *reinterpret_cast<const bf16x8*>(buf + b_frag + (q * BN + j * 32) * 128 + sw);
      }
  };
  f32x16 acc[NB][MI][NI];
  auto mfma_block = [&](int set) {
#pragma unroll
    for (int q = 0; q < NB; ++q)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[q][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][q][j], af[set][i], acc[q][i][j], 0, 0, 0);
  };
  // Stage hand-over.  All my loads have landed (s_waitcnt simm16 on gfx9: vmcnt in bits [3:0] and
  // [15:14], expcnt in [6:4], lgkmcnt in [11:8]) and my LDS reads have returned; then everybody meets.
  // Afterwards the new stage may be read and the buffer of the old one refilled.
  auto stage_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  int g = 0;  // global step count of this workgroup: stage buffer = g & 1
  if (any_stage) {
    stage_barrier();
    load_frags(stages, 0, 0);
  }
  while (cc.valid) {
#pragma unroll
    for (int q = 0; q < NB; ++q)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[q][i][j][r] = 0.f;

    // The K loop is rotated: the barrier that opens stage g+1 and the first fragment reads of that stage
    // sit in front of the last MFMA group of stage g, so the matrix pipe has work while LDS answers.
#pragma unroll 1
    for (int s = 0; s < cc.nsteps; ++s, ++g) {
      const char* buf = stages + (g & 1) * STAGE;
      const int nbuf = (g + 1) & 1;
      // a stage g+1 exists (maybe in the next tile); uniform in the workgroup
      const bool next_stage = SKINNY ? early_next : ic.valid;
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) {
        load_frags(buf, kk + 1, (kk + 1) & 1);
        if (!SKINNY && kk < MODSE_DMA_SPREAD) {  // the loads of stage g+1 go out in slices between the MFMA groups
          __builtin_amdgcn_sched_barrier(0);
          issue_slice(nbuf, kk == 0 ? 0 : SLICE0, kk == 0 ? SLICE0 : UPW - SLICE0);
          __builtin_amdgcn_sched_barrier(0);
        }
        mfma_block(kk & 1);
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (!SKINNY) advance_issue();
      // (after the very last step the barrier only retires the buffer: the epilogue stages through it)
      stage_barrier();
      if constexpr (SKINNY) {  // stage g+2 into the buffer of stage g, whose last fragments are in registers
        early_next = ic.valid;
        issue_slice(g & 1, 0, UPW);
        advance_issue();
        __builtin_amdgcn_sched_barrier(0);
      }
      if (next_stage) load_frags(stages + nbuf * STAGE, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      mfma_block(1);
    }

    // ---- epilogue.  For register group r of block (i, j) the lane holds columns n .. n+3 of row m.
    const GemmProblem& CP = *cc.gp;
    const int cM = CP.M, cN = CP.N, cld = CP.ldc;
    if constexpr (EPI == EPI_STORE_F32 || SKINNY) {  // (a skinny tile's output is a few rows: stored directly)
      const int mrow = cc.m0 + wm * WM + (lane & 31);
      const int ncol = cc.n0 + wn * WN + 4 * khalf;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float a[4], b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              a[q] = acc[0][i][j][r * 4 + q];
              b[q] = acc[NB - 1][i][j][r * 4 + q];
            }
            epilogue4<bf16_t, EPI>(CP, mrow + i * 32, ncol + j * 32 + r * 8, a, b, accumulate, save_pre);
          }
    } else {
      // 16-bit outputs go through LDS so that global memory sees whole 128-byte lines: the wave works in
      // units of 32 rows x 64 columns (two MFMA blocks), writes a unit into a 4 KiB slot in accumulator
      // order (8 bytes per lane), reads it back row-wise (16 bytes per lane, 8 lanes per row) and stores.
      // The two slots are the part of the retired stage buffer that only this wave's own loads refill, so
      // no other wave is involved; LDS serves one wave's accesses in program order.
      static_assert(NI % 2 == 0 && UPW >= 8, "staged epilogue: 64-column units, 8 KiB of stage per wave");
      constexpr int NJP = NI / 2, NU = MI * NJP;
      char* const slot0 = stages + ((g + 1) & 1) * STAGE + first_b_unit * 1024;
      char* const slot1 = slot0 + 4096;
      const int er = lane & 31, esw = (er >> 1) & 7;
      const int rrow = lane >> 3, rchunk = lane & 7;
      auto acc_pos = [&](char* slot, int jj, int r) -> bf16x4* {  // 4 columns of accumulator group (jj, r)
        return reinterpret_cast<bf16x4*>(slot + er * 128 + (((jj * 4 + r) ^ esw) << 4) + khalf * 8);
      };
      auto row_pos = [&](char* slot, int it) -> bf16x8* {  // chunk rchunk of row 8 * it + rrow
        const int rr = it * 8 + rrow;
        return reinterpret_cast<bf16x8*>(slot + rr * 128 + ((rchunk ^ ((rr >> 1) & 7)) << 4));
      };
      auto unit_m = [&](int u) { return cc.m0 + wm * WM + (u / NJP) * 32; };
      auto unit_n = [&](int u) { return cc.n0 + wn * WN + (u % NJP) * 64; };
      // element offset of this lane's row-wise chunk of unit u, or -1 outside the matrix
      auto row_off = [&](int u, int it) -> long {
        const int m = unit_m(u) + it * 8 + rrow, n = unit_n(u) + rchunk * 8;
        return (m < cM && n < cN) ? (long)m * cld + n : -1;
      };
      auto put_block = [&](char* slot, int jj, const f32x16& c) {  // one 32 x 32 block of the unit
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          bf16x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = (bf16_t)c[r * 4 + q];
          *acc_pos(slot, jj, r) = v;
        }
      };
      auto put_unit = [&](char* slot, const f32x16& c0, const f32x16& c1) {
        put_block(slot, 0, c0);
        put_block(slot, 1, c1);
      };
      auto store_unit = [&](char* slot, int u, void* C) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const bf16x8 v = *row_pos(slot, it);
          const long o = row_off(u, it);
          if (o >= 0) global_store16(static_cast<bf16_t*>(C) + o, v);
        }
      };
      if constexpr (EPI == EPI_STORE || EPI == EPI_STORE_DUALK) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          if (unit_m(u) >= cM) continue;
          char* slot = (u & 1) ? slot1 : slot0;
          put_unit(slot, acc[0][u / NJP][2 * (u % NJP)], acc[0][u / NJP][2 * (u % NJP) + 1]);
          store_unit(slot, u, CP.C);
        }
      } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          if (unit_m(u) >= cM) continue;
          const int i = u / NJP, j0 = 2 * (u % NJP);
          // h = silu(a) b and the saved term p = dh/da go to the slots four columns at a time; q = dh/db
          // takes b's place in the accumulator and follows once the slot of h is free
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              bf16x4 hv, pv;
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const float a = acc[0][i][j0 + jj][r * 4 + q4], b = acc[1][i][j0 + jj][r * 4 + q4];
                float h, p, q;
                swiglu_terms(a, b, sigmoid_fast(a), h, p, q);
                hv[q4] = (bf16_t)h;
                pv[q4] = (bf16_t)p;
                acc[1][i][j0 + jj][r * 4 + q4] = q;
              }
              *acc_pos(slot0, jj, r) = hv;
              if (save_pre) *acc_pos(slot1, jj, r) = pv;
            }
          store_unit(slot0, u, CP.C);
          if (save_pre) {
            store_unit(slot1, u, CP.C2);
            put_unit(slot0, acc[1][i][j0], acc[1][i][j0 + 1]);
            store_unit(slot0, u, CP.C3);
          }
        }
      } else if constexpr (EPI == EPI_SWIGLU_BWD) {
        // the saved terms p = dh/da and q = dh/db of the unit come in row-wise (whole lines), one unit ahead
        // of the arithmetic; da = dh p and db = dh q replace them in the slots at the positions the lane read
        bf16x8 pa[4], pb[4];
        auto fetch = [&](int u) {
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const long o = row_off(u, it);
            pa[it] = bf16x8{};
            pb[it] = bf16x8{};
            if (o >= 0) {
              pa[it] = global_load16(static_cast<const bf16_t*>(CP.E1) + o);
              pb[it] = global_load16(static_cast<const bf16_t*>(CP.E2) + o);
            }
          }
        };
        fetch(0);
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          const int i = u / NJP, j0 = 2 * (u % NJP);
          const bool active = unit_m(u) < cM;
          if (active) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
              *row_pos(slot0, it) = pa[it];
              *row_pos(slot1, it) = pb[it];
            }
          }
          if (u + 1 < NU) fetch(u + 1);
          if (active) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const bf16x4 av = *acc_pos(slot0, jj, r), bv = *acc_pos(slot1, jj, r);
                bf16x4 da, db;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                  const float dh = acc[0][i][j0 + jj][r * 4 + q];
                  da[q] = (bf16_t)(dh * (float)av[q]);
                  db[q] = (bf16_t)(dh * (float)bv[q]);
                }
                *acc_pos(slot0, jj, r) = da;
                *acc_pos(slot1, jj, r) = db;
              }
            store_unit(slot0, u, CP.C);
            store_unit(slot1, u, CP.C2);
          }
        }
      }
    }
    cc.tile = tile_of_round(first_tile, ++cc.round);
    open_tile(cc);
  }
  // drain: nothing may still be writing LDS when the workgroup's allocation is released
  __builtin_amdgcn_s_waitcnt(0x0070);
}

}  // namespace modse_gemm
