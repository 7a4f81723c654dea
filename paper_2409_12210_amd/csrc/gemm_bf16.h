// bf16 grouped GEMM for gfx950: MFMA 32x32x16, fp32 accumulate, direct global->LDS loads, ping-pong waves
// over a ring of five LDS panels.
//
// One persistent workgroup of 8 waves (WAVES_M x WAVES_N, two per SIMD) walks the tile list.  A tile is
// 256 x 256 (up-projection: 256 x (128 of W1 + 128 of W3)); K advances 64 elements per step.
//
// LDS: five panels of 32 KiB.  A panel holds 64 K-elements of one operand for the whole tile: 256 rows of
// 128 bytes for a K-contiguous operand (the 16-byte chunk index of a row is XOR-ed with ((row >> 1) & 7):
// conflict-free ds_read_b128 on the 64 banks of gfx950), or 64 K-rows of 512 bytes for an operand stored
// [K, X] (16-byte chunk index XOR-ed with 4 * (k & 3), fragments through ds_read_b64_tr_b16).  Step g uses
// panel 2g (A) and 2g+1 (B); panel i lives in slot i mod 5, so a panel can be refilled as soon as the step
// two (B) or three (A) steps back has been read.
//
// Ping-pong: the two waves of a SIMD (wave w and w + 4) run one phase apart.  Every step has four phases
// separated by workgroup barriers.  In a memory phase a wave only reads the MFMA fragments of one K half
// from LDS (12 ds_read_b128); in a compute phase it issues the 16 MFMAs of that half and, in their shadow,
// everything else: its four loads of one panel and the cursor arithmetic.  A wave issues one instruction
// every few cycles, and the matrix pipe takes 32 cycles per MFMA, so the compute phase has issue slots to
// spare while the memory phase has none: measured on MI355X, every scalar instruction added to the memory
// phase lengthens the step, and four loads spread over the MFMAs of the compute phase cost nothing.
// While a wave multiplies, its SIMD partner reads fragments, so the matrix pipe always has work.
//
// Every wave loads units 4w..4w+3 (1 KiB each) of every panel.  The early waves (0..3) issue the B panel
// of the next step in their first compute phase and the A panel two steps ahead in their second one; the
// late waves issue the A panel two steps ahead first and then the B panel two steps ahead (its slot has
// just been retired in the phase before).  A load has between two and five phases to arrive.  The loads
// are issued from inline assembly (the compiler does not know that they write LDS), so every vmcnt wait
// is explicit here.
//
// The accumulator of v_mfma_f32_32x32x16_bf16 holds, per lane, 4 consecutive rows of the instruction's
// first operand.  The B tile is fed as first operand, so those 4 values are consecutive columns of C.
#pragma once
#include "gemm_bf16_util.h"

namespace modse_gemm {

template <int BM, int BN, int NB, int WAVES_M, int WAVES_N>
struct Bf16Tile {
  static constexpr int BK = 64;
  static constexpr int NWAVES = WAVES_M * WAVES_N;
  static constexpr int NT = NWAVES * 64;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int MI = WM / 32, NI = WN / 32;
  static constexpr int PANEL = 256 * 128;  // bytes of one operand panel
  static constexpr int NSLOT = 5;
  static constexpr int UPW = 4;            // 1 KiB load units per wave and panel
  static_assert(BM == 256 && NB * BN == 256 && NWAVES == 8, "panels are 256 rows, loaded by 8 waves");
  static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile must be a multiple of 32");
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

// A GemmProblem in scalar registers.  The plan is read with scalar loads issued from inline assembly: it
// was written by an earlier kernel and nothing writes it while the GEMM runs, and a load the compiler
// emitted as a vector load would make it wait for every panel load in flight before the value is used.
struct ProblemRegs {
  u32x16 lo;  // A, B, A2, B2, C, C2, C3, E1
  u32x8 hi;   // E2, M, N, K, lda, ldb, ldc
  u32x4 tl;   // mtiles, ntiles, magic_group, magic_tail
  __device__ __forceinline__ void load(const GemmProblem* p) {
    static_assert(sizeof(GemmProblem) == 128 && alignof(GemmProblem) == 128, "scalar loads assume this layout");
    asm volatile(
        "s_load_dwordx16 %0, %3, 0x0\n\ts_load_dwordx8 %1, %3, 0x40\n\ts_load_dwordx4 %2, %3, 0x60\n\ts_waitcnt lgkmcnt(0)"
        : "=&s"(lo), "=&s"(hi), "=&s"(tl)
        : "s"(p)
        : "memory");
  }
  __device__ __forceinline__ const char* ptr(int i) const {  // i-th pointer of the struct, i < 8
    return reinterpret_cast<const char*>(((uint64_t)lo[2 * i + 1] << 32) | lo[2 * i]);
  }
  __device__ __forceinline__ const char* A() const { return ptr(0); }
  __device__ __forceinline__ const char* B() const { return ptr(1); }
  __device__ __forceinline__ const char* A2() const { return ptr(2); }
  __device__ __forceinline__ const char* B2() const { return ptr(3); }
  __device__ __forceinline__ void* C() const { return const_cast<char*>(ptr(4)); }
  __device__ __forceinline__ void* C2() const { return const_cast<char*>(ptr(5)); }
  __device__ __forceinline__ void* C3() const { return const_cast<char*>(ptr(6)); }
  __device__ __forceinline__ const void* E1() const { return ptr(7); }
  __device__ __forceinline__ const void* E2() const { return reinterpret_cast<const void*>(((uint64_t)hi[1] << 32) | hi[0]); }
  __device__ __forceinline__ int M() const { return (int)hi[2]; }
  __device__ __forceinline__ int N() const { return (int)hi[3]; }
  __device__ __forceinline__ int K() const { return (int)hi[4]; }
  __device__ __forceinline__ int lda() const { return (int)hi[5]; }
  __device__ __forceinline__ int ldb() const { return (int)hi[6]; }
  __device__ __forceinline__ int ldc() const { return (int)hi[7]; }
  __device__ __forceinline__ int mtiles() const { return (int)tl[0]; }
  __device__ __forceinline__ int ntiles() const { return (int)tl[1]; }
  __device__ __forceinline__ uint32_t magic_group() const { return tl[2]; }
  __device__ __forceinline__ uint32_t magic_tail() const { return tl[3]; }
};
// tile_start[p] and tile_start[p + 1]
__device__ __forceinline__ u32x2 load_tile_range(const int32_t* p) {
  uint32_t a, b;
  asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %2, 0x4\n\ts_waitcnt lgkmcnt(0)" : "=&s"(a), "=&s"(b) : "s"(p) : "memory");
  return u32x2{a, b};
}

// Position in this workgroup's tile sequence.  The tiles of a workgroup come in rising order, so the
// problem index only moves forwards.
struct TileWalk {
  int p, pstart, pend;  // problem of the tile and its range of the tile list
  int mtiles, ntiles;
  uint32_t magic_group, magic_tail;
  int tile, round;
  int m0, n0;
  int valid;  // (an int: a bool that lives across loops is kept as a lane mask and tested with vector compares)
};
// Walks the K steps of one operand's panels, ahead of the MFMAs.
struct LoadCursor {
  TileWalk w;
  int is_a;           // which operand this cursor walks
  const char* base0;  // operand of the first pass
  const char* base1;  // operand of the second pass of a dual-K product
  const char* src;    // the current step's 64 K-elements of the operand (wave-uniform part of the address)
  int rows, ld;       // rows of the stored matrix along the tile (M or N) and its row stride
  int kbytes;         // bytes between consecutive K steps
  int K, nk, step, nsteps;
  int fast;           // the current step exists and is a full one (no zero fill)
};
// The tile being multiplied.
struct ComputeCursor {
  TileWalk w;
  const char *C, *C2, *C3, *E1, *E2;
  int M, N, ldc, nsteps;
};

// LAYOUT bit 0: A is stored [K, M] (M contiguous) instead of [M, K]; bit 1: B is stored [K, N].
template <int BM, int BN, int NB, int WAVES_M, int WAVES_N, int EPI, int LAYOUT = 0>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gg_bf16_kernel(const GemmPlan* __restrict__ plan,
                                                                        int accumulate, int save_pre) {
  using Cfg = Bf16Tile<BM, BN, NB, WAVES_M, WAVES_N>;
  constexpr int BK = Cfg::BK, MI = Cfg::MI, NI = Cfg::NI, UPW = Cfg::UPW, PANEL = Cfg::PANEL, NSLOT = Cfg::NSLOT;
  constexpr int WM = Cfg::WM, WN = Cfg::WN;
  constexpr bool A_T = (LAYOUT & 1) != 0, B_T = (LAYOUT & 2) != 0;
  static_assert(!(B_T && NB != 1), "a [K, N] operand is a single matrix");
  __shared__ __attribute__((aligned(1024))) char ring[NSLOT * PANEL];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const bool grp_y = wave >= Cfg::NWAVES / 2;  // the second wave of each SIMD
  const int total = __builtin_amdgcn_readfirstlane(plan->tile_start[plan->n_prob]);
  const int first_tile = first_tile_of_block();
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane(lds_address(ring));
  const int unit0 = wave * UPW;  // this wave loads units unit0 .. unit0 + 3 of every panel
  const int lrow = lane >> 3;    // row inside a load unit of a K-contiguous operand
  // element offset of the chunk this lane fetches, for even and odd load units: LDS position (row, p)
  // holds logical chunk p ^ ((row >> 1) & 7), and row = 8 * unit + lrow
  const int lchunk_even = ((lane & 7) ^ (lrow >> 1)) * 8;
  const int lchunk_odd = ((lane & 7) ^ (4 | (lrow >> 1))) * 8;
  // [K, X] operands: a load unit is 2 K-rows of 32 chunks; this lane's row inside the unit and its chunk
  const int t_row = lane >> 5, t_chunk = lane & 31;
  // fragment read offsets inside a panel (bytes), without the kk-dependent swizzle term
  const int a_frag = (wm * WM + (lane & 31)) * 128;
  const int b_frag = (wn * WN + (lane & 31)) * 128;
  const int khalf = lane >> 5, lsw = (lane >> 1) & 7;

  // moves w to w.tile; returns true when the problem changed (then P holds the new problem)
  auto walk_to = [&](TileWalk& w, ProblemRegs& P) -> bool {
    w.valid = w.tile < total ? 1 : 0;
    if (!w.valid) return false;
    int changed = 0;
    if (w.p < 0) {  // first tile of this walk
      w.p = 0;
      const u32x2 r = load_tile_range(plan->tile_start);
      w.pstart = (int)r[0];
      w.pend = (int)r[1];
      changed = 1;
    }
    while (w.tile >= w.pend) {  // (problems without tiles are stepped over)
      ++w.p;
      const u32x2 r = load_tile_range(plan->tile_start + w.p);
      w.pstart = (int)r[0];
      w.pend = (int)r[1];
      changed = 1;
    }
    if (changed) {
      P.load(plan->prob + w.p);
      w.mtiles = P.mtiles();
      w.ntiles = P.ntiles();
      w.magic_group = P.magic_group();
      w.magic_tail = P.magic_tail();
    }
    int mt, nt;
    decode_local(w.tile - w.pstart, w.mtiles, w.ntiles, w.magic_group, w.magic_tail, mt, nt);
    w.m0 = mt * BM;
    w.n0 = nt * BN;
    return changed != 0;
  };

  // ---- issue side: two cursors run ahead of the MFMAs, across tile boundaries.  c0 is served in the first
  // compute phase of a step, c1 in the second.  Early waves: c0 = B panels (one step ahead), c1 = A panels
  // (two steps ahead); late waves: c0 = A panels (two ahead), c1 = B panels (two ahead).
  LoadCursor c0, c1;
  uint32_t off0[UPW], off1[UPW];  // byte offset of this lane's chunk per load unit from the cursor's src
  // opens the tile c.w.tile (or a later one: tiles without K steps -- an expert that received no token, in
  // a weight-gradient GEMM -- take no panel)
  auto open_cursor = [&](LoadCursor& c, uint32_t (&off)[UPW]) {
    for (;;) {
      ProblemRegs P;
      if (walk_to(c.w, P)) {
        if (c.is_a) {
          c.base0 = P.A();
          c.base1 = P.A2();
          c.rows = P.M();
          c.ld = P.lda();
          c.kbytes = A_T ? BK * 2 * c.ld : BK * 2;
        } else {
          if (NB == 2) {  // rows 0..127 of the panel come from B (W1), rows 128..255 from B2 (W3)
            c.base0 = c.base1 = unit0 * 8 >= BN ? P.B2() : P.B();
          } else {
            c.base0 = P.B();
            c.base1 = P.B2();
          }
          c.rows = P.N();
          c.ld = P.ldb();
          c.kbytes = B_T ? BK * 2 * c.ld : BK * 2;
        }
        c.base0 = static_cast<const char*>(uniform_ptr(c.base0));  // (otherwise the compiler keeps the cursor in vector registers)
        c.K = P.K();
        c.nk = (c.K + BK - 1) / BK;
        c.nsteps = (EPI == EPI_STORE_DUALK) ? 2 * c.nk : c.nk;
      }
      if (!c.w.valid || c.nsteps != 0) break;
      c.w.tile = tile_of_round(first_tile, ++c.w.round);
    }
    c.fast = 0;
    if (!c.w.valid) return;
    c.step = 0;
    c.src = c.base0;
    c.fast = BK <= c.K ? 1 : 0;
    const bool tr = c.is_a ? A_T : B_T;
    const int x0 = c.is_a ? c.w.m0 : c.w.n0;
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
      const int u = unit0 + i;
      if (tr) {  // unit = K rows 2u, 2u+1; LDS position (k, p) holds 16-byte chunk p ^ (4 * (k & 3))
        const int k = 2 * u + t_row;
        const int c16 = t_chunk ^ (4 * (k & 3));
        off[i] = (uint32_t)(k * c.ld + min(x0 + c16 * 8, c.rows - 8)) * 2u;  // columns past the end repeat the last chunk
      } else {
        const int r = c.is_a ? u * 8 + lrow : (u * 8 + lrow) % BN;
        off[i] = (uint32_t)(min(x0 + r, c.rows - 1) * c.ld + ((u & 1) ? lchunk_odd : lchunk_even)) * 2u;
      }
    }
  };
  // one load unit of the cursor's current (full) step
  auto panel_dst = [&](int slot) -> uint32_t { return lds_base + slot * PANEL + unit0 * 1024; };  // my units of a ring slot
  auto issue_fast = [&](const LoadCursor& c, const uint32_t (&off)[UPW], uint32_t dst, int i) {
    dma_b128_s(c.src, off[i], dst + i * 1024);
  };
  // all load units of a last step that is not a full one: what lies beyond K reads zeros
  auto issue_partial = [&](const LoadCursor& c, const uint32_t (&off)[UPW], uint32_t dst) {
    const int kstep = (EPI == EPI_STORE_DUALK && c.step >= c.nk) ? c.step - c.nk : c.step;
    const bool tr = c.is_a ? A_T : B_T;
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
      const char* p = c.src + off[i];
      const int kfirst = tr ? 2 * (unit0 + i) + t_row : (((unit0 + i) & 1) ? lchunk_odd : lchunk_even);  // first K of this lane's chunk
      if (kstep * BK + kfirst >= c.K) p = reinterpret_cast<const char*>(g_zero_chunk);
      dma_b128(p, dst + i * 1024);
    }
  };
  auto advance = [&](LoadCursor& c, uint32_t (&off)[UPW]) {
    if (!c.w.valid) return;
    c.src += c.kbytes;
    if (++c.step >= c.nsteps) {
      c.w.tile = tile_of_round(first_tile, ++c.w.round);
      open_cursor(c, off);
      return;
    }
    int kstep = c.step;
    if (EPI == EPI_STORE_DUALK && c.step >= c.nk) {
      kstep -= c.nk;
      if (kstep == 0) c.src = c.base1;
    }
    c.fast = (kstep + 1) * BK <= c.K ? 1 : 0;
  };
  // whole panel of a cursor's current step, then on to the next step (prologue)
  auto issue_panel = [&](LoadCursor& c, uint32_t (&off)[UPW], int slot) {
    if (c.fast) {
#pragma unroll
      for (int i = 0; i < UPW; ++i) issue_fast(c, off, panel_dst(slot), i);
    } else if (c.w.valid) {
      issue_partial(c, off, panel_dst(slot));
    }
    advance(c, off);
  };
  ComputeCursor cc;
  auto open_c = [&]() {
    ProblemRegs P;
    if (walk_to(cc.w, P)) {
      cc.C = P.ptr(4);
      cc.C2 = P.ptr(5);
      cc.C3 = P.ptr(6);
      cc.E1 = P.ptr(7);
      cc.E2 = static_cast<const char*>(P.E2());
      cc.M = P.M();
      cc.N = P.N();
      cc.ldc = P.ldc();
      const int nk = (P.K() + BK - 1) / BK;
      cc.nsteps = (EPI == EPI_STORE_DUALK) ? 2 * nk : nk;
    }
  };

  // ---- compute side
  cc.w.p = -1;
  cc.w.tile = first_tile;
  cc.w.round = 0;
  open_c();
  if (!cc.w.valid) return;
  c0.w = cc.w;
  c0.w.p = -1;
  c1.w = c0.w;
  c0.is_a = grp_y ? 1 : 0;
  c1.is_a = grp_y ? 0 : 1;
  open_cursor(c0, off0);
  open_cursor(c1, off1);
  const int any_step = c0.w.valid;
  // panels of step 0 and the A panel of step 1; the late waves also their share of the B panel of step 1.
  // The last panel c1 loads here is completed (a step that is not a full one; the move to the next step) by
  // the first memory phase, like every panel c1 loads later.
  auto issue_fast_panel_dst = [&](LoadCursor& c, uint32_t (&off)[UPW], uint32_t dst) {
    if (c.fast) {
#pragma unroll
      for (int i = 0; i < UPW; ++i) issue_fast(c, off, dst, i);
    }
  };
  auto issue_fast_panel = [&](LoadCursor& c, uint32_t (&off)[UPW], int slot) { issue_fast_panel_dst(c, off, panel_dst(slot)); };
  if (!grp_y) {
    issue_panel(c1, off1, 0);
    issue_panel(c0, off0, 1);
    issue_fast_panel(c1, off1, 2);
  } else {
    issue_panel(c0, off0, 0);
    issue_panel(c1, off1, 1);
    issue_panel(c0, off0, 2);
    issue_fast_panel(c1, off1, 3);
  }
  int a_ahead = 0;  // the youngest UPW loads of this wave belong to an A panel that is not waited for yet

  // Fragments of one K half (two K slices of 16): set kk & 1.
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
      tr_b[j] = rowbyte + ((c16 ^ (4 * kq)) << 4);
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
  auto load_frags = [&](const char* abuf, const char* bbuf, int kk, int set) {
    const int sw = ((kk * 2 + khalf) ^ lsw) << 4;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      if (A_T) af[set][i] = read_tr(abuf + tr_a[i] + kk * 16 * 512);
      else af[set][i] = *reinterpret_cast<const bf16x8*>(abuf + a_frag + i * 32 * 128 + sw);
    }
#pragma unroll
    for (int q = 0; q < NB; ++q)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        if (B_T) bfr[set][q][j] = read_tr(bbuf + tr_b[j] + kk * 16 * 512);
        else bfr[set][q][j] = *reinterpret_cast<const bf16x8*>(bbuf + b_frag + (q * BN + j * 32) * 128 + sw);
      }
  };
  f32x16 acc[NB][MI][NI];
  // The 16 MFMAs of one K half; in their shadow this wave's four loads of cursor c's panel (into ring slot
  // `slot`), one after every fourth MFMA.
  auto mfma_half = [&](LoadCursor& c, uint32_t (&off)[UPW], uint32_t dst, auto always) {
    const int fast = decltype(always)::value ? 1 : c.fast;
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int t = 0; t < 2 * NB * MI * NI; ++t) {
      constexpr int PER = NB * MI * NI;
      const int set = t / PER, r = t % PER, q = r / (MI * NI), i = (r / NI) % MI, j = r % NI;
      acc[q][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][q][j], af[set][i], acc[q][i][j], 0, 0, 0);
      if (t % (2 * PER / UPW) == 1) {
        __builtin_amdgcn_sched_barrier(0);
        if (fast) issue_fast(c, off, dst, t / (2 * PER / UPW));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  // in the memory phase that follows: a step that was not a full one is issued now, and the cursor moves on
  auto after_issue = [&](LoadCursor& c, uint32_t (&off)[UPW], uint32_t dst) {
    if (!c.fast && c.w.valid) issue_partial(c, off, dst);
    advance(c, off);
  };
  // End of a phase: my LDS reads have returned (s_waitcnt simm16 on gfx9: vmcnt in bits [3:0] and [15:14],
  // expcnt in [6:4], lgkmcnt in [11:8]); then everybody meets.
  auto phase_end = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  // All my panel loads have landed except, if `ahead`, the UPW youngest (loads complete in order).
  auto wait_panels = [&](int ahead) {
    __builtin_amdgcn_sched_barrier(0);
    if (ahead) __builtin_amdgcn_s_waitcnt(0x0f70 | UPW);  // vmcnt(UPW)
    else __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  auto slot_add = [&](int s, int d) { return (s + d) >= NSLOT ? s + d - NSLOT : s + d; };
  // how many times a cursor can move on and still stand on a full step of the same tile and pass
  auto fast_left = [&](const LoadCursor& c) -> int {
    if (!c.fast) return 0;
    const int full = c.K / BK;
    const int lim = (EPI == EPI_STORE_DUALK && c.step >= c.nk) ? c.nk + full : full;
    return lim - c.step - 1;
  };

  if (any_step) {
    wait_panels(0);
    phase_end();
  }
  if (grp_y) phase_end();  // the second wave of each SIMD starts one phase late
  const int d0 = grp_y ? 4 : 3, d1 = grp_y ? 0 : 4;  // ring slots of the panels c0 and c1 load, relative to the step's A panel
  int sa = 0;  // ring slot of the current step's A panel; its B panel is in the next slot
  auto zero_acc = [&]() {
#pragma unroll
    for (int q = 0; q < NB; ++q)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[q][i][j][r] = 0.f;
  };
  zero_acc();
  while (cc.w.valid) {
    int s = 0;
#pragma unroll 1
    while (s < cc.nsteps) {
      // Steady stretch: the steps during which both load cursors stay on full steps of their present tile and
      // pass.  Nothing about a cursor has to be decided then: its source moves on by one step, four loads go
      // out in every MFMA phase, and four loads (the youngest) may stay in flight at either wait, for both
      // wave groups alike.
      {
        const int n0 = fast_left(c0), n1 = fast_left(c1);
        int n = n0 < n1 ? n0 : n1;
        n = n < cc.nsteps - s ? n : cc.nsteps - s;
        s += n;
#pragma unroll 1
        for (; n > 0; --n) {
          const char* abuf = ring + sa * PANEL;
          const char* bbuf = ring + slot_add(sa, 1) * PANEL;
          load_frags(abuf, bbuf, 0, 0);
          load_frags(abuf, bbuf, 1, 1);
          __builtin_amdgcn_sched_barrier(0);
          c1.src += c1.kbytes;
          ++c1.step;
          const uint32_t dst0 = panel_dst(slot_add(sa, d0)), dst1 = panel_dst(slot_add(sa, d1));
          phase_end();
          mfma_half(c0, off0, dst0, std::true_type{});
          phase_end();
          load_frags(abuf, bbuf, 2, 0);
          load_frags(abuf, bbuf, 3, 1);
          __builtin_amdgcn_sched_barrier(0);
          c0.src += c0.kbytes;
          ++c0.step;
          wait_panels(1);
          phase_end();
          mfma_half(c1, off1, dst1, std::true_type{});
          wait_panels(1);
          phase_end();
          sa = slot_add(sa, 2);
        }
        if (s >= cc.nsteps) break;
      }
      ++s;
      const char* abuf = ring + sa * PANEL;
      const char* bbuf = ring + slot_add(sa, 1) * PANEL;
      load_frags(abuf, bbuf, 0, 0);
      load_frags(abuf, bbuf, 1, 1);
      __builtin_amdgcn_sched_barrier(0);
      after_issue(c1, off1, panel_dst(slot_add(sa, grp_y ? 3 : 2)));  // (the panel c1 loaded in the step before)
      const uint32_t dst0 = panel_dst(slot_add(sa, d0)), dst1 = panel_dst(slot_add(sa, d1));
      if (grp_y) a_ahead = c0.w.valid;
      phase_end();
      mfma_half(c0, off0, dst0, std::false_type{});
      phase_end();
      load_frags(abuf, bbuf, 2, 0);
      load_frags(abuf, bbuf, 3, 1);
      __builtin_amdgcn_sched_barrier(0);
      after_issue(c0, off0, dst0);
      if (!grp_y) a_ahead = c1.fast;
      // at the end of this phase of the late waves the panels of the next step must be complete
      if (grp_y) wait_panels(a_ahead);
      phase_end();
      mfma_half(c1, off1, dst1, std::false_type{});
      if (!grp_y) wait_panels(a_ahead);
      phase_end();
      sa = slot_add(sa, 2);
    }

    // ---- epilogue.  For register group r of block (i, j) the lane holds columns n .. n+3 of row m.
    // The early waves wait here for the late waves' last MFMA phase, and the late waves wait behind their
    // epilogue for the early waves' first phase of the next tile: both groups then run their epilogues at the
    // same time (the memory latency of one hides behind the other's) and are one phase apart again afterwards.
    // Without the two barriers the phase barriers alone would let one group's epilogue run while the other
    // group waits, one after the other.
    // (The SwiGLU epilogue stages two outputs at once and keeps its two slots per wave; its groups still run
    // one after the other.)
    constexpr bool BOTH_EPI = EPI != EPI_SWIGLU;  // both groups' epilogues at the same time
    if (BOTH_EPI && !grp_y) phase_end();
    // (The lane index goes through an empty asm statement: otherwise the compiler computes the epilogue's
    // per-lane addresses once, ahead of the tile loop, and they occupy dozens of registers in the main loop.)
    int elane = lane;
    asm volatile("" : "+v"(elane));
    const int ekhalf = elane >> 5;
    const int cM = cc.M, cN = cc.N, cld = cc.ldc;
    if constexpr (EPI == EPI_STORE_F32) {
      // float32 output (weight gradients).  A tile inside the matrix that overwrites C goes through LDS, one
      // 32 x 32 block (4 KiB) at a time: written in accumulator order (16 bytes per lane), read back row-wise,
      // so that global memory sees whole 128-byte lines.  The slots are this wave's own load units in the
      // two panels of the step just finished.
      const bool interior = cc.w.m0 + BM <= cM && cc.w.n0 + BN <= cN;
      if (interior && !accumulate && cc.nsteps != 0) {
        // (the late waves have already refilled their units of the A panel's slot: they have one slot, and
        // write a block into it only after the block before has been read back)
        char* const fslot[2] = {ring + slot_add(sa, grp_y ? NSLOT - 1 : NSLOT - 2) * PANEL + unit0 * 1024,
                                ring + slot_add(sa, NSLOT - 1) * PANEL + unit0 * 1024};
        const int er = elane & 31, esw = (er >> 1) & 7, rrow = elane >> 3, rchunk = elane & 7;
        const uint32_t voff = (uint32_t)(rrow * cld + rchunk * 4) * 4u;
        const char* const wave_c = cc.C + ((size_t)(cc.w.m0 + wm * WM) * cld + cc.w.n0 + wn * WN) * 4;
        auto put = [&](int b) {  // block b = i * NI + j
          f32x16& c = acc[0][b / NI][b % NI];
          char* slot = fslot[b & 1];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            f32x4 v = {c[r * 4], c[r * 4 + 1], c[r * 4 + 2], c[r * 4 + 3]};
            *reinterpret_cast<f32x4*>(slot + er * 128 + (((2 * r + ekhalf) ^ esw) << 4)) = v;
#pragma unroll
            for (int q = 0; q < 4; ++q) c[r * 4 + q] = 0.f;
          }
        };
        if (!grp_y) put(0);
#pragma unroll
        for (int b = 0; b < MI * NI; ++b) {
          if (grp_y) put(b);
          else if (b + 1 < MI * NI) put(b + 1);
          char* slot = fslot[b & 1];
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const int rr = it * 8 + rrow;
            const f32x4 v = *reinterpret_cast<const f32x4*>(slot + rr * 128 + ((rchunk ^ ((rr >> 1) & 7)) << 4));
            global_store16_s(wave_c + ((size_t)((b / NI) * 32 + it * 8) * cld + (b % NI) * 32) * 4, voff, v);
          }
        }
      } else {
      const int mrow = cc.w.m0 + wm * WM + (elane & 31);
      const int ncol = cc.w.n0 + wn * WN + 4 * ekhalf;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] = acc[0][i][j][r * 4 + q];
            const int m = mrow + i * 32, n = ncol + j * 32 + r * 8;
            if (m < cM && n < cN) {
              float* c = reinterpret_cast<float*>(const_cast<char*>(cc.C)) + (size_t)m * cld + n;
              if (accumulate) {
                float old[4];
                load4(c, old);
#pragma unroll
                for (int q = 0; q < 4; ++q) a[q] += old[q];
              }
              store4(c, a);
            }
          }
      }
    } else {
      // 16-bit outputs go through LDS so that global memory sees whole 128-byte lines: the wave works in
      // units of 32 rows x 64 columns (two MFMA blocks), writes a unit into a 4 KiB slot in accumulator
      // order (8 bytes per lane), reads it back row-wise (16 bytes per lane, 8 lanes per row) and stores.
      // The two slots are this wave's own load units in the two panels of the step just finished: nobody
      // reads those panels any more, and the next loads into these units are this wave's own, issued after
      // the epilogue.  LDS serves one wave's accesses in program order.
      static_assert(NI % 2 == 0, "staged epilogue: 64-column units");
      constexpr int NJP = NI / 2, NU = MI * NJP;
      // (the late waves have already refilled their units of the A panel's slot: their two slots are one and
      // the same, so everything below writes a slot only after what it held has been read back, in program
      // order)
      // (SwiGLU, groups one after the other: the late waves take their SIMD partner's units of the B panel's
      // slot, which the partner stopped using a phase ago)
      char* const slot0 = !grp_y ? ring + slot_add(sa, NSLOT - 2) * PANEL + unit0 * 1024
                          : BOTH_EPI ? ring + slot_add(sa, NSLOT - 1) * PANEL + unit0 * 1024
                                     : ring + slot_add(sa, NSLOT - 1) * PANEL + (unit0 - Cfg::NWAVES / 2 * UPW) * 1024;
      char* const slot1 = ring + slot_add(sa, NSLOT - 1) * PANEL + unit0 * 1024;
      const int er = elane & 31, esw = (er >> 1) & 7;
      const int rrow = elane >> 3, rchunk = elane & 7;
      auto acc_pos = [&](char* slot, int jj, int r) -> bf16x4* {  // 4 columns of accumulator group (jj, r)
        return reinterpret_cast<bf16x4*>(slot + er * 128 + (((jj * 4 + r) ^ esw) << 4) + ekhalf * 8);
      };
      auto row_pos = [&](char* slot, int it) -> bf16x8* {  // chunk rchunk of row 8 * it + rrow
        const int rr = it * 8 + rrow;
        return reinterpret_cast<bf16x8*>(slot + rr * 128 + ((rchunk ^ ((rr >> 1) & 7)) << 4));
      };
      auto unit_m = [&](int u) { return cc.w.m0 + wm * WM + (u / NJP) * 32; };
      auto unit_n = [&](int u) { return cc.w.n0 + wn * WN + (u % NJP) * 64; };
      // element offset of this lane's row-wise chunk of unit u, or -1 outside the matrix
      auto row_off = [&](int u, int it) -> long {
        const int m = unit_m(u) + it * 8 + rrow, n = unit_n(u) + rchunk * 8;
        return (m < cM && n < cN) ? (long)m * cld + n : -1;
      };
      // one 32 x 32 block of the unit; the accumulator block is cleared for the next tile on the way
      auto put_block = [&](char* slot, int jj, f32x16& c) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          bf16x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            v[q] = (bf16_t)c[r * 4 + q];
            c[r * 4 + q] = 0.f;
          }
          *acc_pos(slot, jj, r) = v;
        }
      };
      auto put_unit = [&](char* slot, f32x16& c0, f32x16& c1) {
        put_block(slot, 0, c0);
        put_block(slot, 1, c1);
      };
      auto store_unit = [&](char* slot, int u, const char* C) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const bf16x8 v = *row_pos(slot, it);
          const long o = row_off(u, it);
          if (o >= 0) global_store16(reinterpret_cast<bf16_t*>(const_cast<char*>(C)) + o, v);
        }
      };
      // A tile that lies inside the matrix needs no masks: its stores take the tile's address from scalar
      // registers and one per-lane offset that is the same for every store of the tile.
      const bool interior = cc.w.m0 + BM <= cM && cc.w.n0 + BN <= cN;
      const uint32_t voff = (uint32_t)(rrow * cld + rchunk * 8) * 2u;
      const char* const wave_c = cc.C + ((size_t)(cc.w.m0 + wm * WM) * cld + cc.w.n0 + wn * WN) * 2;
      // rows of a staged unit to global memory, for a tile inside the matrix: scalar address of the unit's row
      // group + this lane's fixed offset; no masks, no per-lane 64-bit arithmetic, one basic block
      auto store_unit_interior = [&](char* slot, int u, const char* wave_base) {
        const char* ub = wave_base + ((size_t)(u / NJP) * 32 * cld + (u % NJP) * 64) * 2;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const bf16x8 v = *row_pos(slot, it);
          global_store16_s(ub + (size_t)it * 8 * cld * 2, voff, v);
        }
      };
      const size_t wave_off = ((size_t)(cc.w.m0 + wm * WM) * cld + cc.w.n0 + wn * WN) * 2;
      if constexpr (EPI == EPI_STORE || EPI == EPI_STORE_DUALK) {
        if (interior) {
#pragma unroll
          for (int u = 0; u < NU; ++u) {
            char* slot = (u & 1) ? slot1 : slot0;
            put_unit(slot, acc[0][u / NJP][2 * (u % NJP)], acc[0][u / NJP][2 * (u % NJP) + 1]);
            store_unit_interior(slot, u, wave_c);
          }
        } else {
#pragma unroll
          for (int u = 0; u < NU; ++u) {
            if (unit_m(u) >= cM) continue;
            char* slot = (u & 1) ? slot1 : slot0;
            put_unit(slot, acc[0][u / NJP][2 * (u % NJP)], acc[0][u / NJP][2 * (u % NJP) + 1]);
            store_unit(slot, u, cc.C);
          }
        }
      } else if constexpr (EPI == EPI_SWIGLU) {
        // h = silu(a) b and the saved term p = dh/da go to the slots four columns at a time; q = dh/db
        // takes b's place in the accumulator and follows once the slot of h is free
        // (an inference pass, which saves nothing, takes the copy of the code without the arithmetic of p)
        auto swiglu_unit = [&](int u, auto save_tag) {
          constexpr bool SAVE = decltype(save_tag)::value;
          const int i = u / NJP, j0 = 2 * (u % NJP);
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              bf16x4 hv, pv;
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const float a = acc[0][i][j0 + jj][r * 4 + q4], b = acc[1][i][j0 + jj][r * 4 + q4];
                if constexpr (SAVE) {
                  float h, p, q;
                  swiglu_terms(a, b, sigmoid_fast(a), h, p, q);
                  hv[q4] = (bf16_t)h;
                  pv[q4] = (bf16_t)p;
                  acc[1][i][j0 + jj][r * 4 + q4] = q;
                } else {
                  hv[q4] = (bf16_t)(a * sigmoid_fast(a) * b);
                }
              }
              *acc_pos(slot0, jj, r) = hv;
              if constexpr (SAVE) *acc_pos(slot1, jj, r) = pv;
            }
        };
        auto swiglu_tile = [&](auto save_tag) {
          constexpr bool SAVE = decltype(save_tag)::value;
          if (interior) {
#pragma unroll
            for (int u = 0; u < NU; ++u) {
              const int i = u / NJP, j0 = 2 * (u % NJP);
              swiglu_unit(u, save_tag);
              store_unit_interior(slot0, u, cc.C + wave_off);
              if constexpr (SAVE) {
                store_unit_interior(slot1, u, cc.C2 + wave_off);
                put_unit(slot0, acc[1][i][j0], acc[1][i][j0 + 1]);
                store_unit_interior(slot0, u, cc.C3 + wave_off);
              }
            }
          } else {
#pragma unroll
            for (int u = 0; u < NU; ++u) {
              if (unit_m(u) >= cM) continue;
              const int i = u / NJP, j0 = 2 * (u % NJP);
              swiglu_unit(u, save_tag);
              store_unit(slot0, u, cc.C);
              if constexpr (SAVE) {
                store_unit(slot1, u, cc.C2);
                put_unit(slot0, acc[1][i][j0], acc[1][i][j0 + 1]);
                store_unit(slot0, u, cc.C3);
              }
            }
          }
        };
        if (save_pre) swiglu_tile(std::true_type{});
        else swiglu_tile(std::false_type{});
      } else if constexpr (EPI == EPI_SWIGLU_BWD) {
        {
          // dh goes through LDS as float32, one unit (32 rows x 64 columns, 8 KiB = both slots) at a time:
          // written in accumulator order, read back row-wise.  The saved terms p = dh/da and q = dh/db come
          // from global memory row-wise (whole lines) into registers, one unit ahead: each pair of registers
          // is reloaded for the next unit as soon as it has been multiplied.  da = dh p and db = dh q leave
          // row-wise as well.  The loads are never masked (a load that is skipped would break the counting of
          // the waits, and a conditionally assigned register may be copied before its load has returned):
          // rows and chunks beyond the matrix read the last row / chunk instead; the stores are masked.
          const size_t tile_off = ((size_t)cc.w.m0 * cld + cc.w.n0) * 2;
          const char* const tile_c = cc.C + tile_off;
          const char* const tile_c2 = cc.C2 + tile_off;
          const char* const tile_e1 = cc.E1 + tile_off;
          const char* const tile_e2 = cc.E2 + tile_off;
          const int mrel = wm * WM + rrow, nrel = wn * WN + rchunk * 8;   // this lane's position in the tile (unit 0, row group 0)
          const int mmax = cM - 1 - cc.w.m0, nmax = cN - 8 - cc.w.n0;    // last row / chunk of the matrix, tile-relative
          auto lane_off = [&](int u, int it) -> uint32_t {
            const int m = min(mrel + (u / NJP) * 32 + it * 8, mmax), n = min(nrel + (u % NJP) * 64, nmax);
            return (uint32_t)(m * cld + n) * 2u;
          };
          auto inside = [&](int u, int it) { return mrel + (u / NJP) * 32 + it * 8 <= mmax && nrel + (u % NJP) * 64 <= nmax; };
          auto frow = [&](int rr) -> char* { return (rr < 16 ? slot0 : slot1) + (rr & 15) * 256; };
          bf16x8 pa[4], pb[4];
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const uint32_t o = lane_off(0, it);
            pa[it] = global_load16_s(tile_e1, o);
            pb[it] = global_load16_s(tile_e2, o);
          }
#pragma unroll
          for (int u = 0; u < NU; ++u) {
            const int i = u / NJP, j0 = 2 * (u % NJP);
            // rows 0-15 of the unit are staged in slot 0, rows 16-31 in slot 1: the early waves write both at
            // once, the late waves (one slot) the second half after the first has been read back
            auto stage_half = [&](int half) {
              if ((er >> 4) == half) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                  for (int r = 0; r < 4; ++r) {
                    const f32x16& c = acc[0][i][j0 + jj];
                    const f32x4 v = {c[r * 4], c[r * 4 + 1], c[r * 4 + 2], c[r * 4 + 3]};
                    *reinterpret_cast<f32x4*>(frow(er) + (((jj * 8 + 2 * r + ekhalf) ^ (er & 15)) << 4)) = v;
                  }
              }
            };
            stage_half(0);
            if (!grp_y) stage_half(1);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
              __builtin_amdgcn_sched_barrier(0);  // (keeps the compiler from hoisting the address arithmetic of all rows: registers are short here)
              if (it == 2 && grp_y) {
                stage_half(1);
                __builtin_amdgcn_sched_barrier(0);
              }
              f32x4 dhr[2];
              {
                const int rr = it * 8 + rrow;
#pragma unroll
                for (int h = 0; h < 2; ++h) dhr[h] = *reinterpret_cast<const f32x4*>(frow(rr) + (((2 * rchunk + h) ^ (rr & 15)) << 4));
              }
              // loads issued after this pair: the rest of this unit's, and the next unit's reloaded so far
              if (u + 1 < NU || it == 0) wait_loaded<6>(pa[it], pb[it]);
              else if (it == 1) wait_loaded<4>(pa[it], pb[it]);
              else if (it == 2) wait_loaded<2>(pa[it], pb[it]);
              else wait_loaded<0>(pa[it], pb[it]);
              bf16x8 da, db;
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                const float dh = dhr[q / 4][q % 4];
                da[q] = (bf16_t)(dh * (float)pa[it][q]);
                db[q] = (bf16_t)(dh * (float)pb[it][q]);
              }
              if (u + 1 < NU) {
                const uint32_t o = lane_off(u + 1, it);
                pa[it] = global_load16_s(tile_e1, o);
                pb[it] = global_load16_s(tile_e2, o);
              }
              if (inside(u, it)) {
                const uint32_t o = lane_off(u, it);
                global_store16_s(tile_c, o, da);
                global_store16_s(tile_c2, o, db);
              }
            }
          }
        }
      }
    }
    zero_acc();
    if (BOTH_EPI && grp_y) phase_end();
    cc.w.tile = tile_of_round(first_tile, ++cc.w.round);
    open_c();
  }
  if (!grp_y) phase_end();  // the barrier the late waves still owe
  // drain: nothing may still be writing LDS when the workgroup's allocation is released
  __builtin_amdgcn_s_waitcnt(0x0070);
}

}  // namespace modse_gemm
