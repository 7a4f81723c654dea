// C ABI of libmodse: argument checks, workspace carving and the launch sequence of the MoDSE layer
// (forward: route -> permute -> grouped up-GEMM + SwiGLU -> grouped down-GEMM -> combine; backward: the
// chain rule through the same steps).  Nothing here allocates device memory or synchronises, except the
// opt-in per-stage timing.
#include <algorithm>
#include <cstring>

#include "common.h"

namespace {

struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  }
};

size_t esize_of(modse_dtype dt) { return dt == MODSE_F32 ? 4 : 2; }

modse_status check_desc(const modse_desc* desc, int64_t T) {
  if (!desc || !desc->d_ff) return MODSE_ERR_INVALID_ARG;
  if (T < 0) return MODSE_ERR_INVALID_ARG;
  // (the field is read as an integer: a caller may have put any value there, and loading a value that is none of
  // the enumerators through the enumeration type is undefined)
  static_assert(sizeof(modse_dtype) == sizeof(int32_t), "enumeration stored as a 32-bit integer");
  int32_t dtype_bits;
  std::memcpy(&dtype_bits, &desc->dtype, sizeof dtype_bits);
  if (dtype_bits != (int32_t)MODSE_F32 && dtype_bits != (int32_t)MODSE_BF16) return MODSE_ERR_UNSUPPORTED;
  if (desc->n_experts < 1 || desc->d_model < 1) return MODSE_ERR_INVALID_ARG;
  if (desc->top_k < 1 || desc->top_k > desc->n_experts) return MODSE_ERR_INVALID_ARG;
  if (desc->n_experts > MODSE_MAX_EXPERTS) return MODSE_ERR_UNSUPPORTED;
  if (desc->top_k > 2) return MODSE_ERR_UNSUPPORTED;
  if (desc->d_model % 32 != 0) return MODSE_ERR_INVALID_ARG;
  int64_t fmax = 0;
  for (int e = 0; e < desc->n_experts; ++e) {
    const int32_t f = desc->d_ff[e];
    if (f <= 0 || f % 32 != 0) return MODSE_ERR_INVALID_ARG;
    fmax = std::max<int64_t>(fmax, f);
  }
  // kernels index rows and per-expert matrices with 32-bit element offsets
  const int64_t lim = (int64_t)1 << 31;
  if (T * desc->top_k + 64 * desc->n_experts + 64 >= lim / 64) return MODSE_ERR_UNSUPPORTED;
  if ((T + 64) * std::max<int64_t>(fmax, desc->d_model) >= lim) return MODSE_ERR_UNSUPPORTED;
  if (fmax * desc->d_model >= lim) return MODSE_ERR_UNSUPPORTED;
  return MODSE_OK;
}

LayerDims make_dims(const modse_desc* desc, int64_t T) {
  LayerDims L;
  std::memset(&L, 0, sizeof(L));
  L.d = desc->d_model;
  L.N = desc->n_experts;
  L.k = desc->top_k;
  L.T = (int32_t)T;
  for (int e = 0; e < L.N; ++e) {
    L.f[e] = desc->d_ff[e];
    L.foff[e + 1] = L.foff[e] + L.f[e];
    L.order[e] = e;
  }
  std::stable_sort(L.order, L.order + L.N, [&](int a, int b) { return L.f[a] > L.f[b]; });
  return L;
}

// Upper bound of sum_e n_e * d_ff[e]: every token picks top_k distinct experts, so at worst all tokens
// pick the top_k widest ones.
size_t hidden_elems_max(const LayerDims& L) {
  size_t s = 0;
  for (int j = 0; j < L.k; ++j) s += (size_t)L.f[L.order[j]];
  return s * (size_t)L.T;
}

// scratch of the routing kernels (see RouteBufs)
struct RouteScratch {
  size_t blockhist, near_flag, wpad, total;
};
void carve_route(Carver& c, const LayerDims& L, modse_dtype dt, RouteScratch& r) {
  const size_t nb = ((size_t)L.T + MODSE_ROUTE_TOKENS_PER_BLOCK - 1) / MODSE_ROUTE_TOKENS_PER_BLOCK;
  r.blockhist = c.take(nb * (L.N + 1) * 4);
  r.near_flag = c.take((size_t)L.T * 4);
  r.wpad = c.take(route_wpad_bytes(L, esize_of(dt)));
  r.total = c.off;
}
RouteBufs route_bufs(char* base, const RouteScratch& r) {
  return RouteBufs{reinterpret_cast<int32_t*>(base + r.blockhist), reinterpret_cast<int32_t*>(base + r.near_flag),
                   base + r.wpad};
}

struct FwdLayout {
  RouteScratch route;
  size_t topk_idx, topk_w, counts, offsets, row_of, src_of, near_tie, plan_up, plan_down, Xp, H, O, Opart, total;
};

// Decode-sized batches stream the expert weights once; the down-projection then has too few output tiles
// to occupy the chip (d / 256 per expert) and very long K loops, so its K is cut into chunks that become
// problems of their own.  Returns the chunk length (a multiple of 64), or 0 when K is not split.
constexpr int64_t SPLITK_MAX_TOKENS = MODSE_SKINNY_TOKENS;
int splitk_chunk(const LayerDims& L) {
  if (L.T > SPLITK_MAX_TOKENS) return 0;
  int64_t F = 0;
  for (int e = 0; e < L.N; ++e) F += L.f[e];
  const int64_t ntiles_n = (L.d + 511) / 512;
  // two tiles per CU: fewer, longer chunks mean fewer float32 slabs to write and to add up again (measured at the
  // decode configuration of the benchmark: 1024 tiles 0.187 + 0.016 ms for down-projection + combine, 512 tiles
  // 0.176 + 0.012 ms, 256 tiles 0.261 + 0.009 ms; counts that are no multiple of the CU count lose a round)
  int64_t want = std::max<int64_t>(L.N, 512 / ntiles_n);
  want = std::min<int64_t>(want, MODSE_MAX_PROBLEMS - L.N);          // sum_e ceil(f_e / chunk) <= want + N
  const int64_t chunk = align_up((size_t)((F + want - 1) / want), 64);
  return (int)std::max<int64_t>(chunk, 512);
}
int splitk_max_chunks(const LayerDims& L, int kchunk) {
  int m = 0;
  for (int e = 0; e < L.N; ++e) m = std::max(m, (L.f[e] + kchunk - 1) / kchunk);
  return m;
}

// with_saved: the call is given the buffer that carries activations to the backward pass; the permuted rows,
// the hidden activations and the expert outputs then live there and take no workspace
FwdLayout fwd_layout(const LayerDims& L, modse_dtype dt, bool with_saved) {
  FwdLayout w;
  Carver c;
  const size_t es = esize_of(dt), Tk = (size_t)L.T * L.k;
  carve_route(c, L, dt, w.route);
  w.topk_idx = c.take(Tk * 4);
  w.topk_w = c.take(Tk * 4);
  w.counts = c.take(L.N * 4);
  w.offsets = c.take((L.N + 1) * 4);
  w.row_of = c.take(Tk * 4);
  w.src_of = c.take(Tk * 4);
  w.near_tie = c.take(4);
  w.plan_up = c.take(sizeof(GemmPlan));
  w.plan_down = c.take(sizeof(GemmPlan));
  w.Xp = c.take(with_saved ? 0 : Tk * L.d * es);
  w.H = c.take(with_saved ? 0 : hidden_elems_max(L) * es);
  w.O = c.take(with_saved ? 0 : Tk * L.d * es);
  const int kchunk = with_saved ? 0 : splitk_chunk(L);
  w.Opart = c.take(kchunk ? (size_t)splitk_max_chunks(L, kchunk) * Tk * L.d * 4 : 0);
  w.total = c.off;
  return w;
}

struct SavedLayout {
  size_t dHdA, dHdB, H, O, Xp, total;
};

SavedLayout saved_layout(const LayerDims& L, modse_dtype dt) {
  SavedLayout s;
  Carver c;
  const size_t es = esize_of(dt), h = hidden_elems_max(L) * es;
  s.dHdA = c.take(h);
  s.dHdB = c.take(h);
  s.H = c.take(h);
  s.O = c.take((size_t)L.T * L.k * L.d * es);
  s.Xp = c.take((size_t)L.T * L.k * L.d * es);  // permuted token rows: the weight-gradient GEMMs read them again
  s.total = c.off;
  return s;
}

struct BwdLayout {
  size_t plan[3], dO, dA, dB, dXp, dg, dl, du, dgamma_part, dWg_partial, total;
};

BwdLayout bwd_layout(const LayerDims& L, modse_dtype dt) {
  BwdLayout w;
  Carver c;
  const size_t es = esize_of(dt), Tk = (size_t)L.T * L.k;
  const size_t h = hidden_elems_max(L) * es;
  const size_t nb = ((size_t)L.T + MODSE_ROUTE_TOKENS_PER_BLOCK - 1) / MODSE_ROUTE_TOKENS_PER_BLOCK;
  for (int i = 0; i < 3; ++i) w.plan[i] = c.take(sizeof(GemmPlan));
  w.dO = c.take(Tk * L.d * es);
  w.dA = c.take(h);
  w.dB = c.take(h);
  w.dXp = c.take(Tk * L.d * es);
  w.dg = c.take(Tk * 4);
  w.dl = c.take((size_t)L.T * L.N * 4);
  w.du = c.take((size_t)L.T * L.N * 4);
  w.dgamma_part = c.take((((size_t)L.T + 255) / 256) * 4);
  w.dWg_partial = c.take(nb * L.d * L.N * 4);
  w.total = c.off;
  return w;
}

int64_t tiles_bound(const LayerDims& L, int64_t rows_max, const TileShape& t, bool n_is_f) {
  int64_t s = 0;
  for (int e = 0; e < L.N; ++e) {
    const int64_t nt = ((n_is_f ? L.f[e] : L.d) + t.bn - 1) / t.bn;
    s += ((rows_max + t.bm - 1) / t.bm) * nt;
  }
  return s;
}

// ---------------------------------------------------------------- stage timing
struct StageTimer {
  bool on = false;
  static constexpr int MAXEV = 24;
  hipEvent_t ev[2][MAXEV];
  int stage[2][MAXEV];
  int n[2] = {0, 0};
  bool created = false;
};
StageTimer g_timer;

struct Stamp {
  int which;
  hipStream_t s;
  bool on;
  Stamp(int w, hipStream_t st) : which(w), s(st), on(g_timer.on) {
    if (on) {
      g_timer.n[which] = 0;
      mark(-1);
    }
  }
  void mark(int stage) {
    if (!on) return;
    int& n = g_timer.n[which];
    if (n >= StageTimer::MAXEV) return;
    g_timer.stage[which][n] = stage;
    (void)hipEventRecord(g_timer.ev[which][n], s);
    ++n;
  }
};

#define HIP_TRY(expr)                            \
  do {                                           \
    if ((expr) != hipSuccess) return MODSE_ERR_HIP; \
  } while (0)

RoutingPtrs routing_from(const modse_routing* r, char* ws, const FwdLayout& w) {
  RoutingPtrs R;
  if (r) {
    R = {r->topk_idx, r->topk_w, r->counts, r->offsets, r->row_of, r->src_of, r->near_tie_count};
  } else {
    R = {reinterpret_cast<int32_t*>(ws + w.topk_idx), reinterpret_cast<float*>(ws + w.topk_w),
         reinterpret_cast<int32_t*>(ws + w.counts),   reinterpret_cast<int32_t*>(ws + w.offsets),
         reinterpret_cast<int32_t*>(ws + w.row_of),   reinterpret_cast<int32_t*>(ws + w.src_of),
         reinterpret_cast<int32_t*>(ws + w.near_tie)};
  }
  return R;
}

bool routing_complete(const modse_routing* r) {
  return r && r->topk_idx && r->topk_w && r->counts && r->offsets && r->row_of && r->src_of && r->near_tie_count;
}

// A gate extension is usable when every pointer its switched-on parts need is there.
bool ext_complete(const modse_gate_ext* e) {
  if (!e) return true;
  if (e->W_noise && (!e->gamma || !e->noise_pre || !(e->eps >= 0.f))) return false;
  if (e->probs && (!e->aux_f || !e->aux_P || !e->aux_loss)) return false;
  return true;
}

GateExtPtrs ext_ptrs(const modse_gate_ext* e) {
  return GateExtPtrs{e->W_noise, e->gamma, e->eps, e->noise_pre, e->aux_alpha, e->probs, e->aux_f, e->aux_P, e->aux_loss};
}

}  // namespace

extern "C" {

const char* modse_status_string(modse_status s) {
  int32_t code;  // (read as an integer: a C caller may pass any value)
  static_assert(sizeof(modse_status) == sizeof(int32_t), "enumeration stored as a 32-bit integer");
  std::memcpy(&code, &s, sizeof code);
  switch (code) {
    case MODSE_OK: return "ok";
    case MODSE_ERR_INVALID_ARG: return "invalid argument";
    case MODSE_ERR_UNSUPPORTED: return "unsupported configuration";
    case MODSE_ERR_WORKSPACE: return "workspace too small";
    case MODSE_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

modse_status modse_workspace_size(const modse_desc* desc, int64_t T, int need_bwd, size_t* bytes) {
  if (!bytes) return MODSE_ERR_INVALID_ARG;
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  const LayerDims L = make_dims(desc, T);
  if (need_bwd != MODSE_WS_FWD && need_bwd != MODSE_WS_BWD && need_bwd != MODSE_WS_FWD_SAVED) return MODSE_ERR_INVALID_ARG;
  *bytes = need_bwd == MODSE_WS_BWD ? bwd_layout(L, desc->dtype).total
                                    : fwd_layout(L, desc->dtype, need_bwd == MODSE_WS_FWD_SAVED).total;
  return MODSE_OK;
}

modse_status modse_saved_size(const modse_desc* desc, int64_t T, size_t* bytes) {
  if (!bytes) return MODSE_ERR_INVALID_ARG;
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  *bytes = saved_layout(make_dims(desc, T), desc->dtype).total;
  return MODSE_OK;
}

modse_status modse_route(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                         const float* logit_bias, const modse_routing* out, void* ws, size_t ws_bytes,
                         void* hip_stream) {
  return modse_route_ext(desc, T, x, W_gate, logit_bias, nullptr, out, ws, ws_bytes, hip_stream);
}

modse_status modse_route_ext(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                             const float* logit_bias, const modse_gate_ext* ext, const modse_routing* out, void* ws,
                             size_t ws_bytes, void* hip_stream) {
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  if (T == 0) return MODSE_OK;
  if (!x || !W_gate || !ws || !routing_complete(out) || !ext_complete(ext)) return MODSE_ERR_INVALID_ARG;
  GateExtPtrs G;
  if (ext) G = ext_ptrs(ext);
  const LayerDims L = make_dims(desc, T);
  RouteScratch w;  // the routing scratch is the head of the forward workspace; this call needs no more of it
  Carver c;
  carve_route(c, L, desc->dtype, w);
  if (ws_bytes < w.total) return MODSE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const RoutingPtrs R = {out->topk_idx, out->topk_w, out->counts, out->offsets, out->row_of, out->src_of, out->near_tie_count};
  HIP_TRY(launch_route(L, desc->dtype, x, W_gate, logit_bias, R, route_bufs(static_cast<char*>(ws), w), nullptr,
                       ext ? &G : nullptr, s));
  return MODSE_OK;
}

// ---------------------------------------------------------------- modse_route without a workspace
// For callers that cannot hand over a workspace they allocated (HIP graph capture, serving loops that must
// not allocate): the router's scratch -- per-block histograms and near-tie flags -- lives in a device array
// of this library.  Every GPU holds its own copy at its own address; the name below is only the host-side
// handle of the symbol, the address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char g_route_scratch[MODSE_ROUTE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_route_scratch_ptr[kMaxDevices] = {};

}  // namespace

modse_status modse_route_static(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                                const float* logit_bias, const modse_routing* out, void* hip_stream) {
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  if (T == 0) return MODSE_OK;
  if (!x || !W_gate || !routing_complete(out)) return MODSE_ERR_INVALID_ARG;
  const LayerDims L = make_dims(desc, T);
  RouteScratch w;
  Carver c;
  carve_route(c, L, desc->dtype, w);
  if (w.total > MODSE_ROUTE_STATIC_SCRATCH_BYTES) return MODSE_ERR_WORKSPACE;  // more tokens than the array serves
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MODSE_ERR_HIP;
  if (!g_route_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_route_scratch)) != hipSuccess || !p) return MODSE_ERR_HIP;
    g_route_scratch_ptr[dev] = p;
  }
  char* scratch = static_cast<char*>(g_route_scratch_ptr[dev]);
  const RoutingPtrs R = {out->topk_idx, out->topk_w, out->counts, out->offsets, out->row_of, out->src_of, out->near_tie_count};
  // every word of the scratch that a kernel reads has been written by an earlier kernel of this call
  HIP_TRY(launch_route(L, desc->dtype, x, W_gate, logit_bias, R, route_bufs(scratch, w), nullptr, nullptr,
                       static_cast<hipStream_t>(hip_stream)));
  return MODSE_OK;
}

modse_status modse_routing_stats(const modse_desc* desc, int64_t T, const modse_routing* routing,
                                 int32_t* slot_counts, float* summary, void* hip_stream) {
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  if (!routing || !routing->topk_idx || !slot_counts || !summary) return MODSE_ERR_INVALID_ARG;
  const LayerDims L = make_dims(desc, T);
  HIP_TRY(launch_routing_stats(L, routing->topk_idx, slot_counts, summary, static_cast<hipStream_t>(hip_stream)));
  return MODSE_OK;
}

modse_status modse_layer_fwd(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                             const float* logit_bias, const void* W1, const void* W3, const void* W2, void* y,
                             const modse_routing* routing_out, void* saved, void* ws, size_t ws_bytes,
                             void* hip_stream) {
  return modse_layer_fwd_ext(desc, T, x, W_gate, logit_bias, nullptr, W1, W3, W2, y, routing_out, saved, ws, ws_bytes,
                             hip_stream);
}

modse_status modse_layer_fwd_ext(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                                 const float* logit_bias, const modse_gate_ext* ext, const void* W1, const void* W3,
                                 const void* W2, void* y, const modse_routing* routing_out, void* saved, void* ws,
                                 size_t ws_bytes, void* hip_stream) {
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  if (T == 0) return MODSE_OK;
  if (!x || !W_gate || !W1 || !W3 || !W2 || !y || !ws || !ext_complete(ext)) return MODSE_ERR_INVALID_ARG;
  GateExtPtrs G;
  if (ext) G = ext_ptrs(ext);
  if (routing_out && !routing_complete(routing_out)) return MODSE_ERR_INVALID_ARG;
  const modse_dtype dt = desc->dtype;
  const LayerDims L = make_dims(desc, T);
  const FwdLayout w = fwd_layout(L, dt, saved != nullptr);
  if (ws_bytes < w.total) return MODSE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* wsb = static_cast<char*>(ws);
  const RoutingPtrs R = routing_from(routing_out, wsb, w);
  const RouteBufs RB = route_bufs(wsb, w.route);
  Stamp stamp(0, s);

  // with a backward pass to follow, the permuted rows go straight into the saved buffer
  void* Xp = saved ? static_cast<char*>(saved) + saved_layout(L, dt).Xp : wsb + w.Xp;
  HIP_TRY(launch_router(L, dt, x, W_gate, logit_bias, R, RB, ext ? &G : nullptr, s));
  stamp.mark(MODSE_STAGE_ROUTE);

  FwdPlanArgs pa;
  std::memset(&pa, 0, sizeof(pa));
  pa.Xp = Xp; pa.W1 = W1; pa.W3 = W3; pa.W2 = W2;
  if (saved) {
    const SavedLayout sl = saved_layout(L, dt);
    char* sb = static_cast<char*>(saved);
    pa.dHdA = sb + sl.dHdA; pa.dHdB = sb + sl.dHdB; pa.H = sb + sl.H; pa.O = sb + sl.O;
  } else {
    pa.H = wsb + w.H; pa.O = wsb + w.O;
  }
  pa.up = reinterpret_cast<GemmPlan*>(wsb + w.plan_up);
  pa.down = reinterpret_cast<GemmPlan*>(wsb + w.plan_down);
  pa.up_tile = gemm_tile_shape(dt, EPI_SWIGLU, T);
  pa.down_tile = gemm_tile_shape(dt, EPI_STORE, T);
  // inference on a decode-sized batch: split-K down-projection (the backward pass wants O itself)
  const int kchunk = saved ? 0 : splitk_chunk(L);
  pa.kchunk = kchunk;
  pa.Opart = reinterpret_cast<float*>(wsb + w.Opart);
  // histogram, scan (which also writes the tile plans), stable scatter: one launch for all of it on decode-sized
  // batches
  HIP_TRY(launch_permute(L, dt, x, R, RB, Xp, ext ? &G : nullptr, &pa, s));
  stamp.mark(MODSE_STAGE_PERMUTE);

  const int skinny = T <= MODSE_SKINNY_TOKENS;
  HIP_TRY(launch_grouped_gemm(dt, EPI_SWIGLU, pa.up, 0, saved != nullptr, tiles_bound(L, T, pa.up_tile, true), s, -1,
                              skinny));
  stamp.mark(MODSE_STAGE_UP);
  if (kchunk) {
    int64_t nprob = 0;
    for (int e = 0; e < L.N; ++e) nprob += (L.f[e] + kchunk - 1) / kchunk;
    const int64_t bound = nprob * ((T + pa.down_tile.bm - 1) / pa.down_tile.bm) * ((L.d + pa.down_tile.bn - 1) / pa.down_tile.bn);
    HIP_TRY(launch_grouped_gemm(dt, EPI_STORE_F32, pa.down, 0, 0, bound, s, LAYOUT_TN, skinny));
    stamp.mark(MODSE_STAGE_DOWN);
    HIP_TRY(launch_combine_split(L, dt, pa.Opart, kchunk, R, y, s));
    stamp.mark(MODSE_STAGE_COMBINE);
    return MODSE_OK;
  }
  HIP_TRY(launch_grouped_gemm(dt, EPI_STORE, pa.down, 0, 0, tiles_bound(L, T, pa.down_tile, false), s, -1, skinny));
  stamp.mark(MODSE_STAGE_DOWN);
  HIP_TRY(launch_combine(L, dt, pa.O, R, y, s));
  stamp.mark(MODSE_STAGE_COMBINE);
  return MODSE_OK;
}

modse_status modse_layer_bwd(const modse_desc* desc, int64_t T, const void* x, const void* W_gate, const void* W1,
                             const void* W3, const void* W2, const modse_routing* routing, const void* saved,
                             const void* dY, void* dX, float* dW_gate, float* dW1, float* dW3, float* dW2,
                             int accumulate, void* ws, size_t ws_bytes, void* hip_stream) {
  return modse_layer_bwd_ext(desc, T, x, W_gate, nullptr, 0.f, W1, W3, W2, routing, saved, dY, dX, dW_gate, nullptr,
                             nullptr, dW1, dW3, dW2, accumulate, ws, ws_bytes, hip_stream);
}

modse_status modse_layer_bwd_ext(const modse_desc* desc, int64_t T, const void* x, const void* W_gate,
                                 const modse_gate_ext* ext, float aux_grad, const void* W1, const void* W3,
                                 const void* W2, const modse_routing* routing, const void* saved, const void* dY,
                                 void* dX, float* dW_gate, float* dW_noise, float* dgamma, float* dW1, float* dW3,
                                 float* dW2, int accumulate, void* ws, size_t ws_bytes, void* hip_stream) {
  const modse_status st = check_desc(desc, T);
  if (st != MODSE_OK) return st;
  if (T == 0) return MODSE_OK;
  if (!x || !W_gate || !W1 || !W3 || !W2 || !saved || !dY || !dX || !dW_gate || !dW1 || !dW3 || !dW2 || !ws)
    return MODSE_ERR_INVALID_ARG;
  if (!ext_complete(ext) || (ext && ext->W_noise && (!dW_noise || !dgamma))) return MODSE_ERR_INVALID_ARG;
  GateExtPtrs G;
  if (ext) G = ext_ptrs(ext);
  if (!routing_complete(routing)) return MODSE_ERR_INVALID_ARG;
  const modse_dtype dt = desc->dtype;
  const LayerDims L = make_dims(desc, T);
  const BwdLayout w = bwd_layout(L, dt);
  if (ws_bytes < w.total) return MODSE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* wsb = static_cast<char*>(ws);
  const SavedLayout sl = saved_layout(L, dt);
  const char* sb = static_cast<const char*>(saved);
  const RoutingPtrs R = {routing->topk_idx, routing->topk_w, routing->counts, routing->offsets,
                         routing->row_of,   routing->src_of, routing->near_tie_count};
  Stamp stamp(1, s);

  const void* Xp = sb + sl.Xp;
  void* dO = wsb + w.dO;
  float* dg = reinterpret_cast<float*>(wsb + w.dg);
  HIP_TRY(launch_bwd_prep(L, dt, dY, sb + sl.O, R, dO, dg, s));
  BwdPlanArgs pa;
  std::memset(&pa, 0, sizeof(pa));
  pa.Xp = Xp; pa.dO = dO; pa.H = sb + sl.H; pa.dHdA = sb + sl.dHdA; pa.dHdB = sb + sl.dHdB;
  pa.W1 = W1; pa.W3 = W3; pa.W2 = W2;
  pa.dA = wsb + w.dA; pa.dB = wsb + w.dB; pa.dXp = wsb + w.dXp;
  pa.dW1 = dW1; pa.dW3 = dW3; pa.dW2 = dW2;
  pa.dh = reinterpret_cast<GemmPlan*>(wsb + w.plan[0]);
  pa.dx = reinterpret_cast<GemmPlan*>(wsb + w.plan[1]);
  pa.wg = reinterpret_cast<GemmPlan*>(wsb + w.plan[2]);
  pa.dh_tile = gemm_tile_shape(dt, EPI_SWIGLU_BWD, T);
  pa.dx_tile = gemm_tile_shape(dt, EPI_STORE_DUALK, T);
  pa.wg_tile = gemm_tile_shape(dt, EPI_STORE_F32, T);
  HIP_TRY(launch_plan_bwd(L, dt, R.counts, R.offsets, pa, s));
  stamp.mark(MODSE_STAGE_BWD_PREP);

  HIP_TRY(launch_grouped_gemm(dt, EPI_SWIGLU_BWD, pa.dh, 0, 0, tiles_bound(L, T, pa.dh_tile, true), s));
  HIP_TRY(launch_grouped_gemm(dt, EPI_STORE_DUALK, pa.dx, 0, 0, tiles_bound(L, T, pa.dx_tile, false), s));
  stamp.mark(MODSE_STAGE_BWD_DGRAD);

  int64_t fmax = L.f[L.order[0]];
  const int64_t wg13 = tiles_bound(L, fmax, pa.wg_tile, false);
  const int64_t wg2 = tiles_bound(L, L.d, pa.wg_tile, true);
  HIP_TRY(launch_grouped_gemm(dt, EPI_STORE_F32, pa.wg, accumulate, 0, 2 * wg13 + wg2, s));
  stamp.mark(MODSE_STAGE_BWD_WGRAD);

  const BwdRouterBufs rb = {reinterpret_cast<float*>(wsb + w.dl), reinterpret_cast<float*>(wsb + w.du),
                            reinterpret_cast<float*>(wsb + w.dgamma_part),
                            reinterpret_cast<float*>(wsb + w.dWg_partial)};
  HIP_TRY(launch_bwd_router(L, dt, x, W_gate, pa.dXp, dg, R, ext ? &G : nullptr, aux_grad, rb, dX, dW_gate, dW_noise,
                            dgamma, accumulate, s));
  stamp.mark(MODSE_STAGE_BWD_ROUTER);
  return MODSE_OK;
}

modse_status modse_stage_timing_enable(int on) {
  if (on && !g_timer.created) {
    for (int w = 0; w < 2; ++w)
      for (int i = 0; i < StageTimer::MAXEV; ++i)
        if (hipEventCreate(&g_timer.ev[w][i]) != hipSuccess) return MODSE_ERR_HIP;
    g_timer.created = true;
  }
  g_timer.on = on != 0;
  g_timer.n[0] = g_timer.n[1] = 0;
  return MODSE_OK;
}

modse_status modse_stage_times(float* ms) {
  if (!ms) return MODSE_ERR_INVALID_ARG;
  for (int i = 0; i < MODSE_N_STAGES; ++i) ms[i] = 0.f;
  if (!g_timer.created) return MODSE_OK;
  for (int w = 0; w < 2; ++w) {
    const int n = g_timer.n[w];
    if (n < 2) continue;
    if (hipEventSynchronize(g_timer.ev[w][n - 1]) != hipSuccess) return MODSE_ERR_HIP;
    for (int i = 1; i < n; ++i) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, g_timer.ev[w][i - 1], g_timer.ev[w][i]) != hipSuccess) return MODSE_ERR_HIP;
      const int st = g_timer.stage[w][i];
      if (st >= 0 && st < MODSE_N_STAGES) ms[st] += t;
    }
  }
  return MODSE_OK;
}

}  // extern "C"
