// C ABI of libchunkft: argument validation and dispatch to the gfx950 kernels.
// Nothing here computes; every step of the path runs in kernels.hip.

#include "chunkft.h"

#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "internal.h"

using namespace chunkft;

namespace {

constexpr int64_t kMaxI64 = std::numeric_limits<int64_t>::max();

struct Checked {
  int status;
  WgradProblem p;
  bool mfma;
};

// Validates a layer + range and fills the problem (including the token split).
Checked check_layer(const chunkft_layer* L, int64_t begin, int64_t end) {
  Checked c{};
  c.status = CHUNKFT_ERR_INVALID_ARG;
  if (!L) return c;
  if (L->kind < CHUNKFT_LINEAR || L->kind > CHUNKFT_LAYERNORM) { c.status = CHUNKFT_ERR_DTYPE; return c; }
  const bool one_d = L->kind == CHUNKFT_VECTOR || L->kind == CHUNKFT_RMSNORM || L->kind == CHUNKFT_LAYERNORM;
  const bool norm = L->kind == CHUNKFT_RMSNORM || L->kind == CHUNKFT_LAYERNORM;
  const bool embed = L->kind == CHUNKFT_EMBEDDING;
  if (L->dtype != CHUNKFT_F32 && L->dtype != CHUNKFT_BF16) { c.status = CHUNKFT_ERR_DTYPE; return c; }
  if (!L->X || !L->dY) return c;
  if (L->out <= 0 || L->in <= 0 || L->T <= 0) return c;
  if (L->T > (int64_t(1) << 30)) return c;          // the kernels count the tokens of a slab in 32 bits
  if (L->reserved != 0) return c;
  if (L->split_k < 0 || L->split_k > 64) return c;
  if (one_d && L->out != 1) return c;
  if (L->kind != CHUNKFT_LINEAR && L->split_k > 1) return c;
  if (norm && !(L->norm_eps >= 0.0 && std::isfinite(L->norm_eps))) return c;
  if (embed && L->T > kMaxEmbeddingTokens) return c;
  if (!embed && L->ldx < L->in) return c;
  if (L->lddy < (L->kind == CHUNKFT_LINEAR ? L->out : L->in)) return c;
  if (L->in > kMaxI64 / L->out) { c.status = CHUNKFT_ERR_OVERFLOW; return c; }
  // element offsets t * ld + column must stay inside int64
  if ((!embed && L->ldx > kMaxI64 / L->T) || L->lddy > kMaxI64 / L->T) { c.status = CHUNKFT_ERR_OVERFLOW; return c; }
  const int64_t numel = L->out * L->in;
  if (begin < 0 || begin >= end || end > numel) { c.status = CHUNKFT_ERR_RANGE; return c; }
  const uintptr_t esz = L->dtype == CHUNKFT_F32 ? 4 : 2;
  if ((reinterpret_cast<uintptr_t>(L->X) % (embed ? 8 : esz)) || (reinterpret_cast<uintptr_t>(L->dY) % esz)) return c;

  WgradProblem& p = c.p;
  p.X = L->X;
  p.dY = L->dY;
  p.ldx = L->ldx;
  p.lddy = L->lddy;
  p.out = L->out;
  p.in = L->in;
  p.T = L->T;
  p.begin = begin;
  p.end = end;
  c.mfma = L->kind == CHUNKFT_LINEAR && L->dtype == CHUNKFT_BF16 && mfma_path_ok(p);
  const Split sp = pick_split(L->kind, L->dtype, L->out, L->in, L->T, begin, end, L->split_k, c.mfma,
                              device_compute_units());
  p.S = sp.S;
  p.kslab = sp.kslab;
  if (p.S > 1 && (end - begin) > kMaxI64 / 4 / p.S - 64) { c.status = CHUNKFT_ERR_OVERFLOW; return c; }
  c.status = CHUNKFT_OK;
  return c;
}

int check_hparams(const chunkft_adamw_hparams* hp, AdamWConsts* out) {
  if (!hp) return CHUNKFT_ERR_INVALID_ARG;
  if (hp->step < 1) return CHUNKFT_ERR_INVALID_ARG;
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0) || !(hp->beta2 >= 0.0 && hp->beta2 < 1.0)) return CHUNKFT_ERR_INVALID_ARG;
  if (!(hp->lr >= 0.0) || !(hp->eps >= 0.0) || !(hp->weight_decay >= 0.0)) return CHUNKFT_ERR_INVALID_ARG;
  if (!std::isfinite(hp->lr) || !std::isfinite(hp->eps) || !std::isfinite(hp->weight_decay)) return CHUNKFT_ERR_INVALID_ARG;
  const double n = static_cast<double>(hp->step);
  out->beta1 = static_cast<float>(hp->beta1);
  out->one_minus_beta1 = static_cast<float>(1.0 - hp->beta1);
  out->beta2 = static_cast<float>(hp->beta2);
  out->one_minus_beta2 = static_cast<float>(1.0 - hp->beta2);
  out->inv_bias1 = static_cast<float>(1.0 / (1.0 - std::pow(hp->beta1, n)));
  out->inv_bias2 = static_cast<float>(1.0 / (1.0 - std::pow(hp->beta2, n)));
  out->lr = static_cast<float>(hp->lr);
  out->eps = static_cast<float>(hp->eps);
  out->weight_decay = static_cast<float>(hp->weight_decay);
  return CHUNKFT_OK;
}

// Elements from one slab's partial sums to the next: the chunk length rounded up to a 128-byte line.
int64_t slab_pitch(const WgradProblem& p) { return (p.end - p.begin + 31) / 32 * 32; }

size_t workspace_need(const chunkft_layer* L, const WgradProblem& p) {
  if (L->kind == CHUNKFT_RMSNORM || L->kind == CHUNKFT_LAYERNORM) return static_cast<size_t>(p.T) * 8u;
  if (p.S <= 1) return 0;
  return (static_cast<size_t>(p.S) * static_cast<size_t>(slab_pitch(p)) + 32u) * 4u;
}

// Where the slab partials start inside the workspace: at the 128-byte phase of the array the sum
// goes to (g, or master in the fused call), so that the reduction reads and writes whole lines.
void place_partials(Sinks& s, const WgradProblem& p, void* ws, const float* dst) {
  const uintptr_t lead = (reinterpret_cast<uintptr_t>(dst) / 4u - reinterpret_cast<uintptr_t>(ws) / 4u) & 31u;
  s.ws = static_cast<float*>(ws) + lead;
  s.ws_pitch = slab_pitch(p);
}

int check_workspace(const chunkft_layer* L, const WgradProblem& p, void* ws, size_t ws_bytes) {
  const size_t need = workspace_need(L, p);
  if (need == 0) return CHUNKFT_OK;
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15u)) return CHUNKFT_ERR_WORKSPACE;
  return CHUNKFT_OK;
}

int run_wgrad(const chunkft_layer* L, const Checked& c, int mode, const Sinks& s, void* stream) {
  int e;
  if (L->kind == CHUNKFT_VECTOR) e = launch_colsum(c.p, L->dtype, mode, s, stream);
  else if (L->kind == CHUNKFT_EMBEDDING) e = launch_embed_wgrad(c.p, L->dtype, mode, s, stream);
  else if (L->kind == CHUNKFT_RMSNORM || L->kind == CHUNKFT_LAYERNORM)
    e = launch_norm_wgrad(c.p, L->dtype, L->kind == CHUNKFT_LAYERNORM, static_cast<float>(L->norm_eps), s.ws,
                          mode, s, stream);
  else if (c.mfma) e = launch_wgrad_bf16_mfma(c.p, mode, s, stream);
  else e = launch_wgrad_simt(c.p, L->dtype, mode, s, stream);
  return e == 0 ? CHUNKFT_OK : CHUNKFT_ERR_HIP;
}

}  // namespace

extern "C" int chunkft_split_k(const chunkft_layer* L, int64_t begin, int64_t end) {
  const Checked c = check_layer(L, begin, end);
  return c.status != CHUNKFT_OK ? c.status : c.p.S;
}

extern "C" size_t chunkft_workspace_bytes(const chunkft_layer* L, int64_t begin, int64_t end) {
  const Checked c = check_layer(L, begin, end);
  if (c.status != CHUNKFT_OK) return 0;
  return workspace_need(L, c.p);
}

extern "C" int chunkft_chunk_wgrad(const chunkft_layer* L, int64_t begin, int64_t end, float* g,
                                   int accumulate, void* ws, size_t ws_bytes, void* stream) {
  const Checked c = check_layer(L, begin, end);
  if (c.status != CHUNKFT_OK) return c.status;
  if (!g || (reinterpret_cast<uintptr_t>(g) & 3u)) return CHUNKFT_ERR_INVALID_ARG;
  if (accumulate != 0 && accumulate != 1) return CHUNKFT_ERR_INVALID_ARG;
  const int wsr = check_workspace(L, c.p, ws, ws_bytes);
  if (wsr != CHUNKFT_OK) return wsr;
  Sinks s{};
  s.g = g;
  s.ws = static_cast<float*>(ws);
  if (c.p.S > 1) place_partials(s, c.p, ws, g);
  const int final_mode = accumulate ? EMIT_ACCUM : EMIT_STORE;
  if (c.p.S <= 1) return run_wgrad(L, c, final_mode, s, stream);
  const int r = run_wgrad(L, c, EMIT_PARTIAL, s, stream);
  if (r != CHUNKFT_OK) return r;
  return launch_reduce(s.ws, c.p.S, end - begin, final_mode, s, nullptr, stream) == 0 ? CHUNKFT_OK
                                                                                     : CHUNKFT_ERR_HIP;
}

extern "C" int chunkft_adamw_chunk(const float* g, float* master, float* m, float* v, void* W_at_begin,
                                   int32_t w_dtype, int64_t n, const chunkft_adamw_hparams* hp,
                                   void* stream) {
  if (!g || !master || !m || !v) return CHUNKFT_ERR_INVALID_ARG;
  if (n <= 0) return CHUNKFT_ERR_INVALID_ARG;
  if (n > kMaxI64 / 4) return CHUNKFT_ERR_OVERFLOW;
  if (w_dtype != CHUNKFT_F32 && w_dtype != CHUNKFT_BF16) return CHUNKFT_ERR_DTYPE;
  const uintptr_t al = reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(master) |
                       reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(v);
  if (al & 3u) return CHUNKFT_ERR_INVALID_ARG;
  if (W_at_begin && (reinterpret_cast<uintptr_t>(W_at_begin) & (w_dtype == CHUNKFT_F32 ? 3u : 1u)))
    return CHUNKFT_ERR_INVALID_ARG;
  Sinks s{};
  const int hr = check_hparams(hp, &s.c);
  if (hr != CHUNKFT_OK) return hr;
  s.master = master;
  s.m = m;
  s.v = v;
  s.w_kind = !W_at_begin ? W_NONE : (w_dtype == CHUNKFT_BF16 ? W_BF16 : W_F32);
  return launch_adamw(g, n, s, W_at_begin, stream) == 0 ? CHUNKFT_OK : CHUNKFT_ERR_HIP;
}

namespace {

// Pointer checks of the fused calls (after the layer and the range were accepted).
int check_fused_pointers(const chunkft_layer* L, const void* W, const float* master, const float* m, const float* v) {
  if (!master || !m || !v) return CHUNKFT_ERR_INVALID_ARG;
  const uintptr_t al = reinterpret_cast<uintptr_t>(master) | reinterpret_cast<uintptr_t>(m) |
                       reinterpret_cast<uintptr_t>(v);
  if (al & 3u) return CHUNKFT_ERR_INVALID_ARG;
  if (W && (reinterpret_cast<uintptr_t>(W) & (L->dtype == CHUNKFT_F32 ? 3u : 1u))) return CHUNKFT_ERR_INVALID_ARG;
  return CHUNKFT_OK;
}

Sinks fused_sinks(const chunkft_layer* L, void* W, float* master, float* m, float* v, const AdamWConsts& consts) {
  Sinks s{};
  s.c = consts;
  s.master = master;
  s.m = m;
  s.v = v;
  s.W = W;
  s.w_kind = !W ? W_NONE : (L->dtype == CHUNKFT_BF16 ? W_BF16 : W_F32);
  return s;
}

// One validated fused call: the kernels of a segment by itself.
int run_fused(const chunkft_layer* L, const Checked& c, Sinks s, void* ws, void* stream) {
  s.ws = static_cast<float*>(ws);
  if (c.p.S > 1) place_partials(s, c.p, ws, s.master);
  if (c.p.S <= 1) return run_wgrad(L, c, EMIT_ADAMW, s, stream);
  const int r = run_wgrad(L, c, EMIT_PARTIAL, s, stream);
  if (r != CHUNKFT_OK) return r;
  void* w_at = nullptr;
  if (s.W) w_at = static_cast<char*>(s.W) + static_cast<size_t>(c.p.begin) * (L->dtype == CHUNKFT_BF16 ? 2u : 4u);
  return launch_reduce(s.ws, c.p.S, c.p.end - c.p.begin, EMIT_ADAMW, s, w_at, stream) == 0 ? CHUNKFT_OK
                                                                                        : CHUNKFT_ERR_HIP;
}

}  // namespace

extern "C" int chunkft_wgrad_adamw_fused(const chunkft_layer* L, int64_t begin, int64_t end, void* W,
                                         float* master, float* m, float* v,
                                         const chunkft_adamw_hparams* hp, void* ws, size_t ws_bytes,
                                         void* stream) {
  const Checked c = check_layer(L, begin, end);
  if (c.status != CHUNKFT_OK) return c.status;
  const int pr = check_fused_pointers(L, W, master, m, v);
  if (pr != CHUNKFT_OK) return pr;
  AdamWConsts consts;
  const int hr = check_hparams(hp, &consts);
  if (hr != CHUNKFT_OK) return hr;
  const int wsr = check_workspace(L, c.p, ws, ws_bytes);
  if (wsr != CHUNKFT_OK) return wsr;
  return run_fused(L, c, fused_sinks(L, W, master, m, v, consts), ws, stream);
}

namespace {

constexpr int32_t kMaxGroupSegments = 4096;

struct GroupPlan {
  int status = CHUNKFT_OK;
  std::vector<Checked> checked;       // per segment
  std::vector<char> grouped;          // 1: goes into the one-launch kernel
  size_t ws_need = 0;                 // the largest need of a segment that runs by itself
  bool large_tile = false;
};

// Validates every segment and decides which ones the one-launch kernel takes.  Matrix segments
// whose split_k is 0 take one token slab when the group as a whole has the tiles to fill the
// device (more than a quarter of its compute units, the rule of the single call, applied to the
// sum); a segment the kernel cannot take (fp32, a forced split, a shape off the MFMA path, a body
// of a few rows, the other kinds) runs by itself, exactly as chunkft_wgrad_adamw_fused would.
GroupPlan plan_group(const chunkft_group_segment* segs, int32_t n) {
  GroupPlan g;
  g.checked.resize(static_cast<size_t>(n));
  g.grouped.assign(static_cast<size_t>(n), 0);
  const int cus = device_compute_units();
  int64_t tiles = 0;
  for (int32_t i = 0; i < n; ++i) {
    const chunkft_group_segment& sg = segs[i];
    Checked& c = g.checked[static_cast<size_t>(i)];
    c = check_layer(&sg.layer, sg.begin, sg.end);
    if (c.status != CHUNKFT_OK) { g.status = c.status; return g; }
    const int pr = check_fused_pointers(&sg.layer, sg.W, sg.master, sg.m, sg.v);
    if (pr != CHUNKFT_OK) { g.status = pr; return g; }
    if (c.mfma && sg.layer.split_k == 0) {
      const RowSplit rs = split_rows(c.p);
      const int64_t rows = rs.rb1 > rs.rb0 ? rs.rb1 - rs.rb0 : 0;
      const int64_t t = ((rows + kMainTileM - 1) / kMainTileM) * ((c.p.in + kMainTileN - 1) / kMainTileN);
      tiles = tiles > (int64_t(1) << 40) ? tiles : tiles + t;
    }
  }
  const bool full = tiles > cus / 4;
  bool any = false, all_large = true;
  for (int32_t i = 0; i < n; ++i) {
    const chunkft_group_segment& sg = segs[i];
    Checked& c = g.checked[static_cast<size_t>(i)];
    const bool vec = sg.layer.kind == CHUNKFT_VECTOR && sg.layer.dtype == CHUNKFT_BF16;
    bool take = vec;
    if (c.mfma && (sg.layer.split_k == 1 || (sg.layer.split_k == 0 && full))) {
      c.p.S = 1;
      c.p.kslab = (c.p.T + kMainTileK - 1) / kMainTileK * kMainTileK;
      take = group_takes_segment(c.p, false);
      if (!take) {                                     // back to what the single call would do
        const Split sp = pick_split(sg.layer.kind, sg.layer.dtype, sg.layer.out, sg.layer.in, sg.layer.T, sg.begin,
                                    sg.end, sg.layer.split_k, c.mfma, cus);
        c.p.S = sp.S;
        c.p.kslab = sp.kslab;
      }
    }
    g.grouped[static_cast<size_t>(i)] = take ? 1 : 0;
    if (take && !vec) {
      any = true;
      all_large = all_large && fused_takes_large_tile(c.p, cus);
    }
    if (!take) {
      const size_t need = workspace_need(&sg.layer, c.p);
      if (need > g.ws_need) g.ws_need = need;
    }
  }
  g.large_tile = any && all_large;
  return g;
}

}  // namespace

extern "C" size_t chunkft_group_workspace_bytes(const chunkft_group_segment* segs, int32_t n_segs) {
  if (!segs || n_segs < 1 || n_segs > kMaxGroupSegments) return 0;
  const GroupPlan g = plan_group(segs, n_segs);
  return g.status == CHUNKFT_OK ? g.ws_need : 0;
}

extern "C" int chunkft_wgrad_adamw_fused_group(const chunkft_group_segment* segs, int32_t n_segs,
                                               const chunkft_adamw_hparams* hp, void* ws, size_t ws_bytes,
                                               void* stream) {
  if (!segs || n_segs < 1 || n_segs > kMaxGroupSegments) return CHUNKFT_ERR_INVALID_ARG;
  AdamWConsts consts;
  const int hr = check_hparams(hp, &consts);
  if (hr != CHUNKFT_OK) return hr;
  const GroupPlan g = plan_group(segs, n_segs);
  if (g.status != CHUNKFT_OK) return g.status;
  if (g.ws_need > 0 && (!ws || ws_bytes < g.ws_need || (reinterpret_cast<uintptr_t>(ws) & 15u)))
    return CHUNKFT_ERR_WORKSPACE;
  std::vector<GroupSegment> table;
  table.reserve(static_cast<size_t>(n_segs));
  for (int32_t i = 0; i < n_segs; ++i) {
    if (!g.grouped[static_cast<size_t>(i)]) continue;
    const chunkft_group_segment& sg = segs[i];
    GroupSegment t{};
    t.p = g.checked[static_cast<size_t>(i)].p;
    t.s = fused_sinks(&sg.layer, sg.W, sg.master, sg.m, sg.v, consts);
    t.vector = sg.layer.kind == CHUNKFT_VECTOR;
    if (t.vector) { t.p.S = 1; t.p.kslab = t.p.T; }
    table.push_back(t);
  }
  if (launch_fused_group(table.data(), static_cast<int>(table.size()), g.large_tile, stream) != 0) return CHUNKFT_ERR_HIP;
  for (int32_t i = 0; i < n_segs; ++i) {
    if (g.grouped[static_cast<size_t>(i)]) continue;
    const chunkft_group_segment& sg = segs[i];
    const int r = run_fused(&sg.layer, g.checked[static_cast<size_t>(i)],
                            fused_sinks(&sg.layer, sg.W, sg.master, sg.m, sg.v, consts), ws, stream);
    if (r != CHUNKFT_OK) return r;
  }
  return CHUNKFT_OK;
}

extern "C" const char* chunkft_status_string(int status) {
  switch (status) {
    case CHUNKFT_OK: return "ok";
    case CHUNKFT_ERR_INVALID_ARG: return "invalid argument";
    case CHUNKFT_ERR_RANGE: return "element range empty or outside the tensor";
    case CHUNKFT_ERR_DTYPE: return "unknown or unsupported dtype / kind";
    case CHUNKFT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CHUNKFT_ERR_BUFFER_TOO_SMALL: return "output arrays too small; required counts returned";
    case CHUNKFT_ERR_HIP: return "HIP runtime error on launch";
    case CHUNKFT_ERR_OVERFLOW: return "size does not fit in int64";
    case CHUNKFT_ERR_STATIC_WORKSPACE: return "call needs more workspace than the library's static array holds";
    default: return "unknown status";
  }
}

extern "C" int chunkft_version(void) { return 100; }  // 0.1.0
