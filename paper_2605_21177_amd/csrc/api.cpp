// C ABI of libchunkft: argument validation and dispatch to the gfx950 kernels.
// Nothing here computes; every step of the path runs in kernels.hip.

#include "chunkft.h"

#include <cmath>
#include <cstdint>
#include <limits>

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

extern "C" int chunkft_wgrad_adamw_fused(const chunkft_layer* L, int64_t begin, int64_t end, void* W,
                                         float* master, float* m, float* v,
                                         const chunkft_adamw_hparams* hp, void* ws, size_t ws_bytes,
                                         void* stream) {
  const Checked c = check_layer(L, begin, end);
  if (c.status != CHUNKFT_OK) return c.status;
  if (!master || !m || !v) return CHUNKFT_ERR_INVALID_ARG;
  const uintptr_t al = reinterpret_cast<uintptr_t>(master) | reinterpret_cast<uintptr_t>(m) |
                       reinterpret_cast<uintptr_t>(v);
  if (al & 3u) return CHUNKFT_ERR_INVALID_ARG;
  if (W && (reinterpret_cast<uintptr_t>(W) & (L->dtype == CHUNKFT_F32 ? 3u : 1u))) return CHUNKFT_ERR_INVALID_ARG;
  Sinks s{};
  const int hr = check_hparams(hp, &s.c);
  if (hr != CHUNKFT_OK) return hr;
  const int wsr = check_workspace(L, c.p, ws, ws_bytes);
  if (wsr != CHUNKFT_OK) return wsr;
  s.master = master;
  s.m = m;
  s.v = v;
  s.W = W;
  s.w_kind = !W ? W_NONE : (L->dtype == CHUNKFT_BF16 ? W_BF16 : W_F32);
  s.ws = static_cast<float*>(ws);
  if (c.p.S > 1) place_partials(s, c.p, ws, master);
  if (c.p.S <= 1) return run_wgrad(L, c, EMIT_ADAMW, s, stream);
  const int r = run_wgrad(L, c, EMIT_PARTIAL, s, stream);
  if (r != CHUNKFT_OK) return r;
  void* w_at = nullptr;
  if (W) w_at = static_cast<char*>(W) + static_cast<size_t>(begin) * (L->dtype == CHUNKFT_BF16 ? 2u : 4u);
  return launch_reduce(s.ws, c.p.S, end - begin, EMIT_ADAMW, s, w_at, stream) == 0 ? CHUNKFT_OK
                                                                                   : CHUNKFT_ERR_HIP;
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
