// Host-only fuzz of libchunkft's C++ (planner, plan summary, schedule, argument validation,
// token-split and workspace logic), meant to be built with g++ -fsanitize=address,undefined
// from plan.cpp + api.cpp + shape.cpp.  The kernel launchers are replaced by stand-ins that
// launch nothing and instead check, on the host, what a kernel would have been handed: ranges
// inside the tensor, slabs that cover the tokens, partial sums that stay inside the caller's
// workspace.  No GPU, no HIP.  Exit code 0 and a line "ok ..." on success.

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "chunkft.h"
#include "internal.h"

namespace {
long g_launches = 0;
const char* g_fail = nullptr;
uintptr_t g_ws_lo = 0, g_ws_hi = 0;     // the workspace handed to the call under test

void expect(bool ok, const char* what) {
  if (!ok && !g_fail) g_fail = what;
}

void check_problem(const chunkft::WgradProblem& p) {
  expect(p.begin >= 0 && p.begin < p.end, "range order");
  expect(p.out > 0 && p.in > 0 && p.end <= p.out * p.in, "range inside the tensor");
  expect(p.T > 0 && p.S >= 1 && p.kslab > 0, "slab shape");
  expect((int64_t)p.S * p.kslab >= p.T && (int64_t)(p.S - 1) * p.kslab < p.T, "slabs cover the tokens, none empty");
}

void check_partials(const chunkft::WgradProblem& p, const chunkft::Sinks& s) {
  if (p.S <= 1) return;
  const int64_t E = p.end - p.begin;
  expect(s.ws_pitch >= E, "slab pitch");
  const uintptr_t lo = reinterpret_cast<uintptr_t>(s.ws);
  const uintptr_t hi = lo + 4u * (uintptr_t)((int64_t)(p.S - 1) * s.ws_pitch + E);
  expect(lo >= g_ws_lo && hi <= g_ws_hi, "partial sums inside the workspace");
}
}  // namespace

namespace chunkft {
int device_compute_units() { return kDefaultComputeUnits; }
int launch_wgrad_bf16_mfma(const WgradProblem& p, int mode, const Sinks& s, void*) {
  ++g_launches;
  check_problem(p);
  expect(mfma_path_ok(p), "MFMA path taken for a shape it cannot load");
  const RowSplit rs = split_rows(p);
  expect(rs.rb0 % 8 == 0 && rs.rb1 >= rs.rb0 && rs.rb1 <= p.out, "body rows");
  expect(rs.rb1 == rs.rb0 || (rs.rb0 * p.in >= p.begin && rs.rb1 * p.in <= p.end), "body rows lie inside the range");
  expect(rs.lead_base < 0 || (rs.lead_base % 8 == 0 && rs.lead_base + 8 == rs.rb0), "leading group");
  expect(rs.trail_row < rs.rb1 + 1 || rs.trail_row < p.out, "trailing row");
  if (mode == EMIT_PARTIAL) check_partials(p, s);
  return 0;
}
int launch_wgrad_simt(const WgradProblem& p, int, int mode, const Sinks& s, void*) {
  ++g_launches;
  check_problem(p);
  if (mode == EMIT_PARTIAL) check_partials(p, s);
  return 0;
}
int launch_colsum(const WgradProblem& p, int, int, const Sinks&, void*) { ++g_launches; check_problem(p); expect(p.S == 1, "vector split"); return 0; }
int launch_norm_wgrad(const WgradProblem& p, int, bool, float, float* stats, int, const Sinks&, void*) {
  ++g_launches;
  check_problem(p);
  const uintptr_t lo = reinterpret_cast<uintptr_t>(stats);
  expect(lo >= g_ws_lo && lo + 8u * (uintptr_t)p.T <= g_ws_hi, "statistics inside the workspace");
  return 0;
}
int launch_embed_wgrad(const WgradProblem& p, int, int, const Sinks&, void*) { ++g_launches; check_problem(p); expect(p.T <= kMaxEmbeddingTokens, "tokens per call"); return 0; }
int launch_reduce(const float* ws, int32_t S, int64_t E, int, const Sinks& s, void*, void*) {
  ++g_launches;
  const uintptr_t lo = reinterpret_cast<uintptr_t>(ws);
  expect(S >= 2 && E > 0 && s.ws_pitch >= E, "reduction shape");
  expect(lo >= g_ws_lo && lo + 4u * (uintptr_t)((int64_t)(S - 1) * s.ws_pitch + E) <= g_ws_hi, "reduction reads inside the workspace");
  return 0;
}
int launch_fused_group(const GroupSegment* segs, int n, bool, void*) {
  g_launches += n > 0;
  for (int i = 0; i < n; ++i) {
    check_problem(segs[i].p);
    expect(segs[i].p.S == 1, "grouped segment with a token split");
    expect(group_takes_segment(segs[i].p, segs[i].vector), "grouped segment the kernel cannot take");
    if (!segs[i].vector) expect(mfma_path_ok(segs[i].p), "grouped matrix segment off the MFMA path");
  }
  return 0;
}
int launch_adamw(const float*, int64_t n, const Sinks&, void*, void*) { ++g_launches; expect(n > 0, "adamw size"); return 0; }
}  // namespace chunkft

int main() {
  std::mt19937_64 rng(1234);
  long plans = 0, calls = 0, accepted = 0;
  // ---- planner, plan summary, schedule
  for (int it = 0; it < 60000; ++it) {
    const int n = rng() % 6;
    std::vector<chunkft_tensor_desc> t(n);
    for (auto& d : t) {
      d.rows = (rng() % 5 == 0) ? 0 : (int64_t)(rng() % 50);
      d.cols = (int64_t)(rng() % 40);
      if (rng() % 97 == 0) { d.rows = (int64_t)1 << (20 + rng() % 42); d.cols = (int64_t)1 << (rng() % 40); }
      d.dtype = rng() % 2;
      d.kind = rng() % 5;
    }
    int64_t budget = (int64_t)(rng() % 300);
    if (rng() % 31 == 0) budget = INT64_MAX - (int64_t)(rng() % 100);
    const uint32_t flags = rng() % 8;
    int64_t nc = -1, ns = -1;
    int r = chunkft_plan_cycle(t.data(), n, budget, flags, nullptr, 0, &nc, nullptr, 0, &ns);
    if (r == CHUNKFT_ERR_BUFFER_TOO_SMALL || r == CHUNKFT_OK) {
      if (nc > 200000 || ns > 200000) continue;
      std::vector<chunkft_chunk> c(nc + 1);
      std::vector<chunkft_segment> s(ns + 1);
      int64_t nc2 = 0, ns2 = 0;
      r = chunkft_plan_cycle(t.data(), n, budget, flags, c.data(), nc, &nc2, s.data(), ns, &ns2);
      if (r != CHUNKFT_OK || nc2 != nc || ns2 != ns) { printf("count-then-fill mismatch at %d\n", it); return 1; }
      std::vector<int64_t> pos(n, 0);
      for (int64_t i = 0; i < ns; ++i) {
        const auto& g = s[i];
        if (g.tensor < 0 || g.tensor >= n || g.begin != pos[g.tensor] || g.end <= g.begin) { printf("bad segment at %d\n", it); return 1; }
        pos[g.tensor] = g.end;
      }
      for (int i = 0; i < n; ++i) if (pos[i] != t[i].rows * t[i].cols) { printf("coverage at %d\n", it); return 1; }
      for (int64_t k = 0; k < nc; ++k) {
        if (c[k].cost_bytes <= 0 || c[k].cost_bytes > budget || c[k].seg_begin >= c[k].seg_end) { printf("chunk %ld at %d\n", (long)k, it); return 1; }
        int64_t numel = 0;
        for (int64_t i = c[k].seg_begin; i < c[k].seg_end; ++i) {
          if (s[i].chunk_off != numel) { printf("chunk_off at %d\n", it); return 1; }
          numel += s[i].end - s[i].begin;
        }
        if (numel != c[k].numel) { printf("numel at %d\n", it); return 1; }
      }
      if (nc > 0) {
        chunkft_plan_summary sum;
        if (chunkft_plan_stats(c.data(), nc, (int64_t)(rng() % 100000), &sum) != CHUNKFT_OK) { printf("stats at %d\n", it); return 1; }
        if (!(sum.jitter <= sum.jitter_bound * (1 + 1e-12) + 1e-300) || sum.imbalance_bytes < 0) { printf("jitter bound at %d\n", it); return 1; }
      }
      ++plans;
    }
    chunkft_schedule_entry e;
    chunkft_schedule_at((int64_t)(rng() >> (rng() % 64)), 1 + rng() % 9, 1 + (int64_t)(rng() >> (1 + rng() % 63)), &e);
  }
  // ---- device entry points with made-up addresses: validation, token split, workspace placement
  const uintptr_t base = 0x10000000u;
  for (int it = 0; it < 200000; ++it) {
    chunkft_layer L{};
    L.kind = (int32_t)(rng() % 6) - (rng() % 50 == 0);
    L.dtype = (int32_t)(rng() % 2) + (rng() % 60 == 0 ? 5 : 0);
    const bool wide = rng() % 40 == 0;
    L.out = wide ? (int64_t)(rng() >> (rng() % 64)) : (int64_t)(rng() % 3000) * (rng() % 3 ? 8 : 1);
    L.in = wide ? (int64_t)(rng() >> (rng() % 64)) : (int64_t)(rng() % 3000) * (rng() % 3 ? 8 : 1);
    if (L.kind == CHUNKFT_VECTOR || L.kind == CHUNKFT_RMSNORM || L.kind == CHUNKFT_LAYERNORM) L.out = rng() % 20 ? 1 : 2;
    L.T = (int64_t)(rng() % 20000) - (rng() % 80 == 0);
    L.ldx = L.in + (rng() % 4 ? 0 : (int64_t)(rng() % 64) - 8);
    L.lddy = (L.kind == CHUNKFT_LINEAR ? L.out : L.in) + (rng() % 4 ? 0 : (int64_t)(rng() % 64) - 8);
    L.X = rng() % 50 ? (const void*)(base + 16 * (rng() % 1000) + (rng() % 9 ? 0 : rng() % 16)) : nullptr;
    L.dY = rng() % 50 ? (const void*)(base + 16 * (rng() % 1000) + (rng() % 9 ? 0 : rng() % 16)) : nullptr;
    L.split_k = rng() % 3 ? 0 : (int32_t)(rng() % 70) - 2;
    L.reserved = rng() % 90 == 0;
    L.norm_eps = rng() % 70 ? 1e-6 : -1.0;
    const int64_t numel = (L.out > 0 && L.in > 0 && L.in < INT64_MAX / (L.out > 0 ? L.out : 1)) ? L.out * L.in : 1000;
    int64_t begin = (int64_t)(rng() % (uint64_t)(numel > 0 ? numel : 1));
    int64_t end = begin + 1 + (int64_t)(rng() % (uint64_t)(numel - begin > 0 ? numel - begin : 1));
    if (rng() % 60 == 0) end = begin;
    if (rng() % 60 == 0) end = numel + 1 + (int64_t)(rng() % 5);
    const size_t need = chunkft_workspace_bytes(&L, begin, end);
    const int S = chunkft_split_k(&L, begin, end);
    size_t have = need;
    if (rng() % 10 == 0 && need > 0) have = need - 1 - (size_t)(rng() % need);
    void* ws = have || rng() % 2 ? (void*)(base + 0x4000000u + 16 * (rng() % 64) + (rng() % 12 ? 0 : 4)) : nullptr;
    g_ws_lo = reinterpret_cast<uintptr_t>(ws);
    g_ws_hi = g_ws_lo + have;
    float* fp = (float*)(base + 0x2000000u + 4 * (rng() % 64));
    chunkft_adamw_hparams hp{1e-4, 0.9, 0.999, 1e-8, 0.01, (int64_t)(rng() % 5) - (rng() % 40 == 0)};
    const long before = g_launches;
    int r;
    if (rng() % 2) r = chunkft_chunk_wgrad(&L, begin, end, fp, (int)(rng() % 2), ws, have, nullptr);
    else r = chunkft_wgrad_adamw_fused(&L, begin, end, rng() % 2 ? (void*)fp : nullptr, fp, fp, fp, &hp, ws, have, nullptr);
    ++calls;
    if (r == CHUNKFT_OK) {
      ++accepted;
      if (S < 1) { printf("accepted call with split %d at %d\n", S, it); return 1; }
      if (g_launches == before) { printf("accepted call launched nothing at %d\n", it); return 1; }
    } else if (g_launches != before) {
      printf("rejected call (%d) reached a launcher at %d\n", r, it);
      return 1;
    }
    if (g_fail) { printf("launch check failed: %s (iteration %d)\n", g_fail, it); return 1; }
    if (rng() % 8 == 0) {
      const int64_t n = (int64_t)(rng() % 100000) - 3;
      const int ra = chunkft_adamw_chunk(fp, fp, fp, fp, rng() % 2 ? (void*)fp : nullptr, (int32_t)(rng() % 3), n, &hp, nullptr);
      if ((ra == CHUNKFT_OK) != (n > 0 && hp.step >= 1 && ra == 0)) { printf("adamw validation at %d\n", it); return 1; }
    }
  }
  // ---- grouped fused call: random groups of segments on made-up addresses
  long groups = 0, groups_ok = 0;
  for (int it = 0; it < 30000; ++it) {
    const int n = 1 + (int)(rng() % 20);
    std::vector<chunkft_group_segment> sg((size_t)n);
    for (auto& g : sg) {
      chunkft_layer& L = g.layer;
      L = chunkft_layer{};
      L.kind = rng() % 12 == 0 ? (int32_t)(rng() % 5) : (rng() % 4 == 0 ? CHUNKFT_VECTOR : CHUNKFT_LINEAR);
      L.dtype = rng() % 8 == 0 ? CHUNKFT_F32 : CHUNKFT_BF16;
      L.out = L.kind == CHUNKFT_LINEAR || L.kind == CHUNKFT_EMBEDDING ? 8 * (1 + (int64_t)(rng() % 600)) : 1;
      L.in = (rng() % 10 ? 8 : 1) * (1 + (int64_t)(rng() % 600));
      L.T = 1 + (int64_t)(rng() % 9000);
      if (L.kind == CHUNKFT_EMBEDDING && L.T > 8192) L.T = 8192;
      L.ldx = L.in;
      L.lddy = L.kind == CHUNKFT_LINEAR ? L.out : L.in;
      L.X = (const void*)(base + 16 * (rng() % 1000));
      L.dY = (const void*)(base + 16 * (rng() % 1000));
      L.split_k = rng() % 5 ? 0 : (int32_t)(rng() % 5);
      if (L.kind != CHUNKFT_LINEAR) L.split_k = 0;
      L.norm_eps = 1e-6;
      const int64_t numel = L.out * L.in;
      g.begin = (int64_t)(rng() % (uint64_t)numel);
      g.end = g.begin + 1 + (int64_t)(rng() % (uint64_t)(numel - g.begin));
      if (rng() % 400 == 0) g.end = g.begin;
      g.W = rng() % 2 ? (void*)(base + 0x1000000u) : nullptr;
      g.master = g.m = g.v = (float*)(base + 0x2000000u + 4 * (rng() % 64));
      if (rng() % 500 == 0) g.m = nullptr;
    }
    chunkft_adamw_hparams hp{1e-4, 0.9, 0.999, 1e-8, 0.01, 1 + (int64_t)(rng() % 5)};
    const size_t need = chunkft_group_workspace_bytes(sg.data(), n);
    size_t have = need;
    if (need > 0 && rng() % 10 == 0) have = need - 1;
    void* ws = have ? (void*)(base + 0x4000000u) : nullptr;
    g_ws_lo = reinterpret_cast<uintptr_t>(ws);
    g_ws_hi = g_ws_lo + have;
    const long before = g_launches;
    const int r = chunkft_wgrad_adamw_fused_group(sg.data(), n, &hp, ws, have, nullptr);
    ++groups;
    if (r == CHUNKFT_OK) {
      ++groups_ok;
      if (g_launches == before) { printf("accepted group launched nothing at %d\n", it); return 1; }
    } else if (g_launches != before) {
      printf("rejected group (%d) reached a launcher at %d\n", r, it);
      return 1;
    }
    if (g_fail) { printf("group launch check failed: %s (iteration %d)\n", g_fail, it); return 1; }
  }
  if (groups_ok < groups / 4) { printf("too few accepted groups: %ld of %ld\n", groups_ok, groups); return 1; }
  if (accepted < calls / 20) { printf("too few accepted calls: %ld of %ld\n", accepted, calls); return 1; }
  printf("ok: %ld plans, %ld device calls (%ld accepted), %ld grouped calls (%ld accepted), %ld stand-in launches\n", plans, calls,
         accepted, groups, groups_ok, g_launches);
  return 0;
}
