// Cycle planner: byte budget -> ordered chunks of tensor segments (host only).
//
// Follows the paper's Section 3 "Method" (first paragraph) and Algorithm 1
// lines 1-2: every tensor costs numel x bytes-per-element, tensors are taken
// in model order, a chunk is filled until the budget cannot take one more
// element, and a tensor that does not fit is cut at that element, so it spans
// chunks.  The optional training cost per element is the one of Section 3.1
// (parameter + gradient + fp32 master + two moments).  Optionally a tensor is cut
// between rows only (the same opening paragraph of Section 3 splits large matrices
// along the row dimension), in groups of 8 rows.  Integer arithmetic only, except
// the summary of a plan (chunkft_plan_stats: the imbalance and jitter of the paper's
// appendix on memory jitter), which is a handful of doubles.

#include "chunkft.h"

#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

namespace {

constexpr int64_t kStateBytes = 16;  // fp32 gradient + master + m + v

struct Costed {
  int64_t numel;
  int64_t cost;  // bytes charged per element
  int64_t unit;  // cuts inside this tensor fall on multiples of `unit` elements (1: anywhere)
};

// One greedy pass.  With out == nullptr it only counts.
struct Pass {
  int64_t n_chunks = 0;
  int64_t n_segs = 0;
  // Fewest bytes by which the budget must grow before this pass takes a different decision
  // anywhere (a cut lets one more element or group of rows in, or a tensor becomes narrow
  // enough to be cut between rows): every budget in [budget, budget + slack) gives the same plan.
  int64_t slack = std::numeric_limits<int64_t>::max();
};

Pass greedy(const std::vector<Costed>& ts, int64_t budget, chunkft_chunk* chunks,
            chunkft_segment* segs) {
  Pass p;
  int64_t room = budget;
  int64_t filled = 0;        // elements in the open chunk
  int64_t seg_first = 0;     // first segment of the open chunk
  auto close_chunk = [&]() {
    if (chunks) {
      chunkft_chunk& c = chunks[p.n_chunks];
      c.seg_begin = seg_first;
      c.seg_end = p.n_segs;
      c.numel = filled;
      c.cost_bytes = budget - room;
    }
    ++p.n_chunks;
    room = budget;
    filled = 0;
    seg_first = p.n_segs;
  };
  for (size_t t = 0; t < ts.size(); ++t) {
    int64_t pos = 0;
    const int64_t n = ts[t].numel, s = ts[t].cost;
    // Row-aligned cuts need room for one group of rows in an empty chunk; a tensor for
    // which this budget has none is cut anywhere.  With u > 1 every cut of this tensor
    // is a multiple of u, so `pos` is one too.
    const int64_t u = (ts[t].unit > 1 && ts[t].unit <= budget / s) ? ts[t].unit : 1;
    if (n > 0 && ts[t].unit > 1 && u == 1 && ts[t].unit <= std::numeric_limits<int64_t>::max() / s) {
      const int64_t d = ts[t].unit * s - budget;     // > 0: from there on the tensor is cut between rows
      if (d < p.slack) p.slack = d;
    }
    const int64_t us = u * s;                        // bytes of one unit; fits: u <= budget / s
    while (pos < n) {
      // Counting only, at the start of a chunk: the chunks that this tensor fills completely
      // all look alike, so they are counted in one step (a 2^60-element tensor under a small
      // budget would otherwise take 2^50 trips).
      if (!chunks && !segs && filled == 0 && room == budget) {
        const int64_t per_chunk = budget / s / u * u;
        const int64_t whole = per_chunk > 0 ? (n - pos) / per_chunk : 0;
        if (whole > 1) {
          const int64_t d = us - budget % us;        // each of these chunks would take one more unit
          if (d < p.slack) p.slack = d;
          p.n_chunks += whole - 1;
          p.n_segs += whole - 1;
          pos += (whole - 1) * per_chunk;
          seg_first = p.n_segs;
        }
      }
      int64_t take = room / s;
      if (take >= n - pos) take = n - pos;
      else {
        take = take / u * u;             // the tensor is cut here: on a group boundary
        // room for one more unit, or for the whole rest (whose last group may be short), changes the cut
        const int64_t d_unit = us - room % us, d_rest = (n - pos) * s - room;
        const int64_t d = d_unit < d_rest ? d_unit : d_rest;
        if (d < p.slack) p.slack = d;
      }
      if (take == 0) {       // not one more element (group of rows) of this tensor fits
        close_chunk();
        continue;
      }
      if (segs) {
        chunkft_segment& g = segs[p.n_segs];
        g.tensor = static_cast<int32_t>(t);
        g.reserved = 0;
        g.begin = pos;
        g.end = pos + take;
        g.chunk_off = filled;
      }
      ++p.n_segs;
      pos += take;
      filled += take;
      room -= take * s;
    }
  }
  if (filled > 0) close_chunk();
  return p;
}

}  // namespace

extern "C" int chunkft_plan_cycle(const chunkft_tensor_desc* tensors, int32_t n_tensors,
                                  int64_t budget_bytes, uint32_t flags, chunkft_chunk* chunks,
                                  int64_t chunks_cap, int64_t* n_chunks, chunkft_segment* segs,
                                  int64_t segs_cap, int64_t* n_segs) {
  if (!n_chunks || !n_segs) return CHUNKFT_ERR_INVALID_ARG;
  *n_chunks = 0;
  *n_segs = 0;
  if (n_tensors < 0 || (n_tensors > 0 && !tensors)) return CHUNKFT_ERR_INVALID_ARG;
  if (budget_bytes <= 0) return CHUNKFT_ERR_INVALID_ARG;
  if (flags & ~(CHUNKFT_PLAN_TRAINING_COST | CHUNKFT_PLAN_BALANCED | CHUNKFT_PLAN_ROWS8)) return CHUNKFT_ERR_INVALID_ARG;
  if (chunks_cap < 0 || segs_cap < 0) return CHUNKFT_ERR_INVALID_ARG;
  if ((chunks_cap > 0 && !chunks) || (segs_cap > 0 && !segs)) return CHUNKFT_ERR_INVALID_ARG;

  const int64_t kMax = std::numeric_limits<int64_t>::max();
  std::vector<Costed> ts(static_cast<size_t>(n_tensors));
  int64_t total = 0, max_cost = 0;
  for (int32_t t = 0; t < n_tensors; ++t) {
    const chunkft_tensor_desc& d = tensors[t];
    if (d.rows < 0 || d.cols < 0) return CHUNKFT_ERR_INVALID_ARG;
    if (d.kind < CHUNKFT_LINEAR || d.kind > CHUNKFT_LAYERNORM) return CHUNKFT_ERR_DTYPE;
    int64_t s;
    if (d.dtype == CHUNKFT_F32) s = 4;
    else if (d.dtype == CHUNKFT_BF16) s = 2;
    else return CHUNKFT_ERR_DTYPE;
    if (flags & CHUNKFT_PLAN_TRAINING_COST) s += kStateBytes;
    if (d.rows != 0 && d.cols > kMax / d.rows) return CHUNKFT_ERR_OVERFLOW;
    const int64_t n = d.rows * d.cols;
    if (n != 0 && s > kMax / n) return CHUNKFT_ERR_OVERFLOW;
    if (n * s > kMax - total) return CHUNKFT_ERR_OVERFLOW;
    total += n * s;
    if (n > 0) {
      if (s > budget_bytes) return CHUNKFT_ERR_INVALID_ARG;
      if (s > max_cost) max_cost = s;
    }
    int64_t unit = 1;
    if ((flags & CHUNKFT_PLAN_ROWS8) && d.cols <= kMax / 8) unit = 8 * d.cols;
    ts[static_cast<size_t>(t)] = {n, s, unit > 0 ? unit : 1};
  }

  int64_t budget = budget_bytes;
  Pass need = greedy(ts, budget, nullptr, nullptr);
  if ((flags & CHUNKFT_PLAN_BALANCED) && need.n_chunks > 1) {
    const int64_t k = need.n_chunks;
    int64_t b = total / k + (total % k ? 1 : 0);
    b = (b + 3) / 4 * 4;
    if (b < max_cost) b = max_cost;
    // The candidates are b, b + 4, b + 8, ... below the caller's budget, the answer the first
    // one that needs no more than k chunks.  A pass also tells how far the budget can grow
    // before anything in it changes, so the candidates in between are skipped, not tried:
    // a handful of passes where cuts between groups of rows put megabytes between two plans.
    for (;;) {
      if (b >= budget_bytes) { b = budget_bytes; break; }   // greedy(budget_bytes) needs k chunks
      const Pass trial = greedy(ts, b, nullptr, nullptr);
      if (trial.n_chunks <= k) break;
      const int64_t grow = trial.slack > 0 ? trial.slack : 1;
      if (grow >= budget_bytes - b) { b = budget_bytes; break; }
      b += (grow + 3) / 4 * 4;
    }
    budget = b;
    need = greedy(ts, budget, nullptr, nullptr);
  }
  *n_chunks = need.n_chunks;
  *n_segs = need.n_segs;
  if (need.n_chunks > chunks_cap || need.n_segs > segs_cap) return CHUNKFT_ERR_BUFFER_TOO_SMALL;
  greedy(ts, budget, chunks, segs);
  return CHUNKFT_OK;
}

// Closed form of the rotating schedule: with H = interval and K chunks, step t lies in
// visit t / H, which goes to chunk (t / H) mod K and is that chunk's visit number
// t / (H K) (counting from 0); the chunk has then been updated H times per earlier visit
// plus (t mod H) + 1 times in this one.
extern "C" int chunkft_schedule_at(int64_t step, int32_t n_chunks, int64_t interval, chunkft_schedule_entry* out) {
  if (!out || step < 0 || n_chunks < 1 || interval < 1) return CHUNKFT_ERR_INVALID_ARG;
  const int64_t visit = step / interval, within = step % interval;
  if (interval > INT64_MAX / n_chunks) {
    // a cycle longer than int64: the step lies in the first cycle
    out->local_step = within + 1;
  } else {
    const int64_t earlier_visits = step / (interval * n_chunks);
    if (earlier_visits > (INT64_MAX - within - 1) / interval) return CHUNKFT_ERR_OVERFLOW;
    out->local_step = earlier_visits * interval + within + 1;
  }
  out->active = (int32_t)(visit % n_chunks);
  out->load_before = within == 0;
  out->offload_after = within == interval - 1;
  out->reserved = 0;
  return CHUNKFT_OK;
}

// Summary of a plan in the terms of the paper's appendix on memory jitter: with the step memory
// M_k = resident + B(C_k) (activations and temporaries left out), the mean chunk cost, the
// imbalance eps_B = max_k |B(C_k) - mean|, the jitter (max_k M_k - min_k M_k) / mean_k M_k and
// the bound 2 eps_B / (resident + mean) that the appendix gives for it.
extern "C" int chunkft_plan_stats(const chunkft_chunk* chunks, int64_t n_chunks, int64_t resident_bytes,
                                  chunkft_plan_summary* out) {
  if (!chunks || !out || n_chunks < 1 || resident_bytes < 0) return CHUNKFT_ERR_INVALID_ARG;
  int64_t lo = std::numeric_limits<int64_t>::max(), hi = 0;
  long double sum = 0.0L;
  for (int64_t k = 0; k < n_chunks; ++k) {
    const int64_t c = chunks[k].cost_bytes;
    if (c < 0) return CHUNKFT_ERR_INVALID_ARG;
    if (c < lo) lo = c;
    if (c > hi) hi = c;
    sum += static_cast<long double>(c);
  }
  const long double mean = sum / static_cast<long double>(n_chunks);
  // |B - mean| is largest at one of the two extremes
  const long double up = static_cast<long double>(hi) - mean, down = mean - static_cast<long double>(lo);
  const long double eps_b = up > down ? up : down;
  const long double mean_mem = static_cast<long double>(resident_bytes) + mean;
  out->n_chunks = n_chunks;
  out->min_cost_bytes = lo;
  out->max_cost_bytes = hi;
  out->mean_cost_bytes = static_cast<double>(mean);
  out->imbalance_bytes = static_cast<double>(eps_b);
  out->jitter = mean_mem > 0.0L ? static_cast<double>(static_cast<long double>(hi - lo) / mean_mem) : 0.0;
  out->jitter_bound = mean_mem > 0.0L ? static_cast<double>(2.0L * eps_b / mean_mem) : 0.0;
  return CHUNKFT_OK;
}
