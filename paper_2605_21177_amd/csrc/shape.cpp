// Host-side shape logic of the weight-gradient calls: which rows the MFMA kernel tiles, whether
// a call can take the MFMA path, and into how many token slabs it is split.  Pure functions of
// their arguments (no HIP), so that they can be built and fuzzed on a machine without a GPU.

#include <cstdint>

#include "internal.h"

namespace chunkft {

namespace {
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
// rounds of work for w tiles per compute unit: a partly filled round costs 0.6 + 0.4 x its fill
inline double round_cost(double w) {
  const double fl = (double)(int64_t)w, fr = w - fl;
  return fl + (fr > 1e-9 ? 0.6 + 0.4 * fr : 0.0);
}
}  // namespace

// Body = complete rows from the first multiple of 8 on.  Everything before it
// lies in the one 8-row group [rb0 - 8, rb0) (at most the partial first row and
// 7 complete rows); after it there is at most the partial last row.
RowSplit split_rows(const WgradProblem& p) {
  RowSplit rs{};
  const int64_t r0 = p.begin / p.in, c0 = p.begin % p.in;
  const int64_t r1 = (p.end - 1) / p.in, c1 = (p.end - 1) % p.in + 1;
  const int64_t full0 = r0 + (c0 != 0 ? 1 : 0);           // first complete row
  const int64_t full1 = r1 + 1 - (c1 != p.in ? 1 : 0);    // one past the last complete row
  const int64_t rb0 = (full0 + 7) / 8 * 8;
  const bool body = full1 > rb0;
  rs.rb0 = rb0;
  rs.rb1 = body ? full1 : rb0;
  rs.lead_base = r0 < rb0 ? rb0 - 8 : -1;
  const int64_t first_after = body ? full1 : rb0;          // rows from here on are not in the lead group
  rs.trail_row = r1 >= first_after ? r1 : -1;
  return rs;
}

// The edge rows ride in the MFMA kernel if it has the tile rows that carry them (more than 128 body
// rows = two tile rows of the small tile; the same rule for both tile sizes, so that every call sums
// every element in the same order).
bool edge_rows_folded(const RowSplit& rs) { return rs.rb1 - rs.rb0 > 128; }

bool group_takes_segment(const WgradProblem& p, bool vector) {
  if (vector) return true;
  const RowSplit rs = split_rows(p);
  // a body for the MFMA kernel, its edge rows (if any) carried by it, one token slab
  return p.S == 1 && rs.rb1 > rs.rb0 && (edge_rows_folded(rs) || (rs.lead_base < 0 && rs.trail_row < 0));
}

bool mfma_path_ok(const WgradProblem& p) {
  const auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
  if (!(p.in % 8 == 0 && p.out % 8 == 0 && p.ldx % 8 == 0 && p.lddy % 8 == 0 && a16(p.X) && a16(p.dY)))
    return false;
  if (p.in >= (1 << 21)) return false;      // the epilogue's 32-bit tile offsets
  // the 32-bit byte offsets of the global->LDS loads: a row / column index plus up to 63 tokens
  if (p.out + 64 * p.lddy >= (int64_t(1) << 31) || p.in + 64 * p.ldx >= (int64_t(1) << 31)) return false;
  return true;
}

// Which tile the plain gradient takes.  The 256 x 256 tile (one workgroup per compute unit) runs its
// rounds faster the more tokens a slab has -- measured ratio of a full round against the 128 x 256
// tile's (two workgroups per unit): 1.05 at 768 tokens, 0.99 at 1024, 0.95 at 1536, 0.91 at 2048,
// 0.88 at 3072, 0.85 at 8192, fitted by 0.83 + 160 / T -- but pays for a partly filled last round in
// whole tiles where the small tile pays in half ones.  With w = tiles / compute units, a partly
// filled round costs about 0.6 + 0.4 x (its fill) of a full one (the units that work alone run
// faster): cost(w) = floor(w) + (0.6 + 0.4 frac(w) if frac(w) > 0), and the small tile's cost in the
// same unit is cost(2 w) / 2.  On 75 measured cases (12 shapes, 768 - 8192 tokens) the rule below is
// within 0.3 % of the better tile on average and never more than 4 % off; "small tile up to 2048
// tokens" was 2.5 % off on average and up to 15 %.
bool plain_takes_large_tile(int64_t large_tiles, int64_t slab_tokens, int compute_units) {
  const double cus = compute_units > 0 ? compute_units : kDefaultComputeUnits;
  if (large_tiles <= (int64_t)(cus / 2)) return false;          // too few tiles to fill the device: twice as many small ones
  const double w = (double)large_tiles / cus;
  const double round_ratio = 0.83 + 160.0 / (double)(slab_tokens > 0 ? slab_tokens : 1);
  return round_ratio * round_cost(w) / (round_cost(2.0 * w) / 2.0) < 0.99;
}

// Which tile the fused call takes.  Its AdamW epilogue is HBM-bound and overlaps the partner's loop
// only on the small tile, so the large tile pays only when the loops dominate: measured ratio of the
// large tile's time to the small one's on fully filled rounds 1.05 - 1.10 at 3072 - 4096 tokens, 0.98 -
// 0.99 (in = 4096) and 0.89 (in = 8192) at 6144, 0.84 - 0.93 at 8192, fitted by 0.55 + 2600 / T; partly
// filled rounds are priced as for the plain gradient.  The rule agrees with the faster tile in all 16
// measured cases (four shapes x 3072 - 8192 tokens; X from 24 to 224 MiB).
bool fused_takes_large_tile(const WgradProblem& p, int compute_units) {
  const double cus = compute_units > 0 ? compute_units : kDefaultComputeUnits;
  const RowSplit rs = split_rows(p);
  const int64_t rows = rs.rb1 > rs.rb0 ? rs.rb1 - rs.rb0 : 0;
  const int64_t tiles = ceil_div(rows, kMainTileM) * ceil_div(p.in, kMainTileN) * (p.S > 0 ? p.S : 1);
  if (tiles <= (int64_t)(cus / 2)) return false;
  const int64_t slab_tokens = p.S > 1 ? p.kslab : p.T;
  const double w = (double)tiles / cus;
  const double round_ratio = 0.55 + 2600.0 / (double)(slab_tokens > 0 ? slab_tokens : 1);
  return round_ratio * round_cost(w) / (round_cost(2.0 * w) / 2.0) < 0.99;
}

Split pick_split(int32_t kind, int32_t dtype, int64_t out, int64_t in, int64_t T, int64_t begin,
                 int64_t end, int32_t forced, bool mfma, int compute_units) {
  (void)out; (void)dtype;
  if (kind != 0) return {1, T};                       // only linear layers are ever split
  const int64_t bm = mfma ? kMainTileM : kSimtTileM, bn = mfma ? kMainTileN : kSimtTileN;
  const int64_t bk = mfma ? kMainTileK : kSimtTileK;
  int64_t S = forced;
  if (S <= 0) {
    int64_t rows = (end - 1) / in - begin / in + 1;
    if (mfma) {                                       // the MFMA kernel tiles the body rows only
      WgradProblem tmp{};
      tmp.begin = begin;
      tmp.end = end;
      tmp.in = in;
      const RowSplit rs = split_rows(tmp);
      rows = rs.rb1 > rs.rb0 ? rs.rb1 - rs.rb0 : 1;
    }
    const int64_t tiles = ceil_div(rows, bm) * ceil_div(in, bn);
    S = 1;
    const int64_t slots = compute_units > 0 ? compute_units : kDefaultComputeUnits;   // resident workgroups
    if (mfma && tiles <= slots / 4) {
      // Splitting pays only when the 256 x 256 tiles fill at most a quarter of the compute units.
      // A slab costs its tokens' share of the loop, every further slab 8 bytes per element of
      // partial traffic plus one more set-up and epilogue per tile: time ~ a T / S + b S tiles,
      // least at S = sqrt(a T / (b tiles)).  a / b = 1 / 12 fits the measured grid (16 - 192
      // tiles x 1024 - 8192 tokens x 1 - 16 slabs, plain and fused call, in = 4096); more than 8
      // slabs never won, and from 128 tiles on one slab is best.
      S = 1;
      while ((S + 1) * (S + 1) * 12 * tiles <= T && S < 8) ++S;
      if (S > slots / tiles) S = slots / tiles;
      if (S > T / 256) S = T / 256 > 0 ? T / 256 : 1;    // never slabs of fewer than 256 tokens
    }
  }
  int64_t kslab = ceil_div(ceil_div(T, S), bk) * bk;
  S = ceil_div(T, kslab);                             // no empty slab
  return {(int32_t)S, kslab};
}

}  // namespace chunkft
