// Internal interface between the C ABI (api.cpp) and the gfx950 kernels (kernels.hip).
#ifndef CHUNKFT_INTERNAL_H
#define CHUNKFT_INTERNAL_H

#include <cstddef>
#include <cstdint>

namespace chunkft {

// AdamW constants, rounded once from double on the host.
struct AdamWConsts {
  float beta1, one_minus_beta1;
  float beta2, one_minus_beta2;
  float inv_bias1;   // 1 / (1 - beta1^n)
  float inv_bias2;   // 1 / (1 - beta2^n)
  float lr, eps, weight_decay;
};

// What a gradient value is turned into.
enum EmitMode : int {
  EMIT_STORE = 0,    // g[i] = val
  EMIT_ACCUM = 1,    // g[i] += val
  EMIT_PARTIAL = 2,  // ws[slab * ws_pitch + i] = val   (split over tokens)
  EMIT_ADAMW = 3     // AdamW on master/m/v[i], low-precision copy at W[flat]
};

enum WKind : int { W_NONE = 0, W_BF16 = 1, W_F32 = 2 };

struct Sinks {
  float* g;          // EMIT_STORE / EMIT_ACCUM
  float* ws;         // EMIT_PARTIAL: slab s at ws + s * ws_pitch (also the statistics scratch of the norm kinds)
  int64_t ws_pitch;  // elements from one slab's partial sums to the next
  float* master;     // EMIT_ADAMW
  float* m;
  float* v;
  void* W;           // tensor base, or nullptr
  int32_t w_kind;    // WKind
  AdamWConsts c;
};

constexpr int kMaxEdgeRows = 9;

struct WgradProblem {
  const void* X;
  const void* dY;
  int64_t ldx, lddy;
  int64_t out, in, T;
  int64_t begin, end;     // flat range, E = end - begin
  int32_t S;              // token slabs
  int64_t kslab;          // tokens per slab (multiple of the kernel's K tile)
};

// Shape of the token split for a call: S slabs of kslab tokens (last one short).
struct Split {
  int32_t S;
  int64_t kslab;
};

// Row decomposition of a chunk [begin, end) of W [out, in] for the MFMA kernel.
struct RowSplit {
  int64_t rb0, rb1;     // MFMA body rows [rb0, rb1), empty if rb1 <= rb0
  int64_t lead_base;    // 8-aligned group holding the leading edge rows, or -1
  int64_t trail_row;    // partial last row outside the body, or -1
};
RowSplit split_rows(const WgradProblem& p);               // needs p.begin, p.end, p.in only
bool plain_takes_large_tile(int64_t large_tiles, int64_t slab_tokens, int compute_units);   // tile of the plain gradient
bool edge_rows_folded(const RowSplit& rs);                // the MFMA kernel carries the edge rows itself

// Tile of the plain MFMA gradient and of the FMA kernel: what the token split is chosen from.
constexpr int64_t kMainTileM = 256, kMainTileN = 256, kMainTileK = 32;
constexpr int64_t kSimtTileM = 64, kSimtTileN = 64, kSimtTileK = 16;

constexpr int kMaxDevices = 64;
constexpr int kDefaultComputeUnits = 256;                 // MI355X
int device_compute_units();                               // of the current device (kernels.hip)

// shape.cpp: pure functions of the shapes (and of the compute-unit count they are given)
bool mfma_path_ok(const WgradProblem& p);                 // alignment / shape rules of the MFMA kernel
Split pick_split(int32_t kind, int32_t dtype, int64_t out, int64_t in, int64_t T, int64_t begin,
                 int64_t end, int32_t forced, bool mfma, int compute_units);

// The fused call takes the 256 x 256 tile (one workgroup per compute unit) instead of the 128 x 256
// one (two per compute unit) when it is compute-bound and its operands are too large to stay in
// the last-level cache (shape.cpp).
bool fused_takes_large_tile(const WgradProblem& p, int compute_units);

// One segment of a grouped fused call: a bf16 matrix segment for the MFMA kernel (S = 1) or a
// bf16 scale-vector segment whose normalised input the caller supplies.
struct GroupSegment {
  WgradProblem p;
  Sinks s;
  bool vector;
};
// Whether the one-launch kernel can take this segment (else the caller runs it by itself).
bool group_takes_segment(const WgradProblem& p, bool vector);
// All segments in as few launches as the kernel's argument table allows (12 segments each).
int launch_fused_group(const GroupSegment* segs, int n, bool large_tile, void* stream);

// All launchers return a hipError_t as int (0 = success).
int launch_wgrad_bf16_mfma(const WgradProblem& p, int mode, const Sinks& s, void* stream);
int launch_wgrad_simt(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream);
int launch_colsum(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream);
// Scale vector of RMSNorm / LayerNorm with the normalisation done here: p.X is the raw input,
// stats is a device scratch of 2 * T floats.
int launch_norm_wgrad(const WgradProblem& p, int dtype, bool subtract_mean, float eps, float* stats, int mode,
                      const Sinks& s, void* stream);
// Embedding table: p.X holds the int64 token ids, p.dY is [T, in], the table is [out, in];
// at most kMaxEmbeddingTokens tokens per call.
constexpr int64_t kMaxEmbeddingTokens = 8192;
int launch_embed_wgrad(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream);
// g = sum over slabs (EMIT_STORE / EMIT_ACCUM) or AdamW on that sum (EMIT_ADAMW).
// W_at_begin is already offset to the first element.
int launch_reduce(const float* ws, int32_t S, int64_t E, int mode, const Sinks& s, void* W_at_begin,
                  void* stream);
// AdamW with the gradient read from g.
int launch_adamw(const float* g, int64_t n, const Sinks& s, void* W_at_begin, void* stream);

}  // namespace chunkft
#endif
