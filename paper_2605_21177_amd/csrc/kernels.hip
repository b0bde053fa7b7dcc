// gfx950 (CDNA4) kernels of the ChunkFT hot path.
//
//   wgrad_mfma_kernel   bf16 chunk-restricted weight gradient: LDS-staged dY and X
//                       token slabs, LDS transpose reads, 32x32x16 bf16 MFMA, fp32
//                       accumulators; epilogue stores g, a slab partial, or applies
//                       AdamW straight from the accumulators.
//   wgrad_simt_kernel   the same contraction with fp32 FMAs for the fp32 configuration
//                       and for shapes the MFMA kernel's 16-byte loads cannot take.
//   colsum_kernel       1-D scale-vector gradient sum_t dY[t,j] * X[t,j].
//   elementwise_kernel  AdamW over a chunk and/or the fixed-order sum of slab partials.
//
// The operations are those of the paper's Section 3.1 (gradient of the active
// slices only) and Algorithm 1 lines 19-21 (AdamW with the chunk's own counter).

#include <hip/hip_runtime.h>

#include <cstdint>

#include "internal.h"

namespace chunkft {

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));   // 16 bytes at any dword
typedef unsigned int u32x2_a8 __attribute__((ext_vector_type(2), aligned(8)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) {
  return __uint_as_float(((unsigned int)b) << 16);
}

template <typename T> __device__ __forceinline__ float load_as_f32(const T* p);
template <> __device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_f32<unsigned short>(const unsigned short* p) {
  return bf16_bits_to_f32(*p);
}

// One AdamW update in fp32 (Algorithm 1 lines 19-21).  Every path that updates
// state goes through this function so that fused and un-fused calls agree bit
// for bit; contraction is written out (the file is built with -ffp-contract=off).
__device__ __forceinline__ void adamw_update(float g, float& theta, float& m, float& v,
                                             const AdamWConsts& c) {
  const float m_new = fmaf(c.beta1, m, c.one_minus_beta1 * g);
  const float v_new = fmaf(c.beta2, v, c.one_minus_beta2 * (g * g));
  const float m_hat = m_new * c.inv_bias1;
  const float v_hat = v_new * c.inv_bias2;
  const float step = m_hat / (sqrtf(v_hat) + c.eps) + c.weight_decay * theta;
  theta = fmaf(-c.lr, step, theta);
  m = m_new;
  v = v_new;
}

// Turn one gradient value into its destination.  i = chunk-local index,
// flat = element index in the tensor, slab = token slab of a split call.
template <int MODE>
__device__ __forceinline__ void emit(const Sinks& s, int64_t E, int32_t slab, int64_t i,
                                     int64_t flat, float val) {
  if constexpr (MODE == EMIT_STORE) {
    s.g[i] = val;
  } else if constexpr (MODE == EMIT_ACCUM) {
    s.g[i] += val;
  } else if constexpr (MODE == EMIT_PARTIAL) {
    s.ws[(int64_t)slab * E + i] = val;
  } else {
    float th = s.master[i], mm = s.m[i], vv = s.v[i];
    adamw_update(val, th, mm, vv, s.c);
    s.master[i] = th;
    s.m[i] = mm;
    s.v[i] = vv;
    if (s.w_kind == W_BF16) ((unsigned short*)s.W)[flat] = f32_to_bf16_rne(th);
    else if (s.w_kind == W_F32) ((float*)s.W)[flat] = th;
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA weight-gradient kernel
// ---------------------------------------------------------------------------
// Row decomposition of the chunk [begin, end) of W [out, in]:
//   body rows [rb0, rb1): complete rows, rb0 a multiple of 8 (16-byte dY loads);
//   edge rows: the partial first row, the up-to-7 complete rows before rb0, and
//   the partial last row -- at most kMaxEdgeRows of them, computed by FMA.
struct MfmaParams {
  WgradProblem p;
  int64_t rb0, rb1;
  int32_t tiles_m, tiles_n;
  int32_t n_tile_items;        // tiles_m * tiles_n * S
  int32_t n_edge_items;        // column blocks of the edge rows (0 if no edge rows)
  int32_t n_edge_rows;
  int32_t group_m;
  int64_t edge_row[kMaxEdgeRows];
  Sinks s;
};

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
  static constexpr int NT = 64 * WM * WN;
  static constexpr int TM = BM / WM / 32;           // 32x32 blocks per wave along rows
  static constexpr int TN = BN / WN / 32;
  static constexpr int LDA = BM + 32;               // +64 B per LDS row: 8 rows of a transpose read hit all banks
  static constexpr int LDB = BN + 32;
  static constexpr int STAGE = BK * (LDA + LDB);    // bf16 elements per stage
  static constexpr int CA = BK * BM / 8 / NT;       // 16-byte pieces per thread per stage
  static constexpr int CB = BK * BN / 8 / NT;
  static constexpr int EDGE_COLS = 128;
  static constexpr int TG = NT / 64;                // token groups of the edge path
  static constexpr size_t LDS_MAIN = 2 * STAGE * 2;
  static constexpr size_t LDS_EDGE = (size_t)TG * kMaxEdgeRows * EDGE_COLS * 4;
  static constexpr size_t LDS_BYTES = LDS_MAIN > LDS_EDGE ? LDS_MAIN : LDS_EDGE;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 16 == 0, "tile shape");
  static_assert((BK * BM / 8) % NT == 0 && (BK * BN / 8) % NT == 0, "loader shape");
};

template <class C, int MODE>
__device__ __forceinline__ void edge_item(const MfmaParams& q, int item, unsigned short* lds_raw) {
  // One block of EDGE_COLS columns, all edge rows at once: every thread owns two
  // adjacent columns and a residue class of tokens; partial sums meet in LDS and
  // are added in token-group order.
  const WgradProblem& p = q.p;
  float* red = reinterpret_cast<float*>(lds_raw);           // [TG][kMaxEdgeRows][EDGE_COLS]
  const int lane = threadIdx.x & 63;
  const int tg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t c = (int64_t)item * C::EDGE_COLS + lane * 2;
  const unsigned short* X = (const unsigned short*)p.X;
  const unsigned short* dY = (const unsigned short*)p.dY;
  float acc[kMaxEdgeRows][2];
#pragma unroll
  for (int e = 0; e < kMaxEdgeRows; ++e) acc[e][0] = acc[e][1] = 0.f;
  if (c < p.in) {                                           // in % 8 == 0: both columns valid
    for (int64_t t = tg; t < p.T; t += C::TG) {
      const unsigned int xx = *(const unsigned int*)(X + t * p.ldx + c);
      const float x0 = __uint_as_float(xx << 16), x1 = __uint_as_float(xx & 0xffff0000u);
#pragma unroll
      for (int e = 0; e < kMaxEdgeRows; ++e) {
        if (e < q.n_edge_rows) {
          const float d = bf16_bits_to_f32(dY[t * p.lddy + q.edge_row[e]]);
          acc[e][0] = fmaf(d, x0, acc[e][0]);
          acc[e][1] = fmaf(d, x1, acc[e][1]);
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < kMaxEdgeRows; ++e) {
    red[(tg * kMaxEdgeRows + e) * C::EDGE_COLS + lane * 2 + 0] = acc[e][0];
    red[(tg * kMaxEdgeRows + e) * C::EDGE_COLS + lane * 2 + 1] = acc[e][1];
  }
  __syncthreads();
  const int64_t E = p.end - p.begin;
  for (int idx = threadIdx.x; idx < q.n_edge_rows * C::EDGE_COLS; idx += C::NT) {
    const int e = idx / C::EDGE_COLS, cc = idx % C::EDGE_COLS;
    const int64_t col = (int64_t)item * C::EDGE_COLS + cc;
    const int64_t flat = q.edge_row[e] * p.in + col;
    if (col < p.in && flat >= p.begin && flat < p.end) {
      float sum = red[(0 * kMaxEdgeRows + e) * C::EDGE_COLS + cc];
      for (int g = 1; g < C::TG; ++g) sum += red[(g * kMaxEdgeRows + e) * C::EDGE_COLS + cc];
      const int64_t i = flat - p.begin;
      if constexpr (MODE == EMIT_PARTIAL) {
        // the edge rows take all tokens at once: slab 0 carries the sum, the rest zero
        q.s.ws[i] = sum;
        for (int32_t sl = 1; sl < p.S; ++sl) q.s.ws[(int64_t)sl * E + i] = 0.f;
      } else {
        emit<MODE>(q.s, E, 0, i, flat, sum);
      }
    }
  }
}

template <class C, int MODE>
__global__ __launch_bounds__(C::NT) void wgrad_mfma_kernel(const MfmaParams q) {
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
  const WgradProblem& p = q.p;

  // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD one
  // contiguous run of work items so that tiles sharing dY rows / X columns
  // meet in the same L2.
  const int n_items = q.n_tile_items + q.n_edge_items;
  const int per_xcd = (n_items + 7) >> 3;
  const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (item >= n_items) return;
  if (item >= q.n_tile_items) {
    edge_item<C, MODE>(q, item - q.n_tile_items, lds);
    return;
  }

  // ---- which tile, which token slab
  const int n_tiles = q.tiles_m * q.tiles_n;
  const int slab = item / n_tiles;
  const int tile = item - slab * n_tiles;
  const int per_group = q.group_m * q.tiles_n;
  const int grp = tile / per_group;
  const int first_m = grp * q.group_m;
  const int gsz = (q.tiles_m - first_m < q.group_m) ? q.tiles_m - first_m : q.group_m;
  const int in_grp = tile - grp * per_group;
  const int tile_m = first_m + in_grp % gsz;
  const int tile_n = in_grp / gsz;
  const int64_t row0 = q.rb0 + (int64_t)tile_m * C::BM;
  const int64_t col0 = (int64_t)tile_n * C::BN;
  const int64_t k_begin = (int64_t)slab * p.kslab;
  const int64_t k_end = (k_begin + p.kslab < p.T) ? k_begin + p.kslab : p.T;
  const int nk = (int)((k_end - k_begin + C::BK - 1) / C::BK);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm0 = (wave / C::WN) * (C::BM / C::WM);
  const int wn0 = (wave % C::WN) * (C::BN / C::WN);

  const unsigned short* dY = (const unsigned short*)p.dY;
  const unsigned short* X = (const unsigned short*)p.X;

  // ---- global -> register staging: 16-byte pieces, rows of the tile contiguous
  uint4 ra[C::CA], rb[C::CB];
  auto fetch = [&](int kt) {
    const int64_t k0 = k_begin + (int64_t)kt * C::BK;
#pragma unroll
    for (int i = 0; i < C::CA; ++i) {
      const int id = tid + i * C::NT;
      const int kr = id / (C::BM / 8), mc = id % (C::BM / 8);
      const int64_t t = k0 + kr, r = row0 + mc * 8;
      ra[i] = (t < k_end && r < p.out) ? *(const uint4*)(dY + t * p.lddy + r) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < C::CB; ++i) {
      const int id = tid + i * C::NT;
      const int kr = id / (C::BN / 8), nc = id % (C::BN / 8);
      const int64_t t = k0 + kr, cc = col0 + nc * 8;
      rb[i] = (t < k_end && cc < p.in) ? *(const uint4*)(X + t * p.ldx + cc) : make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&](int stage) {
    unsigned short* A = lds + stage * C::STAGE;
    unsigned short* B = A + C::BK * C::LDA;
#pragma unroll
    for (int i = 0; i < C::CA; ++i) {
      const int id = tid + i * C::NT;
      const int kr = id / (C::BM / 8), mc = id % (C::BM / 8);
      *(uint4*)(A + kr * C::LDA + mc * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < C::CB; ++i) {
      const int id = tid + i * C::NT;
      const int kr = id / (C::BN / 8), nc = id % (C::BN / 8);
      *(uint4*)(B + kr * C::LDB + nc * 8) = rb[i];
    }
  };

  // ---- LDS transpose-read addressing.  In a block of 16 lanes, lane j reads 4
  // consecutive row indices of token (j / 4); the instruction hands lane i the 4
  // tokens of row index i.  Lanes 0-31 take tokens 0-7 of a 16-token step, lanes
  // 32-63 tokens 8-15: exactly the operand layout of the 32x32x16 MFMA.
  const int blk = lane >> 4, i16 = lane & 15;
  const int tr_k = (blk >> 1) * 8 + (i16 >> 2);
  const int tr_m = (blk & 1) * 16 + (i16 & 3) * 4;
  const int offA = tr_k * C::LDA + wm0 + tr_m;
  const int offB = tr_k * C::LDB + wn0 + tr_m;

  f32x16 acc[C::TM][C::TN];
#pragma unroll
  for (int a = 0; a < C::TM; ++a)
#pragma unroll
    for (int b = 0; b < C::TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  fetch(0);
  stash(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) fetch(kt + 1);
    const unsigned short* A = lds + (kt & 1) * C::STAGE;
    const unsigned short* B = A + C::BK * C::LDA;
#pragma unroll
    for (int ks = 0; ks < C::BK / 16; ++ks) {
      bf16x8 fa[C::TM], fb[C::TN];
#pragma unroll
      for (int a = 0; a < C::TM; ++a) {
        const unsigned short* src = A + offA + (ks * 16) * C::LDA + a * 32;
        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(src));
        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(src + 4 * C::LDA));
        fa[a] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int b = 0; b < C::TN; ++b) {
        const unsigned short* src = B + offB + (ks * 16) * C::LDB + b * 32;
        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(src));
        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(src + 4 * C::LDB));
        fb[b] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int a = 0; a < C::TM; ++a)
#pragma unroll
        for (int b = 0; b < C::TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    if (kt + 1 < nk) stash((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue.  Accumulator register v of a 32x32 block holds
  // row (v / 4) * 8 + (lane / 32) * 4 + v % 4, column lane % 32: for a fixed
  // register a half-wave covers 32 consecutive columns of one row (128 B of fp32).
  const int64_t E = p.end - p.begin;
  const bool interior = (row0 + C::BM <= q.rb1) && (col0 + C::BN <= p.in);
#pragma unroll
  for (int a = 0; a < C::TM; ++a) {
#pragma unroll
    for (int b = 0; b < C::TN; ++b) {
      const int64_t col = col0 + wn0 + b * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = row0 + wm0 + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (interior || (row < q.rb1 && col < p.in)) {
          const int64_t flat = row * p.in + col;
          emit<MODE>(q.s, E, slab, flat - p.begin, flat, acc[a][b][v]);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// FMA weight-gradient kernel (fp32 configuration and unaligned bf16 shapes)
// ---------------------------------------------------------------------------
struct SimtParams {
  WgradProblem p;
  int64_t r0;
  int32_t tiles_m, tiles_n;
  Sinks s;
};

template <typename T, int MODE>
__global__ __launch_bounds__(256) void wgrad_simt_kernel(const SimtParams q) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const WgradProblem& p = q.p;
  const int n_tiles = q.tiles_m * q.tiles_n;
  const int slab = blockIdx.x / n_tiles;
  const int tile = blockIdx.x - slab * n_tiles;
  const int tile_m = tile / q.tiles_n, tile_n = tile % q.tiles_n;
  const int64_t row0 = q.r0 + (int64_t)tile_m * BM;
  const int64_t col0 = (int64_t)tile_n * BN;
  const int64_t k_begin = (int64_t)slab * p.kslab;
  const int64_t k_end = (k_begin + p.kslab < p.T) ? k_begin + p.kslab : p.T;
  const T* dY = (const T*)p.dY;
  const T* X = (const T*)p.X;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * 256;
      const int kr = id >> 6, mm = id & 63;
      const int64_t t = k0 + kr;
      const int64_t r = row0 + mm, c = col0 + mm;
      As[kr][mm] = (t < k_end && r < p.out) ? load_as_f32<T>(dY + t * p.lddy + r) : 0.f;
      Bs[kr][mm] = (t < k_end && c < p.in) ? load_as_f32<T>(X + t * p.ldx + c) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  const int64_t E = p.end - p.begin;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = row0 + ty * 4 + i;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = col0 + tx * 4 + j;
      const int64_t flat = row * p.in + col;
      if (col < p.in && flat >= p.begin && flat < p.end)
        emit<MODE>(q.s, E, slab, flat - p.begin, flat, acc[i][j]);
    }
  }
}

// ---------------------------------------------------------------------------
// scale-vector gradient: g[j] = sum_t dY[t, j] * X[t, j]
// ---------------------------------------------------------------------------
template <typename T, int MODE>
__global__ __launch_bounds__(1024) void colsum_kernel(const WgradProblem p, const Sinks s) {
  constexpr int TG = 16;
  __shared__ float red[TG][64];
  const int lane = threadIdx.x & 63, tg = threadIdx.x >> 6;
  const int64_t j = p.begin + (int64_t)blockIdx.x * 64 + lane;
  const T* dY = (const T*)p.dY;
  const T* X = (const T*)p.X;
  float acc = 0.f;
  if (j < p.end)
    for (int64_t t = tg; t < p.T; t += TG)
      acc = fmaf(load_as_f32<T>(dY + t * p.lddy + j), load_as_f32<T>(X + t * p.ldx + j), acc);
  red[tg][lane] = acc;
  __syncthreads();
  if (tg == 0 && j < p.end) {
    float sum = red[0][lane];
    for (int g = 1; g < TG; ++g) sum += red[g][lane];
    emit<MODE>(s, p.end - p.begin, 0, j - p.begin, j, sum);
  }
}

// ---------------------------------------------------------------------------
// element-wise pass: AdamW and/or the sum of slab partials (HBM-bound)
// ---------------------------------------------------------------------------
struct ElemParams {
  const float* src;     // g (S = 0) or the slab partials [S][n]
  int32_t S;            // 0: src is g itself
  int64_t n;
  int64_t head;         // elements before the first 4-element group
  float* g_out;         // EMIT_STORE / EMIT_ACCUM
  float* master;
  float* m;
  float* v;
  void* W;              // already offset to element 0, or nullptr
  int32_t w_kind;
  AdamWConsts c;
};

template <int MODE>
__device__ __forceinline__ void elem_one(const ElemParams& q, int64_t i) {
  float val;
  if (q.S == 0) {
    val = q.src[i];
  } else {
    val = q.src[i];
    for (int32_t sl = 1; sl < q.S; ++sl) val += q.src[(int64_t)sl * q.n + i];
  }
  if constexpr (MODE == EMIT_STORE) {
    q.g_out[i] = val;
  } else if constexpr (MODE == EMIT_ACCUM) {
    q.g_out[i] += val;
  } else {
    float th = q.master[i], mm = q.m[i], vv = q.v[i];
    adamw_update(val, th, mm, vv, q.c);
    q.master[i] = th;
    q.m[i] = mm;
    q.v[i] = vv;
    if (q.w_kind == W_BF16) ((unsigned short*)q.W)[i] = f32_to_bf16_rne(th);
    else if (q.w_kind == W_F32) ((float*)q.W)[i] = th;
  }
}

template <int MODE>
__global__ __launch_bounds__(256) void elementwise_kernel(const ElemParams q) {
  const int64_t nvec = (q.n - q.head) >> 2;
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    // the few elements before and after the 4-element groups
    const int64_t tail0 = q.head + (nvec << 2);
    const int64_t i = threadIdx.x < 4 ? (int64_t)threadIdx.x : tail0 + (threadIdx.x - 4);
    const bool ok = threadIdx.x < 4 ? (i < q.head) : (i < q.n);
    if (ok) elem_one<MODE>(q, i);
  }
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < nvec; j += stride) {
    const int64_t i = q.head + (j << 2);
    f32x4_u val = *(const f32x4_u*)(q.src + i);
    for (int32_t sl = 1; sl < q.S; ++sl) {
      const f32x4_u part = *(const f32x4_u*)(q.src + (int64_t)sl * q.n + i);
      val += part;
    }
    if constexpr (MODE == EMIT_STORE) {
      *(f32x4_u*)(q.g_out + i) = val;
    } else if constexpr (MODE == EMIT_ACCUM) {
      f32x4_u old = *(const f32x4_u*)(q.g_out + i);
      old += val;
      *(f32x4_u*)(q.g_out + i) = old;
    } else {
      f32x4_u th = *(const f32x4_u*)(q.master + i);
      f32x4_u mm = *(const f32x4_u*)(q.m + i);
      f32x4_u vv = *(const f32x4_u*)(q.v + i);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float t = th[e], a = mm[e], b = vv[e];
        adamw_update(val[e], t, a, b, q.c);
        th[e] = t; mm[e] = a; vv[e] = b;
      }
      *(f32x4_u*)(q.master + i) = th;
      *(f32x4_u*)(q.m + i) = mm;
      *(f32x4_u*)(q.v + i) = vv;
      if (q.w_kind == W_BF16) {
        // head was chosen so that this address is 8-byte aligned
        u32x2_a8 pk;
        pk[0] = (unsigned int)f32_to_bf16_rne(th[0]) | ((unsigned int)f32_to_bf16_rne(th[1]) << 16);
        pk[1] = (unsigned int)f32_to_bf16_rne(th[2]) | ((unsigned int)f32_to_bf16_rne(th[3]) << 16);
        *(u32x2_a8*)((unsigned short*)q.W + i) = pk;
      } else if (q.w_kind == W_F32) {
        *(f32x4_u*)((float*)q.W + i) = th;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {

constexpr int kNumCU = 256;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

using MainCfg = TileCfg<256, 256, 32, 2, 4>;   // 512 threads, wave tile 128 x 64

struct RowSplit {
  int64_t rb0, rb1;
  int n_edge;
  int64_t edge_row[kMaxEdgeRows];
};

RowSplit split_rows(const WgradProblem& p) {
  RowSplit rs{};
  const int64_t r0 = p.begin / p.in, c0 = p.begin % p.in;
  const int64_t r1 = (p.end - 1) / p.in, c1 = (p.end - 1) % p.in + 1;
  const int64_t full0 = r0 + (c0 != 0 ? 1 : 0);           // first complete row
  const int64_t full1 = r1 + 1 - (c1 != p.in ? 1 : 0);    // one past the last complete row
  int64_t rb0 = (full0 + 7) / 8 * 8;
  int64_t rb1 = full1;
  if (rb1 <= rb0) { rb0 = rb1 = 0; }
  rs.rb0 = rb0;
  rs.rb1 = rb1;
  // edge rows: everything in [r0, r1] outside [rb0, rb1)
  int n = 0;
  if (rb1 > rb0) {
    for (int64_t r = r0; r < rb0; ++r) rs.edge_row[n++] = r;
    for (int64_t r = rb1; r <= r1; ++r) rs.edge_row[n++] = r;
  } else {
    for (int64_t r = r0; r <= r1; ++r) rs.edge_row[n++] = r;   // caller guarantees <= kMaxEdgeRows
  }
  rs.n_edge = n;
  return rs;
}

template <class C, int MODE>
int launch_mfma_mode(const MfmaParams& q, int grid, hipStream_t st) {
  static bool attr_set = false;   // raising the dynamic LDS limit is idempotent; a race only repeats it
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)wgrad_mfma_kernel<C, MODE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  hipLaunchKernelGGL((wgrad_mfma_kernel<C, MODE>), dim3(grid), dim3(C::NT), C::LDS_BYTES, st, q);
  return (int)hipGetLastError();
}

}  // namespace

bool mfma_path_ok(const WgradProblem& p) {
  const auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
  if (!(p.in % 8 == 0 && p.out % 8 == 0 && p.ldx % 8 == 0 && p.lddy % 8 == 0 && a16(p.X) && a16(p.dY)))
    return false;
  // rows outside the 8-aligned body must fit the edge path
  const int64_t r0 = p.begin / p.in, r1 = (p.end - 1) / p.in;
  const int64_t c0 = p.begin % p.in, c1 = (p.end - 1) % p.in + 1;
  const int64_t full0 = r0 + (c0 != 0 ? 1 : 0), full1 = r1 + 1 - (c1 != p.in ? 1 : 0);
  const int64_t rb0 = (full0 + 7) / 8 * 8;
  if (full1 <= rb0) return (r1 - r0 + 1) <= kMaxEdgeRows;
  return true;
}

Split pick_split(int32_t kind, int32_t dtype, int64_t out, int64_t in, int64_t T, int64_t begin,
                 int64_t end, int32_t forced, bool mfma) {
  (void)out; (void)dtype;
  if (kind != 0) return {1, T};                       // scale vectors are never split
  const int64_t bm = mfma ? MainCfg::BM : 64, bn = mfma ? MainCfg::BN : 64;
  const int64_t bk = mfma ? MainCfg::BK : 16;
  int64_t S = forced;
  if (S <= 0) {
    const int64_t rows = (end - 1) / in - begin / in + 1;
    const int64_t tiles = ceil_div(rows, bm) * ceil_div(in, bn);
    S = 1;
    if (mfma && tiles < kNumCU) {
      S = (2 * kNumCU) / tiles;                       // about two work items per CU
      const int64_t max_by_len = T / 256 > 0 ? T / 256 : 1;   // keep slabs of >= 256 tokens
      if (S > max_by_len) S = max_by_len;
      if (S > 64) S = 64;
      if (S < 1) S = 1;
    }
  }
  int64_t kslab = ceil_div(ceil_div(T, S), bk) * bk;
  S = ceil_div(T, kslab);                             // no empty slab
  return {(int32_t)S, kslab};
}

int launch_wgrad_bf16_mfma(const WgradProblem& p, int mode, const Sinks& s, void* stream) {
  using C = MainCfg;
  MfmaParams q{};
  q.p = p;
  q.s = s;
  const RowSplit rs = split_rows(p);
  q.rb0 = rs.rb0;
  q.rb1 = rs.rb1;
  q.n_edge_rows = rs.n_edge;
  for (int e = 0; e < kMaxEdgeRows; ++e) q.edge_row[e] = e < rs.n_edge ? rs.edge_row[e] : 0;
  q.tiles_m = (int32_t)ceil_div(rs.rb1 - rs.rb0, C::BM);
  q.tiles_n = (int32_t)ceil_div(p.in, C::BN);
  q.n_tile_items = q.tiles_m * q.tiles_n * p.S;
  q.n_edge_items = rs.n_edge > 0 ? (int32_t)ceil_div(p.in, C::EDGE_COLS) : 0;
  q.group_m = 8;
  const int n_items = q.n_tile_items + q.n_edge_items;
  const int grid = (n_items + 7) / 8 * 8;
  hipStream_t st = (hipStream_t)stream;
  switch (mode) {
    case EMIT_STORE: return launch_mfma_mode<C, EMIT_STORE>(q, grid, st);
    case EMIT_ACCUM: return launch_mfma_mode<C, EMIT_ACCUM>(q, grid, st);
    case EMIT_PARTIAL: return launch_mfma_mode<C, EMIT_PARTIAL>(q, grid, st);
    default: return launch_mfma_mode<C, EMIT_ADAMW>(q, grid, st);
  }
}

template <typename T>
static int launch_simt_t(const SimtParams& q, int grid, int mode, hipStream_t st) {
  switch (mode) {
    case EMIT_STORE: hipLaunchKernelGGL((wgrad_simt_kernel<T, EMIT_STORE>), dim3(grid), dim3(256), 0, st, q); break;
    case EMIT_ACCUM: hipLaunchKernelGGL((wgrad_simt_kernel<T, EMIT_ACCUM>), dim3(grid), dim3(256), 0, st, q); break;
    case EMIT_PARTIAL: hipLaunchKernelGGL((wgrad_simt_kernel<T, EMIT_PARTIAL>), dim3(grid), dim3(256), 0, st, q); break;
    default: hipLaunchKernelGGL((wgrad_simt_kernel<T, EMIT_ADAMW>), dim3(grid), dim3(256), 0, st, q); break;
  }
  return (int)hipGetLastError();
}

int launch_wgrad_simt(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream) {
  SimtParams q{};
  q.p = p;
  q.s = s;
  q.r0 = p.begin / p.in;
  const int64_t rows = (p.end - 1) / p.in - q.r0 + 1;
  q.tiles_m = (int32_t)ceil_div(rows, 64);
  q.tiles_n = (int32_t)ceil_div(p.in, 64);
  const int64_t grid = (int64_t)q.tiles_m * q.tiles_n * p.S;
  if (grid > 0x7fffffff) return (int)hipErrorInvalidValue;
  hipStream_t st = (hipStream_t)stream;
  return dtype == 0 ? launch_simt_t<float>(q, (int)grid, mode, st)
                    : launch_simt_t<unsigned short>(q, (int)grid, mode, st);
}

template <typename T>
static int launch_colsum_t(const WgradProblem& p, int grid, int mode, const Sinks& s, hipStream_t st) {
  switch (mode) {
    case EMIT_STORE: hipLaunchKernelGGL((colsum_kernel<T, EMIT_STORE>), dim3(grid), dim3(1024), 0, st, p, s); break;
    case EMIT_ACCUM: hipLaunchKernelGGL((colsum_kernel<T, EMIT_ACCUM>), dim3(grid), dim3(1024), 0, st, p, s); break;
    default: hipLaunchKernelGGL((colsum_kernel<T, EMIT_ADAMW>), dim3(grid), dim3(1024), 0, st, p, s); break;
  }
  return (int)hipGetLastError();
}

int launch_colsum(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream) {
  const int64_t grid = ceil_div(p.end - p.begin, 64);
  if (grid > 0x7fffffff) return (int)hipErrorInvalidValue;
  hipStream_t st = (hipStream_t)stream;
  return dtype == 0 ? launch_colsum_t<float>(p, (int)grid, mode, s, st)
                    : launch_colsum_t<unsigned short>(p, (int)grid, mode, s, st);
}

static int launch_elem(ElemParams& q, int mode, hipStream_t st) {
  // the first 4-element group starts where the low-precision store is 8-byte
  // aligned (bf16), else where the fp32 state is 16-byte aligned
  int64_t head;
  if (q.w_kind == W_BF16 && mode == EMIT_ADAMW)
    head = ((8 - (reinterpret_cast<uintptr_t>(q.W) & 7u)) & 7u) / 2;
  else {
    const void* ref = mode == EMIT_ADAMW ? (const void*)q.master : (const void*)q.g_out;
    head = ((16 - (reinterpret_cast<uintptr_t>(ref) & 15u)) & 15u) / 4;
  }
  if (head > q.n) head = q.n;
  q.head = head;
  const int64_t nvec = (q.n - head) >> 2;
  int64_t blocks = ceil_div(nvec, 256);
  const int64_t cap = (int64_t)kNumCU * 16;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  switch (mode) {
    case EMIT_STORE: hipLaunchKernelGGL((elementwise_kernel<EMIT_STORE>), dim3((int)blocks), dim3(256), 0, st, q); break;
    case EMIT_ACCUM: hipLaunchKernelGGL((elementwise_kernel<EMIT_ACCUM>), dim3((int)blocks), dim3(256), 0, st, q); break;
    default: hipLaunchKernelGGL((elementwise_kernel<EMIT_ADAMW>), dim3((int)blocks), dim3(256), 0, st, q); break;
  }
  return (int)hipGetLastError();
}

int launch_reduce(const float* ws, int32_t S, int64_t E, int mode, const Sinks& s, void* W_at_begin,
                  void* stream) {
  ElemParams q{};
  q.src = ws;
  q.S = S;
  q.n = E;
  q.g_out = s.g;
  q.master = s.master;
  q.m = s.m;
  q.v = s.v;
  q.W = W_at_begin;
  q.w_kind = W_at_begin ? s.w_kind : W_NONE;
  q.c = s.c;
  return launch_elem(q, mode, (hipStream_t)stream);
}

int launch_adamw(const float* g, int64_t n, const Sinks& s, void* W_at_begin, void* stream) {
  ElemParams q{};
  q.src = g;
  q.S = 0;
  q.n = n;
  q.master = s.master;
  q.m = s.m;
  q.v = s.v;
  q.W = W_at_begin;
  q.w_kind = W_at_begin ? s.w_kind : W_NONE;
  q.c = s.c;
  return launch_elem(q, EMIT_ADAMW, (hipStream_t)stream);
}

}  // namespace chunkft
