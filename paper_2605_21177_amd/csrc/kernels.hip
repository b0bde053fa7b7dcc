// gfx950 (CDNA4) kernels of the ChunkFT hot path.
//
//   wgrad_mfma_kernel   bf16 chunk-restricted weight gradient: LDS-staged dY and X
//                       token slabs, LDS transpose reads, 32x32x16 bf16 MFMA, fp32
//                       accumulators; epilogue stores g, a slab partial, or applies
//                       AdamW straight from the accumulators.
//   wgrad_simt_kernel   the same contraction with fp32 FMAs for the fp32 configuration
//                       and for shapes the MFMA kernel's 16-byte loads cannot take.
//   wgrad_edge_kernel   the up-to-9 partial / unaligned rows of a chunk that has too few
//                       rows for the MFMA kernel to carry them (plain FMA).
//   colsum_kernel       1-D scale-vector gradient sum_t dY[t,j] * X[t,j], X normalised by the
//                       caller or here (norm_stats_kernel: per-token mean and 1/std).
//   embed_wgrad_kernel  embedding table gradient: per table row the sum of the dY rows of
//                       the tokens that name it, in token order.
//   elementwise_kernel  AdamW over a chunk and/or the fixed-order sum of slab partials.
//
// The operations are those of the paper's Section 3.1 (gradient of the active
// slices only, through the chunk-aware operators of Algorithm 1 line 8) and
// Algorithm 1 lines 19-21 (AdamW with the chunk's own counter).

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstdlib>

#include "internal.h"

namespace chunkft {

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));   // 16 bytes at any dword
typedef unsigned int u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));   // 8 bytes at any bf16
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// Compile-time loop: the body sees its index as a constant, so register arrays
// indexed by it never fall back to scratch memory.
template <int I> struct IntC { static constexpr int value = I; };
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(IntC<I>{});
    static_for<N, I + 1>(f);
  }
}

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
// The last line is theta - lr * (m_hat / (sqrt(v_hat) + eps) + wd * theta).
__device__ __forceinline__ void adamw_update(float g, float& theta, float& m, float& v,
                                             const AdamWConsts& c) {
  const float m_new = fmaf(c.beta1, m, c.one_minus_beta1 * g);
  const float v_new = fmaf(c.beta2, v, c.one_minus_beta2 * (g * g));
  const float m_hat = m_new * c.inv_bias1;
  const float v_hat = v_new * c.inv_bias2;
  // v_sqrt_f32 and v_rcp_f32 are accurate to 1 ulp: far inside the 1e-5 the update is held to,
  // and an order of magnitude fewer instructions than the correctly rounded sequences
  const float step = fmaf(m_hat, __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v_hat) + c.eps), c.weight_decay * theta);
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
    s.ws[(int64_t)slab * s.ws_pitch + i] = val;
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

// Four consecutive gradient values at once.  The 16-byte fp32 accesses work at
// any 4-byte alignment but stream about 15% faster when 16-byte aligned, whereas
// the 8-byte bf16 store costs next to nothing at 2-byte alignment: callers align
// their groups of four to the fp32 arrays.  Pointers are already offset to the
// first of the four elements.
struct Vec4Sink {
  float* g;        // EMIT_STORE / EMIT_ACCUM / EMIT_PARTIAL destination
  float* master;
  float* m;
  float* v;
  void* W;         // low-precision copy (bf16 or fp32) or nullptr
};

// Chunk state and gradients are streamed: read once, written once, never reused
// by the same kernel, and far larger than the caches.  All these accesses carry
// the non-temporal hint.
struct State4 {
  f32x4_u th, mm, vv;
};

template <int MODE>
__device__ __forceinline__ State4 load_state4(const Vec4Sink& d) {
  State4 st;
  if constexpr (MODE == EMIT_ACCUM) {
    st.th = __builtin_nontemporal_load((const f32x4_u*)d.g);
  } else if constexpr (MODE == EMIT_ADAMW) {
    st.th = __builtin_nontemporal_load((const f32x4_u*)d.master);
    st.mm = __builtin_nontemporal_load((const f32x4_u*)d.m);
    st.vv = __builtin_nontemporal_load((const f32x4_u*)d.v);
  }
  return st;
}

template <int MODE>
__device__ __forceinline__ void finish4(const Vec4Sink& d, int w_kind, const AdamWConsts& c, f32x4_u val,
                                        State4 st) {
  if constexpr (MODE == EMIT_STORE || MODE == EMIT_PARTIAL) {
    // the gradient is read again by the next kernel (AdamW or the slab reduction):
    // a plain store lets the 256 MB memory-side cache keep it
    *(f32x4_u*)d.g = val;
  } else if constexpr (MODE == EMIT_ACCUM) {
    st.th += val;
    *(f32x4_u*)d.g = st.th;
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t = st.th[e], a = st.mm[e], b = st.vv[e];
      adamw_update(val[e], t, a, b, c);
      st.th[e] = t; st.mm[e] = a; st.vv[e] = b;
    }
    __builtin_nontemporal_store(st.th, (f32x4_u*)d.master);
    __builtin_nontemporal_store(st.mm, (f32x4_u*)d.m);
    __builtin_nontemporal_store(st.vv, (f32x4_u*)d.v);
    if (w_kind == W_BF16) {
      u32x2_a2 pk;
      pk[0] = (unsigned int)f32_to_bf16_rne(st.th[0]) | ((unsigned int)f32_to_bf16_rne(st.th[1]) << 16);
      pk[1] = (unsigned int)f32_to_bf16_rne(st.th[2]) | ((unsigned int)f32_to_bf16_rne(st.th[3]) << 16);
      __builtin_nontemporal_store(pk, (u32x2_a2*)d.W);
    } else if (w_kind == W_F32) {
      __builtin_nontemporal_store(st.th, (f32x4_u*)d.W);
    }
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA weight-gradient kernel
// ---------------------------------------------------------------------------
// Row decomposition of the chunk [begin, end) of W [out, in]:
//   body rows [rb0, rb1): complete rows, rb0 a multiple of 8 (16-byte dY loads),
//   computed by the MFMA kernel with no range mask beyond the row bound;
//   edge rows: the partial first row, the up-to-7 complete rows before rb0, and
//   the partial last row -- at most kMaxEdgeRows of them.  The workgroups of the
//   first tile row, which stream every X column tile anyway, carry them as one
//   extra 32-row MFMA block; only when the body has at most 128 rows (a chunk of a
//   few rows) does the small FMA edge kernel compute them.
// Diagnostic build only (-DCHUNKFT_TIMELINE, a library of its own: libchunkft_timeline.so): every
// workgroup of the MFMA kernel notes when it starts, when the first fragments of its tile are in
// registers, when its loop ends and when its epilogue ends (the 100 MHz constant counter), and where
// it ran, in 8 words per work item of a buffer that the caller hands over with
// chunkft_timeline_buffer().  The product library has none of this.
#ifdef CHUNKFT_TIMELINE
static unsigned long long* g_timeline = nullptr;
static size_t g_timeline_words = 0;
extern "C" int chunkft_timeline_buffer(void* device_buffer, size_t bytes) {
  g_timeline = static_cast<unsigned long long*>(device_buffer);
  g_timeline_words = bytes / 8;
  return 0;
}
#define TIMELINE_STAMP(q, item, k)                                                                  \
  do {                                                                                              \
    if ((q).timeline && threadIdx.x == 0) (q).timeline[(size_t)(item) * 8 + (k)] = __builtin_amdgcn_s_memrealtime(); \
  } while (0)
#else
#define TIMELINE_STAMP(q, item, k) do { } while (0)
#endif

struct MfmaParams {
  WgradProblem p;
  int64_t rb0, rb1;
  int32_t tiles_m, tiles_n;
  int32_t n_tile_items;        // tiles_m * tiles_n * S
  int32_t group_m;
  int32_t stagger;             // start delay of every second resident workgroup, in units of 8128 cycles
  int64_t lead_base;           // edge rows folded into the first tile row (-1: none), as in EdgeParams
  int64_t trail_row;
  Sinks s;
#ifdef CHUNKFT_TIMELINE
  unsigned long long* timeline;
#endif
};

struct EdgeParams {
  WgradProblem p;
  int64_t lead_base;   // first row of the 8-row group that holds the leading edge rows, or -1
  int64_t trail_row;   // the partial last row, or -1
  Sinks s;
};

// Tile configuration of the MFMA kernel: a (128 WM) x 256 output tile per workgroup
// of 4 WM waves (WM x 4, each wave 128 x 64 = 4 x 2 blocks of 32 x 32), tokens in
// slabs of 32, and a ring of NS slabs in LDS filled by global->LDS loads.
//   WM = 1, NS = 3: 128 x 256 tiles, 4 waves, 75 KB of LDS -- two workgroups share a
//   compute unit, so the store-bound epilogue of one runs under the MFMA loop of the other;
//   WM = 2, NS = 4: 256 x 256 tiles, 8 waves, 132 KB -- one workgroup per compute unit,
//   a third less operand traffic per flop.
template <int WM_, int NS_, int MI_ = 32>
struct RingCfg {
  static constexpr int WM = WM_, WN = 4, BM = 128 * WM, BN = 256, BK = 32, NS = NS_;
  static constexpr int MI = MI_;                      // MFMA shape: 32 (32x32x16) or 16 (16x16x32)
  static constexpr int NW = WM * WN, NT = 64 * NW;
  static constexpr int TM = BM / WM / MI, TN = BN / WN / MI;
  static constexpr int A_BYTES = BK * BM * 2, B_BYTES = BK * BN * 2;
  // edge block: per token 16 row values = the 8-row group of the leading edge rows and
  // the 8-row group that holds the trailing row (32 B per token, 1 KB per slab)
  static constexpr int E_BYTES = BK * 32;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES + E_BYTES;
  static constexpr int LA = A_BYTES / 1024 / NW;     // 1 KB wave-loads per wave per slab
  static constexpr int LB = B_BYTES / 1024 / NW;
  static constexpr int L = LA + LB;
  // epilogue staging: half a tile (BM / 2 rows x 256 columns of fp32) at a time; a row
  // pitch of 264 floats puts the two half-waves of a ds_write_b32 on disjoint banks
  // (with the 16 x 16 blocks of the other MFMA shape a write spans four row groups: 260 floats spread them)
  static constexpr int EPI_PITCH = MI == 32 ? BN + 8 : BN + 4;
  static constexpr size_t EPI_BYTES = (size_t)(BM / 2) * EPI_PITCH * 4;
  static constexpr size_t RING_BYTES = (size_t)NS * STAGE_BYTES;
  static constexpr size_t LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
  static constexpr int RA = BM * 2, RB = BN * 2;     // bytes of one token in the A / B image of a slab
  static_assert((MI == 32 || MI == 16) && TM * MI == 128 && TN * MI == 64 && (WM == 1 || WM == 2) && L >= 4 &&
                    L <= 6 && NS >= 3,
                "the main loops are written out for this shape");
};

// Edge rows of a chunk whose body is too short to carry them in the MFMA kernel: the leading ones all
// lie in one 8-aligned group of rows (one 16-byte piece of dY per token), the trailing one is a single
// row.  A block is 32 columns over all tokens, done by 512 (token group, 8-column group) pairs -- 8
// "virtual waves" of 64 lanes, lane l = 8-column group l % 4 of token group 16 vw + l / 4, tokens
// t = token group (mod 128) in ascending order: per token one 16-byte piece of X, one of dY and the
// trailing row's value feed 72 FMAs (with one column and 2-byte loads per lane the kernel was bound by
// its load instructions: 300 us at 4096 tokens, eight times what it takes now).  The 16 token groups
// of a virtual wave are added by a butterfly over the lanes, the 8 virtual waves meet in LDS and are
// added in order.  A workgroup of NT threads takes the virtual waves NT / 64 at a time; the sums do not
// depend on NT.
constexpr int kEdgeCols = 32;
constexpr int kEdgeVW = 8;                        // virtual waves per block
constexpr int kEdgeTG = 16 * kEdgeVW;             // token groups
constexpr int kEdgeThreads = 64 * kEdgeVW;
constexpr int kEdgeUnroll = 4;

template <int NT, int MODE>
__device__ __forceinline__ void edge_rows_block(const WgradProblem& p, const Sinks& s, const int64_t lead_base,
                                                const int64_t trail_row, const int64_t block,
                                                float (*red)[kMaxEdgeRows][kEdgeCols]) {
  static_assert(NT % 64 == 0 && kEdgeThreads % NT == 0, "whole virtual waves per pass");
  const unsigned short* X = (const unsigned short*)p.X;
  const unsigned short* dY = (const unsigned short*)p.dY;
  const bool has_lead = lead_base >= 0, has_trail = trail_row >= 0;
  const int lane = threadIdx.x & 63;
  const int cg = lane & 3, tgl = lane >> 2;
  const int64_t col8 = block * kEdgeCols + cg * 8;               // in % 8 == 0: a group of 8 columns is whole or absent
  const bool col_ok = col8 < p.in;
  for (int vw = threadIdx.x >> 6; vw < kEdgeVW; vw += NT / 64) {
    float acc[kMaxEdgeRows][8];
#pragma unroll
    for (int e = 0; e < kMaxEdgeRows; ++e)
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[e][c] = 0.f;
    for (int64_t t0 = vw * 16 + tgl; t0 < p.T; t0 += (int64_t)kEdgeTG * kEdgeUnroll) {
      uint4 xs[kEdgeUnroll], ld[kEdgeUnroll];
      unsigned short tr[kEdgeUnroll];
#pragma unroll
      for (int u = 0; u < kEdgeUnroll; ++u) {
        const int64_t t = t0 + (int64_t)u * kEdgeTG;
        const bool ok = t < p.T && col_ok;
        xs[u] = ok ? *(const uint4*)(X + t * p.ldx + col8) : make_uint4(0, 0, 0, 0);
        ld[u] = (ok && has_lead) ? *(const uint4*)(dY + t * p.lddy + lead_base) : make_uint4(0, 0, 0, 0);
        tr[u] = (ok && has_trail) ? dY[t * p.lddy + trail_row] : (unsigned short)0;
      }
#pragma unroll
      for (int u = 0; u < kEdgeUnroll; ++u) {
        const unsigned int xw[4] = {xs[u].x, xs[u].y, xs[u].z, xs[u].w};
        const unsigned int dw[4] = {ld[u].x, ld[u].y, ld[u].z, ld[u].w};
        float x[8], d[kMaxEdgeRows];
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          x[2 * h] = __uint_as_float(xw[h] << 16);
          x[2 * h + 1] = __uint_as_float(xw[h] & 0xffff0000u);
          d[2 * h] = __uint_as_float(dw[h] << 16);
          d[2 * h + 1] = __uint_as_float(dw[h] & 0xffff0000u);
        }
        d[8] = bf16_bits_to_f32(tr[u]);
#pragma unroll
        for (int e = 0; e < kMaxEdgeRows; ++e)
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[e][c] = fmaf(d[e], x[c], acc[e][c]);
      }
    }
    // the 16 token groups of this virtual wave: lanes that differ in bits 2-5
#pragma unroll
    for (int e = 0; e < kMaxEdgeRows; ++e)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float v = acc[e][c];
        v += __shfl_xor(v, 4);
        v += __shfl_xor(v, 8);
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        if (tgl == 0) red[vw][e][cg * 8 + c] = v;
      }
  }
  __syncthreads();
  for (int o = threadIdx.x; o < kMaxEdgeRows * kEdgeCols; o += NT) {
    const int e = o / kEdgeCols, c = o & (kEdgeCols - 1);
    const int64_t col = block * kEdgeCols + c;
    const int64_t row = e < 8 ? (has_lead ? lead_base + e : -1) : trail_row;   // -1: nothing to emit
    const int64_t flat = row * p.in + col;
    if (col < p.in && row >= 0 && flat >= p.begin && flat < p.end) {
      float sum = red[0][e][c];
      for (int g = 1; g < kEdgeVW; ++g) sum += red[g][e][c];
      const int64_t E = p.end - p.begin, i = flat - p.begin;
      if constexpr (MODE == EMIT_PARTIAL) {
        // the edge rows take all tokens at once: slab 0 carries the sum, the rest zero
        s.ws[i] = sum;
        for (int32_t sl = 1; sl < p.S; ++sl) s.ws[(int64_t)sl * s.ws_pitch + i] = 0.f;
      } else {
        emit<MODE>(s, E, 0, i, flat, sum);
      }
    }
  }
}

template <int MODE>
__global__ __launch_bounds__(kEdgeThreads) void wgrad_edge_kernel(const EdgeParams q) {
  __shared__ float red[kEdgeVW][kMaxEdgeRows][kEdgeCols];
  edge_rows_block<kEdgeThreads, MODE>(q.p, q.s, q.lead_base, q.trail_row, blockIdx.x, red);
}


// LDS transpose read issued as opaque assembly: the compiler must not know that
// it reads LDS, or it would wait for every outstanding global->LDS load before
// it.  The counterpart is that waiting for its result is also done by hand
// (WAIT_HALVES below).
template <int OFF>
__device__ __forceinline__ bf16x4 lds_tr_read(unsigned addr) {
  bf16x4 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
  return r;
}
// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, others "no wait")
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}
#define WAIT_HALVES(h)                                                                                   \
  asm volatile("s_waitcnt lgkmcnt(0)"                                                                    \
               : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]),     \
                 "+v"(h[7]), "+v"(h[8]), "+v"(h[9]), "+v"(h[10]), "+v"(h[11])::"memory")

#define WAIT_HALVES_E(h, he)                                                                             \
  asm volatile("s_waitcnt lgkmcnt(0)"                                                                    \
               : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]),     \
                 "+v"(h[7]), "+v"(h[8]), "+v"(h[9]), "+v"(h[10]), "+v"(h[11]), "+v"(he[0]), "+v"(he[1])::"memory")

// Epilogue of one tile of the MFMA kernels.  Accumulator register v of a 32x32 block holds
// row (v / 4) * 8 + (lane / 32) * 4 + v % 4, column lane % 32 -- a layout that
// could only be stored 4 bytes per lane.  The tile is therefore staged through
// LDS (the ring is free by now), half of it at a time, and leaves as whole rows:
// a wave handles one row of 256 columns per trip, 16 bytes per lane, 1 KB per
// instruction, for the gradient as well as for the AdamW state.
// stage_half(h, stage, sft) writes the wave's share of half h into the staging area; emit_edge(E) emits
// the edge block's elements (both know the accumulator layout of the MFMA shape in use).
template <class C, int MODE, class StageHalf, class EmitEdge>
__device__ __forceinline__ void tile_epilogue(const MfmaParams& q, unsigned char* ldsb, int64_t row0, int64_t col0,
                                              int slab, int wave, int lane, int tid,
                                              StageHalf&& stage_half, EmitEdge&& emit_edge) {
  const WgradProblem& p = q.p;
  const int wn0 = (wave % C::WN) * (C::BN / C::WN);
  const int64_t E = p.end - p.begin;
  const int64_t origin = row0 * p.in + col0 - p.begin;             // chunk-local index of the tile corner
  const int rows_valid = (int)((q.rb1 - row0 < C::BM) ? q.rb1 - row0 : C::BM);
  const int cols_valid = (int)((p.in - col0 < C::BN) ? p.in - col0 : C::BN);
  float* const stage = reinterpret_cast<float*>(ldsb);
  const int wmi = wave / C::WN;
  constexpr int WR = C::BM / C::WM / 2;   // rows of one wave row in a staged half
  constexpr int HALF_ROWS = C::WM * WR;   // rows staged per pass
  float* const g_dst = MODE == EMIT_PARTIAL ? q.s.ws + (int64_t)slab * q.s.ws_pitch : q.s.g;
  // Groups of four columns start where the fp32 destination is 16-byte aligned:
  // at tile-local column delta (the same for every row, because in % 8 == 0).
  // The delta leading and 4 - delta trailing columns of a row that are left over
  // are taken one element per thread (128 rows x 4 = 512 of them per half tile).
  const float* const align_ref = MODE == EMIT_ADAMW ? q.s.master : g_dst;
  const int delta = (int)((4 - ((reinterpret_cast<uintptr_t>(align_ref) >> 2) + (uint64_t)origin) % 4) % 4);
  const int c4 = delta + lane * 4;
  const bool vec_lane = delta == 0 || lane < 63;
  // The staged copy of a row is shifted right by sft columns, so that the groups of four
  // that start at column delta sit on 16-byte boundaries in LDS too: one conflict-free
  // 16-byte read per lane (the row pitch leaves room for the shift).
  const int sft = (4 - delta) & 3;
  auto sink_at = [&](int64_t i) {
    Vec4Sink d;
    d.g = g_dst + i;
    d.master = q.s.master + i;
    d.m = q.s.m + i;
    d.v = q.s.v + i;
    d.W = q.s.w_kind == W_BF16 ? (void*)((unsigned short*)q.s.W + i + p.begin)
                               : (void*)((float*)q.s.W + i + p.begin);
    return d;
  };
  emit_edge(E);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    __syncthreads();                       // ring reads / previous half's row reads are done
    stage_half(h, stage + (wmi * WR) * C::EPI_PITCH + sft + wn0);
    __syncthreads();
    // The left-over element of this thread (delta != 0): in the fused call its state is requested
    // now and used after the row loop, so that this second round of loads costs no extra wait.
    bool lo_ok = false;
    int64_t lo_i = 0;
    float lo_val = 0.f, lo_th = 0.f, lo_m = 0.f, lo_v = 0.f;
    if (delta != 0) {
      static_assert(C::NT / 4 >= HALF_ROWS, "one thread per left-over element of a staged half tile");
      const int rr = tid >> 2, e = tid & 3;
      const int tile_row = (rr / WR) * (2 * WR) + h * WR + rr % WR;
      const int lc = e < delta ? e : cols_valid - 4 + e;      // cols_valid is a multiple of 8
      lo_ok = rr < HALF_ROWS && tile_row < rows_valid;
      if (lo_ok) {
        lo_i = origin + (int64_t)tile_row * p.in + lc;
        lo_val = stage[rr * C::EPI_PITCH + sft + lc];
        if constexpr (MODE == EMIT_ADAMW) {
          lo_th = q.s.master[lo_i];
          lo_m = q.s.m[lo_i];
          lo_v = q.s.v[lo_i];
        }
      }
    }
    if (vec_lane && c4 + 4 <= cols_valid) {
      // RPT rows per trip: their state loads are issued together, then the updates
      // (four measured best for the fused call: 226 us against 228 / 248 us with two / one)
      constexpr int RPT = 4;
      for (int j0 = 0; j0 < HALF_ROWS / C::NW; j0 += RPT) {
        Vec4Sink d[RPT];
        State4 st[RPT];
        bool ok[RPT];
#pragma unroll
        for (int u = 0; u < RPT; ++u) {
          const int rr = (j0 + u) * C::NW + wave;                        // staged row, 0..HALF_ROWS-1
          const int tile_row = (rr / WR) * (2 * WR) + h * WR + rr % WR;
          ok[u] = tile_row < rows_valid;
          d[u] = sink_at(origin + (int64_t)tile_row * p.in + c4);
          if (ok[u]) st[u] = load_state4<MODE>(d[u]);
        }
#pragma unroll
        for (int u = 0; u < RPT; ++u) {
          if (ok[u]) {
            const float4 q4 = *reinterpret_cast<const float4*>(stage + ((j0 + u) * C::NW + wave) * C::EPI_PITCH + sft + c4);
            const f32x4_u val = {q4.x, q4.y, q4.z, q4.w};
            finish4<MODE>(d[u], q.s.w_kind, q.s.c, val, st[u]);
          }
        }
      }
    }
    if (lo_ok) {
      if constexpr (MODE == EMIT_ADAMW) {
        adamw_update(lo_val, lo_th, lo_m, lo_v, q.s.c);
        q.s.master[lo_i] = lo_th;
        q.s.m[lo_i] = lo_m;
        q.s.v[lo_i] = lo_v;
        if (q.s.w_kind == W_BF16) ((unsigned short*)q.s.W)[lo_i + p.begin] = f32_to_bf16_rne(lo_th);
        else if (q.s.w_kind == W_F32) ((float*)q.s.W)[lo_i + p.begin] = lo_th;
      } else {
        emit<MODE>(q.s, E, slab, lo_i, lo_i + p.begin, lo_val);
      }
    }
  }
}

// One 256 x 256 tile of body rows over one slab of tokens.
//
// Data movement.  dY and X are [token][row] / [token][column]: both operands have
// the contraction index outermost, the opposite of what an MFMA lane wants (8
// consecutive tokens of one row).  A slab of 32 tokens x 256 rows is copied as it
// is (512 B per token) into LDS by buffer_load_dwordx4 ... lds -- no VGPR staging, up
// to NS-1 slabs in flight -- and transposed on the way out by ds_read_b64_tr_b16.
// A wave-load writes 1 KB = tokens 2j, 2j+1; lane l lands in token 2j + l/32,
// physical 16-byte slot l%32.  To keep the 8 tokens that one transpose read
// touches on different banks, slot s of token k holds logical slot
// s ^ (sw(k) << 2), sw(k) = (k & 3) | ((k >> 3 & 1) << 2): the swizzle is applied
// to the source offset each lane fetches from, LDS writes stay linear.
//
// Schedule.  Per 32-token slab a wave issues 16 MFMAs in two 16-token steps.
// The transpose reads of the NEXT step are issued behind the first three MFMAs
// of a step and the global->LDS loads of a later slab behind the last five of the
// second step, so their latency runs under MFMAs instead of in front of a wait.
// One s_barrier per slab, between its two steps: it publishes slab kt+1 (every
// wave waited for its own loads of it) and retires slab kt, whose ring slot the
// loads of slab kt+NS then overwrite -- the whole ring is in flight.
template <class C, int MODE>
__device__ __forceinline__ void mfma_tile(const MfmaParams& q, const int item, unsigned char* ldsb) {
  const WgradProblem& p = q.p;
  TIMELINE_STAMP(q, item, 0);
#ifdef CHUNKFT_TIMELINE
  // where: XCC_ID (hardware register 20) and HW_ID (4: wave, SIMD, compute unit, shader engine)
  if (q.timeline && threadIdx.x == 0)
    q.timeline[(size_t)item * 8 + 4] = ((unsigned long long)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 20) << 32) |
                                       (unsigned)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 4);
#endif

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
  const int klen = (int)(k_end - k_begin);
  const int nk = (klen + C::BK - 1) / C::BK;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / C::WN) * (C::BM / C::WM);
  const int wn0 = (wave % C::WN) * (C::BN / C::WN);
  const unsigned short* dY = (const unsigned short*)p.dY;
  const unsigned short* X = (const unsigned short*)p.X;
  const unsigned lds_base = (unsigned)(uintptr_t)ldsb;

  // ---- global->LDS loads.  A load names its source as a uniform base (scalar registers:
  // the first row / column of the token the slab begins with, advanced one slab per fetch by
  // scalar adds) plus a per-lane byte offset that never changes -- the buffer form of the
  // load.  The form with a 64-bit per-lane address needs a vector add per load to advance,
  // and that add waits in the vector pipe behind the MFMAs: measured, every such load then
  // costs the matrix cores about 25 cycles, while the scalar-base form costs them nothing.
  // Rows / columns past the tensor are redirected to the tile's first ones (valid
  // memory, results masked in the epilogue); tokens past the end are clamped to
  // the last token and zeroed in the A fragments (mask_halves).
  unsigned voa[C::LA], vob[C::LB];
  int ka[C::LA], kb[C::LB];
  const unsigned lddy2 = (unsigned)(p.lddy * 2), ldx2 = (unsigned)(p.ldx * 2);    // bytes per token
  // A wave-load writes 1 KB: 1024 / RA tokens, RA / 16 lanes (16-byte slots) per token.
  constexpr int LPT_A = C::RA / 16, TPL_A = 64 / LPT_A;
#pragma unroll
  for (int i = 0; i < C::LA; ++i) {
    const int k = TPL_A * (wave * C::LA + i) + lane / LPT_A;
    const int swk = C::WM == 2 ? ((k & 3) | (((k >> 3) & 1) << 2)) : (k & 3);
    const int lc = (lane % LPT_A) ^ (swk << 2);
    int64_t r = row0 + lc * 8;
    if (r >= p.out) r = row0;
    ka[i] = k;
    voa[i] = (unsigned)r * 2u + (unsigned)k * lddy2;
  }
#pragma unroll
  for (int i = 0; i < C::LB; ++i) {
    const int k = 2 * (wave * C::LB + i) + (lane >> 5);
    const int lc = (lane & 31) ^ (((k & 3) | (((k >> 3) & 1) << 2)) << 2);
    int64_t cc = col0 + lc * 8;
    if (cc >= p.in) cc = col0;
    kb[i] = k;
    vob[i] = (unsigned)cc * 2u + (unsigned)k * ldx2;
  }
  // row 0 / column 0 of the first token of slab `next_fetch`
  const unsigned char* ga = (const unsigned char*)(dY + k_begin * p.lddy);
  const unsigned char* gb = (const unsigned char*)(X + k_begin * p.ldx);
  const int64_t stepA = (int64_t)C::BK * p.lddy * 2, stepB = (int64_t)C::BK * p.ldx * 2;     // bytes per slab
  int next_fetch = 0;   // slab index the bases stand at
  auto load_to_lds = [&](const unsigned char* base, unsigned voff, unsigned dst) {
    // raw buffer over the whole address range behind `base`: the per-lane offsets are kept below 4 GB
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, -1, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (LDS_PTR(void))(uintptr_t)dst, 16, (int)voff, 0, 0, 0);
  };
  auto next_slab = [&]() {
    ga += stepA;
    gb += stepB;
    ++next_fetch;
  };

  // ---- edge block (first tile row only).  One extra wave-load per slab, issued by
  // wave 0: lane l fetches, for token l/2, the 8-row group of the leading edge rows
  // (l even) or the one holding the trailing row (l odd); a missing group is
  // replaced by the tile's first rows (valid memory, masked in the epilogue).
  // With 8 waves, waves w and w + 4 share 64 columns and take one of the two 32-column
  // blocks each (workgroups of tile row 0); with 4 waves the workgroups of tile rows 0 and
  // 1 take one block each (the launcher folds the edge in only if there are two tile rows).
  const bool has_edge = (C::WM == 2 ? tile_m == 0 : tile_m < 2) && (q.lead_base >= 0 || q.trail_row >= 0);
  const int edge_blk = C::WM == 2 ? (wave >> 2) : tile_m;
  const int ke = lane >> 1;
  unsigned voe;
  {
    const int64_t lead = q.lead_base >= 0 ? q.lead_base : q.rb0;
    const int64_t trail = q.trail_row >= 0 ? (q.trail_row & ~(int64_t)7) : q.rb0;
    voe = (unsigned)((lane & 1) ? trail : lead) * 2u + (unsigned)ke * lddy2;
  }
  auto issue_edge = [&](auto stagec) {
    constexpr int STAGE = decltype(stagec)::value;
    const int stage = STAGE >= 0 ? STAGE : next_fetch % C::NS;
    const bool ragged = STAGE >= 0 ? false : (next_fetch + 1) * C::BK > klen;
    unsigned vo = voe;
    if (ragged) {      // the base stands at this slab: a token past the end steps back to the last one
      const int64_t over = k_begin + (int64_t)next_fetch * C::BK + ke - (p.T - 1);
      if (over > 0) vo -= (unsigned)over * lddy2;
    }
    load_to_lds(ga, vo, lds_base + stage * C::STAGE_BYTES + C::A_BYTES + C::B_BYTES);
  };
  // One of the L loads of slab `next_fetch`.  STAGE >= 0: the steady-state form, ring
  // slot known at compile time and the slab known to be complete; STAGE < 0: the general
  // form for the first and last slabs.
  auto issue_one = [&](auto idxc, auto stagec) {
    constexpr int idx = decltype(idxc)::value, STAGE = decltype(stagec)::value;
    const int stage = STAGE >= 0 ? STAGE : next_fetch % C::NS;
    const bool ragged = STAGE >= 0 ? false : (next_fetch + 1) * C::BK > klen;     // only the last slab can be
    if constexpr (idx < C::LA) {
      constexpr int i = idx;
      unsigned vo = voa[i];
      if (ragged) {
        const int64_t over = k_begin + (int64_t)next_fetch * C::BK + ka[i] - (p.T - 1);
        if (over > 0) vo -= (unsigned)over * lddy2;
      }
      load_to_lds(ga, vo, lds_base + stage * C::STAGE_BYTES + (wave * C::LA + i) * 1024);
    } else {
      constexpr int i = idx - C::LA;
      unsigned vo = vob[i];
      if (ragged) {
        const int64_t over = k_begin + (int64_t)next_fetch * C::BK + kb[i] - (p.T - 1);
        if (over > 0) vo -= (unsigned)over * ldx2;
      }
      load_to_lds(gb, vo, lds_base + stage * C::STAGE_BYTES + C::A_BYTES + (wave * C::LB + i) * 1024);
    }
  };

  // ---- transpose-read addressing.  In a block of 16 lanes, lane j reads 4
  // consecutive row indices of token (j / 4); the instruction hands lane i the 4
  // tokens of row index i.  Lanes 0-31 take tokens 0-7 of a 16-token step, lanes
  // 32-63 tokens 8-15: the operand layout of the 32x32x16 MFMA.  The swizzle
  // term of a lane is the same for every step: sw = (i16 / 4) | ((blk / 2) << 2).
  const int blk = lane >> 4, i16 = lane & 15;
  const int tr_k = (blk >> 1) * 8 + (i16 >> 2);
  const int swl = (i16 >> 2) | ((blk >> 1) << 2);
  const int low = (blk & 1) * 2 + ((i16 & 3) >> 1);     // low two bits of the 16-byte slot index
  const int sub = (i16 & 1) * 8;                        // byte offset inside the slot
  // Two bases 64 KB apart per block: with the ring slot known at compile time every
  // read then has an immediate offset (the field holds 16 bits) and costs no VALU add.
  unsigned addrA[C::TM], addrB[C::TN], addrA_hi[C::TM], addrB_hi[C::TN];
#pragma unroll
  for (int a = 0; a < C::TM; ++a) {
    addrA[a] = lds_base + tr_k * C::RA + ((((wm0 >> 3) + a * 4) ^ ((C::WM == 2 ? swl : (i16 >> 2)) << 2)) + low) * 16 + sub;
    addrA_hi[a] = addrA[a] + 65536;
  }
#pragma unroll
  for (int b = 0; b < C::TN; ++b) {
    addrB[b] = lds_base + C::A_BYTES + tr_k * C::RB + ((((wn0 >> 3) + b * 4) ^ (swl << 2)) + low) * 16 + sub;
    addrB_hi[b] = addrB[b] + 65536;
  }

  // Edge block reads: token t of a slab sits at byte 32 t, its 16 row values behind it.
  // Lanes 16-31 and 48-63 (MFMA rows 16-31) re-read rows 0-15; those output rows are dropped.
  const unsigned addrE = lds_base + C::A_BYTES + C::B_BYTES + tr_k * 32 + (i16 & 3) * 8;
  const unsigned addrE_hi = addrE + 65536;
  bf16x4 he0[2], he1[2];
  f32x16 acc_e;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_e[v] = 0.f;
  auto read_edge = [&](bf16x4* he, unsigned so, auto ksc) {
    constexpr int ks = decltype(ksc)::value;
    he[0] = lds_tr_read<ks * 16 * 32>(addrE + so);
    he[1] = lds_tr_read<(ks * 16 + 4) * 32>(addrE + so);
  };
  auto read_edge_at = [&](bf16x4* he, auto stagec, auto ksc) {
    constexpr int st = decltype(stagec)::value, ks = decltype(ksc)::value;
    constexpr int so = st * C::STAGE_BYTES;
    constexpr int off = (so & 0xFFFF) + ks * 16 * 32;
    static_assert(off + 4 * 32 < 65536, "LDS offset field");
    he[0] = lds_tr_read<off>(so < 65536 ? addrE : addrE_hi);
    he[1] = lds_tr_read<off + 4 * 32>(so < 65536 ? addrE : addrE_hi);
  };
  // the edge MFMA of a wave uses one of its two B blocks
  // (the B block is picked by value, four selects, and not by a branch around two MFMAs: the
  // branch made the compiler keep two copies of the accumulator block and move 16 registers,
  // behind a full MFMA latency, in every step)
  auto edge_mma = [&](const bf16x4* he, const bf16x4* h) {
    const bf16x8 fe = __builtin_shufflevector(he[0], he[1], 0, 1, 2, 3, 4, 5, 6, 7);
    const u32x4_t b0 = __builtin_bit_cast(u32x4_t, __builtin_shufflevector(h[8], h[9], 0, 1, 2, 3, 4, 5, 6, 7));
    const u32x4_t b1 = __builtin_bit_cast(u32x4_t, __builtin_shufflevector(h[10], h[11], 0, 1, 2, 3, 4, 5, 6, 7));
    u32x4_t bs;
#pragma unroll
    for (int e = 0; e < 4; ++e) bs[e] = edge_blk == 0 ? b0[e] : b1[e];
    acc_e = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fe, __builtin_bit_cast(bf16x8, bs), acc_e, 0, 0, 0);
  };

  // Fragment halves: unit u < 8 is A block u/2 (tokens 0-3 | 8-11 if u is even,
  // 4-7 | 12-15 if odd), unit u >= 8 is B block (u-8)/2 likewise.
  bf16x4 h0[12], h1[12];
  auto read_unit = [&](bf16x4* h, unsigned so, auto ksc, auto uc) {
    constexpr int ks = decltype(ksc)::value, u = decltype(uc)::value;
    constexpr int off = (ks * 16 + (u & 1) * 4) * (u < 8 ? C::RA : C::RB);
    if constexpr (u < 8) h[u] = lds_tr_read<off>(addrA[u / 2] + so);
    else h[u] = lds_tr_read<off>(addrB[(u - 8) / 2] + so);
  };
  auto read_unit_at = [&](bf16x4* h, auto stagec, auto ksc, auto uc) {      // ring slot at compile time
    constexpr int st = decltype(stagec)::value, ks = decltype(ksc)::value, u = decltype(uc)::value;
    constexpr int so = st * C::STAGE_BYTES;
    constexpr int off = (so & 0xFFFF) + (ks * 16 + (u & 1) * 4) * (u < 8 ? C::RA : C::RB);
    static_assert(off < 65536, "LDS offset field");
    if constexpr (u < 8) h[u] = lds_tr_read<off>(so < 65536 ? addrA[u / 2] : addrA_hi[u / 2]);
    else h[u] = lds_tr_read<off>(so < 65536 ? addrB[(u - 8) / 2] : addrB_hi[(u - 8) / 2]);
  };
  auto frag = [&](const bf16x4* h, int u) {
    return __builtin_shufflevector(h[u], h[u + 1], 0, 1, 2, 3, 4, 5, 6, 7);
  };
  auto mask_halves = [&](bf16x4* h, bf16x4* he, int kt, int ks) {
    if (kt == nk - 1 && (klen % C::BK) != 0) {
      const int kv = klen - kt * C::BK - ks * 16 - (lane >> 5) * 8;   // valid tokens among this lane's 8
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((u & 1) * 4 + e >= kv) h[u][e] = (__bf16)0.f;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (u * 4 + e >= kv) he[u][e] = (__bf16)0.f;
    }
  };

  f32x16 acc[C::TM][C::TN];
#pragma unroll
  for (int a = 0; a < C::TM; ++a)
#pragma unroll
    for (int b = 0; b < C::TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // ---- prologue: the whole ring (NS slabs) in flight, first step of slab 0 in registers
#pragma unroll
  for (int s = 0; s < C::NS; ++s)
    if (s < nk) {
      static_for<C::L>([&](auto ic) { issue_one(ic, IntC<-1>{}); });
      if (has_edge && wave == 0) issue_edge(IntC<-1>{});
      next_slab();
    }
  // wave 0 of an edge workgroup has one more load per slab in flight than the others
  const bool five = has_edge && wave == 0;
  if (C::NS - 1 < nk) {
    if (five) wait_vmcnt<(C::NS - 1) * (C::L + 1)>(); else wait_vmcnt<(C::NS - 1) * C::L>();
  } else {
    wait_vmcnt<0>();
  }
  __builtin_amdgcn_s_barrier();
  static_for<12>([&](auto uc) { read_unit(h0, 0u, IntC<0>{}, uc); });
  he0[0] = he0[1] = he1[0] = he1[1] = bf16x4{};
  if (has_edge) read_edge(he0, 0u, IntC<0>{});
  WAIT_HALVES_E(h0, he0);
  mask_halves(h0, he0, 0, 0);
  TIMELINE_STAMP(q, item, 1);

  // One slab: sixteen MFMAs in two steps of eight, numbered i = 2a + b within a
  // step.  The twelve transpose reads of the next step follow MFMAs 0-2 (four
  // each), so the last of them has five MFMAs of time to return.  Between the two
  // steps sits the slab's one barrier: before it every wave has finished reading
  // ring slot kt (the reads of the second step were waited for) and has seen its
  // own loads of slab kt+1 land, so behind it slot kt is free -- the loads of
  // slab kt+NS go there, behind MFMAs 3-7 of the second step -- and slab kt+1 is
  // complete for the reads of that step.  A slab thus has NS-1 slab times to
  // arrive.  KM >= 0 is the steady-state form (kt mod NS known at compile time,
  // a later slab always fetched, nothing ragged): no branch, no address
  // arithmetic.  KM < 0 is the general form used for the last slabs.
  auto do_slab = [&](int kt, auto kmc, auto edgec) {
    constexpr int KM = decltype(kmc)::value;
    constexpr bool FAST = KM >= 0, EDGE = decltype(edgec)::value;
    const bool fetch = FAST || kt + C::NS < nk;
    const bool more = FAST || kt + 1 < nk;
    const unsigned so = (unsigned)((kt % C::NS) * C::STAGE_BYTES);
    const unsigned so_next = (unsigned)(((kt + 1) % C::NS) * C::STAGE_BYTES);
    constexpr int ST_FETCH = FAST ? KM : -1;
    static_for<8>([&](auto ic) {
      constexpr int i = decltype(ic)::value, a = i / 2, b = (a & 1) ? 1 - i % 2 : i % 2;
      __builtin_amdgcn_sched_barrier(0);
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(h0, 2 * a), frag(h0, 8 + 2 * b), acc[a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (i < 3) {
        static_for<4>([&](auto jc) {
          constexpr int u = 4 * i + decltype(jc)::value;
          if constexpr (FAST) read_unit_at(h1, IntC<(KM >= 0 ? KM : 0)>{}, IntC<1>{}, IntC<u>{});
          else read_unit(h1, so, IntC<1>{}, IntC<u>{});
        });
      } else if constexpr (EDGE && i == 3) {
        if constexpr (FAST) read_edge_at(he1, IntC<(KM >= 0 ? KM : 0)>{}, IntC<1>{});
        else read_edge(he1, so, IntC<1>{});
      }
    });
    if constexpr (EDGE) edge_mma(he0, h0);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (EDGE) WAIT_HALVES_E(h1, he1); else WAIT_HALVES(h1);
    if constexpr (!FAST) mask_halves(h1, he1, kt, 1);
    // slab kt+1 has landed once at most the NS-2 younger slabs are outstanding
    if (FAST || kt + C::NS - 1 < nk) {
      if (EDGE && wave == 0) wait_vmcnt<(C::NS - 2) * (C::L + 1)>(); else wait_vmcnt<(C::NS - 2) * C::L>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    static_for<8>([&](auto ic) {
      constexpr int i = decltype(ic)::value, a = i / 2, b = (a & 1) ? 1 - i % 2 : i % 2;
      __builtin_amdgcn_sched_barrier(0);
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(h1, 2 * a), frag(h1, 8 + 2 * b), acc[a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (i < 3) {
        static_for<4>([&](auto jc) {
          constexpr int u = 4 * i + decltype(jc)::value;
          if constexpr (FAST) read_unit_at(h0, IntC<(KM >= 0 ? (KM + 1) % C::NS : 0)>{}, IntC<0>{}, IntC<u>{});
          else if (more) read_unit(h0, so_next, IntC<0>{}, IntC<u>{});
        });
      } else {
        if constexpr (EDGE && i == 3) {
          if constexpr (FAST) read_edge_at(he0, IntC<(KM >= 0 ? (KM + 1) % C::NS : 0)>{}, IntC<0>{});
          else if (more) read_edge(he0, so_next, IntC<0>{});
        }
        // loads of slab kt+NS: one behind each of MFMAs 3-6, the rest behind MFMA 7
        static_for<C::L>([&](auto lc) {
          constexpr int l = decltype(lc)::value;
          if constexpr ((l < 4 ? l + 3 : 7) == i) {
            if constexpr (FAST) issue_one(lc, IntC<ST_FETCH>{});
            else if (fetch) issue_one(lc, IntC<-1>{});
          }
        });
        if constexpr (EDGE && i == 7) {
          if (fetch && wave == 0) issue_edge(IntC<ST_FETCH>{});
        }
      }
    });
    if (fetch) next_slab();
    if constexpr (EDGE) edge_mma(he1, h1);
    __builtin_amdgcn_sched_barrier(0);
    if (more) {
      if constexpr (EDGE) WAIT_HALVES_E(h0, he0); else WAIT_HALVES(h0);
      if constexpr (!FAST) mask_halves(h0, he0, kt + 1, 0);
    }
  };

  // Steady state: slabs whose fetch (of slab kt + NS) exists and is complete, in
  // groups of NS so that the ring slot is a compile-time constant.
  const bool last_ragged = (klen % C::BK) != 0;
  const int n_fast_raw = (nk - C::NS - (last_ragged ? 1 : 0)) / C::NS * C::NS;
  const int n_fast = n_fast_raw > 0 ? n_fast_raw : 0;
  auto run_slabs = [&](auto edgec) {
    int kt = 0;
    for (; kt < n_fast; kt += C::NS)
      static_for<C::NS>([&](auto kmc) { do_slab(kt + decltype(kmc)::value, kmc, edgec); });
    for (; kt < nk; ++kt) do_slab(kt, IntC<-1>{}, edgec);
  };
  if (has_edge) run_slabs(IntC<1>{}); else run_slabs(IntC<0>{});
  TIMELINE_STAMP(q, item, 2);

  // accumulator register v of a 32 x 32 block: row (v / 4) * 8 + (lane / 32) * 4 + v % 4, column lane % 32
  auto stage_half = [&](int h, float* dst) {      // dst: the wave's first row and column in the staging area
    static_for<(C::TM / 2) * C::TN>([&](auto blk_c) {
      constexpr int a2 = decltype(blk_c)::value / C::TN, b = decltype(blk_c)::value % C::TN;
      float* base = dst + (a2 * 32 + (lane >> 5) * 4) * C::EPI_PITCH + b * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float x = h == 0 ? acc[a2][b][v] : acc[C::TM / 2 + a2][b][v];
        base[((v >> 2) * 8 + (v & 3)) * C::EPI_PITCH] = x;
      }
    });
  };
  auto emit_edge = [&](int64_t E) {
    if (!has_edge) return;
    // Edge block: MFMA rows 0-7 are the leading group, 8-15 the group of the trailing row
    // (registers v = 0..7 of the block); one element at a time, masked by the chunk's range.
    const int64_t col = col0 + wn0 + edge_blk * 32 + (lane & 31);
#pragma unroll
    for (int v = 0; v < 8; ++v) {
      const int r8 = (lane >> 5) * 4 + (v & 3);
      int64_t row;
      if (v < 4) row = q.lead_base >= 0 ? q.lead_base + r8 : -1;
      else row = (q.trail_row >= 0 && (q.trail_row & 7) == r8) ? q.trail_row : -1;
      const int64_t flat = row * p.in + col;
      if (row >= 0 && col < p.in && flat >= p.begin && flat < p.end)
        emit<MODE>(q.s, E, slab, flat - p.begin, flat, acc_e[v]);
    }
  };
  tile_epilogue<C, MODE>(q, ldsb, row0, col0, slab, wave, lane, tid, stage_half, emit_edge);
  TIMELINE_STAMP(q, item, 3);
}

// The same tile with the 16x16x32 MFMA (which holds a higher clock under the part's power limit).
// A wave's 128 x 64 sub-tile is 8 x 4 blocks of 16 x 16; an MFMA takes all 32 tokens of a slab, so
// a slab is 32 MFMAs in two halves of 16: the upper four row blocks, then the lower four, each against
// the slab's four column blocks.  Operand layout of the MFMA: lane l holds row (column) l % 16 and the
// 8 tokens 8 (l / 16) ... + 7; a transpose read hands a 16-lane block 4 tokens of 16 rows, so an
// operand block is two reads (tokens +0..3, +4..7).  A half-wave of such a read touches 8 tokens x 32
// bytes; the 16-byte slots of a token row are therefore XOR-swizzled in bits 1-3 by
// (k & 3) | ((k >> 3 & 1) << 2), which puts the 8 tokens on the 8 different 32-byte groups of the
// 256-byte bank window (applied to the source offsets of the global->LDS loads, as in the other form).
// Registers: the MFMAs of a half go column block by column block, so that in the lower half a
// column block's registers are free after its four MFMAs and take the next slab's block at once; the
// row blocks of one half are read while the other half's MFMAs run.  The ring keeps the A images of
// all slabs together, then the B images, then the edge blocks: every read of an operand block is then
// one base register plus an immediate offset, whatever the ring slot.
#define WAIT8(h)                                                                                         \
  asm volatile("s_waitcnt lgkmcnt(0)"                                                                    \
               : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]),     \
                 "+v"(h[7])::"memory")
#define WAIT8_8_2(ha, hb, he)                                                                            \
  asm volatile("s_waitcnt lgkmcnt(0)"                                                                    \
               : "+v"(ha[0]), "+v"(ha[1]), "+v"(ha[2]), "+v"(ha[3]), "+v"(ha[4]), "+v"(ha[5]),           \
                 "+v"(ha[6]), "+v"(ha[7]), "+v"(hb[0]), "+v"(hb[1]), "+v"(hb[2]), "+v"(hb[3]),           \
                 "+v"(hb[4]), "+v"(hb[5]), "+v"(hb[6]), "+v"(hb[7]), "+v"(he[0]), "+v"(he[1])::"memory")
// all LDS reads but the last two issued (the next slab's last column block) have returned
#define WAIT8_6_2_BUT2(ha, hb, he)                                                                       \
  asm volatile("s_waitcnt lgkmcnt(2)"                                                                    \
               : "+v"(ha[0]), "+v"(ha[1]), "+v"(ha[2]), "+v"(ha[3]), "+v"(ha[4]), "+v"(ha[5]),           \
                 "+v"(ha[6]), "+v"(ha[7]), "+v"(hb[0]), "+v"(hb[1]), "+v"(hb[2]), "+v"(hb[3]),           \
                 "+v"(hb[4]), "+v"(hb[5]), "+v"(he[0]), "+v"(he[1])::"memory")
// the two reads issued before the last eight have returned
#define WAIT2_BEFORE8(hb) asm volatile("s_waitcnt lgkmcnt(8)" : "+v"(hb[6]), "+v"(hb[7])::"memory")

template <class C, int MODE>
__device__ __forceinline__ void mfma_tile16(const MfmaParams& q, const int item, unsigned char* ldsb) {
  static_assert(C::MI == 16 && C::TM == 8 && C::TN == 4, "written out for 8 x 4 blocks of 16 x 16 per wave");
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  const WgradProblem& p = q.p;
  TIMELINE_STAMP(q, item, 0);
#ifdef CHUNKFT_TIMELINE
  if (q.timeline && threadIdx.x == 0)
    q.timeline[(size_t)item * 8 + 4] = ((unsigned long long)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 20) << 32) |
                                       (unsigned)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 4);
#endif

  // ---- which tile, which token slab (as in mfma_tile)
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
  const int klen = (int)(k_end - k_begin);
  const int nk = (klen + C::BK - 1) / C::BK;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / C::WN) * (C::BM / C::WM);
  const int wn0 = (wave % C::WN) * (C::BN / C::WN);
  const unsigned short* dY = (const unsigned short*)p.dY;
  const unsigned short* X = (const unsigned short*)p.X;
  const unsigned lds_base = (unsigned)(uintptr_t)ldsb;

  // ---- global->LDS loads (as in mfma_tile; the slot swizzle is the one described above)
  // A wave's loads of one operand name tokens 4 apart (A) or 2 apart (B); tokens 4 apart have the same
  // swizzle, so loads i and i + (4 tokens) share their per-lane offset and differ in a scalar offset.
  constexpr int LPT_A = C::RA / 16, TPL_A = 64 / LPT_A;
  constexpr int VA = TPL_A >= 4 ? 1 : (C::LA < 4 / TPL_A ? C::LA : 4 / TPL_A);   // distinct per-lane offsets
  constexpr int VB = C::LB < 2 ? C::LB : 2;
  unsigned voa[VA], vob[VB];
  const unsigned lddy2 = (unsigned)(p.lddy * 2), ldx2 = (unsigned)(p.ldx * 2);
  auto swz = [](int k) { return ((k & 3) | (((k >> 3) & 1) << 2)) << 1; };
  auto tok_a = [&](int i) { return TPL_A * (wave * C::LA + i) + lane / LPT_A; };
  auto tok_b = [&](int i) { return 2 * (wave * C::LB + i) + (lane >> 5); };
  static_assert((TPL_A * C::LA == 4 || TPL_A * C::LA == 8) && (2 * C::LB == 4 || 2 * C::LB == 8),
                "a wave's tokens of one operand are an aligned group of 4 or 8: tokens 4 apart share bit 3");
#pragma unroll
  for (int i = 0; i < VA; ++i) {
    const int k = tok_a(i);
    const int lc = (lane % LPT_A) ^ swz(k);
    int64_t r = row0 + lc * 8;
    if (r >= p.out) r = row0;
    voa[i] = (unsigned)r * 2u + (unsigned)k * lddy2;
  }
#pragma unroll
  for (int i = 0; i < VB; ++i) {
    const int k = tok_b(i);
    const int lc = (lane & 31) ^ swz(k);
    int64_t cc = col0 + lc * 8;
    if (cc >= p.in) cc = col0;
    vob[i] = (unsigned)cc * 2u + (unsigned)k * ldx2;
  }
  const unsigned char* ga = (const unsigned char*)(dY + k_begin * p.lddy);
  const unsigned char* gb = (const unsigned char*)(X + k_begin * p.ldx);
  const int64_t stepA = (int64_t)C::BK * p.lddy * 2, stepB = (int64_t)C::BK * p.ldx * 2;
  int next_fetch = 0;
  auto load_to_lds = [&](const unsigned char* base, unsigned voff, unsigned soff, unsigned dst) {
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, -1, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (LDS_PTR(void))(uintptr_t)dst, 16, (int)voff, (int)soff, 0, 0);
  };
  auto next_slab = [&]() {
    ga += stepA;
    gb += stepB;
    ++next_fetch;
  };

  // ---- edge block: 16 rows per token (the 8-row group of the leading edge rows, the 8-row group of
  // the trailing row), one 16 x 16 row block.  The two workgroups (waves) that share 64 columns take
  // two of its four 16-column blocks each.
  const bool has_edge = (C::WM == 2 ? tile_m == 0 : tile_m < 2) && (q.lead_base >= 0 || q.trail_row >= 0);
  const int edge_blk = C::WM == 2 ? (wave >> 2) : tile_m;
  const int ke = lane >> 1;
  unsigned voe;
  {
    const int64_t lead = q.lead_base >= 0 ? q.lead_base : q.rb0;
    const int64_t trail = q.trail_row >= 0 ? (q.trail_row & ~(int64_t)7) : q.rb0;
    voe = (unsigned)((lane & 1) ? trail : lead) * 2u + (unsigned)ke * lddy2;
  }
  auto issue_edge = [&](auto stagec) {
    constexpr int STAGE = decltype(stagec)::value;
    const int stage = STAGE >= 0 ? STAGE : next_fetch % C::NS;
    const bool ragged = STAGE >= 0 ? false : (next_fetch + 1) * C::BK > klen;
    unsigned vo = voe;
    if (ragged) {
      const int64_t over = k_begin + (int64_t)next_fetch * C::BK + ke - (p.T - 1);
      if (over > 0) vo -= (unsigned)over * lddy2;
    }
    load_to_lds(ga, vo, 0u, lds_base + C::NS * (C::A_BYTES + C::B_BYTES) + stage * C::E_BYTES);
  };
  auto issue_one = [&](auto idxc, auto stagec) {
    constexpr int idx = decltype(idxc)::value, STAGE = decltype(stagec)::value;
    const int stage = STAGE >= 0 ? STAGE : next_fetch % C::NS;
    const bool ragged = STAGE >= 0 ? false : (next_fetch + 1) * C::BK > klen;
    if constexpr (idx < C::LA) {
      constexpr int i = idx;
      unsigned vo = voa[i % VA];
      if (ragged) {
        const int64_t over = k_begin + (int64_t)next_fetch * C::BK + tok_a(i) - (p.T - 1);
        if (over > 0) vo -= (unsigned)over * lddy2;
      }
      load_to_lds(ga, vo, (unsigned)(i / VA) * (unsigned)(TPL_A * VA) * lddy2,
                  lds_base + stage * C::A_BYTES + (wave * C::LA + i) * 1024);
    } else {
      constexpr int i = idx - C::LA;
      unsigned vo = vob[i % VB];
      if (ragged) {
        const int64_t over = k_begin + (int64_t)next_fetch * C::BK + tok_b(i) - (p.T - 1);
        if (over > 0) vo -= (unsigned)over * ldx2;
      }
      load_to_lds(gb, vo, (unsigned)(i / VB) * (unsigned)(2 * VB) * ldx2,
                  lds_base + C::NS * C::A_BYTES + stage * C::B_BYTES + (wave * C::LB + i) * 1024);
    }
  };

  // ---- transpose-read addressing
  const int blk = lane >> 4, i16 = lane & 15;
  const int tr_k = blk * 8 + (i16 >> 2);                     // first of the 4 + 4 tokens this lane's reads name
  const int swl = ((i16 >> 2) | ((blk & 1) << 2)) << 1;      // the swizzle of those tokens
  const int low = (i16 & 3) >> 1;
  const int sub = (i16 & 1) * 8;
  static_assert((C::NS - 1) * C::A_BYTES + 4 * C::RA < 65536 && (C::NS - 1) * C::B_BYTES + 4 * C::RB < 65536,
                "LDS offset field");
  unsigned addrA[C::TM], addrB[C::TN];
#pragma unroll
  for (int a = 0; a < C::TM; ++a)
    addrA[a] = lds_base + tr_k * C::RA + ((((wm0 >> 3) + a * 2) ^ swl) + low) * 16 + sub;
#pragma unroll
  for (int b = 0; b < C::TN; ++b)
    addrB[b] = lds_base + C::NS * C::A_BYTES + tr_k * C::RB + ((((wn0 >> 3) + b * 2) ^ swl) + low) * 16 + sub;
  const unsigned addrE = lds_base + C::NS * (C::A_BYTES + C::B_BYTES) + tr_k * 32 + (i16 & 3) * 8;

  // Fragment halves: unit u of a row half is row block u / 2 of that half (tokens +0..3 if u is
  // even, +4..7 if odd); unit u of the column set is column block u / 2 likewise.
  bf16x4 ha0[8], ha1[8], hb[8], he[2];
  // RH: which four row blocks (0: upper, 1: lower); st: ring slot
  auto read_a = [&](bf16x4* h, auto rhc, int st, auto uc) {
    constexpr int RH = decltype(rhc)::value, u = decltype(uc)::value;
    h[u] = lds_tr_read<(u & 1) * 4 * C::RA>(addrA[4 * RH + u / 2] + (unsigned)(st * C::A_BYTES));
  };
  auto read_a_at = [&](bf16x4* h, auto rhc, auto stagec, auto uc) {
    constexpr int RH = decltype(rhc)::value, st = decltype(stagec)::value, u = decltype(uc)::value;
    h[u] = lds_tr_read<st * C::A_BYTES + (u & 1) * 4 * C::RA>(addrA[4 * RH + u / 2]);
  };
  auto read_b = [&](int st, auto uc) {
    constexpr int u = decltype(uc)::value;
    hb[u] = lds_tr_read<(u & 1) * 4 * C::RB>(addrB[u / 2] + (unsigned)(st * C::B_BYTES));
  };
  auto read_b_at = [&](auto stagec, auto uc) {
    constexpr int st = decltype(stagec)::value, u = decltype(uc)::value;
    hb[u] = lds_tr_read<st * C::B_BYTES + (u & 1) * 4 * C::RB>(addrB[u / 2]);
  };
  auto read_e = [&](int st) {
    he[0] = lds_tr_read<0>(addrE + (unsigned)(st * C::E_BYTES));
    he[1] = lds_tr_read<4 * 32>(addrE + (unsigned)(st * C::E_BYTES));
  };
  auto read_e_at = [&](auto stagec) {
    constexpr int st = decltype(stagec)::value;
    he[0] = lds_tr_read<st * C::E_BYTES>(addrE);
    he[1] = lds_tr_read<st * C::E_BYTES + 4 * 32>(addrE);
  };
  auto frag = [&](const bf16x4* h, int u) {
    return __builtin_shufflevector(h[u], h[u + 1], 0, 1, 2, 3, 4, 5, 6, 7);
  };
  // tokens past the end of a ragged last slab: zero in the row-block operands
  auto mask_units = [&](bf16x4* h, int kt) {
    if (kt == nk - 1 && (klen % C::BK) != 0) {
      const int kv = klen - kt * C::BK - blk * 8;            // valid tokens among this lane's 8
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((u & 1) * 4 + e >= kv) h[u][e] = (__bf16)0.f;
    }
  };
  auto mask_edge = [&](int kt) {
    if (kt == nk - 1 && (klen % C::BK) != 0) {
      const int kv = klen - kt * C::BK - blk * 8;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (u * 4 + e >= kv) he[u][e] = (__bf16)0.f;
    }
  };

  f32x4_t acc[C::TM][C::TN], acc_e[2];
#pragma unroll
  for (int a = 0; a < C::TM; ++a)
#pragma unroll
    for (int b = 0; b < C::TN; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc_e[j][v] = 0.f;

  // ---- prologue: the whole ring in flight, the operands of slab 0's upper half in registers
#pragma unroll
  for (int s = 0; s < C::NS; ++s)
    if (s < nk) {
      static_for<C::L>([&](auto ic) { issue_one(ic, IntC<-1>{}); });
      if (has_edge && wave == 0) issue_edge(IntC<-1>{});
      next_slab();
    }
  const bool five = has_edge && wave == 0;
  if (C::NS - 1 < nk) {
    if (five) wait_vmcnt<(C::NS - 1) * (C::L + 1)>(); else wait_vmcnt<(C::NS - 1) * C::L>();
  } else {
    wait_vmcnt<0>();
  }
  __builtin_amdgcn_s_barrier();
  static_for<8>([&](auto uc) { read_a(ha0, IntC<0>{}, 0, uc); });
  static_for<8>([&](auto uc) { read_b(0, uc); });
  he[0] = he[1] = bf16x4{};
  if (has_edge) read_e(0);
  WAIT8_8_2(ha0, hb, he);
  mask_units(ha0, 0);
  mask_edge(0);
  TIMELINE_STAMP(q, item, 1);

  // the edge MFMAs of a wave use two of its four column blocks (picked by value, as in mfma_tile)
  auto edge_mma = [&]() {
    const bf16x8 fe = __builtin_shufflevector(he[0], he[1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const u32x4_t lo = __builtin_bit_cast(u32x4_t, __builtin_shufflevector(hb[2 * j], hb[2 * j + 1], 0, 1, 2, 3, 4, 5, 6, 7));
      const u32x4_t hi = __builtin_bit_cast(u32x4_t, __builtin_shufflevector(hb[4 + 2 * j], hb[5 + 2 * j], 0, 1, 2, 3, 4, 5, 6, 7));
      u32x4_t bs;
#pragma unroll
      for (int e = 0; e < 4; ++e) bs[e] = edge_blk == 0 ? lo[e] : hi[e];
      acc_e[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fe, __builtin_bit_cast(bf16x8, bs), acc_e[j], 0, 0, 0);
    }
  };

  // One slab.  Upper half: its 16 MFMAs (column block by column block), the reads of the lower row
  // blocks behind the first two; the last column block, whose reads were issued last in the slab
  // before, is waited for in front of its first MFMA.  Then the slab's one barrier (as in mfma_tile:
  // slot kt is consumed, slab kt+1 has landed).  Lower half: its 16 MFMAs; behind them the reads of
  // slab kt+1 -- upper row blocks and edge block first, each column block as soon as its four MFMAs
  // are issued -- and the loads of slab kt+NS.
  auto do_slab = [&](int kt, auto kmc, auto edgec) {
    constexpr int KM = decltype(kmc)::value;
    constexpr bool FAST = KM >= 0, EDGE = decltype(edgec)::value;
    const bool fetch = FAST || kt + C::NS < nk;
    const bool more = FAST || kt + 1 < nk;
    const int st = kt % C::NS, st_next = (kt + 1) % C::NS;
    constexpr int ST_FETCH = FAST ? KM : -1;
    constexpr int ST_NEXT = FAST ? (KM + 1) % C::NS : 0;
    static_for<16>([&](auto ic) {
      constexpr int i = decltype(ic)::value, b = i / 4, a = (b & 1) ? 3 - i % 4 : i % 4;
      if constexpr (i == 12) WAIT2_BEFORE8(hb);   // (nothing to wait for in slab 0: the prologue waited for everything)
      __builtin_amdgcn_sched_barrier(0);
      acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(ha0, 2 * a), frag(hb, 2 * b), acc[a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (i < 2) {
        static_for<4>([&](auto jc) {
          constexpr int u = 4 * i + decltype(jc)::value;
          if constexpr (FAST) read_a_at(ha1, IntC<1>{}, IntC<(KM >= 0 ? KM : 0)>{}, IntC<u>{});
          else read_a(ha1, IntC<1>{}, st, IntC<u>{});
        });
      }
    });
    if constexpr (EDGE) edge_mma();
    __builtin_amdgcn_sched_barrier(0);
    WAIT8(ha1);
    if constexpr (!FAST) mask_units(ha1, kt);
    if (FAST || kt + C::NS - 1 < nk) {
      if (EDGE && wave == 0) wait_vmcnt<(C::NS - 2) * (C::L + 1)>(); else wait_vmcnt<(C::NS - 2) * C::L>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    static_for<16>([&](auto ic) {
      constexpr int i = decltype(ic)::value, b = i / 4, a = (b & 1) ? 3 - i % 4 : i % 4;
      __builtin_amdgcn_sched_barrier(0);
      acc[4 + a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(ha1, 2 * a), frag(hb, 2 * b), acc[4 + a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (i < 2) {
        static_for<4>([&](auto jc) {
          constexpr int u = 4 * i + decltype(jc)::value;
          if constexpr (FAST) read_a_at(ha0, IntC<0>{}, IntC<ST_NEXT>{}, IntC<u>{});
          else if (more) read_a(ha0, IntC<0>{}, st_next, IntC<u>{});
        });
      }
      if constexpr (EDGE && i == 2) {
        if constexpr (FAST) read_e_at(IntC<ST_NEXT>{});
        else if (more) read_e(st_next);
      }
      if constexpr (i % 4 == 3) {                  // column block b has had its last MFMA of this slab
        static_for<2>([&](auto jc) {
          constexpr int u = 2 * b + decltype(jc)::value;
          if constexpr (FAST) read_b_at(IntC<ST_NEXT>{}, IntC<u>{});
          else if (more) read_b(st_next, IntC<u>{});
        });
      }
      // loads of slab kt+NS: one behind each of MFMAs 4, 5, 6, 8, 9, 10
      static_for<C::L>([&](auto lc) {
        constexpr int l = decltype(lc)::value;
        if constexpr ((l < 3 ? 4 + l : 5 + l) == i) {
          if constexpr (FAST) issue_one(lc, IntC<ST_FETCH>{});
          else if (fetch) issue_one(lc, IntC<-1>{});
        }
      });
      if constexpr (EDGE && i == 12) {
        if (fetch && wave == 0) issue_edge(IntC<ST_FETCH>{});
      }
    });
    if (fetch) next_slab();
    __builtin_amdgcn_sched_barrier(0);
    if (more) {
      WAIT8_6_2_BUT2(ha0, hb, he);
      if constexpr (!FAST) {
        mask_units(ha0, kt + 1);
        if constexpr (EDGE) mask_edge(kt + 1);
      }
    }
  };

  // Steady state: slabs whose fetch (of slab kt + NS) exists and is complete, in groups of NS so that
  // the ring slot is a compile-time constant.
  const bool last_ragged = (klen % C::BK) != 0;
  const int n_fast_raw = (nk - C::NS - (last_ragged ? 1 : 0)) / C::NS * C::NS;
  const int n_fast = n_fast_raw > 0 ? n_fast_raw : 0;
  auto run_slabs = [&](auto edgec) {
    int kt = 0;
    for (; kt < n_fast; kt += C::NS)
      static_for<C::NS>([&](auto kmc) { do_slab(kt + decltype(kmc)::value, kmc, edgec); });
    for (; kt < nk; ++kt) do_slab(kt, IntC<-1>{}, edgec);
  };
  if (has_edge) run_slabs(IntC<1>{}); else run_slabs(IntC<0>{});
  TIMELINE_STAMP(q, item, 2);

  // accumulator register v of a 16 x 16 block: row (lane / 16) * 4 + v, column lane % 16
  auto stage_half = [&](int h, float* dst) {
    static_for<4 * C::TN>([&](auto blk_c) {
      constexpr int a = decltype(blk_c)::value / C::TN, b = decltype(blk_c)::value % C::TN;
      float* base = dst + (a * 16 + (lane >> 4) * 4) * C::EPI_PITCH + b * 16 + (lane & 15);
#pragma unroll
      for (int v = 0; v < 4; ++v) base[v * C::EPI_PITCH] = h == 0 ? acc[a][b][v] : acc[4 + a][b][v];
    });
  };
  auto emit_edge = [&](int64_t E) {
    if (!has_edge) return;
    // edge block rows 0-7 are the leading group, 8-15 the group of the trailing row
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t col = col0 + wn0 + (2 * edge_blk + j) * 16 + (lane & 15);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = (lane >> 4) * 4 + v;
        int64_t row;
        if (r < 8) row = q.lead_base >= 0 ? q.lead_base + r : -1;
        else row = (q.trail_row >= 0 && (q.trail_row & 7) == r - 8) ? q.trail_row : -1;
        const int64_t flat = row * p.in + col;
        if (row >= 0 && col < p.in && flat >= p.begin && flat < p.end)
          emit<MODE>(q.s, E, slab, flat - p.begin, flat, acc_e[j][v]);
      }
    }
  };
  tile_epilogue<C, MODE>(q, ldsb, row0, col0, slab, wave, lane, tid, stage_half, emit_edge);
  TIMELINE_STAMP(q, item, 3);
}

// Workgroup ids are dealt round-robin to the 8 XCDs; each XCD gets one contiguous run of work
// items so that tiles sharing dY rows / X columns meet in the same L2.  Returns -1 for the
// padding workgroups at the end of the grid.
__device__ __forceinline__ int xcd_work_item(int n_items) {
  const int per_xcd = (n_items + 7) >> 3;
  const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  return item < n_items ? item : -1;
}

// Two workgroups share a compute unit.  Started together they run their MFMA loops
// together and then their HBM-bound epilogues together; with stagger > 0 the second
// one of each pair (workgroups are dealt to the 32 compute units of an XCD in order:
// the first 32 fill one slot each, the next 32 the other) starts late instead, so that
// one tends to be in its loop while the other is in its epilogue.  With one workgroup per
// compute unit (the large tile, fused call only) every second compute unit starts late.
template <class C, int MODE>
__device__ __forceinline__ void start_offset(int stagger) {
  const int j = (int)(blockIdx.x >> 3);
  bool late = false;
  if constexpr (C::WM == 1) late = j >= 32 && j < 64;
  else if constexpr (MODE == EMIT_ADAMW) late = j < 32 && (j & 1);
  if (late)
    for (int i = 0; i < stagger; ++i) __builtin_amdgcn_s_sleep(127);
}

// The parameters stay in the kernel-argument memory and are read where they are used (the index
// below is always 0, which the compiler cannot know): taken by value they are all loaded into scalar
// registers up front, and the loop then runs out of registers (14 spilled vector registers in the
// 128 x 256 configuration against 2).
struct MfmaArgs {
  MfmaParams q[1];
};

template <class C, int MODE>
__global__ __launch_bounds__(C::NT, 2) void wgrad_mfma_kernel(const MfmaArgs args) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char ldsb[];
  const MfmaParams& q = args.q[blockIdx.y];
  const int n_items = q.n_tile_items;
  const int per_xcd = (n_items + 7) >> 3;
  const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (item >= n_items) return;
  if constexpr (C::WM == 1) {
    const int j = (int)(blockIdx.x >> 3);
    if (j >= 32 && j < 64)
      for (int i = 0; i < q.stagger; ++i) __builtin_amdgcn_s_sleep(127);
  } else if constexpr (MODE == EMIT_ADAMW) {
    const int j = (int)(blockIdx.x >> 3);
    if (j < 32 && (j & 1))
      for (int i = 0; i < q.stagger; ++i) __builtin_amdgcn_s_sleep(127);
  }
  if constexpr (C::MI == 16) mfma_tile16<C, MODE>(q, item, ldsb);
  else mfma_tile<C, MODE>(q, item, ldsb);
}

// ---------------------------------------------------------------------------
// one launch for all segments of a chunk (fused call only)
// ---------------------------------------------------------------------------
// The work items of up to kGroupMax segments are laid end to end: the tiles of each bf16 matrix
// segment (parameters as for wgrad_mfma_kernel) and, for a bf16 scale-vector segment (tiles_m = 0),
// blocks of 64 elements.  A workgroup finds its segment by its item number and then does exactly
// what the single-segment kernels do, in the same order, so the results are theirs bit for bit.
constexpr int kGroupMax = 12;

struct GroupParams {
  int32_t n_segs, n_items, stagger, reserved;
  int32_t item_start[kGroupMax + 1];     // first work item of each segment; [n_segs] = n_items
  MfmaParams seg[kGroupMax];
};
static_assert(sizeof(GroupParams) <= 4096, "the table travels as a kernel argument");

// 64 elements of a scale-vector segment: the arithmetic of colsum_kernel (16 token groups, each summed
// in ascending token order, then added in group order), with the workgroup's waves taking the token
// groups in turn.
template <class C, int MODE>
__device__ __forceinline__ void colsum_item(const MfmaParams& q, const int block, unsigned char* ldsb) {
  constexpr int TG = 16;
  float (*red)[64] = reinterpret_cast<float (*)[64]>(ldsb);
  const WgradProblem& p = q.p;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t j = p.begin + (int64_t)block * 64 + lane;
  const unsigned short* dY = (const unsigned short*)p.dY;
  const unsigned short* X = (const unsigned short*)p.X;
  for (int tg = wave; tg < TG; tg += C::NW) {
    float acc = 0.f;
    if (j < p.end)
#pragma unroll 8
      for (int64_t t = tg; t < p.T; t += TG) {
        const float x = bf16_bits_to_f32(X[t * p.ldx + j]);
        acc = fmaf(bf16_bits_to_f32(dY[t * p.lddy + j]), x, acc);
      }
    red[tg][lane] = acc;
  }
  __syncthreads();
  if (wave == 0 && j < p.end) {
    float sum = red[0][lane];
    for (int g = 1; g < TG; ++g) sum += red[g][lane];
    emit<MODE>(q.s, p.end - p.begin, 0, j - p.begin, j, sum);
  }
}

template <class C>
__global__ __launch_bounds__(C::NT, 2) void wgrad_group_kernel(const GroupParams gp) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char ldsb[];
  const int item = xcd_work_item(gp.n_items);
  if (item < 0) return;
  start_offset<C, EMIT_ADAMW>(gp.stagger);
  int si = 0;
  while (si + 1 < gp.n_segs && item >= gp.item_start[si + 1]) ++si;
  const MfmaParams& q = gp.seg[si];
  const int local = item - gp.item_start[si];
  if (q.tiles_m == 0) colsum_item<C, EMIT_ADAMW>(q, local, ldsb);
  else if constexpr (C::MI == 16) mfma_tile16<C, EMIT_ADAMW>(q, local, ldsb);
  else mfma_tile<C, EMIT_ADAMW>(q, local, ldsb);
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
// With NORM the operator normalises its input itself: X is the raw input and stats[2t],
// stats[2t+1] are the token's mean (0 for RMSNorm) and reciprocal standard deviation.
template <typename T, int MODE, int NORM>
__global__ __launch_bounds__(1024) void colsum_kernel(const WgradProblem p, const Sinks s, const float* stats) {
  constexpr int TG = 16;
  __shared__ float red[TG][64];
  const int lane = threadIdx.x & 63, tg = threadIdx.x >> 6;
  const int64_t j = p.begin + (int64_t)blockIdx.x * 64 + lane;
  const T* dY = (const T*)p.dY;
  const T* X = (const T*)p.X;
  float acc = 0.f;
  if (j < p.end)
#pragma unroll 8                                   // eight tokens' loads in flight; the sum keeps its order
    for (int64_t t = tg; t < p.T; t += TG) {
      float x = load_as_f32<T>(X + t * p.ldx + j);
      if constexpr (NORM) x = (x - stats[2 * t]) * stats[2 * t + 1];
      acc = fmaf(load_as_f32<T>(dY + t * p.lddy + j), x, acc);
    }
  red[tg][lane] = acc;
  __syncthreads();
  if (tg == 0 && j < p.end) {
    float sum = red[0][lane];
    for (int g = 1; g < TG; ++g) sum += red[g][lane];
    emit<MODE>(s, p.end - p.begin, 0, j - p.begin, j, sum);
  }
}

// Per-token statistics of RMSNorm (SUB = 0) or LayerNorm (SUB = 1): one wave per token, two
// passes over the row (mean first, then the centred sum of squares), fp32.
template <typename T, int SUB>
__global__ __launch_bounds__(256) void norm_stats_kernel(const T* X, int64_t ldx, int64_t n, int64_t tokens,
                                                         float eps, float* stats) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= tokens) return;
  const T* row = X + t * ldx;
  auto wave_sum = [](float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
  };
  float mean = 0.f;
  if constexpr (SUB) {
    float s1 = 0.f;
    for (int64_t j = lane; j < n; j += 64) s1 += load_as_f32<T>(row + j);
    mean = wave_sum(s1) / (float)n;
  }
  float s2 = 0.f;
  for (int64_t j = lane; j < n; j += 64) {
    const float d = load_as_f32<T>(row + j) - mean;
    s2 = fmaf(d, d, s2);
  }
  const float var = wave_sum(s2) / (float)n;
  if (lane == 0) {
    stats[2 * t] = mean;
    stats[2 * t + 1] = 1.0f / sqrtf(var + eps);
  }
}

// ---------------------------------------------------------------------------
// embedding table gradient: g[r, :] = sum over the tokens t with ids[t] = r of dY[t, :]
// ---------------------------------------------------------------------------
// A workgroup of 8 waves owns kEmbRows = 64 consecutive table rows and a block of 1024
// columns (blockIdx.y).  It first turns the token ids into "which of my rows, if any" in LDS
// (one coalesced pass over the ids per workgroup), its first wave compacts that in place into
// the short list of tokens that hit any of the 64 rows (token order kept), and then every
// wave takes 8 of the rows one after the other: it walks the list, picks the entries of its
// row and adds their dY rows in ascending token order -- no atomics, the order of the sum is
// fixed.  The loads of four tokens are issued before their additions, so a row that several
// tokens name does not cost one memory latency per token; a row that very many name (token
// frequencies are heavy-tailed: the commonest token can be a tenth of a batch) is summed by
// all eight waves together, wave w taking every eighth hit, and the eight partial sums are
// added in wave order -- still a fixed order.  A lane holds the columns 256 i + 4 lane + e (i < kEmbIter, e < 4), so loads and
// stores of a wave are 1 KB (fp32) pieces.  HBM-bound: the rows are written (or updated)
// once, whether any token names them or not -- except when the result is added to g
// (accumulation over micro-batches), where only the named rows are touched.
constexpr int kEmbWaves = 8;
constexpr int kEmbRows = 64;       // rows per workgroup, kEmbRows / kEmbWaves per wave
constexpr int kEmbIter = 4;        // 256-column pieces per workgroup
constexpr int kEmbTok = 8192;      // most tokens per call (their list lives in LDS)
constexpr int kEmbHot = 32;        // hits from which a row is summed by all waves together ...
constexpr int kEmbHotMax = 2;      // ... for at most this many rows of a workgroup

template <typename T> __device__ __forceinline__ void load4_as_f32(const T* p, int valid, float (&o)[4]);
template <> __device__ __forceinline__ void load4_as_f32<float>(const float* p, int valid, float (&o)[4]) {
  if (valid >= 4) {
    const f32x4_u v = *(const f32x4_u*)p;
    o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = e < valid ? p[e] : 0.f;
  }
}
template <> __device__ __forceinline__ void load4_as_f32<unsigned short>(const unsigned short* p, int valid,
                                                                         float (&o)[4]) {
  if (valid >= 4) {
    const u32x2_a2 v = *(const u32x2_a2*)p;
    o[0] = __uint_as_float(v[0] << 16); o[1] = __uint_as_float(v[0] & 0xffff0000u);
    o[2] = __uint_as_float(v[1] << 16); o[3] = __uint_as_float(v[1] & 0xffff0000u);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = e < valid ? bf16_bits_to_f32(p[e]) : 0.f;
  }
}

template <typename T, int MODE>
__global__ __launch_bounds__(64 * kEmbWaves) void embed_wgrad_kernel(const WgradProblem p, const Sinks s) {
  __shared__ int list[kEmbTok];
  __shared__ int list_len, n_hot;
  __shared__ int hits_of[kEmbRows], hot_row[kEmbHotMax];
  __shared__ float part[kEmbWaves][256 * kEmbIter];
  __shared__ float hot_sum[kEmbHotMax][256 * kEmbIter];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // column blocks of one group of rows are neighbours in the launch order, so that a row's
  // pieces are touched at about the same time
  const int n_cblk = (int)((p.in + 256 * kEmbIter - 1) / (256 * kEmbIter));
  const int64_t row_base = p.begin / p.in + (int64_t)(blockIdx.x / n_cblk) * kEmbRows;
  const int64_t row_last = (p.end - 1) / p.in;
  const int64_t cbase = (int64_t)(blockIdx.x % n_cblk) * (256 * kEmbIter);
  const int64_t* ids = (const int64_t*)p.X;
  const T* dY = (const T*)p.dY;
  const int n = (int)p.T;                                   // <= kEmbTok, checked by the launcher
  for (int i = threadIdx.x; i < n; i += 64 * kEmbWaves) {
    const int64_t d = ids[i] - row_base;
    list[i] = (d >= 0 && d < kEmbRows) ? (int)d : -1;
  }
  __syncthreads();
  // wave 0: in-place compaction to entries (token << 6 | row), in token order; the write
  // position never passes the read position
  if (wave == 0) {
    int count = 0;
    for (int t0 = 0; t0 < n; t0 += 64) {
      const int w = t0 + lane < n ? list[t0 + lane] : -1;
      const unsigned long long hits = __ballot(w >= 0);
      if (w >= 0) list[count + __popcll(hits & ((1ull << lane) - 1ull))] = ((t0 + lane) << 6) | w;
      count += __popcll(hits);
    }
    if (lane == 0) list_len = count;
  }
  __syncthreads();
  const int len = list_len;
  const int64_t E = p.end - p.begin;
  // adding to g: rows that no token names stay as they are, their traffic is saved
  if (MODE == EMIT_ACCUM && len == 0) return;               // the same for every thread

  // NT tokens at a time into `into`: all their loads, then their additions in token order
  auto add_tokens = [&](float (&into)[kEmbIter][4], auto ntc, int ta, int tb, int tc, int td) {
    constexpr int NT = decltype(ntc)::value;
    const int tok[4] = {ta, tb, tc, td};
    float x[NT][kEmbIter][4];
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const T* src = dY + (int64_t)tok[k] * p.lddy;
#pragma unroll
      for (int i = 0; i < kEmbIter; ++i) {
        const int64_t c = cbase + i * 256 + 4 * lane;
        if (c < p.in) load4_as_f32<T>(src + c, (int)(p.in - c < 4 ? p.in - c : 4), x[k][i]);
        else x[k][i][0] = x[k][i][1] = x[k][i][2] = x[k][i][3] = 0.f;
      }
    }
#pragma unroll
    for (int k = 0; k < NT; ++k)
#pragma unroll
      for (int i = 0; i < kEmbIter; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) into[i][e] += x[k][i][e];
  };
  // Sum of the hits of local row `r` that `mine(ordinal)` selects, ordinal = 0, 1, ... in token order.
  auto gather = [&](float (&into)[kEmbIter][4], int r, auto mine) {
    int q0 = 0, q1 = 0, q2 = 0, pending = 0, ordinal = 0;     // the last tokens found, oldest in q2
    for (int j = 0; j < len; ++j) {
      const int e = list[j];                                  // the same for every lane
      if ((e & 63) != r) continue;
      if (!mine(ordinal++)) continue;
      const int t = e >> 6;
      if (pending == 3) {
        add_tokens(into, IntC<4>{}, q2, q1, q0, t);
        pending = 0;
      } else {
        q2 = q1; q1 = q0; q0 = t;
        ++pending;
      }
    }
    if (pending == 3) { add_tokens(into, IntC<2>{}, q2, q1, 0, 0); add_tokens(into, IntC<1>{}, q0, 0, 0, 0); }
    else if (pending == 2) add_tokens(into, IntC<2>{}, q1, q0, 0, 0);
    else if (pending == 1) add_tokens(into, IntC<1>{}, q0, 0, 0, 0);
  };

  // ---- rows with very many hits: all waves together
  for (int i = threadIdx.x; i < kEmbRows; i += 64 * kEmbWaves) hits_of[i] = 0;
  __syncthreads();
  for (int j = threadIdx.x; j < len; j += 64 * kEmbWaves) atomicAdd(&hits_of[list[j] & 63], 1);
  __syncthreads();
  if (threadIdx.x == 0) {
    int nh = 0;
    for (int r = 0; r < kEmbRows && nh < kEmbHotMax; ++r)
      if (hits_of[r] >= kEmbHot) hot_row[nh++] = r;
    n_hot = nh;
  }
  __syncthreads();
  const int nh = n_hot;
  for (int h = 0; h < nh; ++h) {
    float pacc[kEmbIter][4];
#pragma unroll
    for (int i = 0; i < kEmbIter; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) pacc[i][e] = 0.f;
    gather(pacc, hot_row[h], [&](int ordinal) { return (ordinal & (kEmbWaves - 1)) == wave; });
#pragma unroll
    for (int i = 0; i < kEmbIter; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) part[wave][i * 256 + 4 * lane + e] = pacc[i][e];
    __syncthreads();
    for (int c = threadIdx.x; c < 256 * kEmbIter; c += 64 * kEmbWaves) {
      float sum = part[0][c];
#pragma unroll
      for (int w = 1; w < kEmbWaves; ++w) sum += part[w][c];
      hot_sum[h][c] = sum;
    }
    __syncthreads();
  }

  for (int sub = 0; sub < kEmbRows / kEmbWaves; ++sub) {
    const int local = sub * kEmbWaves + wave;               // consecutive rows go to different waves
    const int64_t row = row_base + local;
    if (row > row_last) break;
    if (MODE == EMIT_ACCUM && hits_of[local] == 0) continue;
    float acc[kEmbIter][4];
#pragma unroll
    for (int i = 0; i < kEmbIter; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][e] = 0.f;
    // The row's state is requested first, so that it travels while the hit list is walked.
    Vec4Sink d[kEmbIter];
    State4 st[kEmbIter];
    bool whole[kEmbIter];
#pragma unroll
    for (int i = 0; i < kEmbIter; ++i) {
      const int64_t c = cbase + i * 256 + 4 * lane;
      const int64_t flat = row * p.in + c;
      whole[i] = c + 4 <= p.in && flat >= p.begin && flat + 4 <= p.end;
      const int64_t k = flat - p.begin;
      d[i].g = s.g + k;
      d[i].master = s.master + k;
      d[i].m = s.m + k;
      d[i].v = s.v + k;
      d[i].W = s.w_kind == W_BF16 ? (void*)((unsigned short*)s.W + flat) : (void*)((float*)s.W + flat);
      if (whole[i]) st[i] = load_state4<MODE>(d[i]);
    }
    int hot = -1;
    for (int h = 0; h < nh; ++h)
      if (hot_row[h] == local) hot = h;
    if (hot >= 0) {
#pragma unroll
      for (int i = 0; i < kEmbIter; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][e] = hot_sum[hot][i * 256 + 4 * lane + e];
    } else {
      gather(acc, local, [](int) { return true; });
    }

#pragma unroll
    for (int i = 0; i < kEmbIter; ++i) {
      const int64_t c = cbase + i * 256 + 4 * lane;
      if (c >= p.in) continue;
      const int64_t flat = row * p.in + c;
      if (whole[i]) {
        const f32x4_u val = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
        finish4<MODE>(d[i], s.w_kind, s.c, val, st[i]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (c + e < p.in && flat + e >= p.begin && flat + e < p.end)
            emit<MODE>(s, E, 0, flat + e - p.begin, flat + e, acc[i][e]);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// element-wise pass: AdamW and/or the sum of slab partials (HBM-bound)
// ---------------------------------------------------------------------------
struct ElemParams {
  const float* src;     // g (S = 0) or the slab partials, slab sl at src + sl * pitch
  int32_t S;            // 0: src is g itself
  int64_t n;
  int64_t pitch;
  int64_t head;         // elements before the first 4-element group (at most 31)
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
    for (int32_t sl = 1; sl < q.S; ++sl) val += q.src[(int64_t)sl * q.pitch + i];
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

template <int MODE, int U = 1>
__global__ __launch_bounds__(256) void elementwise_kernel(const ElemParams q) {
  const int64_t nvec = (q.n - q.head) >> 2;
  if (blockIdx.x == 0 && threadIdx.x < 36) {
    // the few elements before (at most 31) and after (at most 3) the 4-element groups
    const int64_t tail0 = q.head + (nvec << 2);
    const int64_t i = threadIdx.x < 32 ? (int64_t)threadIdx.x : tail0 + (threadIdx.x - 32);
    const bool ok = threadIdx.x < 32 ? (i < q.head) : (i < q.n);
    if (ok) elem_one<MODE>(q, i);
  }
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  // U 4-element groups per trip, all loads ahead of the arithmetic
  for (int64_t j0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j0 < nvec; j0 += U * stride) {
    Vec4Sink d[U];
    State4 st[U];
    f32x4_u val[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t j = j0 + u * stride;
      ok[u] = j < nvec;
      const int64_t i = q.head + (j << 2);
      d[u].g = q.g_out + i;
      d[u].master = q.master + i;
      d[u].m = q.m + i;
      d[u].v = q.v + i;
      d[u].W = q.w_kind == W_BF16 ? (void*)((unsigned short*)q.W + i) : (void*)((float*)q.W + i);
      if (ok[u]) {
        val[u] = __builtin_nontemporal_load((const f32x4_u*)(q.src + i));
        for (int32_t sl = 1; sl < q.S; ++sl)
          val[u] += __builtin_nontemporal_load((const f32x4_u*)(q.src + (int64_t)sl * q.pitch + i));
        st[u] = load_state4<MODE>(d[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) finish4<MODE>(d[u], q.w_kind, q.c, val[u], st[u]);
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Start delay (units of 8128 cycles) of the second workgroup of each compute unit in the fused
// call, whose epilogue is long and HBM-bound: measured best at 6 for 1024 tokens (196 us against
// 200 us at 8, 208 us at 0), flat between 6 and 10 for 4096 and 8192; the plain gradient gains
// nothing.
constexpr int kStaggerAdamW = 6;
// The large tile has one workgroup per compute unit: there every second compute unit of an XCD starts
// late, so that the epilogues of half the part fall into the loops of the other half (measured at
// T = 8192: 1 - 3 % at 10, nothing from 24 on).
constexpr int kStaggerAdamWLarge = 10;
// 256 x 256 tiles, four slabs of 33 KB in LDS, one workgroup per compute unit: both waves of a SIMD are in
// the loop together, which the 16x16x32 MFMA needs (a wave then issues one MFMA per 32 cycles; alone
// on its SIMD it would have to issue one per 16 cycles beside its reads and loads, and cannot)
using MainCfg = RingCfg<2, 4, 16>;
// 128 x 256 tiles, three slabs of 25 KB, two workgroups per compute unit: while its partner is in its
// epilogue a workgroup's waves are alone on their SIMDs, so this one keeps the 32x32x16 MFMA (with the
// other shape its loops were 10 % slower).  The two shapes give the same bits: the hardware adds the
// tokens of either in the same order.
using FusedCfg = RingCfg<1, 3, 32>;
                                  // (the fused call, and plain gradients with few tiles)

template <class C, int MODE>
int launch_mfma_mode(const MfmaParams& q, int grid, hipStream_t st) {
  // The dynamic LDS limit is a per-device attribute of the kernel; raising it is idempotent, so
  // a race between threads only repeats the call.
  static std::atomic<bool> attr_set[kMaxDevices] = {};
  const auto kern = &wgrad_mfma_kernel<C, MODE>;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev >= kMaxDevices || !attr_set[dev].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::LDS_BYTES);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev < kMaxDevices) attr_set[dev].store(true, std::memory_order_release);
  }
  MfmaArgs args;
  args.q[0] = q;
#ifdef CHUNKFT_TIMELINE
  args.q[0].timeline = g_timeline_words >= (size_t)q.n_tile_items * 8 ? g_timeline : nullptr;
#endif
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS_BYTES, st, args);
  return (int)hipGetLastError();
}

}  // namespace

static_assert(MainCfg::BM == kMainTileM && MainCfg::BN == kMainTileN && MainCfg::BK == kMainTileK,
              "the token split is chosen from these tile sizes");

// Compute units of the current device, asked once per device (a launch-shape input: how many
// workgroups fill the part).  Without a device -- the host-only size queries on a machine
// that has none -- the count of the MI355X this library is written for.
int device_compute_units() {
  static std::atomic<int> cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return kDefaultComputeUnits; }
  if (dev < kMaxDevices) {
    const int c = cached[dev].load(std::memory_order_relaxed);
    if (c > 0) return c;
  }
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return kDefaultComputeUnits;
  }
  if (dev < kMaxDevices) cached[dev].store(cus, std::memory_order_relaxed);
  return cus;
}

// Parameters of the MFMA kernel for a call.  False if the work items cannot be counted in 32 bits.
template <class C>
bool fill_mfma_params(const WgradProblem& p, int mode, const Sinks& s, const RowSplit& rs, MfmaParams& q) {
  const bool folded = edge_rows_folded(rs);
  q = MfmaParams{};
  q.p = p;
  q.s = s;
  q.rb0 = rs.rb0;
  q.rb1 = rs.rb1;
  q.lead_base = folded ? rs.lead_base : -1;
  q.trail_row = folded ? rs.trail_row : -1;
  const int64_t tiles_m = ceil_div(rs.rb1 - rs.rb0, C::BM), tiles_n = ceil_div(p.in, C::BN);
  if (tiles_m > 0x3fffffff || tiles_n > 0x3fffffff || tiles_m * tiles_n > 0x3fffffff / p.S) return false;
  q.tiles_m = (int32_t)tiles_m;
  q.tiles_n = (int32_t)tiles_n;
  q.n_tile_items = (int32_t)(tiles_m * tiles_n * p.S);
  // Order of the tiles inside an XCD's run of work items: groups of 8 tile rows (4 of the fused
  // call's smaller tiles), column tile by column tile, so that X tiles stay in that L2.  Measured
  // for the fused call on 4096 x 14336 at T = 4096: 571 us in groups of 4 against 736 us row-major;
  // on 14336 x 4096 at T = 1024: 313 against 335 us.
  q.group_m = mode == EMIT_ADAMW ? 4 : 8;
  q.stagger = mode == EMIT_ADAMW ? (C::WM == 1 ? kStaggerAdamW : kStaggerAdamWLarge) : 0;
  return true;
}

int launch_edge_rows(const WgradProblem& p, int mode, const Sinks& s, const RowSplit& rs, hipStream_t st) {
  EdgeParams e{};
  e.p = p;
  e.s = s;
  e.lead_base = rs.lead_base;
  e.trail_row = rs.trail_row;
  const dim3 grid((unsigned)ceil_div(p.in, kEdgeCols)), block(kEdgeThreads);
  switch (mode) {
    case EMIT_STORE: hipLaunchKernelGGL((wgrad_edge_kernel<EMIT_STORE>), grid, block, 0, st, e); break;
    case EMIT_ACCUM: hipLaunchKernelGGL((wgrad_edge_kernel<EMIT_ACCUM>), grid, block, 0, st, e); break;
    case EMIT_PARTIAL: hipLaunchKernelGGL((wgrad_edge_kernel<EMIT_PARTIAL>), grid, block, 0, st, e); break;
    default: hipLaunchKernelGGL((wgrad_edge_kernel<EMIT_ADAMW>), grid, block, 0, st, e); break;
  }
  return (int)hipGetLastError();
}

template <class C>
int launch_mfma_cfg(const WgradProblem& p, int mode, const Sinks& s, hipStream_t st) {
  const RowSplit rs = split_rows(p);
  if (!edge_rows_folded(rs) && (rs.lead_base >= 0 || rs.trail_row >= 0)) {
    const int err = launch_edge_rows(p, mode, s, rs, st);
    if (err != 0) return err;
  }
  if (rs.rb1 <= rs.rb0) return 0;
  MfmaParams q;
  if (!fill_mfma_params<C>(p, mode, s, rs, q)) return (int)hipErrorInvalidValue;   // work items are counted in 32 bits
  const int grid = (q.n_tile_items + 7) / 8 * 8;
  switch (mode) {
    case EMIT_STORE: return launch_mfma_mode<C, EMIT_STORE>(q, grid, st);
    case EMIT_ACCUM: return launch_mfma_mode<C, EMIT_ACCUM>(q, grid, st);
    case EMIT_PARTIAL: return launch_mfma_mode<C, EMIT_PARTIAL>(q, grid, st);
    default: return launch_mfma_mode<C, EMIT_ADAMW>(q, grid, st);
  }
}

int launch_wgrad_bf16_mfma(const WgradProblem& p, int mode, const Sinks& s, void* stream) {
  // The plain gradient (short epilogue) is a little faster on the large tile; the fused call,
  // whose epilogue moves 26 bytes per element, gains from two workgroups per compute unit.
  if (mode == EMIT_ADAMW) {
    if (fused_takes_large_tile(p, device_compute_units())) return launch_mfma_cfg<MainCfg>(p, mode, s, (hipStream_t)stream);
    return launch_mfma_cfg<FusedCfg>(p, mode, s, (hipStream_t)stream);
  }
  // The plain gradient takes whichever tile is faster for its number of tiles and tokens
  // (plain_takes_large_tile, csrc/shape.cpp); every element is summed over the tokens in the same
  // order either way.
  const RowSplit rs = split_rows(p);
  const int64_t big_tiles = ceil_div(rs.rb1 - rs.rb0, MainCfg::BM) * ceil_div(p.in, MainCfg::BN) * p.S;
  const int64_t slab_tokens = p.S > 1 ? p.kslab : p.T;
  if (!plain_takes_large_tile(big_tiles, slab_tokens, device_compute_units()))
    return launch_mfma_cfg<FusedCfg>(p, mode, s, (hipStream_t)stream);
  return launch_mfma_cfg<MainCfg>(p, mode, s, (hipStream_t)stream);
}

// ---- grouped fused call
template <class C>
static int launch_group_cfg(const GroupSegment* segs, int n, hipStream_t st) {
  static std::atomic<bool> attr_set[kMaxDevices] = {};
  const auto kern = &wgrad_group_kernel<C>;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev >= kMaxDevices || !attr_set[dev].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::LDS_BYTES);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev < kMaxDevices) attr_set[dev].store(true, std::memory_order_release);
  }
  for (int first = 0; first < n; first += kGroupMax) {
    const int count = n - first < kGroupMax ? n - first : kGroupMax;
    GroupParams gp{};
    int64_t items = 0;
    for (int i = 0; i < count; ++i) {
      const GroupSegment& g = segs[first + i];
      MfmaParams& q = gp.seg[i];
      gp.item_start[i] = (int32_t)items;
      if (g.vector) {
        q = MfmaParams{};
        q.p = g.p;
        q.s = g.s;
        q.tiles_m = 0;
        items += ceil_div(g.p.end - g.p.begin, 64);
      } else {
        if (!fill_mfma_params<C>(g.p, EMIT_ADAMW, g.s, split_rows(g.p), q)) return (int)hipErrorInvalidValue;
        gp.stagger = q.stagger;
        items += q.n_tile_items;
      }
      if (items > 0x3fffffff) return (int)hipErrorInvalidValue;
    }
    if (gp.stagger == 0) gp.stagger = C::WM == 1 ? kStaggerAdamW : kStaggerAdamWLarge;
    gp.item_start[count] = (int32_t)items;
    gp.n_segs = count;
    gp.n_items = (int32_t)items;
    const int grid = (gp.n_items + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS_BYTES, st, gp);
    const int err = (int)hipGetLastError();
    if (err != 0) return err;
  }
  return 0;
}

int launch_fused_group(const GroupSegment* segs, int n, bool large_tile, void* stream) {
  if (n <= 0) return 0;
  return large_tile ? launch_group_cfg<MainCfg>(segs, n, (hipStream_t)stream)
                    : launch_group_cfg<FusedCfg>(segs, n, (hipStream_t)stream);
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
  const int64_t tiles_m = ceil_div(rows, 64), tiles_n = ceil_div(p.in, 64);
  if (tiles_m > 0x7fffffff || tiles_n > 0x7fffffff || tiles_m * tiles_n > 0x7fffffff / p.S)
    return (int)hipErrorInvalidValue;                  // the grid is counted in 32 bits
  q.tiles_m = (int32_t)tiles_m;
  q.tiles_n = (int32_t)tiles_n;
  const int64_t grid = tiles_m * tiles_n * p.S;
  hipStream_t st = (hipStream_t)stream;
  return dtype == 0 ? launch_simt_t<float>(q, (int)grid, mode, st)
                    : launch_simt_t<unsigned short>(q, (int)grid, mode, st);
}

template <typename T, int NORM>
static int launch_colsum_t(const WgradProblem& p, int grid, int mode, const Sinks& s, const float* stats,
                           hipStream_t st) {
  switch (mode) {
    case EMIT_STORE: hipLaunchKernelGGL((colsum_kernel<T, EMIT_STORE, NORM>), dim3(grid), dim3(1024), 0, st, p, s, stats); break;
    case EMIT_ACCUM: hipLaunchKernelGGL((colsum_kernel<T, EMIT_ACCUM, NORM>), dim3(grid), dim3(1024), 0, st, p, s, stats); break;
    default: hipLaunchKernelGGL((colsum_kernel<T, EMIT_ADAMW, NORM>), dim3(grid), dim3(1024), 0, st, p, s, stats); break;
  }
  return (int)hipGetLastError();
}

int launch_colsum(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream) {
  const int64_t grid = ceil_div(p.end - p.begin, 64);
  if (grid > 0x7fffffff) return (int)hipErrorInvalidValue;
  hipStream_t st = (hipStream_t)stream;
  return dtype == 0 ? launch_colsum_t<float, 0>(p, (int)grid, mode, s, nullptr, st)
                    : launch_colsum_t<unsigned short, 0>(p, (int)grid, mode, s, nullptr, st);
}

int launch_norm_wgrad(const WgradProblem& p, int dtype, bool subtract_mean, float eps, float* stats, int mode,
                      const Sinks& s, void* stream) {
  const int64_t grid = ceil_div(p.end - p.begin, 64), sgrid = ceil_div(p.T, 4);
  if (grid > 0x7fffffff || sgrid > 0x7fffffff) return (int)hipErrorInvalidValue;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == 0) {
    if (subtract_mean) hipLaunchKernelGGL((norm_stats_kernel<float, 1>), dim3((int)sgrid), dim3(256), 0, st, (const float*)p.X, p.ldx, p.in, p.T, eps, stats);
    else hipLaunchKernelGGL((norm_stats_kernel<float, 0>), dim3((int)sgrid), dim3(256), 0, st, (const float*)p.X, p.ldx, p.in, p.T, eps, stats);
  } else {
    if (subtract_mean) hipLaunchKernelGGL((norm_stats_kernel<unsigned short, 1>), dim3((int)sgrid), dim3(256), 0, st, (const unsigned short*)p.X, p.ldx, p.in, p.T, eps, stats);
    else hipLaunchKernelGGL((norm_stats_kernel<unsigned short, 0>), dim3((int)sgrid), dim3(256), 0, st, (const unsigned short*)p.X, p.ldx, p.in, p.T, eps, stats);
  }
  const int err = (int)hipGetLastError();
  if (err != 0) return err;
  return dtype == 0 ? launch_colsum_t<float, 1>(p, (int)grid, mode, s, stats, st)
                    : launch_colsum_t<unsigned short, 1>(p, (int)grid, mode, s, stats, st);
}

template <typename T>
static int launch_embed_t(const WgradProblem& p, dim3 grid, int mode, const Sinks& s, hipStream_t st) {
  // The update streams seven arrays: it runs 8 % faster with one workgroup per CU than with the
  // two that fit (4.06 against 3.73 TB/s), so that mode asks for LDS it does not use; the plain
  // gradient only writes and is faster with two.
  const size_t pad = mode == EMIT_ADAMW ? 40 * 1024 : 0;
  switch (mode) {
    case EMIT_STORE: hipLaunchKernelGGL((embed_wgrad_kernel<T, EMIT_STORE>), grid, dim3(64 * kEmbWaves), pad, st, p, s); break;
    case EMIT_ACCUM: hipLaunchKernelGGL((embed_wgrad_kernel<T, EMIT_ACCUM>), grid, dim3(64 * kEmbWaves), pad, st, p, s); break;
    default: hipLaunchKernelGGL((embed_wgrad_kernel<T, EMIT_ADAMW>), grid, dim3(64 * kEmbWaves), pad, st, p, s); break;
  }
  return (int)hipGetLastError();
}

int launch_embed_wgrad(const WgradProblem& p, int dtype, int mode, const Sinks& s, void* stream) {
  const int64_t rows = (p.end - 1) / p.in - p.begin / p.in + 1;
  const int64_t gx = ceil_div(rows, kEmbRows), gy = ceil_div(p.in, 256 * kEmbIter);
  if (gy > 65535 || gx > 0x7fffffff / gy || p.T > kEmbTok) return (int)hipErrorInvalidValue;
  const dim3 grid((unsigned)(gx * gy));
  return dtype == 0 ? launch_embed_t<float>(p, grid, mode, s, (hipStream_t)stream)
                    : launch_embed_t<unsigned short>(p, grid, mode, s, (hipStream_t)stream);
}

static int launch_elem(ElemParams& q, int mode, hipStream_t st) {
  // the first 4-element group starts where the fp32 arrays are 128-byte aligned (judged by the
  // master weights for the update, by the output gradient otherwise): the 1 KB a wave requests
  // per array is then eight whole lines; at a 16-byte phase inside a line it is nine, and the
  // pass 14 % slower (measured)
  const void* ref = mode == EMIT_ADAMW ? (const void*)q.master : (const void*)q.g_out;
  int64_t head = ((128 - (reinterpret_cast<uintptr_t>(ref) & 127u)) & 127u) / 4;
  if (head > q.n) head = q.n;
  q.head = head;
  const int64_t nvec = (q.n - head) >> 2;
  int64_t blocks = ceil_div(nvec, 256);
  // One block of 256 threads per CU, one group of four elements per thread in flight: the
  // seven streams of the update then reach 5.9 - 6.0 TB/s; with twice the blocks, or twice the
  // groups per trip, HBM efficiency drops to 5.3 - 5.4 TB/s (measured sweep).
  const int64_t cap = (int64_t)device_compute_units();
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
  q.pitch = s.ws_pitch;
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
