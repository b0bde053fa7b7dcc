/*
 * libchunkft -- the ChunkFT hot path on one MI355X (gfx950).
 *
 * ChunkFT fine-tunes all parameters of a model by rotating over "chunks":
 * byte-budgeted, contiguous element ranges of the flattened row-major
 * parameter tensors.  At each step only the active chunk gets a gradient
 * (never a dense one) and an AdamW update whose fp32 master weights and
 * moments exist for that chunk alone.  This library is that step:
 *
 *   chunkft_plan_cycle         byte budget -> chunks covering every element once
 *   chunkft_chunk_wgrad        g[chunk] = (dY^T X)[chunk], dense dW never formed
 *   chunkft_adamw_chunk        AdamW on the chunk's fp32 state (+ bf16 write-back)
 *   chunkft_wgrad_adamw_fused  both, g never leaving the chip when it need not
 *
 * Conventions
 *   - A linear layer computes y = x W^T; W is [out, in] row-major, X is
 *     [T, in], dY is [T, out], T = batch x sequence flattened.
 *   - A chunk segment on one tensor is the flat element range [begin, end),
 *     flat = r * in + c.  It may start and end mid-row.
 *   - Chunk-local arrays (g, master, m, v) hold element `begin + i` at index i.
 *   - All sizes and offsets are in ELEMENTS unless the name ends in _bytes.
 *   - Pointers marked (device) must be device memory reachable from the
 *     current HIP device; pointers marked (host) are ordinary host memory.
 *   - The library allocates no device memory and keeps no data between
 *     calls (its only process state is, per device, the number of compute
 *     units and a flag per kernel that its LDS size attribute has been set).
 *     Every buffer is owned by the caller.
 *   - Device entry points validate their arguments synchronously, then
 *     enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without waiting.  They return CHUNKFT_OK or
 *     a negative chunkft_status; nothing throws or aborts across this ABI.
 *     On every status but CHUNKFT_ERR_HIP nothing has been enqueued and no
 *     buffer has been touched.  CHUNKFT_ERR_HIP means the runtime refused a
 *     launch: a call that takes several kernels (a token split, a chunk of a
 *     few rows) may then have enqueued the earlier ones, so the outputs and
 *     the workspace of that call are unspecified.
 *   - Identical inputs give bit-identical outputs on every call.
 */
#ifndef CHUNKFT_H
#define CHUNKFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CHUNKFT_OK = 0,
  CHUNKFT_ERR_INVALID_ARG = -1,      /* null pointer, non-positive size, bad stride, bad hyper-parameter */
  CHUNKFT_ERR_RANGE = -2,            /* [begin, end) empty or outside the tensor */
  CHUNKFT_ERR_DTYPE = -3,            /* unknown dtype / kind, or a combination not supported */
  CHUNKFT_ERR_WORKSPACE = -4,        /* workspace missing, misaligned or smaller than chunkft_workspace_bytes */
  CHUNKFT_ERR_BUFFER_TOO_SMALL = -5, /* planner output arrays too short; required counts were written */
  CHUNKFT_ERR_HIP = -6,              /* the HIP runtime refused a launch */
  CHUNKFT_ERR_OVERFLOW = -7,         /* an element or byte count does not fit int64 */
  CHUNKFT_ERR_STATIC_WORKSPACE = -8  /* the call needs more workspace than CHUNKFT_STATIC_WORKSPACE_BYTES */
} chunkft_status;

typedef enum { CHUNKFT_F32 = 0, CHUNKFT_BF16 = 1 } chunkft_dtype;

/* The chunk-aware backward operators (Algorithm 1 line 8 and the paper's list of
 * supported modules: Linear, Embedding, LayerNorm, RMSNorm).
 *   LINEAR     a weight matrix of y = x W^T.
 *   VECTOR     a 1-D scale vector whose NORMALISED input the caller supplies
 *              (rows = 1, cols = length).
 *   EMBEDDING  a lookup table y[t] = W[ids[t]] of rows x cols.
 *   RMSNORM    the scale vector of y = w * x / sqrt(mean(x^2) + eps); the operator
 *   LAYERNORM  the scale vector of y = w * (x - mean) / sqrt(var + eps) + b;
 *              both normalise the raw input themselves (rows = 1). */
typedef enum {
  CHUNKFT_LINEAR = 0, CHUNKFT_VECTOR = 1, CHUNKFT_EMBEDDING = 2, CHUNKFT_RMSNORM = 3, CHUNKFT_LAYERNORM = 4
} chunkft_kind;

/* ------------------------------------------------------------------------
 * Cycle planner (host only)
 *
 * Paper: Section 3 "Method", first paragraph, and Algorithm 1 lines 1-2: the
 * size of a tensor is numel x element_size; parameters are accumulated in
 * model order until a byte budget is reached; a tensor larger than what is
 * left is split and so spans several chunks.  The chunks are a disjoint
 * partition of all trainable elements (Section 3.2).
 * ---------------------------------------------------------------------- */
typedef struct {
  int64_t rows, cols;   /* W is rows x cols (out x in); VECTOR: rows = 1 */
  int32_t dtype;        /* chunkft_dtype of the stored parameter */
  int32_t kind;         /* chunkft_kind */
} chunkft_tensor_desc;

typedef struct {
  int32_t tensor;       /* index into the tensor array */
  int32_t reserved;     /* written as 0 */
  int64_t begin, end;   /* flat element range of that tensor */
  int64_t chunk_off;    /* index of `begin` in the chunk-local state arrays */
} chunkft_segment;

typedef struct {
  int64_t seg_begin, seg_end; /* this chunk's segments are segs[seg_begin, seg_end) */
  int64_t numel;              /* elements in the chunk = length of its g/master/m/v */
  int64_t cost_bytes;         /* bytes charged against the budget */
} chunkft_chunk;

/* flags */
#define CHUNKFT_PLAN_GREEDY 0u
/* Charge each element its full training footprint instead of its storage size:
 * parameter + fp32 gradient + fp32 master + fp32 m + fp32 v = element_size + 16
 * (the cost listed in Section 3.1, first paragraph). */
#define CHUNKFT_PLAN_TRAINING_COST 1u
/* Keep the greedy chunk count K but lower the per-chunk budget to the
 * smallest multiple of 4 bytes >= ceil(total / K) for which K chunks still
 * suffice, so every chunk is close to the mean cost (byte-balance condition,
 * Appendix "Analysis of Memory Jitter"). */
#define CHUNKFT_PLAN_BALANCED 2u
/* Cut a tensor between rows only, in groups of 8 rows: where the open chunk cannot
 * take the rest of a tensor it takes the largest whole number of 8-row groups that
 * fits (none: the chunk is closed and the tensor goes on in the next one), so that
 * every segment begins and ends on a row that is a multiple of 8 or at an end of
 * its tensor (Section 3 "Method", first paragraph, splits large matrices along the
 * row dimension; the multiple of 8 is what the gradient kernel can do without its
 * edge-row path).
 * A tensor of which not even one 8-row group fits an empty chunk is cut anywhere,
 * as without the flag.  Chunks may stay below the budget by up to one group. */
#define CHUNKFT_PLAN_ROWS8 4u

/*
 * tensors (host, in)   n_tensors descriptors in model order.
 * budget_bytes         > 0 and >= the per-element cost of every non-empty tensor.
 * chunks (host, out)   array of chunks_cap entries, may be NULL when chunks_cap = 0.
 * segs (host, out)     array of segs_cap entries, may be NULL when segs_cap = 0.
 * n_chunks, n_segs (host, out, required)  always receive the counts the plan needs.
 *
 * Count-then-fill: if either capacity is short the counts are still written,
 * the arrays are left untouched and CHUNKFT_ERR_BUFFER_TOO_SMALL is returned.
 * Zero-element tensors produce no segment; an empty tensor list gives 0 chunks.
 * Errors: CHUNKFT_ERR_INVALID_ARG (null required pointer, budget too small,
 * negative shape, unknown flag), CHUNKFT_ERR_DTYPE, CHUNKFT_ERR_OVERFLOW.
 */
int chunkft_plan_cycle(const chunkft_tensor_desc* tensors, int32_t n_tensors,
                       int64_t budget_bytes, uint32_t flags,
                       chunkft_chunk* chunks, int64_t chunks_cap, int64_t* n_chunks,
                       chunkft_segment* segs, int64_t segs_cap, int64_t* n_segs);

/* ------------------------------------------------------------------------
 * Summary of a plan (host only)
 *
 * Paper: appendix "Analysis of Memory Jitter".  With the step memory of chunk k
 * taken as M_k = resident_bytes + B(C_k) (the appendix's 2M + B(C_k), activations
 * and temporary buffers left out) and B(C_k) = chunks[k].cost_bytes:
 *   mean_cost_bytes  (1/K) sum_k B(C_k)
 *   imbalance_bytes  eps_B = max_k | B(C_k) - mean |
 *   jitter           (max_k M_k - min_k M_k) / ((1/K) sum_k M_k)
 *   jitter_bound     2 eps_B / (resident_bytes + mean), which the appendix gives
 *                    as the bound of the jitter (it holds exactly for this M_k).
 * Plan with CHUNKFT_PLAN_TRAINING_COST for B to be the appendix's
 * parameter + gradient + master + optimizer bytes; resident_bytes is then
 * 2 bytes per parameter of the whole model for bf16 weights.
 * ---------------------------------------------------------------------- */
typedef struct {
  int64_t n_chunks;
  int64_t min_cost_bytes, max_cost_bytes;
  double mean_cost_bytes, imbalance_bytes, jitter, jitter_bound;
} chunkft_plan_summary;

/* chunks (host, in)  n_chunks >= 1 entries as chunkft_plan_cycle wrote them (only
 *                    cost_bytes is read, each >= 0);  resident_bytes >= 0;
 * out (host, out).   Errors: CHUNKFT_ERR_INVALID_ARG. */
int chunkft_plan_stats(const chunkft_chunk* chunks, int64_t n_chunks, int64_t resident_bytes,
                       chunkft_plan_summary* out);

/* ------------------------------------------------------------------------
 * Rotating schedule (host only)
 *
 * Paper: Algorithm 1, the loop over training steps: the same chunk is optimised
 * for `interval` consecutive steps, then the next one in round-robin order;
 * its state is brought in before the first of those steps and sent back after
 * the last; every chunk counts its own updates for the bias correction.
 * ---------------------------------------------------------------------- */
typedef struct {
  int32_t active;         /* chunk that is optimised at this training step */
  int32_t load_before;    /* 1: the chunk becomes active at this step */
  int32_t offload_after;  /* 1: the chunk is switched out after this step */
  int32_t reserved;       /* written as 0 */
  int64_t local_step;     /* the chunk's own update count n after this step's
                             increment: pass it as chunkft_adamw_hparams.step */
} chunkft_schedule_entry;

/* step >= 0 (training steps count from 0), n_chunks >= 1, interval >= 1.
 * A pure function of its arguments; writes *out.
 * Errors: INVALID_ARG, OVERFLOW. */
int chunkft_schedule_at(int64_t step, int32_t n_chunks, int64_t interval, chunkft_schedule_entry* out);

/* ------------------------------------------------------------------------
 * Layer operands of one backward step
 * ---------------------------------------------------------------------- */
typedef struct {
  int32_t kind;      /* chunkft_kind */
  int32_t dtype;     /* chunkft_dtype of X, dY (and of W in the fused call) */
  int64_t out, in;   /* W shape; the 1-D kinds: out = 1, in = vector length;
                        EMBEDDING: out = table rows, in = embedding width */
  int64_t T;         /* tokens, 1 .. 2^30 */
  const void* X;     /* (device) LINEAR: [T, in] layer input.  VECTOR: [T, in] the
                        normalised activations that the scale multiplies.
                        RMSNORM / LAYERNORM: [T, in] the operator's raw input.
                        EMBEDDING: T <= 8192 token ids as int64 (ids outside the
                        table rows of the range are ignored; a longer batch is
                        passed in pieces with accumulate = 1) */
  int64_t ldx;       /* row stride of X in elements, >= in (EMBEDDING: ignored) */
  const void* dY;    /* (device) LINEAR: [T, out] output gradient.  Others: [T, in] */
  int64_t lddy;      /* row stride of dY in elements */
  int32_t split_k;   /* 0: the library picks the number of token slabs S from the
                        shape alone; 1..64: use exactly this S (LINEAR only;
                        the other kinds always use one slab) */
  int32_t reserved;  /* must be 0 */
  double norm_eps;   /* RMSNORM / LAYERNORM: the eps under the square root, >= 0;
                        other kinds: ignored */
} chunkft_layer;

/* Number of token slabs S the two wgrad entry points will use for this call
 * (pure function of the layer shape, the range and split_k), or a negative
 * status.  Host only. */
int chunkft_split_k(const chunkft_layer* L, int64_t begin, int64_t end);

/* Bytes of device workspace the two wgrad entry points need for this call:
 * LINEAR: 0 when S = 1, else 4 * (S * P + 32) for the per-slab partial sums,
 * P = end - begin rounded up to a multiple of 32 (the library places them at the
 * 128-byte phase of the array their sum goes to);
 * RMSNORM / LAYERNORM: 8 * T for the per-token statistics; other kinds 0.
 * Returns 0 also for invalid arguments (the call itself reports those). */
size_t chunkft_workspace_bytes(const chunkft_layer* L, int64_t begin, int64_t end);

/* ------------------------------------------------------------------------
 * Chunk-restricted weight gradient
 *
 * Paper: Section 3.1, equation g^(k) = grad_{theta^(k)} L -- the backward pass
 * produces the gradient of the active slices only, into an auxiliary fp32
 * buffer, never a dense gradient (also Algorithm 1 line 18).  For y = x W^T:
 *   LINEAR     g[i] = sum_t dY[t, r] * X[t, c],  begin + i = r * in + c
 *   VECTOR     g[i] = sum_t dY[t, j] * X[t, j],  j = begin + i
 *   EMBEDDING  g[i] = sum over the tokens t with ids[t] = r of dY[t, c], in
 *              ascending token order (no atomics: the result is reproducible)
 *   RMSNORM    g[i] = sum_t dY[t, j] * X[t, j] * rstd[t],
 *              rstd[t] = 1 / sqrt(mean_j X[t, j]^2 + eps)
 *   LAYERNORM  g[i] = sum_t dY[t, j] * (X[t, j] - mean[t]) * rstd[t],
 *              rstd[t] = 1 / sqrt(var[t] + eps), biased variance
 * (the paper names the last three operators without formulas; these are the
 * textbook gradients of the forms given with chunkft_kind).
 * Products and sums are fp32 (bf16 inputs are multiplied exactly); the sum
 * over tokens is taken slab by slab in a fixed order.
 *
 * g (device, out)   end - begin floats.  accumulate = 0: overwritten;
 *                   accumulate = 1: g += result (gradient accumulation over
 *                   micro-batches, Algorithm 1 line 14).
 * ws (device)       workspace of at least chunkft_workspace_bytes(), 16-byte
 *                   aligned; may be NULL when that is 0.  Contents on entry
 *                   are ignored; on return they are unspecified.
 * Only elements [0, end - begin) of g are written; nothing else is touched.
 * Layout: any 4-byte aligned g is accepted.  The LINEAR kernels run fastest when
 * g (and master, m, v in the fused call) has the 128-byte phase of the tensor,
 * ((uintptr_t)g / 4 - begin) % 32 == 0 for a row length that is a multiple of
 * 32: the 16-byte groups and the memory lines of a row of the chunk are then
 * those of the same row of W (measured on the fused call: 7 % faster).
 * master, m and v are walked together: when they lie a whole number of MiB apart
 * (129 MiB for 128 MiB arrays was the worst case measured: the fused call 203 -
 * 229 us instead of 188 us) their streams can meet on the same memory channels;
 * a whole number of MiB plus 256 KiB apart was never slower than the best.
 * Errors: INVALID_ARG, RANGE, DTYPE, WORKSPACE, HIP.
 * ---------------------------------------------------------------------- */
int chunkft_chunk_wgrad(const chunkft_layer* L, int64_t begin, int64_t end,
                        float* g, int accumulate,
                        void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * AdamW on a chunk
 *
 * Paper: Algorithm 1 lines 19-21, element by element, in fp32:
 *   m <- b1 m + (1 - b1) g          v <- b2 v + (1 - b2) g^2
 *   mhat = m / (1 - b1^n)           vhat = v / (1 - b2^n)
 *   theta <- theta - lr * ( mhat / (sqrt(vhat) + eps) + wd * theta )
 * with theta on the right the value before the update and n the chunk's own
 * update counter after its increment (Section 3.1: each chunk keeps a local
 * counter for bias correction).  The library never counts: pass n as `step`.
 * ---------------------------------------------------------------------- */
typedef struct {
  double lr, beta1, beta2, eps, weight_decay;
  int64_t step;   /* n >= 1 */
} chunkft_adamw_hparams;

/*
 * g (device, in)            n floats.
 * master, m, v (device)     n floats each, updated in place.
 * W_at_begin (device, out)  NULL, or the low-precision parameter copy ALREADY
 *                           offset to the chunk's first element; receives
 *                           round-to-nearest-even(master) as w_dtype (only
 *                           CHUNKFT_BF16 makes sense; CHUNKFT_F32 copies).
 * n                         elements, > 0.  No alignment is required of any
 *                           pointer beyond that of its element type.
 * Errors: INVALID_ARG (null pointer, n <= 0, step < 1, betas outside [0,1),
 * negative lr/eps), DTYPE, HIP.
 */
int chunkft_adamw_chunk(const float* g, float* master, float* m, float* v,
                        void* W_at_begin, int32_t w_dtype, int64_t n,
                        const chunkft_adamw_hparams* hp, void* stream);

/* ------------------------------------------------------------------------
 * Fused: chunk gradient straight into the AdamW update
 *
 * Same arithmetic as chunkft_chunk_wgrad (accumulate = 0) followed by
 * chunkft_adamw_chunk on its result, bit for bit, but g is consumed from the
 * accumulators (S = 1) or from the slab partials (S > 1) and never stored
 * (the "temporary chunk gradients" of Algorithm 1 line 22 do not exist).
 *
 * W (device, out)   BASE of the low-precision tensor [out, in] (NOT offset);
 *                   elements [begin, end) receive the rounded master.  May be
 *                   NULL (fp32 training: the master is the parameter).  With
 *                   dtype F32 a non-NULL W receives an fp32 copy.
 * master, m, v      (device) chunk-local, end - begin floats each, in place.
 * Elements of W outside [begin, end) are never written.
 * Errors: as the two calls above.
 * ---------------------------------------------------------------------- */
int chunkft_wgrad_adamw_fused(const chunkft_layer* L, int64_t begin, int64_t end,
                              void* W, float* master, float* m, float* v,
                              const chunkft_adamw_hparams* hp,
                              void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Fused call for all segments of a chunk at once
 *
 * Paper: Algorithm 1 line 18 runs ONE chunk-aware backward over all slices of the
 * active chunk C_k, and lines 19-21 one update of the chunk; a chunk that crosses
 * tensors has one segment per tensor (chunkft_plan_cycle).  This call takes them
 * together: the tiles of all bf16 matrix segments and the blocks of all bf16 VECTOR
 * segments become the work items of a single kernel launch (12 segments per launch),
 * so that a small segment (a k or v projection, a norm vector) shares the device
 * with the large ones instead of running alone on a fraction of it.
 * Each segment's result is, bit for bit, that of chunkft_wgrad_adamw_fused on it
 * with the same token split.  The split: a matrix segment with split_k = 0 takes one
 * slab when the group's matrix segments together have more 256 x 256 tiles than a
 * quarter of the compute units (the single call's rule applied to the sum), else
 * what the single call would choose; split_k >= 1 is obeyed.  Segments the one-launch
 * kernel cannot take (fp32, more than one token slab, shapes off the MFMA path, bodies
 * of a few rows, EMBEDDING / RMSNORM / LAYERNORM) are run by themselves inside this
 * call, one after the other on `stream`, sharing `ws`.
 *
 * segs (host, in)   n_segs >= 1 (at most 4096) segments; ranges on the same tensor
 *                   must not overlap, and no two segments may share state elements.
 *   layer           operands of the tensor's backward step (as for the single call)
 *   begin, end      flat range on that tensor
 *   W               (device) tensor base or NULL
 *   master, m, v    (device) chunk-local arrays ALREADY offset to the segment
 *                   (state + chunk_off), end - begin floats each
 * hp                one set of hyper-parameters and one step count for the chunk
 * ws (device)       at least chunkft_group_workspace_bytes(), 16-byte aligned; may be
 *                   NULL when that is 0 (always, when the kernel takes every segment)
 * Errors: those of chunkft_wgrad_adamw_fused, for the first segment that has one.
 * ---------------------------------------------------------------------- */
typedef struct {
  chunkft_layer layer;
  int64_t begin, end;
  void* W;
  float* master;
  float* m;
  float* v;
} chunkft_group_segment;

size_t chunkft_group_workspace_bytes(const chunkft_group_segment* segs, int32_t n_segs);   /* host only */

int chunkft_wgrad_adamw_fused_group(const chunkft_group_segment* segs, int32_t n_segs,
                                    const chunkft_adamw_hparams* hp,
                                    void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The fused call without a workspace argument
 *
 * For callers that cannot allocate device memory or have none to hand over: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid
 * allocation.  The same call as chunkft_wgrad_adamw_fused, bit for bit and with the
 * same argument rules, but whatever workspace it needs (token-slab partial sums,
 * per-token statistics of the normalising kinds) lies in a device array of
 * CHUNKFT_STATIC_WORKSPACE_BYTES that is part of the library: every GPU the library
 * runs on holds one copy from the first such call on it until the process ends.
 * A call that would need more returns CHUNKFT_ERR_STATIC_WORKSPACE, nothing enqueued
 * (chunkft_workspace_bytes tells beforehand).  Neither this call nor anything under
 * it allocates or frees memory.  The first call on a device asks the runtime for the
 * array's address (make it outside a graph capture).  All calls on one GPU share the
 * one array: two that overlap in time (different streams, or graphs replayed side by
 * side) race on it; calls on one stream are ordered and safe.  Nothing in the array
 * is read before the same call has written it, so no clearing is needed between calls.
 * ---------------------------------------------------------------------- */
#define CHUNKFT_STATIC_WORKSPACE_BYTES (64u << 20)

int chunkft_wgrad_adamw_fused_static(const chunkft_layer* L, int64_t begin, int64_t end,
                                     void* W, float* master, float* m, float* v,
                                     const chunkft_adamw_hparams* hp, void* stream);

const char* chunkft_status_string(int status);
int chunkft_version(void);   /* major * 10000 + minor * 100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* CHUNKFT_H */
