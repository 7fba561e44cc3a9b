/*
 * moe.h - C ABI of the MI355X (gfx950) MoE expert-layer library.
 *
 * One top-k Mixture-of-Experts block, forward and backward, as the paper describes it
 * (arxiv 2504.03871, Section 2.1): a gate scores every expert for each token, the token goes to its
 * top-k experts, the expert outputs are weighted by the scores and summed.  "Dispatch" groups token
 * rows by expert, "combine" brings the expert outputs back (Section 2.1, expert parallelism).  Every
 * call can be restricted to one GPU's share of each expert's tokens, which is how the asymmetric
 * expert assignment of Section 4.2 appears at this level: a half-open range [lo_e, hi_e) over the
 * kept-token list of expert e.
 *
 * Conventions for every entry point (the two host-only planner calls moe_asymea_* state their own)
 *   - Returns MOE_OK (0) or a negative MOE_ERR_* code.  Arguments are validated before anything is
 *     launched; on an argument error nothing has been enqueued and no output is touched.
 *   - `cfg` is a host pointer.  Every other pointer is a DEVICE pointer owned by the caller and must
 *     be 16-byte aligned; the library allocates nothing, frees nothing and keeps no state between
 *     calls (except the last HIP error code, per host thread).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work is enqueued on
 *     it; no call synchronises with the host and none reads device memory from the host.
 *   - Activations (x, x_perm, y_perm, saved, d_out, dy_perm, dx_perm, out, dx) and expert weights
 *     (W1, W1b, W2) have the storage type cfg->dtype: fp32, or bf16 or fp16 (round-to-nearest-even; the
 *     paper trains in FP16 mixed precision, Section 6.1) with fp32 accumulation on the matrix cores.  Router tensors (Wr, bias, logits, topk_w, d_topk_w, d_logits, dWr) and
 *     expert weight gradients (dW1, dW1b, dW2) are always fp32.  Index tensors are int32.
 *   - All matrices are dense row-major: x[T][d_model], W1[E][d_model][d_ff], W2[E][d_ff][d_model],
 *     Wr[d_model][E], topk_*[T][k], permuted buffers [T*k][...].
 *   - Assignment a = t*k + j is slot j of token t.  Expert e's list holds its assignments in ascending
 *     token order; the first kept[e] = min(counts[e], capacity) of them own rows
 *     offsets[e] .. offsets[e]+kept[e]-1 of the permuted buffers; later ones are dropped
 *     (row_of = -1) and contribute nothing.
 *   - slice_lo / slice_hi: device int32[E], positions in expert e's kept list that THIS GPU
 *     computes.  Both NULL = everything.  On the device they are clamped to [0, kept[e]] and an
 *     inverted range is empty.  Rows of permuted buffers outside the shares are never read for a
 *     result and never written.
 *   - Shapes: 1 <= k <= min(E, MOE_MAX_K), E <= MOE_MAX_E, T >= 0 (T = 0 is a no-op),
 *     T*k <= 2^30.  bf16 / fp16: d_model and d_ff multiples of 64; fp32: multiples of 4.  The kernels address
 *     one operand through 32-bit byte offsets, so T*k * max(d_model, d_ff) * (bytes per element) and
 *     d_model * d_ff * 4 must both stay below 2^32 (MOE_ERR_BAD_SHAPE otherwise).
 *   - `ws` is the caller's device workspace and `ws_bytes` its size; a call that uses it returns
 *     MOE_ERR_WORKSPACE, before launching anything, when ws_bytes < moe_workspace_bytes(cfg).
 *   - An expert id in topk_idx outside [0, E) is treated as a dropped assignment (row_of = -1, not
 *     counted, contributes nothing); it never indexes memory.
 *   - Calls that use the same workspace or output buffers must not overlap in time.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_API __attribute__((visibility("default")))

#define MOE_MAX_E 256
#define MOE_MAX_K 8

enum { MOE_DTYPE_F32 = 0, MOE_DTYPE_BF16 = 1, MOE_DTYPE_F16 = 2 };
enum { MOE_ACT_GELU = 0, MOE_ACT_SWIGLU = 1 };

enum {
  MOE_OK = 0,
  MOE_ERR_NULL = -1,      /* a required pointer is NULL */
  MOE_ERR_BAD_SHAPE = -2, /* T, d_model, d_ff, E, k out of the supported range or misaligned sizes */
  MOE_ERR_BAD_DTYPE = -3, /* dtype or act not one of the enumerators */
  MOE_ERR_BAD_SLICE = -4, /* exactly one of slice_lo / slice_hi is NULL */
  MOE_ERR_ALIGN = -5,     /* a device pointer is not 16-byte aligned */
  MOE_ERR_HIP = -6,       /* a launch failed; see moe_last_hip_error() */
  MOE_ERR_WORKSPACE = -7  /* ws_bytes is smaller than moe_workspace_bytes(cfg) */
};

/*
 * Benchmark aid, not a step of the layer: timing brackets owned by the CALLER.  A moe_cfg whose `prof`
 * points at one of these makes every launch of kernel `which` with n[which] > 0 record
 * hipEventRecord(start[which][i]) / hipEventRecord(stop[which][i]) on the launch's stream around it,
 * i = count[which]++ modulo n[which].  start/stop hold hipEvent_t handles created by the caller; the
 * struct and the arrays are HOST memory that must stay valid during the call.  The library keeps no
 * pointer to it after the call returns.  Do not use under graph capture.
 */
enum {
  MOE_PROF_GEMM1_FWD = 0,   /* x_perm W1 (+ activation) */
  MOE_PROF_GEMM2_FWD = 1,   /* H W2 */
  MOE_PROF_DH_BWD = 2,      /* dy W2^T (+ activation derivative); bf16 with few tiles: the same launch also does H^T dy */
  MOE_PROF_DW2_BWD = 3,     /* H^T dy, when it has a launch of its own */
  MOE_PROF_DW1_BWD = 4,     /* x_perm^T dA (SwiGLU: both weight gradients), those with a launch of their own */
  MOE_PROF_DX_BWD = 5,      /* dA W1^T; bf16 with few tiles: the same launch also does x_perm^T dA */
  MOE_PROF_GATHER = 6,      /* row gather of moe_dispatch */
  MOE_PROF_COMBINE = 7,     /* moe_combine kernel */
  MOE_PROF_COMBINE_BWD = 8, /* moe_combine_bwd kernel */
  MOE_PROF_ROUTE = 9,       /* moe_route kernel */
  MOE_PROF_COUNT = 10
};
typedef struct moe_prof {
  void** start[MOE_PROF_COUNT];
  void** stop[MOE_PROF_COUNT];
  int32_t n[MOE_PROF_COUNT];
  int64_t count[MOE_PROF_COUNT];
} moe_prof;

typedef struct moe_cfg {
  int32_t T;        /* tokens */
  int32_t d_model;  /* embedding width d */
  int32_t d_ff;     /* expert hidden width f */
  int32_t E;        /* experts */
  int32_t k;        /* experts per token */
  int32_t dtype;    /* MOE_DTYPE_* : storage type of activations and expert weights */
  int32_t act;      /* MOE_ACT_GELU: gelu_erf(x W1) W2 ; MOE_ACT_SWIGLU: (silu(x W1) * (x W1b)) W2 */
  int32_t capacity; /* rows kept per expert; <= 0 = unlimited */
  moe_prof* prof;   /* HOST pointer to caller-owned timing brackets, or NULL (the normal case) */
} moe_cfg;

/* Static text for a return code (never NULL). */
MOE_API const char* moe_error_string(int code);
/* hipError_t value of the last failed HIP call made by this host thread (0 if none). */
MOE_API int moe_last_hip_error(void);

/* Bytes of device workspace `ws` sufficient for every call below with this cfg. */
MOE_API int moe_workspace_bytes(const moe_cfg* cfg, size_t* bytes);
/* Bytes of the `saved` buffer of moe_expert_ffn_fwd: (2 for GELU, 3 for SwiGLU) * T*k * d_ff elements. */
MOE_API int moe_saved_bytes(const moe_cfg* cfg, size_t* bytes);

/*
 * Gate (Section 2.1: confidence score per expert, top-k).  logits = x Wr (+ bias), fp32 accumulate,
 * written to logits_out[T][E].  If logits_in is non-NULL the matrix product is skipped and those
 * logits are used instead (x, Wr may then be NULL).  Selection is made on the fp32 logits as stored:
 * descending value, equal values by ascending expert id; slot 0 is the best.
 * topk_w[t][j] = exp(l_j - l_0) / sum_i exp(l_i - l_0) over the k selected logits.
 * bias[E] may be NULL.  logits_out may be NULL only when logits_in is given.
 * bf16 and fp16: the product runs on the matrix cores with the fp32 gate weight split into two bf16 terms
 * (about 16 mantissa bits; fp16 activations enter exactly, as two bf16 terms each); ws (moe_workspace_bytes,
 * device) holds the re-laid-out weight and is required unless logits_in is given.  fp32: plain fp32 FMAs on
 * the stored values, ws may be NULL.
 */
MOE_API int moe_route(const moe_cfg* cfg, const void* x, const float* Wr, const float* bias,
              const float* logits_in, float* logits_out, int32_t* topk_idx, float* topk_w,
              void* ws, size_t ws_bytes, void* stream);

/*
 * Dispatch (Section 2.1: token embeddings go to their experts; locally a stable group-by-expert).
 * Writes counts[E] (routed), kept[E], offsets[E+1] (exclusive scan of kept), row_of[T*k]
 * (row of each assignment or -1), src_of[T*k] (assignment of each row, -1 from offsets[E] on) and
 * gathers x_perm[row] = x[src_of[row] / k] for the rows inside this GPU's shares.
 * x_perm may be NULL: only the index arrays are produced.
 */
MOE_API int moe_dispatch(const moe_cfg* cfg, const void* x, const int32_t* topk_idx,
                 const int32_t* slice_lo, const int32_t* slice_hi,
                 int32_t* counts, int32_t* kept, int32_t* offsets, int32_t* row_of, int32_t* src_of,
                 void* x_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_dispatch for callers that cannot allocate or carry a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as moe_dispatch
 * minus `ws`: the per-block histograms live in a device array that is part of the library's code object
 * (MOE_DISPATCH_STATIC_BYTES per GPU, held until the process ends; its address is looked up once per
 * device on the first call there).  Allocates nothing.  Limit: (ceil(T*k / 1024) + 1) * E * 4 bytes must fit
 * the array, else MOE_ERR_WORKSPACE before anything is launched.  All calls on one GPU share the array, so
 * two calls that overlap in time on one GPU (different streams or host threads) race; calls in stream order
 * are fine, and nothing in the array has to be cleared between calls (every entry a call reads, it has
 * written first).
 */
#define MOE_DISPATCH_STATIC_BYTES (1 << 20)
MOE_API int moe_dispatch_static(const moe_cfg* cfg, const void* x, const int32_t* topk_idx,
                        const int32_t* slice_lo, const int32_t* slice_hi,
                        int32_t* counts, int32_t* kept, int32_t* offsets, int32_t* row_of, int32_t* src_of,
                        void* x_perm, void* stream);

/*
 * Expert FFN forward on the in-share rows (Section 2.1: experts are FFNs made of GEMMs).
 * GELU:   A = x_perm W1[e], H = gelu_erf(A), y_perm = H W2[e];          saved = [A | H]
 * SwiGLU: G = x_perm W1[e], U = x_perm W1b[e], H = silu(G) * U, y_perm = H W2[e];  saved = [G | U | H]
 * Each saved plane is [T*k][d_ff] in the storage type.  W1b must be NULL for GELU.
 */
MOE_API int moe_expert_ffn_fwd(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b,
                       const void* W2, const int32_t* offsets, const int32_t* kept,
                       const int32_t* slice_lo, const int32_t* slice_hi,
                       void* saved, void* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_expert_ffn_fwd for a layer whose activations are checkpointed (Section 6.1): the same two GEMMs, but of
 * the saved planes only the hidden activation H is written, to `hidden` ([T*k][d_ff] in the storage type), because
 * the second GEMM reads it; the pre-activations (A, or G and U) are not stored, which removes one (GELU) or two
 * (SwiGLU) of the first GEMM's output planes from its HBM writes.  H and y_perm are bit-identical to
 * moe_expert_ffn_fwd's.  Before the backward the caller refills a full `saved` buffer with
 * moe_expert_ffn_recompute.  Other arguments as in moe_expert_ffn_fwd.
 */
MOE_API int moe_expert_ffn_fwd_light(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b,
                             const void* W2, const int32_t* offsets, const int32_t* kept,
                             const int32_t* slice_lo, const int32_t* slice_hi,
                             void* hidden, void* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * Activation checkpointing (the paper trains with it, Section 6.1): the first half of
 * moe_expert_ffn_fwd again.  Fills every plane of `saved` from x_perm and the first-layer weights with
 * the same kernel the forward call uses, so the planes are bit-identical to the forward's, and does
 * nothing else (no W2, no y_perm).  A caller that checkpoints keeps ONE `saved` buffer for all layers:
 * before a layer's backward it repeats moe_route and moe_dispatch for that layer's input, calls this,
 * then moe_expert_ffn_bwd as usual.  Costs the FLOPs of GEMM1 (2 T k d_model d_ff, SwiGLU twice that)
 * and saves (planes - 1) x T k d_ff elements per layer of resident activations.
 * Arguments as in moe_expert_ffn_fwd.
 */
MOE_API int moe_expert_ffn_recompute(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b,
                             const int32_t* offsets, const int32_t* kept, const int32_t* slice_lo,
                             const int32_t* slice_hi, void* saved, void* ws, size_t ws_bytes, void* stream);

/*
 * Combine (Section 2.1: outputs weighted by the scores and summed).
 * out[t] = sum over slots j = 0..k-1, in that order, of topk_w[t][j] * y_perm[row_of[t*k+j]],
 * taking only slots that are kept and inside this GPU's shares; fp32 accumulation.
 * topk_w == NULL means unit weights (the un-permute of the input gradient).  accumulate != 0 adds
 * to `out` instead of overwriting it.
 */
MOE_API int moe_combine(const moe_cfg* cfg, const void* y_perm, const float* topk_w, const int32_t* topk_idx,
                const int32_t* row_of, const int32_t* offsets, const int32_t* kept,
                const int32_t* slice_lo, const int32_t* slice_hi,
                void* out, int32_t accumulate, void* stream);

/*
 * Combine backward (Section 5: the gradient of the block output feeds two branches).
 * For every in-share slot: dy_perm[row] = topk_w[a] * d_out[t] and d_topk_w[a] = <d_out[t], y_perm[row]>;
 * every other slot gets d_topk_w[a] = 0.
 */
MOE_API int moe_combine_bwd(const moe_cfg* cfg, const void* d_out, const void* y_perm, const float* topk_w,
                    const int32_t* topk_idx, const int32_t* row_of, const int32_t* offsets,
                    const int32_t* kept, const int32_t* slice_lo, const int32_t* slice_hi,
                    void* dy_perm, float* d_topk_w, void* stream);

/*
 * Expert FFN backward on the in-share rows.
 * dH = dy_perm W2[e]^T;  dW2[e] = H^T dy_perm;
 * GELU:   dA = dH * gelu'(A);  dW1[e] = x_perm^T dA;  dx_perm = dA W1[e]^T
 * SwiGLU: dU = dH * silu(G), dG = dH * U * silu'(G);  dW1[e] = x_perm^T dG, dW1b[e] = x_perm^T dU;
 *         dx_perm = dG W1[e]^T + dU W1b[e]^T
 * Weight gradients sum over the in-share rows of the expert only; accumulate != 0 adds them to
 * dW1/dW1b/dW2 instead of overwriting (an expert with an empty share then leaves its gradient as is,
 * otherwise it is zero-filled).
 */
MOE_API int moe_expert_ffn_bwd(const moe_cfg* cfg, const void* dy_perm, const void* x_perm, const void* saved,
                       const void* W1, const void* W1b, const void* W2,
                       const int32_t* offsets, const int32_t* kept,
                       const int32_t* slice_lo, const int32_t* slice_hi,
                       void* dx_perm, float* dW1, float* dW1b, float* dW2, int32_t accumulate,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * Gate backward (Section 5: the branch through the confidence scores to the gate weights and to
 * the block input, accumulated with the gradient that comes back through the experts).
 * g = sum_j w_j dw_j;  d_logits[t][e_j] = w_j (dw_j - g), 0 for unselected experts;
 * dWr = x^T d_logits (accumulate = 0: overwritten; 1: added to, for gradient accumulation over
 * micro-batches);  dx += d_logits Wr^T.  dx may be NULL to skip that part, dWr may be NULL to skip the
 * weight gradient (d_logits is always written): the two parts are independent, so a caller can run the
 * weight-gradient part on a second stream next to the expert backward, with a workspace and a d_logits
 * buffer of its own, and add to dx once the gradient through the experts has been written.
 * Sums are fp32 in a fixed order.  bf16 / fp16 storage with more than 16 experts: dWr runs on the matrix cores
 * with d_logits entering as two bf16 terms (about 16 mantissa bits) and x exactly; otherwise plain fp32 FMAs.
 */
MOE_API int moe_route_bwd(const moe_cfg* cfg, const void* x, const float* Wr, const int32_t* topk_idx,
                  const float* topk_w, const float* d_topk_w,
                  float* d_logits, float* dWr, void* dx, int32_t accumulate, void* ws, size_t ws_bytes, void* stream);

/*
 * Planner of the asymmetric expert assignment (Section 4.2 of the paper, Algorithm 1 and the paragraph
 * on memory limits).  HOST-ONLY: runs on the CPU, enqueues nothing, and `o` is a HOST pointer.
 *
 * In the paper's notation: n experts per layer, L layers, M attention GPUs and N expert GPUs in a
 * group (one must divide the other, else MOE_ERR_BAD_SHAPE), T_A_attn = time of one layer's attention
 * module on an attention GPU, T_E_attn = time of one expert module on an attention GPU, T_E_exp = time of
 * one layer's expert module on an expert GPU (any common unit; profile them with the expert batch a GPU
 * sees per micro-batch, Section 5).  A chunk is n_1 = max(1, N/M) experts acquired by each attention GPU
 * = n_2 = n_1 M / N experts offloaded by each expert GPU.  Per layer the bubble T_gather = T_E_exp -
 * T_A_attn is accumulated; whenever it reaches T_squeeze = (T_E_exp N / n) n_1 + (T_E_attn N / n) n_2,
 * floor(bubble / T_squeeze) chunks are offloaded at that layer and their time is taken off the bubble.
 * o[l] (l = 0 .. L-1) receives the number of experts EACH expert GPU offloads at layer l, a multiple
 * of n_2.
 * Memory bounds: n_max >= 0 caps the sum of o at floor(n_max / n_2) chunks (what the attention GPUs can
 * hold), n_min > 0 raises it to ceil(n_min / n_2) chunks (what the expert GPUs cannot hold), through the
 * paper's coefficients alpha and beta on T_gather; n_min <= 0 and n_max < 0: the unmodified algorithm.
 * All arithmetic is IEEE double in the paper's order; since the per-layer step is a rounded quotient, the
 * total can fall one chunk short of a bound it aims at, never beyond n_max.
 * T_gather <= 0 gives all zeros (MOE_ERR_BAD_SHAPE if a positive n_min was asked for).  MOE_ERR_BAD_SHAPE
 * also for n, L < 1, non-finite times, T_squeeze <= 0, n_max < n_min.
 */
MOE_API int moe_asymea_plan(int32_t n, int32_t L, int32_t M, int32_t N, double T_A_attn, double T_E_attn,
                    double T_E_exp, int32_t n_min, int32_t n_max, int32_t* o);

/*
 * From one layer's offload count to the slice arguments of the device entry points.  HOST-ONLY;
 * slice_lo / slice_hi are HOST int32[n] arrays, to be copied to the device by the caller.
 *
 * The paper moves whole experts and leaves open which; here expert e lives on expert GPU e / (n/N)
 * (N must divide n), each expert GPU gives up the LAST o_l of its n/N experts, and the offloaded experts,
 * by ascending id, go to the attention GPUs in equal contiguous runs of o_l N / M.  role 0 = expert GPU
 * `rank` (0 .. N-1), role 1 = attention GPU `rank` (0 .. M-1).  An expert this GPU computes gets
 * [0, INT32_MAX) (the device clamps it to the kept count), every other expert [0, 0).  Over all M + N
 * GPUs the ranges cover every expert exactly once.  o_l must be a multiple of n_2 in [0, n/N].
 */
MOE_API int moe_asymea_shares(int32_t n, int32_t M, int32_t N, int32_t o_l, int32_t role, int32_t rank,
                      int32_t* slice_lo, int32_t* slice_hi);

/*
 * Benchmark aid, not a step of the layer: a one-wave kernel that writes n pairs (shader-clock counter, 100 MHz
 * real-time counter) to `samples` (device uint64[2 n]), pausing `sleeps` (0..1000) sleep instructions of about
 * 8000 shader cycles between pairs.  Launched on a second stream next to other work it shows the clock the chip
 * sustains under that work: (difference of the first) / (difference of the second) x 100 MHz per interval.
 * The loop is bounded (n <= 2^20), so the kernel always ends.
 */
MOE_API int moe_bench_clock_probe(uint64_t* samples, int32_t n, int32_t sleeps, void* stream);

/*
 * Benchmark aid, not a step of the layer: a kernel of nothing but bf16 MFMA instructions on register operands
 * (1024 blocks of eight waves, `iters` (1..10^6) rounds of 32 independent accumulations per wave), to show the
 * rate the chip sustains for an instruction shape under its own power management.  kind 0: 16 x 16 x 32, the
 * instruction the grouped GEMM uses; kind 1: 32 x 32 x 16.  `operand` is device memory of at least 64 KiB that the
 * register operands are read from (random bf16 values give realistic switching activity), `sink` device float[1024 * 512]
 * that receives one sum per lane.  FLOP of one launch: 1024 * 8 * iters * 32 * 16384.
 */
MOE_API int moe_bench_mfma_loop(int32_t kind, int32_t iters, const void* operand, float* sink, void* stream);

/*
 * Introspection for tests, HOST-ONLY (nothing is enqueued, `out` is a HOST int32[6]): which tile block number
 * `block` of a grouped-GEMM launch of the 16-bit path computes, by the same code the kernels run.
 * kind 0, row-tile GEMMs (x W, dy W^T) over n_rt row tiles of which the first n_full_rt are full and the last
 * n_split are split along K into 8 parts, ntn column tiles: out = {1, row tile, -1, column tile, index among the
 * split tiles or -1, K part}.  kind 1, weight-gradient GEMM with ntm x ntn tiles per expert: out = {1, expert slot
 * (position in descending-size order), m tile, n tile, -1, -1}.  out[0] = 0: a surplus block that exits at once.
 */
MOE_API int moe_gemm_block_tile(int32_t kind, int64_t block, int32_t n_rt, int32_t n_full_rt, int32_t n_split,
                        int32_t ntm, int32_t ntn, int32_t* out);

/*
 * Benchmark aid, not a step of the layer: a plain streaming kernel of this library over `bytes` bytes
 * (a multiple of 16; dst and src are device pointers, 16-byte aligned).  mode 0: dst = src (the copy
 * rate is the practical ceiling of the HBM-bound kernels on a given box); mode 1: dst is filled with
 * zeros and src is ignored (used between timed iterations to push earlier data out of the caches).
 */
MOE_API int moe_bench_stream(void* dst, const void* src, size_t bytes, int32_t mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
