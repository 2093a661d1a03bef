/*
 * rf.h - C ABI of the cascaded-reduction library for AMD MI355X (gfx950).
 *
 * A cascaded reduction (paper Section 3.1, Eq. (1)) is a chain of I reductions
 * over one shared axis of length L0, d_i = R_i_{l=1..L0} F_i(X[l], d_1..d_{i-1}),
 * each with an associative, commutative reduce operator (+)_i and a combine
 * operator (x)_i taken from Table 1 (max/min pair with +, sum pairs with *).
 * Every entry point below evaluates one such chain in its single-loop,
 * incremental form (Section 3.3, Eq. (15)-(16)): one pass over the input
 * carries a running state that is rescaled as each tile arrives; partial
 * states of disjoint segments are merged with the level-k fused expression
 * (Section 3.2, Eq. (11)).
 *
 * Conventions shared by all entry points
 *   - Every `data` pointer is a DEVICE pointer into memory owned by the caller
 *     (inputs, outputs and partial-state workspaces alike).  The library never
 *     allocates or frees device memory, and retains none of the caller's.  Its only state
 *     is the fixed scratch array of rf_moe_routing_noalloc.
 *   - rf_tensor describes a dense tensor: shape[] and stride[] in ELEMENTS for
 *     dims 0..ndim-1.  The last dimension must have stride 1; outer dimensions
 *     may be strided.  Base pointers and every outer stride must keep rows
 *     16-byte aligned where a kernel uses 128-bit accesses (checked; a
 *     violation returns RF_ERR_ALIGNMENT).
 *   - Calls only enqueue work on `stream` (a hipStream_t; NULL = the default
 *     stream) and return; nothing synchronises the device.
 *   - Errors are reported by return code only.  All argument checks run on the
 *     host before any launch.  An unsupported dtype or shape is
 *     RF_ERR_UNSUPPORTED, never a silent slow path.  Zero-sized problems are
 *     RF_OK and launch nothing.
 *   - All internal state (m, l, acc, sum of squares) is fp32.
 */
#ifndef RF_H_
#define RF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define RF_API __attribute__((visibility("default")))
#else
#define RF_API
#endif

typedef enum {
  RF_OK = 0,
  RF_ERR_INVALID_ARG = 1, /* null pointer, bad ndim, shapes that do not agree   */
  RF_ERR_UNSUPPORTED = 2, /* dtype / head dim / axis the kernels do not cover   */
  RF_ERR_ALIGNMENT = 3,   /* pointer or stride not aligned for 128-bit access   */
  RF_ERR_WORKSPACE = 4,   /* partial-state tensors have the wrong shape         */
  RF_ERR_LAUNCH = 5       /* the HIP runtime rejected a launch                  */
} rf_status;

typedef enum { RF_F32 = 0, RF_BF16 = 1, RF_I32 = 2, RF_FP8_E4M3 = 3 /* OCP E4M3, 1 byte */ } rf_dtype;

/* (+)_i and (x)_i of Table 1. */
typedef enum { RF_RED_MAX = 0, RF_RED_MIN = 1, RF_RED_SUM = 2 } rf_reduce_op;
typedef enum { RF_COMB_ADD = 0, RF_COMB_MUL = 1 } rf_combine_op;
typedef struct {
  rf_reduce_op reduce;
  rf_combine_op combine;
} rf_stage;

#define RF_MAX_DIMS 5
typedef struct {
  void* data;                  /* device pointer, caller-owned */
  rf_dtype dtype;
  int32_t ndim;                /* 1..RF_MAX_DIMS */
  int64_t shape[RF_MAX_DIMS];
  int64_t stride[RF_MAX_DIMS]; /* in elements */
} rf_tensor;

typedef void* rf_stream; /* hipStream_t */

/* Human-readable name of a status code (static storage, never NULL). */
RF_API const char* rf_status_string(rf_status s);

/*
 * The chain of (reduce, combine) stages an entry point implements, in
 * dependency order (Section 3.1; operators from Table 1).  `entry` is the
 * entry-point name, e.g. "rf_cascade_attention" -> {MAX,ADD},{SUM,MUL},{SUM,MUL}.
 * Writes at most `cap` stages to `out` (host memory) and returns the chain
 * length, or -1 for an unknown name.
 */
RF_API int rf_describe_cascade(const char* entry, rf_stage* out, int cap);

/*
 * Safe softmax over the last axis (Section 2.2): the cascade
 *   m = max_j x[j];  t = sum_j exp(x[j]-m);  y[j] = exp(x[j]-m)/t
 * computed with one read of x and one write of y.
 *   x, y : same shape, ndim 1..5, last axis contiguous; dtype bf16->bf16 or
 *          f32->f32.  Leading dims are flattened to rows; they must be
 *          expressible with one row pitch (contiguous, or 2-D with a pitch).
 *   axis : must name the last axis (ndim-1 or -1); otherwise RF_ERR_UNSUPPORTED.
 *   y may alias x exactly (in place); any other overlap is undefined.
 */
RF_API rf_status rf_safe_softmax(const rf_tensor* x, rf_tensor* y, int axis, rf_stream stream);

/*
 * Mean and population variance over the last axis (paper Appendix, evaluation on
 * non-ML workloads): the cascade
 *   m = (1/L) sum_l x[l];   var = (1/L) sum_l (x[l] - m)^2
 * computed with one read of x.  The running state is (count, mean, M2) and is
 * merged pairwise (Section 3.2, level-k fused expression, for this cascade).
 *   x    : ndim 1..5, last axis contiguous and non-empty, f32 or bf16; leading
 *          dims must be expressible with one row pitch.
 *   mean, var : f32, contiguous, shape = x.shape without the last axis
 *          (shape [1] when x is 1-D).
 */
RF_API rf_status rf_variance(const rf_tensor* x, rf_tensor* mean, rf_tensor* var,
                             rf_stream stream);

/*
 * MoE routing (Appendix A.2, "MoE routing"): the scores GEMM feeding the cascade
 *   p[e] = sum_c x[c] w[c,e];  m = max_e p[e];  t = sum_e exp(p[e]-m);  s = TopK_e p[e]
 * with output exp(s - m) / t, the softmax probability of each selected expert.
 * TopK acts on the raw scores (softmax keeps their order); the k results are in
 * descending order of score, equal scores in ascending order of expert index.
 * The contraction axis is split over workgroups (multi-segment strategy,
 * Section 4.3); fp32 partial scores pass through `workspace`.
 *   x    : [S, hd] bf16, tokens.            hd % 128 == 0.
 *   w    : [hd, E] bf16, router weights.    E in {32, 64, 128}.
 *   topk : 1 .. min(E, 16).
 *   prob : [S, topk] f32;  idx : [S, topk] i32 (expert indices).
 *   workspace : device memory, 16-byte aligned, at least
 *          rf_moe_routing_workspace_bytes(S, hd, E) bytes; contents need no
 *          initialisation and are undefined afterwards.  Too small or misaligned:
 *          RF_ERR_WORKSPACE.  Concurrent calls must not share a workspace.
 */
RF_API size_t rf_moe_routing_workspace_bytes(int64_t S, int64_t hd, int64_t E);
RF_API rf_status rf_moe_routing(const rf_tensor* x, const rf_tensor* w, int topk, rf_tensor* prob,
                                rf_tensor* idx, void* workspace, size_t workspace_bytes,
                                rf_stream stream);

/*
 * rf_moe_routing for callers that cannot allocate device memory or hand over a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as rf_moe_routing, but the fp32 partial
 * scores live in a device array inside the library (RF_MOE_ROUTING_NOALLOC_MAX_BYTES bytes,
 * held by every GPU the library is used on until the process ends) instead of a caller's
 * workspace; the call allocates and frees nothing.
 *   A problem whose rf_moe_routing_workspace_bytes(S, hd, E) exceeds
 *   RF_MOE_ROUTING_NOALLOC_MAX_BYTES is refused with RF_ERR_WORKSPACE before any launch.
 *   The device of `stream` must be the current device.  All calls on one GPU share that
 *   GPU's array: calls that overlap in time on one GPU (different streams, different host
 *   threads) race on it and must be serialised by the caller.  Nothing in the array needs
 *   a particular value between calls.
 */
#define RF_MOE_ROUTING_NOALLOC_MAX_BYTES ((size_t)8 << 20)
RF_API rf_status rf_moe_routing_noalloc(const rf_tensor* x, const rf_tensor* w, int topk,
                                        rf_tensor* prob, rf_tensor* idx, rf_stream stream);

/*
 * FP8 per-token quantisation fused with a GEMM (Section 3.4, case study): the cascade
 *   m = max_k |a[k]|;   c[n] = sum_k q(MAX a[k] / m) w[n,k]
 * (q = rounding to OCP E4M3, nearest-even, MAX = 448), returned as c * m / MAX, an
 * approximation of a @ w^T, computed in ONE pass over k with the incremental form of
 * Section 3.4: the running maximum m' of the row prefix seen so far scales the elements that
 * arrive, and the accumulator is rescaled by m'_old / m'_new whenever the maximum moves.
 * Rounding sits between the two reductions, so the one-pass value is not bit-identical to the
 * two-pass definition above: an element is quantised with some prefix maximum m' <= m that
 * includes it.  What is promised, for any way the kernel cuts the row into prefixes:
 *   - every dequantised element (m'/MAX) q(MAX a[k]/m') is within 2^-4 |a[k]| + 2^-10 m / MAX
 *     of a[k], as in the two-pass definition, so
 *       |c - c_twopass| <= 2 sum_k (2^-4 |a[k]| + 2^-10 m / MAX) |w[n,k]|
 *     plus fp32 accumulation and the bf16 rounding of c;
 *   - a token whose maximum is its first element is quantised exactly as in the two-pass
 *     definition; an all-zero token gives an all-zero output row.
 *   a : [M, K] bf16.  K % 128 == 0.
 *   w : [N, K] FP8 E4M3, row n = output channel n (already quantised; any weight scale is
 *       the caller's to apply).  N % 8 == 0.
 *   c : [M, N] bf16.
 */
RF_API rf_status rf_fp8_quant_gemm(const rf_tensor* a, const rf_tensor* w, rf_tensor* c,
                                   rf_stream stream);

/*
 * Fused attention, single-segment strategy (Section 4.3; Appendix A.2):
 *   P = scale * Q K^T;  m = max_j P;  t = sum_j exp(P-m);  O = sum_j exp(P-m)/t * V[j]
 * with the running state (m, l, acc) kept on chip and acc divided by l once
 * at the end.
 *   q : [B, Hq, Lq, d]     k, v : [B, Hkv, Lk, d]     o : [B, Hq, Lq, d]
 *   all four tensors f32, or all four bf16; d in {64, 128}; Hq % Hkv == 0,
 *   query head h reads KV head h / (Hq/Hkv).
 *   causal != 0: query i sees key j iff j <= i + (Lk - Lq).
 *   A query row with no visible key (or Lk == 0) produces zeros.
 */
RF_API rf_status rf_cascade_attention(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v,
                               rf_tensor* o, float scale, int causal, rf_stream stream);

/*
 * Multi-segment strategy, first half (Section 4.3; Appendix A.4 partial
 * kernel): the key axis is cut into num_splits chunks, chunk c covering keys
 * [c*ceil(Lk/S), min(Lk,(c+1)*ceil(Lk/S))), and each chunk's state is written:
 *   part_m, part_l : [B, Hq, Lq, S]     f32   (row max, sum of exp)
 *   part_acc       : [B, Hq, Lq, S, d]  f32   UNNORMALISED sum_j exp(P-m_c) V[j]
 * An empty or fully masked chunk stores the identity state (-inf, 0, 0...).
 *   q, k, v as for rf_cascade_attention, bf16 only, d == 128.
 *   The three partial-state tensors must be contiguous and of exactly these
 *   shapes (RF_ERR_WORKSPACE otherwise).
 */
RF_API rf_status rf_cascade_attention_splitk(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v,
                                      int num_splits, rf_tensor* part_m, rf_tensor* part_l,
                                      rf_tensor* part_acc, float scale, int causal,
                                      rf_stream stream);

/*
 * Multi-segment strategy, second half: the level-k fused expression
 * (Section 3.2 Eq. (11); Appendix A.2 level-k form) over the S partial states
 *   m = max_c m_c;  l = sum_c l_c exp(m_c-m);  O = sum_c acc_c exp(m_c-m) / l.
 *   part_m, part_l : [B, Hq, Lq, S] f32; part_acc : [B, Hq, Lq, S, d] f32,
 *   contiguous; o : [B, Hq, Lq, d] bf16 or f32; any S >= 1; d % 4 == 0.
 *   Rows whose l is 0 produce zeros.
 */
RF_API rf_status rf_merge_states(const rf_tensor* part_m, const rf_tensor* part_l,
                          const rf_tensor* part_acc, rf_tensor* o, rf_stream stream);

/*
 * RMSNorm fused with a linear layer: the "sum + sum" cascade (Appendix A.2)
 *   ss_i = sum_k x[i,k]^2
 *   y[i,n] = sum_k x[i,k] g[k] w[k,n] * (ss_i/K + eps)^(-1/2)
 * as one GEMM pass over K with a side accumulator for ss and one per-row
 * rescale in the epilogue.
 *   x : [M, K] bf16   g : [K] bf16   w : [K, N] bf16 (row-major)   y : [M, N] bf16
 *   K % 64 == 0 and N % 8 == 0 are required, and the row pitches of x and w must be below
 *   2^24 elements (RF_ERR_UNSUPPORTED otherwise); M is arbitrary.
 */
RF_API rf_status rf_rmsnorm_gemm(const rf_tensor* x, const rf_tensor* g, const rf_tensor* w,
                          rf_tensor* y, float eps, rf_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* RF_H_ */
