/*
 * molora.h -- C ABI of the MI355X (gfx950) routed-LoRA hot path.
 *
 * The library computes the per-token routed LoRA projection of the MoLoRA paper
 * (Eq. "pertok"):
 *
 *     h_i = x_i W + x_i A_{r(i)} B_{r(i)},        r : [N] -> [C]
 *
 * in the execution order of the paper's physical pipeline (Fig. "molora", right):
 * router -> histogram & group by adapter -> grouped GEMM -> scatter back to the
 * original positions.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - Every pointer marked DEVICE is device memory owned by the caller (for example a
 *    torch tensor's data_ptr()); pointers marked HOST are ordinary host memory read
 *    during the call.  The library never allocates, frees or retains caller memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call
 *    only enqueues work on it and returns without synchronising; results are valid
 *    once the stream has reached that point.
 *  - Layouts are dense row-major with no strides (stacked weight shapes of Table
 *    "tab:moe_adapter": A is (C, d_in, rank), B is (C, rank, d_out)):
 *        x [N][d_in] bf16      W [d_in][d_out] bf16      G [d_in][C] bf16
 *        A [C][d_in][rank] bf16          B [C][rank][d_out] bf16
 *        r [N] int32           offsets [C+1] int32       perm [N] int32
 *        h [N][d_out] fp32
 *    bf16 values are raw 16-bit patterns.  Device pointers must be 16-byte aligned.
 *  - Return value: MOLORA_OK, or a negative code.  Problems the host can see (null
 *    pointer, bad size, misalignment, workspace too small) are reported before anything
 *    is enqueued and leave all outputs untouched.  A failed launch maps to MOLORA_EHIP.
 *  - Data-dependent problems (a routing target outside [0, C)) cannot be seen by the
 *    host without a synchronisation; they are reported through an optional DEVICE flag
 *    and handled as "this token has no adapter" (see molora_bucket).
 *  - Inputs are expected to be finite.  The argmax is a scan from target 0 that moves on a
 *    strict ">": a NaN logit at a target above 0 is never selected, a NaN at target 0 is
 *    kept unless a later logit compares greater (never, against NaN), so it yields r = 0.
 */
#ifndef MOLORA_H
#define MOLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int molora_status;

enum {
    MOLORA_OK = 0,
    MOLORA_EINVAL = -1,     /* null pointer, non-positive or unsupported size          */
    MOLORA_EALIGN = -2,     /* a device pointer is not 16-byte aligned                 */
    MOLORA_EWORKSPACE = -3, /* workspace_bytes smaller than molora_apply_workspace_bytes */
    MOLORA_EHIP = -5        /* the HIP runtime reported an error at launch            */
};

/* Limits of this implementation (checked, MOLORA_EINVAL beyond them). */
#define MOLORA_MAX_TARGETS 1024 /* C                                   */
#define MOLORA_MAX_RANK 128     /* rank, which must be a multiple of 8 */
#define MOLORA_MAX_BREAKS 64    /* M of molora_route_vocab             */
#define MOLORA_MAX_HIDDEN 256   /* H of molora_route_mlp, a multiple of 8 */
#define MOLORA_MAX_TOPK 4       /* k of molora_route_mlp / molora_apply_mix */
#define MOLORA_STATIC_WORKSPACE_BYTES (8u << 20) /* scratch of molora_apply_static, per GPU */

/*
 * Learned routing with one selected adapter per token (Sec. "Router Architecture"
 * with k = 1: the softmax over the single selected logit is 1, which leaves Eq.
 * "pertok").  The gate is the linear, bias-free form of Table "tab:moe_adapter":
 *
 *     r[i] = argmax_c sum_k x[i][k] * G[k][c],     lowest c on ties.
 *
 * Each logit is accumulated in fp32 in ascending k, one rounded addition per term
 * (the bf16 x bf16 products are exact in fp32), so r is a deterministic function of
 * the input bits.
 *   x DEVICE bf16 [N][d_in]; G DEVICE bf16 [d_in][C]; r DEVICE int32 [N] (written).
 *   N >= 0; d_in >= 1 and a multiple of 8; 1 <= C <= MOLORA_MAX_TARGETS.
 */
molora_status molora_route(const void *x, const void *G, int32_t *r,
                           int64_t N, int32_t d_in, int32_t C, void *stream);

/*
 * Vocabulary routing (Def. "Vocabulary Routing"): with breaks b_0 < b_1 < ... < b_M the
 * token id v routes to the 0-based range m with b_m <= v < b_{m+1}; ids outside
 * [b_0, b_M) get -1 ("no adapter").
 *   v DEVICE int32 [N]; breaks HOST int32 [M+1], strictly increasing, copied during the
 *   call; r DEVICE int32 [N] (written).  1 <= M <= MOLORA_MAX_BREAKS.
 */
molora_status molora_route_vocab(const int32_t *v, const int32_t *breaks, int32_t M,
                                 int32_t *r, int64_t N, void *stream);

/*
 * Dispatch (Sec. "Unified Dispatch Infrastructure", Alg. "Unified Dispatch Kernel"):
 * histogram of tokens per target and a position for every token inside its target's
 * list.  Where the paper hands out positions with an atomic counter (any order inside a
 * list), this library orders every list by ascending token index, which makes the
 * result unique; offsets + perm carry the same information as the paper's per-target
 * pointer arrays xs/ys (row p of the grouped problem is x[perm[p]] and lands in
 * h[perm[p]]).
 *
 *     offsets[0] = 0,  offsets[c+1] = offsets[c] + |{t : r[t] = c}|      (c < C)
 *     perm[offsets[c] .. offsets[c+1]) = tokens with r = c, ascending
 *     perm[offsets[C] .. N)            = tokens with r outside [0, C), ascending
 *
 * so perm is always a permutation of 0..N-1 and offsets[C] <= N counts the routed
 * tokens.  If err_flag is not NULL it is set to 1 when some r[t] is outside [0, C) and
 * left unchanged otherwise (the caller zeroes it).
 *   r DEVICE int32 [N]; offsets DEVICE int32 [C+1]; perm DEVICE int32 [N];
 *   err_flag DEVICE int32 [1] or NULL.  0 <= N < 2^31; 1 <= C <= MOLORA_MAX_TARGETS.
 */
molora_status molora_bucket(const int32_t *r, int32_t *offsets, int32_t *perm,
                            int64_t N, int32_t C, int32_t *err_flag, void *stream);

/*
 * Bytes of DEVICE workspace molora_apply / molora_apply_bucketed need for these sizes
 * (0 if the sizes are invalid).  The workspace holds the bucketing (molora_apply only),
 * the low-rank intermediate t = x A_r in sorted order and, for small batches, the partial
 * sums of a shrink whose K range is split over workgroups; its contents are scratch and
 * need no initialisation.
 */
size_t molora_apply_workspace_bytes(int64_t N, int32_t d_in, int32_t d_out,
                                    int32_t C, int32_t rank);

/*
 * The routed projection, Eq. "pertok":  h[i][:] = x[i] W + (x[i] A[r[i]]) B[r[i]].
 * Buckets r internally (as molora_bucket), computes the grouped shrink t = x A_c, then
 * one GEMM pass that adds the grouped expand t B_c in the epilogue of x W and writes
 * every row of h once, at its original position.  A token whose r[i] is outside [0, C)
 * gets h[i] = x[i] W.  bf16 products are accumulated in fp32; t is carried as a pair of
 * bf16 values (high part + remainder), so its rounding does not limit the result.
 *   x, W, A, B, r DEVICE (read); h DEVICE fp32 [N][d_out] (every element written);
 *   workspace DEVICE, 256-byte aligned, workspace_bytes >= molora_apply_workspace_bytes.
 *   0 <= N < 2^31; d_in, d_out >= 8 and multiples of 8; rank a multiple of 8,
 *   8 <= rank <= MOLORA_MAX_RANK; 1 <= C <= MOLORA_MAX_TARGETS.  For N > 512 (where the
 *   tiled kernel may be taken) x and W must each be smaller than 4 GiB
 *   (N * d_in < 2^31 and d_in * d_out < 2^31 elements): larger ones are MOLORA_EINVAL,
 *   here and in molora_apply_bucketed, molora_base_expand and molora_apply_mix.
 */
molora_status molora_apply(const void *x, const void *W, const void *A, const void *B,
                           const int32_t *r, float *h,
                           int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * molora_apply for callers that cannot allocate device memory and have no workspace to hand
 * in: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and bit-identical h; the workspace is a fixed array of
 * MOLORA_STATIC_WORKSPACE_BYTES (8 MiB) inside the library, one copy per GPU, held until the
 * process ends.  Sizes whose molora_apply_workspace_bytes exceeds it are refused with
 * MOLORA_EWORKSPACE before anything is enqueued (8 MiB covers N = 16384 tokens at rank 32, or
 * 8192 at rank 64, ...).  The call allocates nothing (no hipMalloc / hipFree, no allocating
 * library routine).  All calls on one GPU share that GPU's array: calls that overlap in time
 * on one GPU (two streams, two threads) race on it and must be serialised by the caller;
 * successive calls on one stream are safe.  The array keeps the last call's contents; nothing
 * in it needs to start at zero.  molora_static_workspace_bytes returns the limit.
 */
size_t molora_static_workspace_bytes(void);
molora_status molora_apply_static(const void *x, const void *W, const void *A, const void *B,
                                  const int32_t *r, float *h,
                                  int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                  void *stream);

/*
 * Same as molora_apply for a caller that already holds molora_bucket's output for r
 * (for example several projections that share one routing decision): offsets and perm
 * replace r, and the bucketing step is skipped.
 */
molora_status molora_apply_bucketed(const void *x, const void *W, const void *A, const void *B,
                                    const int32_t *offsets, const int32_t *perm, float *h,
                                    int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                    int32_t rank, void *workspace, size_t workspace_bytes,
                                    void *stream);

/*
 * The two kernels of molora_apply_bucketed as separate calls (same semantics, same
 * kernels), for callers that want to time or schedule them individually.
 *
 * molora_shrink:  t_p = x[perm[p]] A_c  for every routed sorted position p in bucket c
 * (offsets[c] <= p < offsets[c+1]); rows p >= offsets[C] are not touched.  t is written
 * as two bf16 halves per value, t = hi + lo with hi = bf16(t), lo = bf16(t - hi):
 *   t DEVICE bf16 [N][2*rank], row p = [hi_0 .. hi_{rank-1} | lo_0 .. lo_{rank-1}].
 * molora_base_expand:  h[perm[p]][:] = x[perm[p]] W + t_p B_c  (rows without adapter:
 * x W only), every row of h written once.
 * offsets and perm must be molora_bucket's output for this N and C.
 * molora_shrink's workspace is optional DEVICE scratch (256-byte aligned, contents need no
 * initialisation) of molora_shrink_workspace_bytes(...) bytes, which is 0 for most sizes: a
 * batch of a few dozen tokens has too few (adapter, row tile) pairs to occupy the chip, so
 * the K range of t = x A_c is then cut into slices over more workgroups, whose fp32 partial
 * sums pass through the scratch and are added in a fixed order by a second kernel.  With
 * workspace NULL (or smaller than that) K is not split: same t up to the order of the fp32
 * additions, more slowly.
 */
size_t molora_shrink_workspace_bytes(int64_t N, int32_t d_in, int32_t C, int32_t rank);
molora_status molora_shrink(const void *x, const void *A, const int32_t *offsets,
                            const int32_t *perm, void *t, int64_t N, int32_t d_in, int32_t C,
                            int32_t rank, void *workspace, size_t workspace_bytes, void *stream);
molora_status molora_base_expand(const void *x, const void *W, const void *B, const void *t,
                                 const int32_t *offsets, const int32_t *perm, float *h,
                                 int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                 void *stream);

/*
 * Dispatch and shrink in ONE launch, for layers with a few narrow adapters (Alg. "Unified
 * Dispatch Kernel" / Alg. "Compositional Gating Kernel" beside the shrink of Eq. "pertok").
 * The grouped shrink needs the dispatch step's permutation, so the two normally run one after
 * the other, each bound by latency on a batch of a few thousand tokens.  When C * rank <= 64
 * (and N > 512) the shrink can do without the permutation: it computes x_i A_c for EVERY c in
 * token order (the step is bound by reading x; the extra arithmetic costs nothing) and the
 * expand step picks the row's adapter, so both steps fit one launch in which no workgroup
 * waits for another.  molora_dense_shrink_supported says (1 / 0) whether the sizes qualify;
 * the calls below return MOLORA_EINVAL when they do not.  molora_apply takes this path by
 * itself.
 *
 *   molora_bucket_shrink:         r given -> offsets, perm as molora_bucket, and t
 *   molora_gate_dispatch_shrink:  token ids (and request adapters) -> r, offsets, perm as
 *                                 molora_gate_dispatch (C = n_adapters * M), and t
 *   molora_base_expand_dense:     molora_base_expand reading that t
 *
 * t DEVICE bf16 [N][2 * C * rank], the TOKEN-ORDER intermediate: row i =
 * [hi(x_i A_0) .. hi(x_i A_{C-1}) | lo(x_i A_0) .. lo(x_i A_{C-1})], hi = bf16(value),
 * lo = bf16(value - hi).  Other arguments, ordering, err_flag and errors as in molora_bucket /
 * molora_gate_dispatch / molora_shrink / molora_base_expand.
 */
int32_t molora_dense_shrink_supported(int64_t N, int32_t d_in, int32_t C, int32_t rank);
molora_status molora_bucket_shrink(const int32_t *r, const void *x, const void *A, int32_t *offsets,
                                   int32_t *perm, void *t, int64_t N, int32_t d_in, int32_t C,
                                   int32_t rank, int32_t *err_flag, void *stream);
molora_status molora_gate_dispatch_shrink(const int32_t *v, const int32_t *adapter,
                                          const int32_t *breaks, int32_t M, int32_t n_adapters,
                                          const void *x, const void *A, int32_t *r, int32_t *offsets,
                                          int32_t *perm, void *t, int64_t N, int32_t d_in,
                                          int32_t rank, int32_t *err_flag, void *stream);
molora_status molora_base_expand_dense(const void *x, const void *W, const void *B, const void *t,
                                       const int32_t *offsets, const int32_t *perm, float *h,
                                       int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                       int32_t rank, void *stream);

/*
 * Dispatch and shrink in one launch for a batch of at most 64 tokens (a decode step): the
 * targets of the whole batch are one wavefront of keys, so every workgroup of the shrink
 * derives the rows of its adapter from r itself (ascending token index: the stable order of
 * Alg. "Unified Dispatch Kernel") instead of waiting for a dispatch launch, and offsets and perm
 * are written on the side for molora_base_expand.  Same outputs as molora_bucket followed by
 * molora_shrink (offsets, perm bit for bit; t in the bucket-order layout of molora_shrink,
 * [N][2*rank]), same optional workspace as molora_shrink, err_flag as molora_bucket.
 * molora_bucket_shrink_small_supported says (1 / 0) whether the sizes qualify (N <= 64 and a
 * rank above 32, where the shrink is the K-streaming kernel); otherwise MOLORA_EINVAL.
 * molora_apply takes this path by itself.
 */
int32_t molora_bucket_shrink_small_supported(int64_t N, int32_t d_in, int32_t C, int32_t rank);
molora_status molora_bucket_shrink_small(const int32_t *r, const void *x, const void *A,
                                         int32_t *offsets, int32_t *perm, void *t, int64_t N,
                                         int32_t d_in, int32_t C, int32_t rank, void *workspace,
                                         size_t workspace_bytes, int32_t *err_flag, void *stream);

/*
 * A batch of at most 64 tokens in two launches (sizes as molora_bucket_shrink_small_supported):
 *
 *   molora_shrink_base_small:  offsets, perm, t as molora_bucket_shrink_small (K never split)
 *                              AND h = x W, all in one launch.  The base projection of a batch
 *                              of one row tile runs in token order and needs nothing from the
 *                              dispatch step, so the latency-bound shrink (a dozen workgroups,
 *                              each reading one A_c) hides behind the stream of W instead of
 *                              preceding it.
 *   molora_expand_small:       h[perm[p]] += t_p B_c for every routed sorted position p: the
 *                              expand of Eq. "pertok" alone, added to what h holds.
 *
 * One after the other they give what molora_bucket, molora_shrink and molora_base_expand give,
 * up to the order of the fp32 additions.  molora_apply takes this path by itself.  Arguments,
 * layouts and errors as in those calls; h is written by the first call and read and
 * written by the second.
 */
molora_status molora_shrink_base_small(const int32_t *r, const void *x, const void *W, const void *A,
                                       int32_t *offsets, int32_t *perm, void *t, float *h, int64_t N,
                                       int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                       int32_t *err_flag, void *stream);
molora_status molora_expand_small(const void *B, const void *t, const int32_t *offsets,
                                  const int32_t *perm, float *h, int64_t N, int32_t d_out, int32_t C,
                                  int32_t rank, void *stream);

/*
 * The base weight of a decode step in the layout its kernel streams best.  With at most 64
 * rows the step of Eq. "pertok" is one read of W from HBM.  A workgroup owns a group of gc = 64
 * (32 for d_out <= 8192) output columns and its wavefronts take 16 rows of W at a time: in the
 * row-major W such a slab is sixteen pieces of 2*gc bytes, d_out elements apart.  W is constant
 * while a model is served, so it can be stored once with every slab contiguous:
 *
 *     Wp, d_in * d_out bf16 elements: W cut into slabs of 16 rows (slab s = rows 16 s ..;
 *     the last one holds 8 rows when d_in is not a multiple of 16) that start where they
 *     start in W, at element 16 s * d_out; inside a slab of n rows column group g is an
 *     [n][gc] matrix of its own at offset g * n * gc:
 *     Wp[16 s * d_out + g * n * gc + i * gc + c] = W[16 s + i][g * gc + c]
 *
 * The workgroups advance through W together, so at any time the chip reads one contiguous
 * region (measured at 64 x 4096 -> 12288: 27.0 us against 31.4 us for the launch).
 * molora_pack_w_cols(d_out) returns gc, or 0 when d_out is not a multiple of it (no packed
 * form: use molora_shrink_base_small).  molora_pack_w writes Wp from W (device pointers, 16-byte
 * aligned, distinct buffers of d_in * d_out elements; MOLORA_EINVAL for a d_out without packed
 * form).  molora_shrink_base_small_packed is molora_shrink_base_small with Wp in the place of
 * W: the same arithmetic in the same order, so every output is bit-identical; MOLORA_EINVAL in
 * the same cases and for a d_out without packed form.
 *
 * The adapters' B are static too: B [C][rank][d_out] is a [C * rank][d_out] matrix, and
 * molora_pack_w(B, Bp, C * rank, d_out) stores it the same way (with rank a multiple of 16 a
 * slab lies inside one adapter).  molora_expand_small_packed is molora_expand_small with Bp
 * in the place of B: bit-identical h; MOLORA_EINVAL in the same cases, for a rank that is
 * not a multiple of 16 and for a d_out without packed form.
 */
int32_t molora_pack_w_cols(int32_t d_out);
molora_status molora_pack_w(const void *W, void *Wp, int32_t d_in, int32_t d_out, void *stream);
molora_status molora_shrink_base_small_packed(const int32_t *r, const void *x, const void *Wp,
                                              const void *A, int32_t *offsets, int32_t *perm, void *t,
                                              float *h, int64_t N, int32_t d_in, int32_t d_out,
                                              int32_t C, int32_t rank, int32_t *err_flag,
                                              void *stream);
molora_status molora_expand_small_packed(const void *Bp, const void *t, const int32_t *offsets,
                                         const int32_t *perm, float *h, int64_t N, int32_t d_out,
                                         int32_t C, int32_t rank, void *stream);

/*
 * molora_base_expand with the height of the row tiles forced, for the tiling ablation (App.
 * "Adaptive Tiling", Table "tab:adaptive_tiling": tile shape chosen from the load against one
 * fixed shape).  tile_rows = 64 (the streaming kernel, W read once per 64-row tile), 128
 * (128 x 128 output tiles) or 256 (256 x 256 tiles); anything else is MOLORA_EINVAL.  Same
 * result as molora_base_expand up to the order of the fp32 additions.
 */
molora_status molora_base_expand_fixed(const void *x, const void *W, const void *B, const void *t,
                                       const int32_t *offsets, const int32_t *perm, float *h,
                                       int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                       int32_t rank, int32_t tile_rows, void *stream);

/*
 * Learned router with top-k selection (Sec. "Router Architecture"):
 *
 *     logits_i = W2^T GELU(W1^T x_i + b1) + b2,   idx_i = TopK(logits_i, k),
 *     w_i = softmax(logits_i[idx_i])
 *
 * x [N][d_in], W1 [d_in][H], W2 [H][K] bf16 device pointers; b1 [H], b2 [K] fp32 device
 * pointers; idx [N][k] int32 and w [N][k] fp32 device outputs, the selected targets in
 * descending order of their logit (lowest index first among equal logits) and their mixture
 * weights.  H (a multiple of 8, <= MOLORA_MAX_HIDDEN) is 64 in the paper; K <=
 * MOLORA_MAX_TARGETS; 1 <= k <= min(K, MOLORA_MAX_TOPK).  Arithmetic: fp32 throughout, every
 * sum sequential in ascending index order with the bias added last, GELU in its exact erf form
 * evaluated by a fixed sequence of fp32 operations (so the selection is reproducible bit for
 * bit).  workspace: device scratch of molora_route_mlp_workspace_bytes(N, H) bytes, 256-byte
 * aligned, owned by the caller (holds the hidden pre-activations).  Errors as molora_apply.
 */
size_t molora_route_mlp_workspace_bytes(int64_t N, int32_t H);
molora_status molora_route_mlp(const void *x, const void *W1, const float *b1, const void *W2,
                               const float *b2, int32_t *idx, float *w, int64_t N, int32_t d_in,
                               int32_t H, int32_t K, int32_t k, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * Compositional gating (Alg. "Compositional Gating Kernel"): the composite target of token i
 * is  r[i] = adapter[i] * M + m,  m the modality of vocabulary index v[i] as in
 * molora_route_vocab (breaks: HOST pointer to M + 1 ascending ints), adapter[i] the slot of
 * the request the token belongs to.  r[i] = -1 when v[i] is outside [breaks[0], breaks[M]) or
 * adapter[i] outside [0, n_adapters).  v, adapter, r: device int32 [N];
 * n_adapters * M <= MOLORA_MAX_TARGETS.  With the hot-set layout A [S][M][d][r] the composite
 * target indexes the flattened pool directly.
 */
molora_status molora_route_compose(const int32_t *v, const int32_t *adapter, const int32_t *breaks,
                                   int32_t M, int32_t n_adapters, int32_t *r, int64_t N,
                                   void *stream);

/*
 * Gating and dispatch in one launch, the way Alg. "Compositional Gating Kernel" is written:
 * the composite target of molora_route_compose (adapter == NULL: of molora_route_vocab, i.e.
 * n_adapters = 1 and a = 0) is computed inside the dispatch kernel.  Outputs r [N] as the
 * routing call would give it, and offsets [n_adapters * M + 1], perm [N] as molora_bucket
 * would give them for that r (same ordering, same treatment of -1, same err_flag).  Saves a
 * launch and a pass over r for integer routing, where the whole step is latency bound.
 */
molora_status molora_gate_dispatch(const int32_t *v, const int32_t *adapter, const int32_t *breaks,
                                   int32_t M, int32_t n_adapters, int32_t *r, int32_t *offsets,
                                   int32_t *perm, int64_t N, int32_t *err_flag, void *stream);

/*
 * Weighted top-k mixture with an optional slot table (Sec. "Router Architecture", Def.
 * "Hot-Set Layout"):
 *
 *     h[i][:] = x[i] W + sum_{j<k} w[i][j] (x[i] A_s) B_s,   s = slots[idx[i][j]]
 *
 * idx [N][k] int32 targets in [0, C) (an entry outside contributes nothing); w [N][k] fp32
 * weights (NULL: all 1); slots [C] int32 device table from target to position in the pools
 * A [S][d_in][rank], B [S][rank][d_out] (NULL: position = target; the caller guarantees
 * 0 <= slots[c] < S).  Tokens are grouped by their tuple of targets, so C^k must not exceed
 * MOLORA_MAX_TARGETS and k * rank must not exceed MOLORA_MAX_RANK; k <= MOLORA_MAX_TOPK.
 * k = 1, w = NULL, slots = NULL is molora_apply.  workspace as for molora_apply, of
 * molora_apply_mix_workspace_bytes(...) bytes.  Errors as molora_apply.
 */
size_t molora_apply_mix_workspace_bytes(int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                        int32_t rank, int32_t k);
molora_status molora_apply_mix(const void *x, const void *W, const void *A, const void *B,
                               const int32_t *idx, const float *w, const int32_t *slots, float *h,
                               int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                               int32_t k, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Replayable launch sequences (Sec. "CUDA Graph Compatibility": fixed shapes and fixed
 * addresses allow a serving step to be recorded once and replayed).
 *
 * molora_graph_begin puts `stream` (a hipStream_t other than the null stream) into capture
 * mode; every molora_* call issued on that stream until molora_graph_end is recorded instead
 * of executed (all of them are capturable: no allocation, no synchronisation, no host read of
 * device memory).  The once-per-device set-up of molora_init is not a stream operation and
 * must not happen inside a capture: molora_graph_begin runs it before the capture starts; a
 * caller that captures with the HIP API itself calls molora_init() first.  molora_graph_end stops the capture and returns an executable graph, owned
 * by the caller, in *graph (NULL on error).  molora_graph_launch replays it on `stream`
 * (asynchronous, any stream of the same device); the recorded calls read and write the same
 * device addresses as at capture time, so the caller refreshes inputs in place.
 * molora_graph_destroy frees the graph (NULL is ignored; the graph must not be running).
 * Errors: MOLORA_EINVAL for NULL arguments, MOLORA_EHIP when the runtime refuses.
 */
typedef struct molora_graph molora_graph;
molora_status molora_graph_begin(void *stream);
molora_status molora_graph_end(void *stream, molora_graph **graph);
molora_status molora_graph_launch(molora_graph *graph, void *stream);
void molora_graph_destroy(molora_graph *graph);

/*
 * For benchmarks (no passage of the paper: a measuring aid): the device-side duration of one
 * launch of the kernel that holds the base projection, taken from the launch's own dispatch,
 * which is the interval a kernel trace reports.  molora_launch_timer_create makes a timer (two
 * HIP events; the one place where the library creates anything).  molora_launch_timer_arm
 * hands it to the calling thread's next launch of such a kernel -- the tiled GEMM of
 * molora_base_expand* / molora_apply*, the small-batch GEMM of the same calls, the launch of
 * molora_shrink_base_small* -- which records its start and end on it; other launches pass it
 * by, a timer armed later replaces it, and a launch under stream capture must not be given one.
 * molora_launch_timer_elapsed_us waits for that launch to finish (the only call of the
 * library that blocks) and returns its duration; MOLORA_EHIP if no launch took the timer.  A
 * timer can be armed again after it has been read.  molora_launch_timer_destroy frees it
 * (NULL is ignored).  MOLORA_EINVAL for NULL arguments.
 */
typedef struct molora_launch_timer molora_launch_timer;
molora_status molora_launch_timer_create(molora_launch_timer **timer);
molora_status molora_launch_timer_arm(molora_launch_timer *timer);
molora_status molora_launch_timer_elapsed_us(molora_launch_timer *timer, double *us);
void molora_launch_timer_destroy(molora_launch_timer *timer);

/*
 * Once-per-device set-up on the current device: tells the runtime which kernels use more than
 * 64 KB of LDS.  Every entry point does this by itself the first time it runs on a device, so
 * the call is only needed before the caller's own stream capture (see above).  Enqueues
 * nothing, allocates nothing; thread safe.  MOLORA_EHIP if the runtime refuses (no device).
 */
molora_status molora_init(void);

/* Human-readable name of a status code (static storage, never NULL). */
const char *molora_status_string(molora_status status);

/* Library version string, e.g. "molora-gfx950 0.1" (static storage). */
const char *molora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOLORA_H */
