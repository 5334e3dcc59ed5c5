/*
 * sablock.h -- C ABI of the SABlock prefill-time KV-cache compression path on
 * MI355X (gfx950).
 *
 * The five calls are the steps of the paper's method in order:
 *   sablock_score          window attention scores of every cached key   (Sec. 3.2, Eqs. barA, st, Dk)
 *   sablock_refine         segment-guided score refinement               (Alg. 1, Eqs. Ik, Dk, omegak, st_tilde)
 *   sablock_search_blocks  Top-B, implicit budgets, block-size search    (Alg. 2, Eqs. topk, implicit_budget, rk, gk_star)
 *   sablock_select         per-segment token sets and their union        (Alg. 2, Eq. final_selection)
 *   sablock_compact        gather of K/V rows into the retained cache    (end of Sec. 3.3)
 * (sablock_search_select is sablock_search_blocks and sablock_select in one call, with the same results.)
 * In front of them, sablock_segment_count / sablock_segment_offsets turn token ids and a delimiter set into the
 * segment offsets the five calls take (Sec. 3.1), and sablock_window_attention computes the attention of the window
 * queries together with the row statistics that let sablock_score read K once; behind them,
 * sablock_decode_attention is one decode step over the cache they leave (or over the full cache, for comparison).
 * sablock_score_all_heads / sablock_compact_shared are the variant with one retained set per layer.
 *
 * Conventions shared by all calls
 * -------------------------------
 * Problems.  A call covers n_seq sequences x n_layers layers x n_kv_heads KV
 *   heads; every (sequence, layer, KV head) is an independent problem p =
 *   (seq * n_layers + layer) * n_kv_heads + head, and every per-problem array
 *   is dense in that order.  L = seq_len, W = window (observation window, the
 *   paper's n_rcnt), T = L - W (compressible region), G = n_q_heads/n_kv_heads.
 * Pointers.  Every pointer is a DEVICE pointer unless its comment says "host".
 *   The caller owns all buffers; the library allocates no device memory, keeps
 *   no state between calls, reads no environment variable and frees nothing.
 *   Scratch comes from the caller's workspace `ws` (device, 256-byte aligned)
 *   of at least sablock_workspace_bytes() bytes; its contents are undefined
 *   between calls.  (The only thing remembered is each device's compute-unit
 *   count, asked once per device.)
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = default stream).
 *   Calls only enqueue work and return; outputs are valid once the stream
 *   reaches that point; calls on one stream are ordered.  Calls on different
 *   streams (and from different host threads) may overlap as long as each has
 *   its own workspace and output buffers: nothing else is shared between calls.
 *   Only kernels are enqueued (no allocation, copy, memset or synchronisation),
 *   so a sequence of calls can be captured into a HIP graph.
 * Errors.  Status code only (never exceptions/aborts).  Host scalars are
 *   validated before anything is enqueued: on a non-OK status nothing was
 *   launched.  Device-resident data (segment offsets, NaNs) is not validated.
 *   sablock_last_error() returns a thread-local message for the last failure.
 * Segments.  Sequence s owns the offsets seg_off[seg_ptr[s] .. seg_ptr[s+1])
 *   (device int32, CSR), first entry 0, strictly increasing, last entry T; its
 *   segment count is K_s = seg_ptr[s+1] - seg_ptr[s] - 1.  seg_ptr is a HOST
 *   array of n_seq+1 int32.  Segments are shared by all layers and heads of a
 *   sequence.  Per-segment outputs use the row stride max_segments >= max_s K_s
 *   passed by the caller; entries k >= K_s are written as 0.
 * Ranking.  Wherever tokens or blocks are ranked: value descending, index
 *   ascending; -0.0 and +0.0 rank as equal values.
 */
#ifndef SABLOCK_H
#define SABLOCK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SABLOCK_API __attribute__((visibility("default")))

typedef enum {
    SABLOCK_OK = 0,
    SABLOCK_ERR_INVALID_ARG = 1,          /* null pointer, negative or inconsistent host scalar */
    SABLOCK_ERR_UNSUPPORTED = 2,          /* shape outside what the kernels cover */
    SABLOCK_ERR_WORKSPACE_TOO_SMALL = 3,
    SABLOCK_ERR_DEVICE = 4                /* a HIP call or launch failed */
} sablock_status;

typedef enum { SABLOCK_F32 = 0, SABLOCK_BF16 = 1 } sablock_dtype;

/* Launch parameters of this implementation (no passage of the paper: they change how the work is cut into
 * workgroups, never a result).  Part of the shape, so the workspace size and the calls always see the same
 * values; all zero = the library's own plan, which is what every figure quoted for the library was taken with.
 * Out-of-range values are INVALID_ARG. */
typedef struct {
    int32_t compute_units;    /* compute units the launch plans assume; 0 = ask the current device (DEVICE error
                                 if there is none: set it to size a workspace on a host without a GPU) */
    int32_t score_chunk;      /* keys per workgroup of the MFMA scoring kernels, >= 128, rounded down to a multiple
                                 of 128; 0 = whole rounds of one workgroup per compute unit */
    int32_t window_chunk;     /* keys per workgroup of sablock_window_attention and of the one-read row statistics,
                                 >= 32, rounded down to a multiple of 32; 0 = whole rounds of workgroups */
    int32_t topb_slices;      /* workgroups per row of the two Top-B passes of sablock_search_select, 1 .. 64
                                 (1 = the per-row kernel alone); 0 = by problems per compute unit */
    int32_t stats_per_key;    /* which kernel forms the row statistics where two exist (head_dim 128; 129 .. 256
                                 window-query rows per KV head, and G = 4 with W = 32): 1 = the kernel with a lane per
                                 key on blocks of 128 rows (two blocks: K read twice by that pass), 2 = the kernel with a
                                 lane per window query (one read of K for all rows); 0 = the faster one by measurement
                                 (2 above 128 rows, 1 at 128) */
    int32_t reserved[3];      /* must be 0 */
} sablock_tuning;

/* Host scalars describing one call.  Strides are in ELEMENTS for the four outer
 * axes (sequence, layer, head, token); the head_dim axis is contiguous. */
typedef struct {
    int32_t n_seq;
    int32_t n_layers;
    int32_t n_q_heads;        /* multiple of n_kv_heads */
    int32_t n_kv_heads;
    int32_t head_dim;         /* D: multiple of 8, 8 <= D <= 256 */
    int32_t seq_len;          /* L */
    int32_t window;           /* W: 1 <= W <= 64, W < L */
    int32_t dtype;            /* sablock_dtype of Q, K, V and the compacted outputs */
    int64_t q_stride[4];      /* Q window [n_seq][n_layers][n_q_heads][W][D]; token axis = window query */
    int64_t k_stride[4];      /* K [n_seq][n_layers][n_kv_heads][L][D] */
    int64_t v_stride[4];      /* V, same axes as K */
    sablock_tuning tuning;    /* all zero = defaults */
} sablock_shape;

/* Hyperparameters; the paper's defaults are eps 1e-6, alpha 0.9, eta 1.0, tau 0.85 (Sec. 4.1). */
typedef struct { float eps, alpha, eta, tau; } sablock_hparams;

SABLOCK_API const char *sablock_version(void);
SABLOCK_API const char *sablock_last_error(void);

/* Bytes of workspace that any of the calls below may need for this shape, max_segments and budget as passed to
 * the calls.  Host computation only; the launch plans behind it depend on the compute-unit count, which is
 * shape->tuning.compute_units or, when that is 0, the current device's. */
SABLOCK_API sablock_status sablock_workspace_bytes(const sablock_shape *shape, int32_t max_segments,
                                       int32_t budget, size_t *bytes_out /* host */);

/* Window scoring (Sec. 3.2).  For each problem and each key t in [0, L):
 *   A[h,i,t] = softmax over the keys visible to window query i (t <= T+i; causal
 *              inside the window) of <Q[h,i,:], K[t,:]> / sqrt(D)      (Eq. 1)
 *   Abar[i,t] = mean of A over the G query heads of the KV head          (Eq. barA)
 *   s_out[p][t]   = sum_i Abar[i,t]                                      (Eq. st)
 *   ent_out[p][t] = -sum_i Ahat[i,t] ln(Ahat[i,t] + eps), Ahat = Abar/s  (inner sum of Eq. Dk)
 * q_win, k: shape->dtype, laid out by q_stride/k_stride.
 * row_lse: optional [n_seq][n_layers][n_q_heads][W] float, the natural-log
 *   sum-exp of each window query's scaled logits over its visible keys (what a
 *   prefill attention kernel already has); when NULL it is computed here with an
 *   extra pass over K.
 * eps: > 0 (it keeps the logarithm of a masked or underflowed entry finite; INVALID_ARG otherwise).
 * s_out, ent_out: [P][L] float.  Arithmetic: fp32 accumulate and outputs.
 * Any shape within the limits of sablock_shape is accepted.  bf16 with head_dim 64, 96 or 128, W in {8, 16, 32, 64} and
 * any G with G * W <= 128 (e.g. G = 7 with W = 16, G = 3 with W = 32, G = 16 with W = 8), head_dim 256 with the same
 * windows and G * W <= 96 (e.g. G = 2 with W = 32), and head_dim 128 with
 * 129 .. 256 rows of a window of 32 or 64 queries (G = 5 .. 8 with W = 32, G = 3 or 4 with W = 64), runs on the
 * matrix pipe; every other shape and fp32 on a plain vector kernel, ~20 x slower per key. */
SABLOCK_API sablock_status sablock_score(const sablock_shape *shape, const void *q_win, const void *k,
                             const float *row_lse /* nullable */, float eps,
                             float *s_out, float *ent_out,
                             void *ws, size_t ws_bytes, void *stream);

/* sablock_score for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments (minus ws), same kernels, same results as
 * sablock_score; the row statistics that sablock_score keeps in the caller's workspace live in an array that is
 * part of the library's device code (SABLOCK_STATIC_SCRATCH_BYTES per GPU, held from the moment the library is
 * loaded on that GPU until the process ends).  The call allocates and frees nothing, on the device or through
 * any library.
 * Limit: a call whose statistics need more than SABLOCK_STATIC_SCRATCH_BYTES (the sablock_score part of
 *   sablock_workspace_bytes: about 2 KiB per problem and key chunk) returns UNSUPPORTED and launches nothing.  All
 *   five configurations this library is measured on fit (the largest, 1 024 problems of 256 rows, takes 4 MiB).
 *   With row_lse given no scratch is used at all.
 * Sharing: all calls on one GPU use that GPU's one array.  Calls ordered on one stream are safe; calls that may
 *   overlap on one GPU (other streams, other host threads) race on it: give those sablock_score and a workspace
 *   each.  Nothing needs clearing between calls: each call writes every statistic before it reads it. */
#define SABLOCK_STATIC_SCRATCH_BYTES (8u << 20)
SABLOCK_API sablock_status sablock_score_static(const sablock_shape *shape, const void *q_win, const void *k,
                                    const float *row_lse /* nullable */, float eps,
                                    float *s_out, float *ent_out, void *stream);

/* Measurement aid (no step of the method): streams K exactly as the MFMA scoring kernels do - the same split of
 * every problem's keys into workgroups, the same direct-to-LDS ring per wavefront - and computes nothing.  With
 * read_lds != 0 every key tile is also read from LDS into registers, as the scoring kernels do before their
 * matrix products.  With s_out and ent_out given ([P][L] float each; both or neither) it also writes 4 bytes per
 * key into each, with the store pattern of the scoring step's column pass (the values are meaningless).  Its
 * duration is what the memory system delivers to this access pattern, the yardstick the scoring kernels' times
 * are compared with (bench.py --yardstick).  bf16, head_dim 128 only (UNSUPPORTED otherwise); sink: 4 bytes of
 * device memory, practically never written. */
SABLOCK_API sablock_status sablock_stream_probe(const sablock_shape *shape, const void *k, int32_t read_lds,
                                    float *s_out /* nullable */, float *ent_out /* nullable */,
                                    void *sink, void *stream);

/* Segment-guided refinement (Alg. 1).  Per segment S_k of the compressible region:
 *   I_k = mean s_t (Eq. Ik), D_k = mean ent_t (Eq. Dk), omega_k = I_k (1 + eta D_k) (Eq. omegak);
 *   s_tilde_out[p][t] = s_t (1 + alpha omega_k(t)), t in [0, T)            (Eq. st_tilde)
 * s, ent: [P][L] float (as written by sablock_score).  s_tilde_out: [P][T] float.
 * omega_out: optional [P][max_segments] float.  Segment sums are accumulated in fp64. */
SABLOCK_API sablock_status sablock_refine(const sablock_shape *shape, const float *s, const float *ent,
                              const int32_t *seg_off, const int32_t *seg_ptr /* host */,
                              int32_t max_segments, const sablock_hparams *hp /* host */,
                              float *s_tilde_out, float *omega_out /* nullable */,
                              void *ws, size_t ws_bytes, void *stream);

/* Budget-driven block-size search (Alg. 2).  Per problem: T_topB = the min(budget, T)
 * best tokens of s_tilde (Eq. topk); per segment b_k = |T_topB & S_k| (Eq.
 * implicit_budget) and Score_base = sum of s_tilde over T_topB & S_k.  For each
 * candidate g <= min(|S_k|, b_k), largest first: blocks of g tokens from the
 * segment's first token (last block may be short), Phi = block sum, blocks taken
 * in rank order while they fit in b_k, the first that does not fit is cut to its
 * best (b_k - n) tokens; accepted iff Score_k(g) >= tau * Score_base (Eq. rk);
 * g_k* = first accepted (Eq. gk_star); g = 1 is accepted unconditionally.
 * cand: HOST array, ascending, cand[0] == 1, n_cand <= 16.  budget = the paper's B
 *   (entries chosen from the compressible region; may exceed T, may be 0).
 * seg_budget_out (b_k), block_size_out (g_k*, 0 where b_k == 0): [P][max_segments] int32.
 * topb_out: optional [P][2] int32, the Top-B set in closed form: (order-preserving key v of the
 *   min(budget,T)-th best score, index cut c); token t is in T_topB iff key(t) > v or (key(t) == v and
 *   t <= c), key(x) = bits(x) ^ (sign bit of x set ? 0xFFFFFFFF : 0x80000000), -0.0 taken as +0.0.  sablock_select accepts it back and then
 *   skips recomputing it.
 * Block sums, scores and the accept test are evaluated in fp64 on the fp32 inputs. */
SABLOCK_API sablock_status sablock_search_blocks(const sablock_shape *shape, const float *s_tilde,
                                     const int32_t *seg_off, const int32_t *seg_ptr /* host */,
                                     int32_t max_segments,
                                     const int32_t *cand /* host */, int32_t n_cand,
                                     int32_t budget, float tau,
                                     int32_t *seg_budget_out, int32_t *block_size_out,
                                     int32_t *topb_out /* nullable */,
                                     void *ws, size_t ws_bytes, void *stream);

/* Selection (Alg. 2, Eq. final_selection): T_k* = T_k(g_k*) per segment, T* their union.
 * seg_budget, block_size: as written by sablock_search_blocks for the same s_tilde.
 * topb: optional [P][2] int32 as written by sablock_search_blocks for the same s_tilde and budget
 *   (NULL: recomputed here).
 * idx_out: [P][budget] int32, token indices in ascending order, entries past n_sel = -1.
 * n_sel_out: [P] int32 (= min(budget, T)). */
SABLOCK_API sablock_status sablock_select(const sablock_shape *shape, const float *s_tilde,
                              const int32_t *seg_off, const int32_t *seg_ptr /* host */,
                              int32_t max_segments,
                              const int32_t *seg_budget, const int32_t *block_size,
                              const int32_t *topb /* nullable */, int32_t budget,
                              int32_t *idx_out, int32_t *n_sel_out,
                              void *ws, size_t ws_bytes, void *stream);

/* Search and selection in one call: the outputs of sablock_search_blocks and of sablock_select for the same
 * arguments, bit for bit (Alg. 2 as a whole).  When 0 < budget < T, budget <= 16384 and every sequence has fewer
 * than 16383 segments (and not both above 8192), the Top-B kernel also lays out the output rows and the search
 * writes the selected tokens itself, which saves the selection's own passes; otherwise the two sequences simply
 * run one after the other.
 * Workspace: sablock_workspace_bytes covers it. */
SABLOCK_API sablock_status sablock_search_select(const sablock_shape *shape, const float *s_tilde,
                                     const int32_t *seg_off, const int32_t *seg_ptr /* host */,
                                     int32_t max_segments,
                                     const int32_t *cand /* host */, int32_t n_cand,
                                     int32_t budget, float tau,
                                     int32_t *seg_budget_out, int32_t *block_size_out,
                                     int32_t *topb_out /* nullable */,
                                     int32_t *idx_out, int32_t *n_sel_out,
                                     void *ws, size_t ws_bytes, void *stream);

/* Cache construction (end of Sec. 3.3): per problem, rows idx[0..n_sel) of K and V copied
 * bit for bit, rows n_sel..budget-1 zero-filled, then, if append_window, the W most
 * recent rows T..L-1 in order.  k, v: shape->dtype, laid out by k_stride / v_stride.
 * k_out, v_out: dense [P][budget + (append_window ? W : 0)][D] of shape->dtype. */
SABLOCK_API sablock_status sablock_compact(const sablock_shape *shape, const void *k, const void *v,
                               const int32_t *idx, const int32_t *n_sel, int32_t budget,
                               int32_t append_window, void *k_out, void *v_out, void *stream);

/*
 * The head mean taken literally (Eq. barA averages over ALL H query heads of a layer): ONE score row, hence one
 * retained set, per (sequence, layer) instead of one per KV head.
 *   sablock_score_all_heads   as sablock_score, but Abar[i, t] is the mean over all n_q_heads heads of the layer;
 *       s_out / ent_out are [n_seq * n_layers][L].  row_lse as in sablock_score.  Supported: bf16, head_dim 128,
 *       W in {8, 16, 32} and any G with G * W <= 128; otherwise UNSUPPORTED.  With 8 KV
 *       heads, G = 4 and W = 32 the heads of a layer are summed on chip and the workspace
 *       (sablock_score_all_heads_workspace_bytes) holds row statistics only; for the other shapes it also holds
 *       the head-group means of every KV head, 4 * W bytes per key and KV head, before they are averaged.
 *   refine / search_blocks / select then run on the per-layer rows: pass them a shape whose n_q_heads and
 *       n_kv_heads are 1 (a problem is then a (sequence, layer)).
 *   sablock_compact_shared    as sablock_compact with the real head counts, but idx is [n_seq * n_layers][budget]
 *       and n_sel [n_seq * n_layers]: every KV head of a layer gathers the layer's rows.
 */
SABLOCK_API sablock_status sablock_score_all_heads_workspace_bytes(const sablock_shape *shape, size_t *bytes_out);
SABLOCK_API sablock_status sablock_score_all_heads(const sablock_shape *shape, const void *q_win, const void *k,
                                       const float *row_lse, float eps, float *s_out, float *ent_out,
                                       void *ws, size_t ws_bytes, void *stream);
SABLOCK_API sablock_status sablock_compact_shared(const sablock_shape *shape, const void *k, const void *v,
                                      const int32_t *idx, const int32_t *n_sel, int32_t budget,
                                      int32_t append_window, void *k_out, void *v_out, void *stream);

/*
 * The producer of row_lse (Sec. 2.1, Eq. 1): causal attention of the W window queries over all L keys, i.e. the
 * rows of the prefill attention that the scoring step looks at.  Query i (position T + i) attends to keys
 * t <= T + i.  A prefill that computes these rows here (or takes the same two outputs from its own attention
 * kernel) hands row_lse to sablock_score, which then reads K once.
 *   out          [n_seq][n_layers][n_q_heads][W][D] fp32: softmax(q . k / sqrt(D)) @ v
 *   row_lse_out  [P][G * W] fp32, natural log of the softmax denominators, in the layout sablock_score takes
 * Supported: bf16, head_dim 128, W in {8, 16, 32, 64} and any G with G * W <= 256; otherwise UNSUPPORTED.  Probabilities enter
 * the second product rounded to bf16 (the denominators are summed in fp32 before rounding).
 */
SABLOCK_API sablock_status sablock_window_attention_workspace_bytes(const sablock_shape *shape, size_t *bytes_out);
SABLOCK_API sablock_status sablock_window_attention(const sablock_shape *shape, const void *q_win, const void *k,
                                        const void *v, float *out, float *row_lse_out,
                                        void *ws, size_t ws_bytes, void *stream);

/*
 * Punctuation-based segmentation of the compressible region (Sec. 3.1), the step in front of the five calls:
 * delimiter tokens (commas, periods, ...) mark segment boundaries.  A delimiter closes the segment it belongs to:
 * a new segment starts after every token t < n_tokens - 1 whose id is in `delims`; consecutive delimiters give
 * one-token segments; a sequence without delimiters is one segment.  Two calls, because the offsets are CSR
 * with HOST pointers (see "Segments" above):
 *   1. sablock_segment_count writes the segment count K_s of every sequence to seg_count_out (device, n_seq
 *      int32); the caller reads it back and forms seg_ptr[s+1] = seg_ptr[s] + K_s + 1;
 *   2. sablock_segment_offsets writes, for every sequence, 0, the boundaries in ascending order, n_tokens to
 *      seg_off_out[seg_ptr[s] .. seg_ptr[s+1]) (device); entries beyond what seg_ptr leaves room for are dropped.
 * token_ids: device int32, sequence s at token_ids + s * token_stride (elements), n_tokens = T ids each (the
 * compressible region only).  delims: HOST array of n_delim <= 64 token ids (n_delim = 0: one segment each).
 * Errors: INVALID_ARG for NULL pointers, n_seq < 1, n_tokens < 1, token_stride < n_tokens, a seg_ptr that leaves
 * a sequence fewer than 2 or more than n_tokens + 1 offsets; UNSUPPORTED for n_seq > 64 or n_delim > 64.
 */
SABLOCK_API sablock_status sablock_segment_count(const int32_t *token_ids, int64_t token_stride, int32_t n_seq,
                                     int32_t n_tokens, const int32_t *delims, int32_t n_delim,
                                     int32_t *seg_count_out, void *stream);
SABLOCK_API sablock_status sablock_segment_offsets(const int32_t *token_ids, int64_t token_stride, int32_t n_seq,
                                       int32_t n_tokens, const int32_t *delims, int32_t n_delim,
                                       const int32_t *seg_ptr, int32_t *seg_off_out, void *stream);

/*
 * Check of a CSR segment array on the device (Sec. 3.1: the segments S_1 .. S_K partition the compressible
 * region, so every sequence's offsets must read 0 = off[0] < off[1] < ... < off[K] = n_tokens).  The five calls
 * do not look at the values in seg_off (they are device data) and index s, ent and s_tilde with them, so offsets
 * from an untrusted source are checked with this call first; it is no step of the path.
 *   seg_off (device), seg_ptr (host, n_seq + 1 entries): as in the other calls.  n_tokens = T.
 *   n_bad_out (device, n_seq int32): per sequence the number of offsets that break the rule (0 = valid).
 * Enqueues one kernel on `stream`; the caller reads n_bad_out back.  Errors: INVALID_ARG for NULL pointers,
 * n_seq < 1, n_tokens < 1, a seg_ptr that leaves a sequence fewer than 2 or more than n_tokens + 1 offsets;
 * UNSUPPORTED for n_seq > 64.
 */
SABLOCK_API sablock_status sablock_validate_segments(const int32_t *seg_off, const int32_t *seg_ptr, int32_t n_seq,
                                         int32_t n_tokens, int32_t *n_bad_out, void *stream);

/*
 * Decode-time attention of ONE new token over a KV cache (Sec. 2.1, Eq. 1 with a single query position): the
 * step after the path, over the compacted cache that sablock_compact wrote or over the full cache.  For every
 * problem p and each of its G query heads h:  out[h] = softmax_r(<q[h], K[p][r]> / sqrt(D)) . V[p][r].
 *   shape      n_seq, n_layers, heads, head_dim, dtype as in the other calls; seq_len = number of ROWS of the
 *              cache buffers; k_stride / v_stride describe them (elements; [3] = row stride); window and
 *              q_stride are ignored.  A compacted cache is dense: row stride D, head stride rows * D, ...
 *   q          [n_seq][n_layers][n_q_heads][D], dense, dtype of the cache.
 *   n_sel      NULL (every row holds an entry), or device [P]: rows n_sel[p] .. budget-1 of problem p hold no
 *              entry (the zero-filled gap sablock_compact leaves when fewer than `budget` tokens were retained)
 *              and are skipped; rows from `budget` on (the window rows) always count.
 *   out        [n_seq][n_layers][n_q_heads][D] fp32, dense.  A problem without any row gives zeros.
 *   ws         at least sablock_decode_workspace_bytes(shape) bytes (partial results of the row splits).
 * Supported: G <= 8; head_dim * element size / 16 a power of two in [4, 64]; G * head_dim <= 1024;
 * at least 2 rows.  Errors as for the other calls.
 */
SABLOCK_API sablock_status sablock_decode_workspace_bytes(const sablock_shape *shape, size_t *bytes_out);
SABLOCK_API sablock_status sablock_decode_attention(const sablock_shape *shape, const void *q, const void *k_cache,
                                        const void *v_cache, const int32_t *n_sel, int32_t budget, float *out,
                                        void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SABLOCK_H */
