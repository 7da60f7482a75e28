/*
 * spindle.h - C ABI of the MI355X (gfx950) prefill-time KV-cache reduction pass
 * of SpindleKV (arXiv 2507.06517).
 *
 * The operations, each working on `batch * n_kv_heads` independent problems
 * ("units") per call; fold layers into `batch` to process a stack in one call:
 *
 *   spindle_compress_deep     attention-weight token eviction
 *                             (Sec. "Attention Weight Based Token Eviction", Eq. 1-3, 7)
 *   spindle_compress_shallow  similarity codebook replacement
 *                             (Sec. "Similarity Based Token Replacement", Eq. 8-13, Alg. 1);
 *                             spindle_shallow_graph + spindle_shallow_codebook = its two halves
 *   spindle_reconstruct       codebook look-up and rescale (Eq. 14)
 *   spindle_decode_merge      tokens generated later join the stored codebook or extend it
 *                             (same section, the paragraph after Eq. 14)
 *   spindle_layer_budgets, spindle_reserve_ratio
 *                             host arithmetic: layer-wise budgets (Eq. 5-6), reserve ratio (Eq. 15)
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, contiguous in
 *     the stated shape, 16-byte aligned.  The library allocates no device memory;
 *     scratch space is the caller's `workspace` (size from the *_workspace_bytes
 *     query, 256-byte aligned).  No result depends on an earlier call: what the
 *     library keeps per process is the records of spindle_profile, a per-device note
 *     that a kernel's LDS limit has been raised, and the built-in scratch array of
 *     spindle_decode_merge_static.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue
 *     work on it and return without synchronising; all data-dependent counts stay
 *     on the device.
 *   - K, V, Qw and the vector outputs share `dtype`.  head_dim must be 128.
 *   - Inputs are assumed finite; NaN/Inf give undefined selections.
 *   - Return value: SPINDLE_OK or an error code; spindle_last_error() gives a
 *     thread-local message for the last failing call.  Nothing is enqueued when a
 *     call fails validation.
 *   - Two calls that share a workspace must be ordered on one stream.
 */
#ifndef SPINDLE_H
#define SPINDLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPINDLE_OK = 0,
  SPINDLE_ERR_INVALID_ARG = 1,  /* null pointer, bad shape, bad parameter            */
  SPINDLE_ERR_UNSUPPORTED = 2,  /* valid but outside what the kernels handle         */
  SPINDLE_ERR_WORKSPACE = 3,    /* workspace missing, misaligned or too small        */
  SPINDLE_ERR_HIP = 4           /* a HIP runtime call failed (message has the cause) */
} spindle_status;

typedef enum { SPINDLE_F32 = 0, SPINDLE_F16 = 1, SPINDLE_BF16 = 2 } spindle_dtype;

/* Divisor of the accumulated attention score, Eq. 2. */
typedef enum {
  SPINDLE_NORM_PAPER = 0, /* divide the window sum of key a by (l - a), as printed */
  SPINDLE_NORM_NONE = 1   /* plain window sum                                      */
} spindle_norm;

/*
 * Shape of the KV cache of one call: K, V are [batch, n_kv_heads, seq_len, head_dim].
 * stride_b, stride_h, stride_t give the distance, in elements, between consecutive batches,
 * heads and tokens of the INPUT tensors K and V (the head dimension is always contiguous), so
 * that a cache stored as [batch, seq_len, n_kv_heads, head_dim] needs no copy: stride_t =
 * n_kv_heads * head_dim, stride_h = head_dim.  All three zero = contiguous in the stated shape.
 * Each must be a multiple of 8 elements (16-byte rows) and stride_t >= head_dim.  Qw and every
 * output are always contiguous.  spindle_decode_merge takes contiguous new tokens (strides 0).
 */
typedef struct {
  int32_t batch;      /* B   >= 1                                                  */
  int32_t n_kv_heads; /* h_g >= 1                                                  */
  int32_t group_size; /* h_n = query heads per KV head (used by the deep path)     */
  int32_t seq_len;    /* l   >= 1                                                  */
  int32_t head_dim;   /* d_h, must be 128                                          */
  int32_t dtype;      /* spindle_dtype                                             */
  int64_t stride_b;   /* elements between batches of K and V, 0 = contiguous       */
  int64_t stride_h;   /* elements between heads,   0 = contiguous                  */
  int64_t stride_t;   /* elements between tokens,  0 = contiguous                  */
} spindle_kv_desc;

/* ------------------------------------------------------------------------- */
/* Deep layers: attention-weight eviction                                     */
/* ------------------------------------------------------------------------- */

/*
 * Bytes of workspace spindle_compress_deep needs for this shape and window.
 */
spindle_status spindle_deep_workspace_bytes(const spindle_kv_desc *desc, int32_t window,
                                            size_t *bytes);

/*
 * For every unit (b, i):
 *   1. logits of the `window` last queries of the h_n query heads of KV head i
 *      against all keys, causal mask, softmax over the visible keys (Eq. 1);
 *   2. per context key a < l_c = seq_len - window: sum over the window queries,
 *      divided by (l - a) under SPINDLE_NORM_PAPER (Eq. 2), mean over the h_n
 *      heads of the group (Eq. 3);
 *   3. 1-D max pooling over context positions, odd kernel `pool_kernel`, stride 1,
 *      same length, neighbours outside the context ignored (1 = no pooling);
 *   4. the k = budget - window largest pooled scores, equal scores lowest position
 *      first (Eq. 7); kept positions in ascending order followed by the whole
 *      window l_c .. l-1 (the observation window is always kept);
 *   5. K_out = K[kept], V_out = V[kept].
 *
 *   Qw          [B, h_g*h_n, window, d]; query head h serves KV head h / h_n, row w is
 *               the query at position l - window + w.  window*h_n <= 256.
 *   scale       logit scale, normally 1/sqrt(d).
 *   budget      total kept tokens per unit, window included; window <= budget.
 *               budget >= seq_len keeps everything.
 *   budgets     optional device int32 [B*h_g] per-unit budgets overriding `budget`
 *               (each window <= budgets[u]); NULL = uniform.
 *   out_stride  row pitch of the outputs in tokens, >= the largest budget in use
 *               (clamped to seq_len).
 *   kept_idx    [B, h_g, out_stride] int32; entries past a unit's budget are -1.
 *   K_out,V_out [B, h_g, out_stride, d]; rows past a unit's budget are zero.
 *               V and V_out may both be NULL (keys only).
 *   scores_out  optional [B, h_g, l_c] float32 pooled scores (step 3), else NULL.
 */
spindle_status spindle_compress_deep(const spindle_kv_desc *desc, const void *K, const void *V,
                                     const void *Qw, int32_t window, int32_t pool_kernel,
                                     float scale, int32_t norm, int32_t budget,
                                     const int32_t *budgets, int32_t out_stride,
                                     int32_t *kept_idx, void *K_out, void *V_out,
                                     float *scores_out, void *workspace, size_t workspace_bytes,
                                     void *stream);

/* ------------------------------------------------------------------------- */
/* Shallow layers: similarity codebook                                        */
/* ------------------------------------------------------------------------- */

/*
 * Bytes of workspace spindle_compress_shallow needs when `n_tensors` (1 or 2) of
 * K, V are processed in one call.  Dominated by the bit-packed adjacency matrix:
 * seq_len^2 / 8 bytes per unit and tensor.
 */
spindle_status spindle_shallow_workspace_bytes(const spindle_kv_desc *desc, int32_t n_tensors,
                                               size_t *bytes);

/*
 * Alg. 1 for every unit, independently for K (threshold theta_k) and V (theta_v):
 *   m_a = |x_a| (Eq. 8); S_ab = x_a.x_b / (m_a m_b) (Eq. 4; 0 if either norm is 0);
 *   G_ab = [S_ab > theta], G_aa = 1 (Eq. 9); then repeatedly pick the token of highest
 *   degree among the remaining ones (lowest index on ties), append its unit vector to
 *   the codebook, point every remaining neighbour (itself included) to that entry and
 *   remove them (Eq. 10-13), until no token remains.
 * The adjacency decision S_ab > theta is taken exactly as a double-precision
 * evaluation (dimension-order summation) would take it.
 * Codebook cap: only the first `max_codes` entries in pick order are stored; a token
 * whose entry was cut is pointed to the stored entry of highest cosine similarity
 * (lowest entry index on ties).  max_codes >= seq_len never cuts.
 *
 *   K, V        either may be NULL (with all of its outputs) to process one tensor.
 *   Ck, Cv      [B, h_g, max_codes, d] unit vectors in `dtype`; rows >= n_codes are zero.
 *   n_codes_*   [B, h_g] int32 stored entries = min(found, max_codes).  -1 marks a problem whose
 *               construction did not finish; its other outputs are then undefined.  Every
 *               round takes at least the remaining token of the largest key, so this cannot
 *               happen unless the workspace was overwritten while the call ran (a second
 *               call on another stream with the same workspace, or between the two halves).
 *   n_found_*   optional [B, h_g] int32 entries found before the cap, else NULL.
 *   ref_*       [B, h_g, l] int32 code index of each token, in [0, n_codes).
 *   mag_*       [B, h_g, l] float32 magnitudes m_a.
 *   adj_*       optional [B, h_g, l, ceil(l/32)] uint32 adjacency bits (bit b of row a at
 *               word b/32, position b%32), else NULL.
 *   deg_*       optional [B, h_g, l] int32 degrees (row sums of G), else NULL.
 * seq_len <= 65535.
 */
spindle_status spindle_compress_shallow(const spindle_kv_desc *desc, const void *K, const void *V,
                                        float theta_k, float theta_v, int32_t max_codes,
                                        void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v,
                                        int32_t *n_found_k, int32_t *n_found_v,
                                        int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v,
                                        uint32_t *adj_k, uint32_t *adj_v,
                                        int32_t *deg_k, int32_t *deg_v,
                                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * spindle_compress_shallow in two halves, for a caller that overlaps other work with the
 * second one (e.g. the eviction call of another layer on a second stream that waits for an
 * event recorded between the two):
 *   spindle_shallow_graph     magnitudes, similarities, G, degrees and neighbour lists
 *                             (Eq. 4, 8-10): the phase that fills the chip.  Writes mag_*,
 *                             adj_* and deg_* if given, clears C* and sets n_codes_* to -1;
 *                             everything else goes to the workspace
 *   spindle_shallow_codebook  the loop of Alg. 1 (Eq. 11-13), the cap and the outputs C*,
 *                             n_codes_*, n_found_*, ref_*: mostly one workgroup per unit,
 *                             most of the chip is idle meanwhile
 * Both take exactly the arguments of spindle_compress_shallow, validated the same way, and
 * must be given the same values and the same workspace, untouched in between; calling the
 * first and then the second on one stream is the same as the single call.
 */
spindle_status spindle_shallow_graph(const spindle_kv_desc *desc, const void *K, const void *V,
                                     float theta_k, float theta_v, int32_t max_codes,
                                     void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v,
                                     int32_t *n_found_k, int32_t *n_found_v,
                                     int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v,
                                     uint32_t *adj_k, uint32_t *adj_v,
                                     int32_t *deg_k, int32_t *deg_v,
                                     void *workspace, size_t workspace_bytes, void *stream);
spindle_status spindle_shallow_codebook(const spindle_kv_desc *desc, const void *K, const void *V,
                                        float theta_k, float theta_v, int32_t max_codes,
                                        void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v,
                                        int32_t *n_found_k, int32_t *n_found_v,
                                        int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v,
                                        uint32_t *adj_k, uint32_t *adj_v,
                                        int32_t *deg_k, int32_t *deg_v,
                                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * One codebook per layer instead of one per KV head (Sec. "Similarity Based Token Replacement",
 * first paragraph: the copies that repeating K and V for every query head creates have cosine 1
 * and must cost no storage; Eq. 15, whose r_2 counts the entries of a layer, |C_K u C_V|, with
 * no sum over heads).  The rows of all n_kv_heads heads of a batch entry, head after head, are
 * ONE problem of n_kv_heads * seq_len tokens run through Alg. 1 exactly as
 * spindle_compress_shallow runs a head: same thresholds, decisions, tie rules and cap.
 * With K and V repeated per query head (n_kv_heads = the number of query heads,
 * spindle_compress_deep called with group_size 1 on the repeated tensors) the inputs are that
 * call's K_out and V_out as they are, with seq_len = its out_stride, when every unit keeps
 * out_stride rows.
 *   K, V        [B, n_kv_heads, seq_len, d]; the heads of a batch entry must follow each other
 *               in memory (stride_h = seq_len * stride_t, or all strides 0).
 *   Ck, Cv      [B, max_codes, d];  n_codes_*, n_found_* [B]
 *   ref_*       [B, n_kv_heads, seq_len] int32: entry of the layer's codebook, in [0, n_codes)
 *   mag_*       [B, n_kv_heads, seq_len] float32
 * Errors as spindle_compress_shallow; SPINDLE_ERR_UNSUPPORTED if n_kv_heads * seq_len > 65535
 * (evict to fewer rows per head first) or the heads are not adjacent in memory.  The workspace
 * size comes from spindle_shallow_layer_workspace_bytes.
 */
spindle_status spindle_shallow_layer_workspace_bytes(const spindle_kv_desc *desc, int32_t n_tensors,
                                                     size_t *bytes);
spindle_status spindle_compress_shallow_layer(const spindle_kv_desc *desc, const void *K, const void *V,
                                              float theta_k, float theta_v, int32_t max_codes,
                                              void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v,
                                              int32_t *n_found_k, int32_t *n_found_v,
                                              int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v,
                                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Diagnostics of the last spindle_compress_shallow call that used `workspace` with this
 * shape: for each of the batch * n_kv_heads * n_tensors problems i (all K units first,
 * then all V units), with s = stats + 16*i: s[0] = rounds of the parallel codebook
 * construction, s[1] = codebook entries found, s[2] = token pairs whose adjacency was
 * decided in double precision, s[4..13] = microseconds the workgroup that runs the later
 * rounds of the problem spent in their phases (s[4] loading keys and compacting the list of
 * remaining tokens, s[6] one-hop maxima, s[8] two-hop maxima and picks, s[10] degree updates,
 * s[12], s[13] bookkeeping; the odd slots in between are unused), others 0.  `stats` is a HOST
 * buffer of 16 * batch * n_kv_heads * n_tensors int32.  Waits for `stream`.
 */
spindle_status spindle_shallow_stats(const spindle_kv_desc *desc, int32_t n_tensors,
                                     const void *workspace, void *stream, int32_t *stats);

/*
 * Eq. 14: out[u, a, :] = C[u, ref[u, a], :] * mag[u, a] for all units u and tokens a.
 *   C [units, max_codes, d] and out [units, l, d] in `dtype`; ref [units, l] int32;
 *   mag [units, l] float32.  No workspace.
 */
spindle_status spindle_reconstruct(int32_t units, int32_t seq_len, int32_t head_dim, int32_t dtype,
                                   int32_t max_codes, const void *C, const int32_t *ref,
                                   const float *mag, void *out, void *stream);

/* ------------------------------------------------------------------------- */
/* Decode-time merge                                                           */
/* ------------------------------------------------------------------------- */

/*
 * Workspace of spindle_decode_merge for desc (seq_len = new tokens per problem, at most 1024;
 * group_size is ignored) and a codebook table of max_codes rows.  Errors: INVALID_ARG for a
 * bad desc or max_codes < 1; UNSUPPORTED beyond 1024 new tokens.
 */
spindle_status spindle_decode_workspace_bytes(const spindle_kv_desc *desc, int32_t max_codes, size_t *bytes);

/*
 * Sec. "Similarity Based Token Replacement", the paragraph after Eq. 14: new tokens of one
 * tensor (K or V) are merged into the codebooks an earlier spindle_compress_shallow or
 * spindle_decode_merge call left.  Per problem u = (batch, kv-head), with m = desc->seq_len:
 *   1. every new token a takes the stored entry c < n_codes[u] of highest cosine (Eq. 4,
 *      between the raw token and the stored row, the row's own norm in the denominator),
 *      lowest c on ties, provided that cosine exceeds theta (strictly, as Eq. 9);
 *   2. the tokens that found none run through Alg. 1 among themselves (Eq. 9-13, their input
 *      order deciding ties); pick j becomes entry n_codes[u] + j: its unit vector is
 *      written to row n_codes[u] + j of C and its tokens refer to it.
 * Decisions are taken in double precision exactly as spindle_compress_shallow takes them.
 * Entries that do not fit into max_codes rows are not stored and their tokens get ref = -1;
 * n_found tells (n_found[u] > max_codes: rebuild or enlarge the codebook).
 *   X_new     [batch, n_kv_heads, m, d] in desc->dtype (device)
 *   C         [batch, n_kv_heads, max_codes, d] in desc->dtype (device), read and appended to
 *   n_codes   [batch, n_kv_heads] int32 (device): in = stored entries, out = stored entries afterwards
 *   n_found   [batch, n_kv_heads] int32 (device): entries needed in total
 *   n_matched [batch, n_kv_heads] int32 (device), optional: tokens merged in step 1
 *   ref       [batch, n_kv_heads, m] int32 (device): entry of each new token
 *   mag       [batch, n_kv_heads, m] float32 (device): Eq. 8
 * Only enqueues on `stream`; allocates nothing.  Errors: INVALID_ARG (null or misaligned
 * pointers, theta outside (-1, 1), max_codes < 1), UNSUPPORTED (head_dim != 128, m > 1024),
 * WORKSPACE, HIP.
 */
spindle_status spindle_decode_merge(const spindle_kv_desc *desc, const void *X_new, float theta,
                                    int32_t max_codes, void *C, int32_t *n_codes, int32_t *n_found,
                                    int32_t *n_matched, int32_t *ref, float *mag, void *workspace,
                                    size_t workspace_bytes, void *stream);

/*
 * spindle_decode_merge for callers that cannot allocate device memory or carry a workspace
 * around: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments, results and errors as spindle_decode_merge, without `workspace`:
 * the scratch memory (the new tokens as doubles, their magnitudes, one partial result per 512
 * stored entries) is an array of spindle_decode_static_capacity() bytes (6 MiB) inside the
 * library's code object, which every GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing on host or device and only enqueues on `stream`, which
 * must belong to the current device.  (With per-kernel timing switched on, spindle_profile
 * creates HIP events; leave it off for such callers.)
 *   - A call whose spindle_decode_workspace_bytes exceeds the capacity is refused with
 *     SPINDLE_ERR_UNSUPPORTED and a message that names both sizes; nothing is enqueued.
 *     Roughly: batch * n_kv_heads * (new tokens rounded up to 16) <= 5000 at max_codes <= 8192,
 *     e.g. 32 problems x 128 tokens.
 *   - All calls on one GPU share the array: calls that may overlap on one GPU (two streams, two
 *     threads) race; order them on one stream or with events.  Nothing in it needs clearing:
 *     every element a kernel reads was written earlier in the same call.
 */
spindle_status spindle_decode_merge_static(const spindle_kv_desc *desc, const void *X_new, float theta,
                                           int32_t max_codes, void *C, int32_t *n_codes, int32_t *n_found,
                                           int32_t *n_matched, int32_t *ref, float *mag, void *stream);

/* Bytes of the built-in scratch array of spindle_decode_merge_static. */
size_t spindle_decode_static_capacity(void);

/* ------------------------------------------------------------------------- */
/* Host helpers (plain arithmetic on the host, no GPU work)                    */
/* ------------------------------------------------------------------------- */

/*
 * Sec. "Attention Weight Based Token Eviction", Eq. 5-6 and the unnumbered equation before
 * them: layer-wise budgets.  With l_c = seq_len - window and r_c = (reserve_ratio * seq_len -
 * window) / l_c (clamped to [0, 1]), alpha = (1 + beta) / 2:
 *   r_c <= beta          every layer gets r_c,
 *   beta < r_c <= alpha  layer 0 gets 2 r_c - beta, the last layer beta,
 *   alpha < r_c          layer 0 gets 1, the last layer 2 r_c - 1
 * (the printed "0.05" is beta and the printed "1 - 2 r_c" is read as 2 r_c - 1, which keeps the
 * mean at r_c and is continuous at alpha); layers in between are interpolated linearly (Eq. 6).
 *   budgets  HOST buffer of n_layers int32: window + floor(r_c(layer) * l_c), Eq. 7's k plus the
 *            window: the `budget` argument of spindle_compress_deep (it counts the window).
 *            Eq. 6 is evaluated in doubles in the printed order of operations.
 *   ratios   optional HOST buffer of n_layers doubles: r_c(layer).
 * Errors: INVALID_ARG for n_layers < 1, window < 1, window > seq_len, beta outside [0, 1],
 * reserve_ratio outside [0, 1] or a null `budgets`.
 */
spindle_status spindle_layer_budgets(double reserve_ratio, int32_t seq_len, int32_t window,
                                     int32_t n_layers, double beta, int32_t *budgets, double *ratios);

/*
 * Sec. "Experiments", Eq. 15: reserve ratio of one layer, r = r1 * r2 * r3 with
 *   r1 = kept_tokens / total_tokens           (eviction; token counts summed over heads, K and V)
 *   r2 = codebook_entries / kept_tokens       (replacement; entries of the K and V codebooks)
 *   r3 = (head_dim + index_bits / elem_bits + magnitude_bits / elem_bits) / head_dim
 *        (one index and one magnitude per token, in units of cache elements.  The printed
 *        fraction is garbled; it is read as (d_h + int_bit / key_bit + 1) / d_h, whose "+ 1" is a
 *        magnitude as wide as a cache element: magnitude_bits = elem_bits gives exactly that.
 *        The magnitudes spindle_compress_shallow writes are float32: magnitude_bits = 32.)
 * `out` is a HOST buffer of 4 doubles: r1, r2, r3, r.  Errors: INVALID_ARG for counts or widths
 * < 1, kept_tokens > total_tokens, codebook_entries > kept_tokens or a null `out`.
 */
spindle_status spindle_reserve_ratio(int64_t kept_tokens, int64_t total_tokens, int64_t codebook_entries,
                                     int32_t head_dim, int32_t index_bits, int32_t elem_bits,
                                     int32_t magnitude_bits, double *out);

/* ------------------------------------------------------------------------- */
/* Per-kernel timing (measurement aid for the roofline figures)                */
/* ------------------------------------------------------------------------- */

/*
 * enable = 1: every kernel the library launches from now on is bracketed by a pair of HIP
 * events recorded on the stream it is launched on; enable = 2: only the similarity kernel of
 * spindle_compress_shallow ("shallow_gram") is; enable = 0 stops recording.  An event between
 * two kernels of a stream costs about 10 us of idle time on the GPU, so mode 1 lengthens a
 * step by some 5 % and is meant for breakdowns, mode 2 (two events per call) for measuring the
 * dominant kernel inside a timed run.  Every call discards the records collected so far.
 * Process-wide; not meant to be switched while another thread is inside a compress call.
 */
spindle_status spindle_profile(int32_t enable);

/*
 * Waits for the recorded events, writes up to `max` records in launch order
 * (names[i*32 .. i*32+31] = NUL-terminated kernel name, ms[i] = elapsed milliseconds),
 * clears the records and returns how many were written (negative on a HIP error).
 * `names` and `ms` are HOST buffers.
 */
int32_t spindle_profile_read(char *names, float *ms, int32_t max);

/*
 * What this GPU sustains, for reading the roofline figures (neither computes anything the method
 * needs; both enqueue on `stream`, wait for it and time with a pair of HIP events):
 *   spindle_calibrate_mfma        four independent chains of `iters` v_mfma_f32_32x32x16_f16 per
 *                                 wave, eight waves per compute unit, operands in registers: the
 *                                 rate of the matrix cores with no memory traffic and no other
 *                                 work, in TFLOP/s.  `pattern` 0: small non-negative operand
 *                                 values (few bits switch between instructions); 1: pseudo-random
 *                                 values with the signs and magnitudes of the similarity kernel's
 *                                 operands, which draw more power per instruction and so show the
 *                                 clock the part sustains on such data.
 *   spindle_calibrate_similarity  the similarity kernel of spindle_compress_shallow run again on
 *                                 the unit vectors an earlier call with the same desc and n_tensors
 *                                 left in `workspace`, with the same staging, barriers and matrix
 *                                 instructions but without the packing of the results, and
 *                                 nothing written: its duration in milliseconds.  `mode` 0: as
 *                                 just said; 1: also without the loads that stream a chunk's
 *                                 tokens into LDS after its first two stages (the matrix
 *                                 instructions keep reading the same staged tokens); 2: matrix
 *                                 instructions only, both operands from registers.  The three
 *                                 show what the vector work, the streaming and the fragment
 *                                 reads each cost beside the matrix instructions.
 */
spindle_status spindle_calibrate_mfma(int32_t iters, int32_t pattern, void *stream, double *tflops);
/*   spindle_calibrate_copy        a plain copy of `bytes` from src to dst (device buffers, 16-byte
 *                                 aligned), run twice and the second timed: bytes read plus bytes
 *                                 written per second, in GB/s; its known size is also what the HBM
 *                                 traffic counters of a profiler run are scaled by. */
spindle_status spindle_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream, double *gbs);
spindle_status spindle_calibrate_similarity(const spindle_kv_desc *desc, int32_t n_tensors, void *workspace,
                                            size_t workspace_bytes, int32_t mode, void *stream, double *ms);

/* ------------------------------------------------------------------------- */

/* Thread-local message of the last failing call on this thread ("" if none). */
const char *spindle_last_error(void);

/* Library version, major << 16 | minor. */
uint32_t spindle_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPINDLE_H */
