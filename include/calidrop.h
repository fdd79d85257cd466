/*
 * calidrop.h - C ABI of the MI355X (gfx950) CaliDrop hot path.
 *
 * Two operations, both defined by the CaliDrop paper (arXiv 2507.19906):
 *
 *   calidrop_compress  - prefill side, Alg. 1 steps 3-8: apply a SnapKV-style eviction
 *                        strategy f (Sec. 4.1.3: observation window, average pooling) per KV
 *                        head, gather KV_compress, and precompute the calibration state
 *                        (C_q, C_out, log C_weight) of the last prompt query over KV_evict.
 *   calidrop_decode    - decode side, Alg. 2: attention of the current query over
 *                        KV_compress, cosine gate against C_q, and the Eq. 1-2 merge with the
 *                        calibration state.
 *   calidrop_recalibrate - the recomputation branch of Alg. 2 (steps 3-8) for the heads that
 *                        calidrop_decode flagged: refresh the calibration state from KV_evict
 *                        with the current query and calibrate the step's output.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller (for example a torch
 *     tensor's data_ptr(); the one exception is stated at calidrop_recalibrate_packed); they
 *     must stay alive until `stream` has executed the enqueued work.  `p` and the returned strings are HOST memory.  The library keeps no pointer
 *     after a call returns and has no process-wide switches: its only state is a thread-local
 *     error string.
 *   - Calls validate their arguments on the host first (no HIP call is made before
 *     validation passes), then enqueue kernels on `stream` (a hipStream_t; NULL = default
 *     stream) and return without synchronising.  They never allocate or free device memory.
 *   - Return value: CALIDROP_OK (0) or a negative calidrop_status.  On error nothing was
 *     enqueued, except for CALIDROP_EHIP (a launch failed; earlier kernels of the same call
 *     may already be queued).  calidrop_last_error() describes the last failure on this
 *     thread.
 *   - Base pointers must be 16-byte aligned (CALIDROP_EALIGN otherwise).
 *   - head_dim must be 64 or 128, n_q_heads / n_kv_heads an integer G with 1 <= G <= 16,
 *     budget <= 2^24 (CALIDROP_EUNSUPPORTED otherwise).
 *   - Accumulation is always fp32; `dtype` is the storage type of Q/K/V, the compressed cache
 *     and the decode output.  The calibration state is always fp32.
 *   - Logits are scaled by 1/sqrt(head_dim) (Eq. 2) unless `scale` is non-zero.
 */
#ifndef CALIDROP_H
#define CALIDROP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CALIDROP_OK = 0,
  CALIDROP_EINVAL = -1,       /* null pointer, bad struct_size, bad parameter value        */
  CALIDROP_ESHAPE = -2,       /* sizes inconsistent with each other                        */
  CALIDROP_EALIGN = -3,       /* a base pointer is not 16-byte aligned                     */
  CALIDROP_EWORKSPACE = -4,   /* workspace missing or smaller than *_workspace_bytes()     */
  CALIDROP_EUNSUPPORTED = -5, /* head_dim / group size / dtype outside the supported set   */
  CALIDROP_EHIP = -6          /* a kernel launch reported an error                         */
} calidrop_status;

typedef enum { CALIDROP_BF16 = 0, CALIDROP_FP32 = 1 } calidrop_dtype;

/* Flags written by calidrop_decode, one per (sequence, query head): the branch of Alg. 2. */
enum {
  CALIDROP_FLAG_NONE = 0,       /* theta1 <= rho <= theta2: plain compressed attention     */
  CALIDROP_FLAG_CALIBRATED = 1, /* rho > theta2: output merged with C_out by Eq. 1         */
  CALIDROP_FLAG_RECOMPUTE = 2,  /* rho < theta1: the calibration state is stale; the output is
                                   the plain compressed attention until calidrop_recalibrate
                                   has processed the head                                  */
  CALIDROP_FLAG_RECOMPUTED = 3  /* set by calidrop_recalibrate: state recomputed with the
                                   current query and the output calibrated with it         */
};

typedef struct {
  uint32_t struct_size; /* = sizeof(calidrop_params); also accepted: 52, the layout without
                           flags, and 48, the layout without calib_size and flags (the missing
                           fields are then 0)                                                 */
  int32_t dtype;        /* calidrop_dtype                                                   */
  int32_t batch;        /* sequences; a stack of layers is passed as batch = layers * seqs   */
  int32_t n_q_heads;    /* Hq                                                               */
  int32_t n_kv_heads;   /* Hkv; G = Hq / Hkv query heads share one KV head                  */
  int32_t head_dim;     /* D                                                                */
  int32_t window;       /* w >= 1: observation window = the last w prompt positions          */
  int32_t budget;       /* B > w: retained tokens per KV head, window included               */
  int32_t pool_kernel;  /* k odd >= 1: average-pooling width (1 = no pooling)                */
  float scale;          /* logit scale; 0 selects 1/sqrt(D)                                  */
  float theta1, theta2; /* Alg. 2 thresholds, theta1 <= theta2, compared strictly in fp32;
                           (-inf, -inf) calibrates whenever a calibration state exists       */
  int32_t calib_size;   /* m >= 0, the "calibration size" of Sec. 5.3: only the m evicted tokens
                           of highest pooled score (ties to the lower position) form the
                           calibration / offload set, the others are dropped; 0 = every evicted
                           token                                                              */
  uint32_t flags;       /* per-call options, an OR of CALIDROP_OPT_* (0 = none)               */
} calidrop_params;

/* Per-call options in calidrop_params.flags.  They change how a compress call works, never what
 * it returns.
 *   CALIDROP_OPT_WRITE_SCORES    also store the pooled scores in the SCORE workspace region for every
 *                                sequence (otherwise that region is only written for prompts too long
 *                                for the in-LDS selection); costs one extra pass of stores.  For
 *                                inspection by tests and tools.
 *   CALIDROP_OPT_WIDE_SELECTION  run the per-head top-k as the multi-workgroup chain of launches for
 *                                every call (normally only prompts longer than 32768, or pooling widths
 *                                above 15, take it).  Same results (integer selection); for tests and
 *                                tuning.                                                             */
enum { CALIDROP_OPT_WRITE_SCORES = 1u, CALIDROP_OPT_WIDE_SELECTION = 2u };

/* Bytes of device workspace calidrop_compress needs for these shapes (0 on invalid params).
 * total_tokens = sum of prompt lengths, max_seq_len = longest prompt.                       */
size_t calidrop_compress_workspace_bytes(const calidrop_params* p, int64_t total_tokens,
                                         int32_t max_seq_len);

/* Bytes of device workspace calidrop_decode needs (0 on invalid params).                     */
size_t calidrop_decode_workspace_bytes(const calidrop_params* p, int32_t max_cache_len);

/* Named regions inside the compress workspace, for inspection by tests and tools after the
 * stream has finished (SCORE needs CALIDROP_OPT_WRITE_SCORES in the compress call's params).
 * Layouts:
 *   ROW_LSE   float [batch][Hkv][S]: per window-query row, log2 of its softmax denominator over
 *             all visible keys (logits in log2 units); rows of a KV head are ordered (query head in
 *             group, window position) and padded with +inf to the stride S = bytes / (batch*Hkv*4)
 *             (G*w rounded up to a multiple of 128, or of 256 when G*w > 128).
 *   SCORE     float, packed like K with D = 1: pooled score of prefix position j of KV head g
 *             of sequence b at [seq_offsets[b]*Hkv + g*n_b + j], j < n_b - w.
 * Returns CALIDROP_OK and fills offset/bytes, or CALIDROP_EINVAL.                            */
typedef enum { CALIDROP_REGION_ROW_LSE = 0, CALIDROP_REGION_SCORE = 1, CALIDROP_REGION_VOTE_PLANES = 2 } calidrop_region;
int calidrop_compress_workspace_region(const calidrop_params* p, int64_t total_tokens,
                                       int32_t max_seq_len, int32_t region, size_t* offset,
                                       size_t* bytes);

/*
 * calidrop_compress - Alg. 1 steps 3-8 for `batch` independent sequences (one layer each).
 *
 * For every sequence b with prompt length n_b = seq_offsets[b+1] - seq_offsets[b] and every
 * KV head g:
 *   n_b <= B : every position is retained, nothing is evicted, c_lse = -inf, c_out = 0.
 *   n_b >  B : (P = n_b - w)
 *     1. S = scale * Q_win K^T for the G*w window-query rows of the group; window query i sits
 *        at position P+i and sees columns 0..P+i; row softmax over the visible columns.
 *     2. vote[j] = sum over those rows of the probability on prefix column j < P.
 *     3. score = average pool of vote (stride 1, zero padding floor(k/2), divisor k).
 *     4. retained = the B-w prefix positions of largest score (ties to the lower position),
 *        in ascending order, followed by the window positions P..n_b-1.
 *     5. K_c, V_c = the retained rows of K, V (KV_compress); every other prefix row is
 *        KV_evict and stays where it is, in the caller's k / v.
 *     6. for each query head h of the group, with q = q_cal[h] (default Q_{-1}, the last
 *        window query): c_lse[h] = log sum_{t in evict} exp(scale q.K_t) (= log C_weight),
 *        c_out[h] = Att(q, K_evict, V_evict), c_q[h] = q.  With calib_size = m > 0 "evict"
 *        here means the calibration set: the m evicted positions of highest score.
 *
 * Arguments
 *   q_win         [batch][Hq][w][D] dtype: the last w prompt queries (as used by attention).
 *   k, v          packed prompts, dtype: sequence b starts at token seq_offsets[b]; inside a
 *                 sequence the layout is [Hkv][n_b][D].
 *   seq_offsets   [batch+1] int32, ascending, seq_offsets[0] = 0.
 *   total_tokens  = seq_offsets[batch]; max_seq_len >= every n_b (host copies; they size the
 *                 launch grids - a sequence longer than max_seq_len is truncated in scoring).
 *   q_cal         [batch][Hq][D] dtype calibration query, or NULL for Q_{-1}.
 *   k_c, v_c      out, dtype: sequence b at token cache_offsets[b] of capacity
 *                 cap_b = cache_offsets[b+1]-cache_offsets[b] >= min(B, n_b); inside:
 *                 [Hkv][cap_b][D]; the first min(B, n_b) rows of each head are written.
 *   cache_offsets [batch+1] int32.
 *   cache_lens    out [batch] int32 = min(B, n_b).
 *   indices       out [batch][Hkv][B] int32: retained prompt positions, ascending; -1 padded
 *                 when n_b < B.
 *   cal_indices   out [batch][Hkv][calib_size] int32: positions of the calibration set, ascending,
 *                 -1 padded (fewer than calib_size evicted tokens, or n_b <= B).  These are the
 *                 rows a caller would offload.  Required when calib_size > 0, ignored (may be
 *                 NULL) when calib_size = 0.
 *   c_q, c_out    out [batch][Hq][D] fp32.   c_lse  out [batch][Hq] fp32.
 *   workspace     >= calidrop_compress_workspace_bytes(p, total_tokens, max_seq_len) bytes,
 *                 256-byte aligned; contents need no initialisation.
 */
int calidrop_compress(const calidrop_params* p, const void* q_win, const void* k, const void* v,
                      const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len,
                      const void* q_cal, void* k_c, void* v_c, const int32_t* cache_offsets,
                      int32_t* cache_lens, int32_t* indices, int32_t* cal_indices, float* c_q,
                      float* c_out, float* c_lse, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * calidrop_compress_with_lse - calidrop_compress with step 1's normalisers supplied by the caller.
 *
 * The softmax of step 1 needs, for every window query i of every query head, the log-sum-exp of
 * its logits over the keys it may attend to (positions 0..P+i).  The prefill attention that
 * produced the prompt's outputs (Alg. 1 steps 1-2, outside this library) has that number for
 * every query row as the by-product of its own softmax; passing it in saves the pass over K that
 * calidrop_compress spends on it (K is then read once, for the votes, instead of twice).
 *
 *   win_lse   [batch][Hq][w] fp32, natural-log units: log sum_{j <= P+i} exp(scale q_win[h][i].K[g][j])
 *             with the same scale as params.scale.  NULL = compute it (exactly calidrop_compress).
 *             The values are used as given: votes are exp(logit - win_lse), so an lse that is off
 *             by delta scales that row's votes by exp(-delta) and nothing else.
 *
 * Every other argument, the outputs, the workspace and the errors are those of calidrop_compress.
 */
int calidrop_compress_with_lse(const calidrop_params* p, const void* q_win, const void* k,
                               const void* v, const int32_t* seq_offsets, int64_t total_tokens,
                               int32_t max_seq_len, const float* win_lse, const void* q_cal,
                               void* k_c, void* v_c, const int32_t* cache_offsets,
                               int32_t* cache_lens, int32_t* indices, int32_t* cal_indices,
                               float* c_q, float* c_out, float* c_lse, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * calidrop_decode - Alg. 2 for one decode step of `batch` sequences.
 *
 * Per sequence b and query head h (KV head g = h / G):
 *   1. z_r = scale * q_t[h].K_c[g][r] over the cache_lens[b] live rows; a_lse = logsumexp(z)
 *      (= log A_weight); o_a = sum softmax(z)_r V_c[g][r]                (Alg. 2 step 1)
 *   2. rho = cos(q_t[h], c_q[h]), taken as 0 when either norm is 0, in fp32   (step 2)
 *   3. rho < theta1: flag RECOMPUTE, out = o_a.
 *      rho > theta2 and c_lse[h] > -inf: alpha_j = 1/(1+exp(a_lse - c_lse[h])),
 *          out = (1-alpha_j) o_a + alpha_j c_out[h]  (Eq. 1-2), flag CALIBRATED.
 *      otherwise out = o_a, flag NONE.
 *
 * Arguments: q_t [batch][Hq][D] dtype; k_c, v_c, cache_offsets, cache_lens as produced by
 * calidrop_compress (the caller may have appended rows and raised cache_lens).  cache_offsets may
 * be NULL when every sequence has the same capacity and that capacity is max_cache_len (sequence
 * b then starts at token b * max_cache_len): the kernel then needs no offset loads before it can
 * start streaming.  max_cache_len >= every cache_lens[b] (host copy; sizes the grid); c_q, c_out, c_lse the
 * calibration state; out [batch][Hq][D] dtype; a_lse optional out [batch][Hq] fp32 (may be
 * NULL); flags optional out [batch][Hq] uint8 (may be NULL); workspace >=
 * calidrop_decode_workspace_bytes(p, max_cache_len) bytes, 256-byte aligned.
 * A sequence with cache_lens[b] = 0 yields out = 0 and a_lse = -inf.
 */
int calidrop_decode(const calidrop_params* p, const void* q_t, const void* k_c, const void* v_c,
                    const int32_t* cache_offsets, const int32_t* cache_lens,
                    int32_t max_cache_len, const float* c_q, const float* c_out,
                    const float* c_lse, void* out, float* a_lse, uint8_t* flags,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * calidrop_decode_static - calidrop_decode for callers that cannot allocate or bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * Same arguments (minus workspace / workspace_bytes), same validation, same kernels and bit-identical
 * results.  The scratch of the call - the per-split partial outputs of the form of the step that spreads
 * a long cache over several workgroups - lives in a fixed array of CALIDROP_STATIC_SCRATCH_BYTES of
 * device memory inside the library, one copy per GPU, held from the library's load until the process
 * ends.  The call allocates nothing and frees nothing.
 *   - A call whose scratch need, calidrop_decode_workspace_bytes(p, max_cache_len), exceeds
 *     CALIDROP_STATIC_SCRATCH_BYTES returns CALIDROP_EWORKSPACE and enqueues nothing: use
 *     calidrop_decode with a workspace for such shapes.
 *   - Every call on a GPU shares that GPU's array, which keeps the previous call's contents.  Nothing in
 *     it needs to start at zero (every partial a call reads, it has written before), so consecutive
 *     calls on one stream are safe; calls that overlap in time on one GPU (different streams, or
 *     different host threads) race on it and must not be made.
 *   - The array's address on the current device is looked up on the first call on that device
 *     (CALIDROP_EHIP if the lookup fails).
 */
#define CALIDROP_STATIC_SCRATCH_BYTES (8u << 20)
int calidrop_decode_static(const calidrop_params* p, const void* q_t, const void* k_c, const void* v_c,
                           const int32_t* cache_offsets, const int32_t* cache_lens,
                           int32_t max_cache_len, const float* c_q, const float* c_out,
                           const float* c_lse, void* out, float* a_lse, uint8_t* flags, void* stream);

/*
 * calidrop_append - decode-time growth of the compressed cache: tokens generated during decoding
 * are appended and never evicted (the evicted set is fixed at prefill).  For every sequence b
 * the rows k_new[b][g], v_new[b][g] ([batch][Hkv][D] dtype: K and V of the token just generated)
 * are written to position cache_lens[b] of every KV head of k_c / v_c and cache_lens[b] grows by
 * one.  A sequence whose capacity (cache_offsets[b+1] - cache_offsets[b]) is used up is left
 * unchanged.  No workspace.  The next calidrop_decode must be given max_cache_len >= the new
 * lengths (the capacity is always a valid choice).
 */
int calidrop_append(const calidrop_params* p, const void* k_new, const void* v_new, void* k_c,
                    void* v_c, const int32_t* cache_offsets, int32_t* cache_lens, void* stream);

/*
 * calidrop_recalibrate - the rho < theta1 branch of Alg. 2 (steps 3-8), for the heads that the
 * preceding calidrop_decode call of the same step flagged CALIDROP_FLAG_RECOMPUTE.
 *
 * For every such (sequence b, query head h), with KV head g = h / G and KV_evict = the rows of
 * the prompt that are not listed in indices[b][g] (the list holds the window, so these are
 * prefix rows) - or, when calib_size > 0, exactly the rows listed in cal_indices[b][g]:
 *   c_lse[h] = log sum_{t in evict} exp(scale q_t[h].K_t),  c_out[h] = Att(q_t[h], K_evict, V_evict)
 *   (the current query is used, as the text of Sec. 3.2 says), c_q[h] = q_t[h]           (steps 5-7)
 *   out[h] = alpha_i out[h] + alpha_j c_out[h] with alpha_j = 1/(1+exp(a_lse[h] - c_lse[h]))  (step 8)
 *   flags[h] = CALIDROP_FLAG_RECOMPUTED.
 * Heads with any other flag, and their state, are left untouched.  Sequences with nothing evicted
 * (n_b <= B) get c_q = q_t, c_lse = -inf, c_out = 0 and an unchanged output.  KV groups without a
 * flagged head are not streamed at all.
 *
 * Arguments: q_t, out, a_lse, flags as passed to / written by calidrop_decode for this step (out
 * and flags are updated in place; flags must not be NULL here); k, v, seq_offsets, total_tokens,
 * max_seq_len, indices and cal_indices as in / from calidrop_compress (the prompt K/V must still
 * be resident: this is where the "offloaded" evicted cache is read from; cal_indices is required
 * when calib_size > 0 and ignored otherwise); c_q, c_out, c_lse the calibration state,
 * updated in place; workspace >= calidrop_recalibrate_workspace_bytes(p, max_seq_len) bytes,
 * 256-byte aligned.
 */
size_t calidrop_recalibrate_workspace_bytes(const calidrop_params* p, int32_t max_seq_len);
int calidrop_recalibrate(const calidrop_params* p, const void* q_t, const void* k, const void* v,
                         const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len,
                         const int32_t* indices, const int32_t* cal_indices, uint8_t* flags,
                         const float* a_lse, void* out, float* c_q, float* c_out, float* c_lse,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Other eviction strategies f (Alg. 1 step 3).  The method is independent of how the retained
 * set is chosen (Sec. 3.2; Sec. 4.1.3 also evaluates StreamingLLM and H2O), so the steps after
 * the choice - gather of KV_compress, KV_evict = everything else, calibration state - are also
 * available for a retained set that is already known.
 *
 * calidrop_streaming_indices - the StreamingLLM choice (Sec. 4.1.3: a fixed number of attention
 * sinks, the rest of the budget spent on the most recent tokens): for every sequence b and KV
 * head, indices[b][g] = 0..n_sink-1 followed by n_b-(B-n_sink)..n_b-1 when n_b > B, else
 * 0..n_b-1 padded with -1.  Index arithmetic only; the paper's setting is n_sink = 32.
 *   0 <= n_sink <= budget (CALIDROP_EINVAL otherwise); seq_offsets, total_tokens, max_seq_len
 *   as in calidrop_compress; indices out [batch][Hkv][B] int32.  No workspace.
 *
 * calidrop_compress_given - Alg. 1 steps 4-8 for the retained lists in `indices`:
 *   n_b <= B : everything is retained (the library overwrites indices[b] with 0..n_b-1, -1 padded),
 *              c_lse = -inf, c_out = 0.
 *   n_b >  B : indices[b][g] must hold B distinct positions in [0, n_b), ascending (device memory,
 *              so the host cannot check it: an entry outside the range is read as the nearest valid
 *              position by the gather and marks nothing as retained - memory safe, result
 *              meaningless).  K_c, V_c = those rows; KV_evict = every other row of the prompt;
 *              c_lse, c_out = log-weight and attention of q_cal over KV_evict; c_q = q_cal.
 *   `window` and `pool_kernel` of the params play no role here; calib_size must be 0 (the ranking
 *   of evicted tokens needs scores: CALIDROP_EUNSUPPORTED otherwise).  calidrop_decode and
 *   calidrop_recalibrate work on the result unchanged.
 * Arguments: q_cal [batch][Hq][D] dtype (required: the last prompt query Q_{-1}); the others as in
 * calidrop_compress; workspace >= calidrop_compress_given_workspace_bytes(p, max_seq_len) bytes,
 * 256-byte aligned.
 */
size_t calidrop_compress_given_workspace_bytes(const calidrop_params* p, int32_t max_seq_len);
int calidrop_streaming_indices(const calidrop_params* p, int32_t n_sink, const int32_t* seq_offsets,
                               int64_t total_tokens, int32_t max_seq_len, int32_t* indices,
                               void* stream);
int calidrop_compress_given(const calidrop_params* p, const void* q_cal, const void* k,
                            const void* v, const int32_t* seq_offsets, int64_t total_tokens,
                            int32_t max_seq_len, int32_t* indices, void* k_c, void* v_c,
                            const int32_t* cache_offsets, int32_t* cache_lens, float* c_q,
                            float* c_out, float* c_lse, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * calidrop_compress_h2o - Alg. 1 steps 3-8 with H2O as the eviction strategy f (Sec. 4.1.3:
 * importance = accumulated attention score; the budget is split into important and local tokens).
 *
 * For every sequence b with n_b > B and every KV head g:
 *   1. every prompt query i of the G heads of the group attends causally (columns 0..i), logits
 *      scale * q.K, row softmax;  vote[j] = sum over those G * n_b rows of the probability on
 *      column j (a dense n_b x n_b pass per head, on the matrix cores).
 *   2. retained = the n_local most recent positions plus the B - n_local positions of largest
 *      vote among the others (ties to the lower position), ascending.
 *   3. gather, KV_evict, calibration state exactly as in calidrop_compress, with Q_{-1} (the
 *      last row of q_full) as the calibration query; calib_size > 0 ranks the evicted tokens by
 *      the same votes.
 * n_b <= B keeps everything.  n_local = 0 selects B / 2 (the even split the paper uses);
 * otherwise 1 <= n_local < B.  `window` and `pool_kernel` of the params play no role.
 *
 * Arguments: q_full dtype, packed like k but with Hq heads: sequence b starts at token
 * seq_offsets[b], inside [Hq][n_b][D] (every prompt query, as used by attention); all other
 * arguments as in calidrop_compress; batch * n_q_heads <= 65535; workspace >=
 * calidrop_compress_h2o_workspace_bytes(p, n_local, total_tokens, max_seq_len) bytes, 256-byte
 * aligned.
 */
size_t calidrop_compress_h2o_workspace_bytes(const calidrop_params* p, int32_t n_local,
                                             int64_t total_tokens, int32_t max_seq_len);
/* Regions of that workspace for inspection after the stream has finished:
 *   ROW_LSE float [batch][Hq][stride]: log2 of the softmax denominator of every prompt query
 *           (logits in log2 units), stride = bytes / (batch * Hq * 4) >= max_seq_len, +inf padded;
 *   SCORE   float, packed like K with D = 1: vote of position j of KV head g of sequence b at
 *           [seq_offsets[b]*Hkv + g*n_b + j], for the candidates j < n_b - n_local (needs
 *           CALIDROP_OPT_WRITE_SCORES in the call's params unless the prompt is longer than 32768);
 *   VOTE_PLANES float [G][total_tokens*Hkv] (H2O only): plane hh holds, packed like SCORE and for
 *           every position j < n_b, the probability mass position j received from the queries
 *           of query head hh of its group; the score is the sum of the G planes.                  */
int calidrop_compress_h2o_workspace_region(const calidrop_params* p, int32_t n_local,
                                           int64_t total_tokens, int32_t max_seq_len,
                                           int32_t region, size_t* offset, size_t* bytes);
int calidrop_compress_h2o(const calidrop_params* p, int32_t n_local, const void* q_full,
                          const void* k, const void* v, const int32_t* seq_offsets,
                          int64_t total_tokens, int32_t max_seq_len, void* k_c, void* v_c,
                          const int32_t* cache_offsets, int32_t* cache_lens, int32_t* indices,
                          int32_t* cal_indices, float* c_q, float* c_out, float* c_lse,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Offloading KV_evict (Alg. 1 step 4 moves the evicted cache out of GPU memory instead of deleting
 * it; Alg. 2 step 4 reloads it for the recomputation branch; Sec. 3.2).
 *
 * calidrop_pack_evicted - after calidrop_compress / calidrop_compress_given: write the rows of
 * K, V that form KV_evict - or, with calib_size > 0, the calibration set (Sec. 5.3) - of every
 * (sequence, KV head) as one contiguous block, so that the caller can move them (for example to
 * host memory) with plain copies and release the prompt tensors.
 *   rows per KV head of sequence b: E_b = calidrop_packed_rows(p, n_b)
 *        = 0 if n_b <= B, else n_b - B, or min(calib_size, n_b - B) when calib_size > 0.
 *   evict_offsets [batch+1] int32 in: sequence b owns tokens evict_offsets[b]..evict_offsets[b+1]
 *        of the packed buffers, capacity cap_b = their difference >= E_b (a sequence whose
 *        capacity is too small gets evict_lens[b] = 0 and nothing written).
 *   k_e, v_e      out, dtype: inside sequence b [Hkv][cap_b][D]; the first E_b rows of each head are
 *        written, in ascending prompt position.
 *   evict_lens    out [batch] int32 = E_b.
 *   evict_indices out int32, packed like k_e with one int per row: the prompt position of each row.
 *   indices, cal_indices as written by calidrop_compress (cal_indices required when
 *   calib_size > 0, ignored otherwise); k, v, seq_offsets, total_tokens, max_seq_len as there;
 *   workspace >= calidrop_pack_evicted_workspace_bytes(p, max_seq_len) bytes, 256-byte aligned.
 *
 * calidrop_recalibrate_packed - calidrop_recalibrate reading the packed rows instead of the prompt:
 * same results, same in/out arguments (q_t, flags, a_lse, out, c_q, c_out, c_lse).  k_e and v_e may
 * be device memory or page-locked host memory that the device can address (hipHostMalloc): in the
 * second case the kernel pulls the rows of the flagged KV groups over the host link while it
 * computes, and nothing is staged in device memory (the library asks the runtime what kind of
 * memory k_e is - hipPointerGetAttributes, a host-side query - and requests host-resident rows as
 * whole rows, which the host link moves a third faster than the pieces of the matrix-operand
 * layout).  evict_offsets / evict_lens are device memory.
 * max_evict_len >= every evict_lens[b] (host copy; sizes the grid).  workspace >=
 * calidrop_recalibrate_packed_workspace_bytes(p, max_evict_len) bytes, 256-byte aligned.
 */
int32_t calidrop_packed_rows(const calidrop_params* p, int32_t seq_len);   /* -1 on invalid params */
size_t calidrop_pack_evicted_workspace_bytes(const calidrop_params* p, int32_t max_seq_len);
int calidrop_pack_evicted(const calidrop_params* p, const void* k, const void* v,
                          const int32_t* seq_offsets, int64_t total_tokens, int32_t max_seq_len,
                          const int32_t* indices, const int32_t* cal_indices, void* k_e, void* v_e,
                          const int32_t* evict_offsets, int32_t* evict_lens, int32_t* evict_indices,
                          void* workspace, size_t workspace_bytes, void* stream);
size_t calidrop_recalibrate_packed_workspace_bytes(const calidrop_params* p, int32_t max_evict_len);
int calidrop_recalibrate_packed(const calidrop_params* p, const void* q_t, const void* k_e,
                                const void* v_e, const int32_t* evict_offsets,
                                const int32_t* evict_lens, int32_t max_evict_len, uint8_t* flags,
                                const float* a_lse, void* out, float* c_q, float* c_out,
                                float* c_lse, void* workspace, size_t workspace_bytes, void* stream);

/* Host string describing the last error on the calling thread ("" if none). Never NULL.      */
const char* calidrop_last_error(void);

/* Library version as major*10000 + minor*100 + patch.                                        */
int calidrop_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CALIDROP_H */
