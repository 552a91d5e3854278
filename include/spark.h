/*
 * spark.h -- C ABI of the MI355X (gfx950) SparK hot path.
 *
 * SparK ("Query-Aware Unstructured Sparsity with Recoverable KV Cache Channel Pruning")
 * prunes the key cache along the channel axis, per token and per head, at prefill, and
 * restores the pruned entries from one cached statistic while the attention scores are
 * computed at decode.  This library is that data path on one GPU:
 *
 *   spark_prune        prefill:  saliency -> per-token top-T channels -> packed key cache
 *   spark_decode_attn  decode:   one attention step that reads only the packed keys and
 *                                the dense values
 *   spark_unpack       parity / debugging: canonical export of the opaque packed cache
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller unless it is a `const
 *     spark_desc *` (host) or documented otherwise.  The library never allocates, frees or
 *     retains device memory; callers size buffers with the query functions below.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and the call returns after the launches; the library never synchronises.
 *   - Failure is a return code.  Arguments are checked on the host before anything is
 *     launched; a launch error reported by the runtime becomes SPARK_ERR_HIP.  No
 *     exceptions, no global state; calls on distinct streams and buffers are thread safe.
 *   - bfloat16 tensors are raw 16-bit patterns.  Channel stride is 1 everywhere; token and
 *     head strides are in ELEMENTS: K[n,h,j] = k[n*k_token_stride + h*k_head_stride + j]
 *     for global token n in [0,total_tokens), likewise V.  Rows of K and V must be 16-byte
 *     aligned (strides multiples of 8, base pointers 16-byte aligned; checked); q and the window
 *     queries need 2-byte alignment only.
 *   - Inputs are expected to be FINITE.  Infinities and NaNs in K, V, q or the window queries are not
 *     detected.  Every loop in the library is bounded whatever the bits are, so a call with such input
 *     completes without fault; but the mask, kept entries and statistic of a row that contains one (of
 *     every row of a sequence whose window queries contain one) are unspecified, and so is every output
 *     row computed from such a row (it may be NaN).  Rows and sequences without such entries are not
 *     affected: sequences and KV heads are independent.
 *   - Sequences are ragged: cu_seqlens[b] .. cu_seqlens[b+1] are the global token indices
 *     of batch element b (int32 [batch+1], cu_seqlens[0] = 0, cu_seqlens[batch] =
 *     total_tokens).  Query head g reads KV head g / (n_q_heads / n_kv_heads).
 */
#ifndef SPARK_H
#define SPARK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPARK_OK = 0,
    SPARK_ERR_INVALID_ARG = 1,      /* NULL pointer, non-positive size, bad stride/alignment */
    SPARK_ERR_UNSUPPORTED = 2,      /* head_dim != 128, group size not in {1,2,4,8,16}, token stride of K above 2^24 */
    SPARK_ERR_WORKSPACE_TOO_SMALL = 3,
    SPARK_ERR_HIP = 4,              /* the HIP runtime reported an error at launch */
    SPARK_ERR_MISMATCH = 5          /* spark_check_packed: the cache was not written for this description */
} spark_status;

typedef enum { SPARK_PACK_BF16 = 0, SPARK_PACK_INT8 = 1 } spark_pack_dtype;
typedef enum { SPARK_OUT_BF16 = 0, SPARK_OUT_F32 = 1 } spark_out_dtype;
typedef enum { SPARK_RECOVER_GAUSSIAN = 1, SPARK_RECOVER_EXPONENTIAL = 2 } spark_recovery;

/* Problem description shared by all calls (plain data, host memory). */
typedef struct spark_desc {
    int32_t batch;            /* 1 <= B <= 2^18 */
    int32_t n_q_heads;        /* Hq, a multiple of n_kv_heads; Hq/Hkv in {1,2,4,8,16} */
    int32_t n_kv_heads;       /* Hkv >= 1 */
    int32_t head_dim;         /* D, must be 128 */
    int32_t keep;             /* T in [1, D]: channels kept per (token, KV head).  An integer,
                                 not a ratio: the paper's T = floor((1 - lambda) * D). */
    int32_t window;           /* W >= 1: observation-window length (spark_prune only) */
    int32_t pack_dtype;       /* spark_pack_dtype: storage of the kept key entries */
    int32_t out_dtype;        /* spark_out_dtype: element type of spark_decode_attn's output */
    int64_t total_tokens;     /* sum of sequence lengths, <= 2^31 - 256 */
    int64_t k_token_stride, k_head_stride;    /* dense K (spark_prune only) */
    int64_t v_token_stride, v_head_stride;    /* dense V (spark_decode_attn only) */
    float   softmax_scale;    /* 0 => 1/sqrt(head_dim) */
    int32_t n_splits;         /* decode: > 0 cuts every sequence into this many blocks per KV head; 0 => the
                                 library cuts sequences in proportion to their length (ragged batches:
                                 long sequences get more blocks), and batches of 32 to 256 short sequences
                                 (with at least two 64-token tiles per resident wavefront) are dealt out
                                 tile by tile to independent wavefronts (the balanced cut; see max_seqlen);
                                 -1 asks for the balanced cut whenever it exists (batch <= 256, at most 8
                                 query heads per KV head; spark_decode_attn and spark_decode_attn_tail; the
                                 other entry points cut by length).  Must be the same for the workspace
                                 query, its init and the calls. */
    int32_t keep_v;           /* T_v in [1, D]: channels kept per (token, KV head) of the VALUE cache, used by
                                 the *_values entry points only; 0 where values stay dense */
    int32_t stats;            /* 1: spark_prune also stores, per (token, KV head), the mean and the standard
                                 deviation of the saliency over all channels (8 bytes more per row; needed by
                                 spark_decode_attn_sampled); 0: not stored */
    int32_t tail_capacity;    /* rows per sequence in the appended-token buffers of spark_decode_attn_tail;
                                 0 elsewhere.  Enters the decode workspace size: keep it the same for the
                                 workspace query, its init and the calls. */
    int32_t max_seqlen;       /* decode, a hint: the longest sequence of the batch in tokens where the caller
                                 knows it (the lengths themselves are on the device), 0 where not.  With
                                 n_splits = 0 a batch whose longest sequence is within 9/8 of the average is
                                 balanced as it is and keeps one block per sequence, which is 3 to 5 %
                                 cheaper there than the balanced cut.  Never affects results; enters the
                                 workspace size like n_splits. */
} spark_desc;

/* Size in bytes of the packed key cache for this description (depends on batch, n_kv_heads,
 * keep, pack_dtype, total_tokens).  0 if the description is invalid. */
size_t spark_packed_bytes(const spark_desc *desc);

/* Scratch sizes in bytes (0 is possible; then NULL may be passed as the workspace). */
size_t spark_prune_workspace(const spark_desc *desc);
size_t spark_decode_workspace(const spark_desc *desc);

/*
 * Prepares a decode workspace: zeroes the per-(batch, KV head) arrival counters, which sit at its
 * start (batch * n_kv_heads 32-bit words, at a position that does not depend on token counts,
 * split counts or tail capacity; the partial softmax states follow).  Call once after allocating
 * (or overwriting) the workspace and whenever batch or n_kv_heads change; spark_decode_attn leaves
 * the counters zeroed, so one workspace that is large enough serves any number of successive calls
 * on one stream, also for descriptions that differ in total_tokens, n_splits or tail_capacity.
 * Two calls that overlap in time need two workspaces.
 */
spark_status spark_decode_workspace_init(const spark_desc *desc, void *workspace,
                                         size_t workspace_bytes, void *hip_stream);

/* Number of blocks per KV head spark_decode_attn uses for a sequence of average length; 0 where
 * spark_decode_attn and spark_decode_attn_tail take the balanced cut instead (see n_splits). */
int32_t spark_decode_splits(const spark_desc *desc);

/*
 * Prefill-time channel pruning of the key cache.
 * [Sec. "Problem Formulation and Analysis", Eq. (7) and the greedy Top_T solution;
 *  Sec. "SparK", mean query over the observation window, "Saliency Measurement and
 *  Unstructured Pruning"; App. "Caching Pruned Channel Statistics", mean over the pruned set]
 *
 *   qbar[b,g,:] = mean over the W window queries of head g
 *   a[b,h,j]    = mean over the heads g of KV head h of |qbar[b,g,j]|   (float64, rounded to float32)
 *   w[n,h,j]    = a[b,h,j] * |K[n,h,j]|                                 (one float32 multiply)
 *   kept(n,h)   = the T channels of largest w; equal w: lower channel first
 *   mu[n,h]     = mean of w over the D-T pruned channels (0 if T == D)
 * and writes, per (token, KV head): the 128-bit channel mask, the kept entries (original
 * bf16 bits, ascending channel; or int8 codes = round(k / scale), scale = max|k| / 127, for
 * SPARK_PACK_INT8) and mu, plus a per (batch, KV head); all inside `packed_out`.
 *
 *   k_bf16     in   dense keys, bf16, addressed with k_*_stride; k_token_stride <= 2^24 elements
 *                   (SPARK_ERR_UNSUPPORTED beyond that)
 *   qwin_bf16  in   [batch, n_q_heads, window, 128] bf16, contiguous
 *   cu_seqlens in   int32 [batch+1]
 *   packed_out out  spark_packed_bytes(desc) bytes, 256-byte aligned; fully overwritten
 *   workspace       spark_prune_workspace(desc) bytes (may be NULL when that is 0)
 * Every token given is pruned, window tokens included.  V is not touched.
 */
spark_status spark_prune(const spark_desc *desc, const void *k_bf16, const void *qwin_bf16,
                         const int32_t *cu_seqlens, void *packed_out, void *workspace,
                         size_t workspace_bytes, void *hip_stream);

/*
 * One decode step of attention over the packed key cache.
 * [Sec. "SparK", "Channel Recovery" with the degenerate recovery function
 *  ktilde[n,h,j] = mu[n,h] / a[b,h,j] for pruned entries; Sec. "Preliminaries", Eq. (4)]
 *
 *   s[g,n]  = scale * ( sum_{j kept} q[g,j] K[n,h,j] + sum_{j pruned} q[g,j] mu[n,h]/a[b,h,j] )
 *   out[b,g,:] = sum_n softmax_n(s[g,:])[n] * V[n,h,:]       over the tokens n of sequence b
 * (a[b,h,j] == 0 recovers 0).  The dense K-tilde is never written to memory.  A sequence of
 * length 0 gives a zero output row.
 *
 *   q_bf16     in   [batch, n_q_heads, 128] bf16, contiguous
 *   packed     in   written by spark_prune with the same batch / n_kv_heads / keep /
 *                   pack_dtype / total_tokens and the same cu_seqlens
 *   v_bf16     in   dense values, bf16, addressed with v_*_stride
 *   out        out  [batch, n_q_heads, 128], bf16 or float32 per desc->out_dtype, 8-byte aligned
 *   workspace       spark_decode_workspace(desc) bytes, 16-byte aligned, prepared with
 *                   spark_decode_workspace_init (split partials and arrival counters)
 * One kernel launch: the sequence is split over blocks, and the block that finishes last for a
 * (batch, KV head) pair merges the partial softmax states and writes the output.
 */
spark_status spark_decode_attn(const spark_desc *desc, const void *q_bf16, const void *packed,
                               const void *v_bf16, const int32_t *cu_seqlens, void *out,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Canonical export of a packed cache, for parity tests and debugging (not a hot path).
 * Any output pointer may be NULL to skip it.
 *   mask_out  uint32 [total_tokens, n_kv_heads, 4]   bit j%32 of word j/32 = channel j kept
 *   vals_out  [total_tokens, n_kv_heads, keep]       kept entries, ascending channel:
 *                                                    uint16 bf16 bits, or int8 codes
 *   mu_out    float  [total_tokens, n_kv_heads]
 *   scale_out float  [total_tokens, n_kv_heads]      int8 scales (SPARK_PACK_INT8 only)
 *   a_out     float  [batch, n_kv_heads, 128]
 */
spark_status spark_unpack(const spark_desc *desc, const void *packed, uint32_t *mask_out,
                          void *vals_out, float *mu_out, float *scale_out, float *a_out,
                          void *hip_stream);

/*
 * Debugging aid: does this packed cache belong to this description?  The decode and unpack calls
 * trust the description they are given (they read rows at the stride it implies and cannot report a
 * mismatch without a device-to-host round trip); this call makes that round trip.  It copies the
 * cache's 64-byte header to the host, WAITS for `hip_stream`, and compares magic word, kept-channel
 * count, storage type, statistics flag, batch, n_kv_heads, total_tokens and row length with what
 * `desc` implies.  `is_value_cache` = 0 checks a key cache written by spark_prune (against keep,
 * pack_dtype, stats), 1 a value cache written by spark_prune_values (against keep_v).
 * Returns SPARK_OK, SPARK_ERR_MISMATCH, or the usual argument / runtime errors.  Not a hot path.
 */
spark_status spark_check_packed(const spark_desc *desc, const void *packed, int32_t is_value_cache,
                                void *hip_stream);

/*
 * One decode step with a SAMPLED recovery function.
 * [Sec. "SparK", "Channel Recovery": a saliency w~ is sampled for every pruned entry from the cached
 *  statistics and the key entry is back-computed as w~ / a; Gaussian: w~ ~ N(mu, sigma^2); Exponential:
 *  w~ ~ Exp(1/mu); App. "Caching Pruned Channel Statistics": mu, sigma over all channels of the token]
 *
 *   ktilde[n,h,j] = K[n,h,j] if kept, else w~[n,h,j] / a[b,h,j]  (0 if a == 0); then scores, softmax, P V
 *   as in spark_decode_attn.
 * The paper does not say how the samples are drawn.  Here they are a pure function of (seed, n, h, j):
 *   mix(x): x ^= x >> 16; x *= 0x85EBCA6B; x ^= x >> 13; x *= 0xC2B2AE35; x ^= x >> 16   (32-bit words)
 *   base = mix(mix(mix(n) + seed_lo) + h * 0x9E3779B9 + seed_hi),  x_c = mix(base + c * 0x9E3779B9),
 *   u_c  = ((x_c >> 9) + 0.5) / 2^23
 *   Gaussian, channels 2m, 2m+1:  w~ = mu + sigma * sqrt(-2 ln u_2m) * {cos, sin}(2 pi u_(2m+1))
 *   Exponential, channel j:        w~ = -mu * ln u_j
 * so a call with the same seed repeats, and a caller that wants fresh samples per step changes the seed.
 * A Gaussian sample may be negative (it is not clamped).
 *
 *   packed    written by spark_prune with desc->stats = 1 (bf16 or int8 storage of the kept entries)
 *   recovery  spark_recovery
 *   seed      64 bits: seed_lo = low word, seed_hi = high word
 * Other arguments as spark_decode_attn.  This variant draws 128 - keep variates per (token, KV head) and is
 * bound by arithmetic, not by memory.
 */
spark_status spark_decode_attn_sampled(const spark_desc *desc, const void *q_bf16, const void *packed,
                                       const void *v_bf16, const int32_t *cu_seqlens, void *out,
                                       void *workspace, size_t workspace_bytes, int32_t recovery,
                                       uint64_t seed, void *hip_stream);

/* Export of the per-row statistics of a cache written with desc->stats = 1 (parity tests, debugging):
 *   mu_all_out, sigma_out  float [total_tokens, n_kv_heads]; either may be NULL. */
spark_status spark_unpack_stats(const spark_desc *desc, const void *packed, float *mu_all_out,
                                float *sigma_out, void *hip_stream);

/*
 * One decode step when tokens have been appended after prefill.
 * [Sec. "Preliminaries": every decode step concatenates the new token's key and value to the cache;
 *  Sec. "SparK": channels are pruned once, at prefill -- so appended rows are kept dense]
 *
 * The cache of sequence b is its pruned prefix (packed keys + dense values, as in spark_decode_attn)
 * followed by tail_len[b] appended rows; scores of appended rows are plain scale * <q, k>; one softmax
 * runs over prefix and appended rows together, and the output sums over both value sets.
 *
 *   tail_k_bf16, tail_v_bf16  in  [batch, tail_capacity, n_kv_heads, 128] bf16, contiguous, 16-byte aligned;
 *                                 row i < tail_len[b] of sequence b is its i-th appended token
 *   tail_len                  in  int32 [batch] (device), 0 <= tail_len[b] <= desc->tail_capacity
 * Everything else as spark_decode_attn (same workspace).  Appending a token is the caller's copy into row
 * tail_len[b]; re-pruning a full tail into a new packed cache is a spark_prune call on those rows.
 * Still one launch: extra blocks of the decode grid (one per 256 rows of capacity and (batch, KV head)) leave
 * the appended rows' softmax state in spare workspace slots and are counted like sequence splits.
 */
spark_status spark_decode_attn_tail(const spark_desc *desc, const void *q_bf16, const void *packed,
                                    const void *v_bf16, const int32_t *cu_seqlens, const void *tail_k_bf16,
                                    const void *tail_v_bf16, const int32_t *tail_len, void *out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Channel pruning of the value cache.
 * [App. "Pruning Value Cache Channels": per token the importance of a value channel is the magnitude of
 *  the entry itself; only the top-T_v channels are retained; values need no scaling or recombination
 *  because the weighted sum consumes them directly -- read here as: a pruned entry contributes 0]
 *
 *   kept_v(n,h) = the keep_v channels of largest |V[n,h,j]|; equal magnitudes: lower channel first
 * and writes, per (token, KV head), the 128-bit channel mask and the kept entries (original bf16 bits,
 * ascending channel) into `packed_v_out`.  No query, window or sequence boundary enters.
 *
 *   v_bf16        in   dense values, bf16, addressed with v_*_stride (v_token_stride <= 2^24 elements)
 *   packed_v_out  out  spark_packed_values_bytes(desc) bytes, 256-byte aligned; fully overwritten
 * Uses desc->n_kv_heads, head_dim, keep_v, total_tokens and the v strides.
 */
size_t spark_packed_values_bytes(const spark_desc *desc);   /* 0 if the description is invalid or keep_v == 0 */
spark_status spark_prune_values(const spark_desc *desc, const void *v_bf16, void *packed_v_out,
                                void *hip_stream);

/*
 * One decode step of attention over the packed key cache AND the packed value cache.
 * [Sec. "SparK", Channel Recovery, for the scores, as in spark_decode_attn; App. "Pruning Value Cache
 *  Channels" for the values: a pruned value entry contributes 0 to the weighted sum]
 *
 *   out[b,g,:] = sum_n softmax_n(s[g,:])[n] * Vtilde[n,h,:],  Vtilde[n,h,j] = V[n,h,j] if kept_v else 0
 *
 * Arguments as spark_decode_attn, with `packed_v` (written by spark_prune_values with the same
 * n_kv_heads / keep_v / total_tokens) in place of the dense values; the kept key entries may be stored
 * as bf16 or as int8 codes (desc->pack_dtype), the kept value entries are always bf16.  Workspace and split
 * count are those of spark_decode_attn.
 */
spark_status spark_decode_attn_values(const spark_desc *desc, const void *q_bf16, const void *packed,
                                      const void *packed_v, const int32_t *cu_seqlens, void *out,
                                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* spark_decode_attn_values with appended, never-pruned rows (arguments as in spark_decode_attn_tail; the
 * appended values are dense like the appended keys). */
spark_status spark_decode_attn_values_tail(const spark_desc *desc, const void *q_bf16, const void *packed,
                                           const void *packed_v, const int32_t *cu_seqlens,
                                           const void *tail_k_bf16, const void *tail_v_bf16,
                                           const int32_t *tail_len, void *out, void *workspace,
                                           size_t workspace_bytes, void *hip_stream);

/*
 * Canonical export of a packed value cache (parity tests and debugging).  Either output may be NULL.
 *   mask_out  uint32 [total_tokens, n_kv_heads, 4]       bit j%32 of word j/32 = channel j kept
 *   vals_out  uint16 [total_tokens, n_kv_heads, keep_v]  kept entries (bf16 bits), ascending channel
 */
spark_status spark_unpack_values(const spark_desc *desc, const void *packed_v, uint32_t *mask_out,
                                 void *vals_out, void *hip_stream);

/*
 * The top-p variant of the pruning: no fixed number of channels per row.
 * [Sec. "Adaptive Variants of SparK", table "Ablation study on variants": per token, the fewest most salient
 *  channels whose saliencies together account for 99 % of the row's total saliency are kept]
 *
 *   w[n,h,j]   as in spark_prune (one float32 multiply); order: w descending, equal w lower channel first
 *   count(n,h) = the smallest m >= 1 whose m most salient channels hold at least p of the row's saliency
 *   kept, mask, mu (mean of w over the 128 - count pruned channels, 0 if none) as in spark_prune
 * The count is an integer decided by sums, so the decision is taken in integers, which any summation order
 * reproduces: every w of a row is expressed in units of the last place of the row's largest saliency, rounded
 * down (q < 2^24), p is given in basis points, and count = the smallest m >= 1 with
 *   10000 * (sum of the m largest q)  >=  p_basis_points * (sum of all q).
 * An all-zero row keeps one channel (channel 0).
 *
 *   p_basis_points  1 .. 10000 (9900 = the paper's 99 %)
 *   packed_out      spark_packed_topp_bytes(desc) bytes, 256-byte aligned: sized for the worst case (every row
 *                   keeps all 128 channels); rows are 24 bytes (mask, mu, count) plus two bytes per kept entry
 *                   in a value stream, and only the used part of the stream is written or ever read
 * Uses batch, head counts, window, total_tokens and the k strides of `desc`; desc->keep is not used;
 * bf16 storage only (SPARK_ERR_UNSUPPORTED for SPARK_PACK_INT8 or stats).  Other arguments as spark_prune.
 */
size_t spark_packed_topp_bytes(const spark_desc *desc);
spark_status spark_prune_topp(const spark_desc *desc, const void *k_bf16, const void *qwin_bf16,
                              const int32_t *cu_seqlens, int32_t p_basis_points, void *packed_out,
                              void *hip_stream);

/*
 * One decode step over a cache written by spark_prune_topp: scores, softmax and output exactly as in
 * spark_decode_attn (degenerate recovery mu / a for the pruned entries of every row), with every row walked to
 * its own count.  Arguments, workspace and split count as spark_decode_attn.
 */
spark_status spark_decode_attn_topp(const spark_desc *desc, const void *q_bf16, const void *packed,
                                    const void *v_bf16, const int32_t *cu_seqlens, void *out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Canonical export of a top-p cache (parity tests and debugging).  Any output may be NULL.
 *   mask_out   uint32 [total_tokens, n_kv_heads, 4]
 *   count_out  int32  [total_tokens, n_kv_heads]        kept channels of the row
 *   vals_out   uint16 [total_tokens, n_kv_heads, 128]   kept entries (bf16 bits), ascending channel, then zeros
 *   mu_out     float  [total_tokens, n_kv_heads];   a_out float [batch, n_kv_heads, 128]
 */
spark_status spark_unpack_topp(const spark_desc *desc, const void *packed, uint32_t *mask_out,
                               int32_t *count_out, void *vals_out, float *mu_out, float *a_out,
                               void *hip_stream);

/*
 * spark_decode_attn for callers that can neither allocate device memory nor hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result
 * as spark_decode_attn, without the workspace: split partials and arrival counters live in an array of
 * SPARK_STATIC_WORKSPACE_BYTES inside the library's device image (one copy per GPU, held until the process
 * ends).  The call allocates nothing, frees nothing and prepares the array itself (no init call).
 *   - SPARK_ERR_WORKSPACE_TOO_SMALL if the partial states do not fit SPARK_STATIC_WORKSPACE_BYTES (all five
 *     benchmark shapes fit; the largest needs 2.7 MB; where the balanced cut of a ragged batch would not fit
 *     but the cut by length does, the call uses the cut by length);
 *   - the first call on a GPU looks the array's address up (hipGetSymbolAddress): make it outside a capture;
 *   - every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (two streams) race.
 */
#define SPARK_STATIC_WORKSPACE_BYTES (4u << 20)
spark_status spark_decode_attn_static(const spark_desc *desc, const void *q_bf16, const void *packed,
                                      const void *v_bf16, const int32_t *cu_seqlens, void *out,
                                      void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *spark_status_string(spark_status status);

#ifdef __cplusplus
}
#endif
#endif /* SPARK_H */
