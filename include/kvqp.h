/*
 * kvqp.h -- C ABI of the quantized-pruned KV cache for MI355X (gfx950).
 *
 * Method: "More Tokens, Lower Precision" (arXiv 2412.12706), Section 3:
 * at prefill the cache is first pruned along the token axis to a fixed budget
 * ("KV Pruning": keep s < n tokens) and the survivors are then quantized
 * ("KV Quantization": z = min, m = max, s = (m - z)/(2^B - 1),
 * Q(G) = round((G - z)/s)); at decode the attention of Eq. (3),
 * Softmax(h_Q X_K^T) X_V, runs on the dequantized survivors G' = Q(G) s + z
 * ("Quantized Pruning").  Grouping axes follow Section 2 / Section 6.3: keys
 * per channel, values per token (KIVI), or keys per token as the ablation
 * (FlexGen).  The paper's Limitations section names the missing piece this
 * library supplies: dequantization fused into the attention products.
 *
 * Everything the paper leaves open (how prompt tokens are scored, the bit
 * layout, the precision of stored scales) is stated below; the library and
 * its independent CPU checker both implement these statements.
 *
 * General rules
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates or frees device memory, never synchronises the device,
 *     and enqueues work only on the HIP stream passed in (hipStream_t cast to
 *     void*, NULL = default stream).  Inputs are never modified.
 *   - cfg / cache structs are HOST memory, read during the call only.
 *   - Return value: KVQP_OK or a negative KVQP_ERR_* code; nothing throws.
 *     Arguments are validated on the host before anything is launched.
 *   - One call handles one layer.  `batch` is the number of independent
 *     caches, so several layers with identical shapes may be passed as a
 *     larger batch when their buffers are contiguous.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - binary16 ("half") everywhere data is 16-bit floating point.
 */
#ifndef KVQP_H
#define KVQP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVQP_OK 0
#define KVQP_ERR_INVALID_ARG (-1)  /* bad shape, NULL pointer, inconsistent fields       */
#define KVQP_ERR_UNSUPPORTED (-2)  /* valid request outside what this build implements   */
#define KVQP_ERR_WORKSPACE (-3)    /* workspace NULL or smaller than kvqp_workspace_bytes */
#define KVQP_ERR_HIP (-4)          /* a HIP call failed (launch error etc.)              */

#define KVQP_KEY_PER_CHANNEL 0 /* a key group = G consecutive kept tokens of one channel */
#define KVQP_KEY_PER_TOKEN 1   /* a key group = G consecutive channels of one token      */

/*
 * Problem statement of one layer (Section 3; the scoring parameters window
 * and pool_kernel belong to the attention-score pruning rule below).
 * Supported in this build: head_dim == 128; n_q_heads / n_kv_heads in
 * {1,2,4,8}; bits in {2,4,8,16}; group_size in {32,64,128};
 * outlier_threshold 0, or > 0 with bits in {2,4,8}; decode_cache_hint one of KVQP_CACHE_*;
 * window * (n_q_heads/n_kv_heads) <= 256; pool_kernel odd, <= 63;
 * seq_len - window <= 131072.
 */
typedef struct kvqp_cfg {
    int32_t batch;        /* number of independent caches                                */
    int32_t n_q_heads;    /* Hq                                                          */
    int32_t n_kv_heads;   /* Hkv, divides Hq                                             */
    int32_t head_dim;     /* D                                                           */
    int32_t seq_len;      /* L, prompt length (compress only)                            */
    int32_t window;       /* W: the last W prompt tokens score the prefix and stay half  */
    int32_t pool_kernel;  /* odd; 1 = no pooling                                         */
    int32_t budget;       /* prefix tokens kept in low precision; n_kept = min(budget, L-W) */
    int32_t bits;         /* B: 2, 4, 8, or 16 (16 = keep half, no scale/zero)           */
    int32_t group_size;   /* G; must divide D                                            */
    int32_t key_axis;     /* KVQP_KEY_PER_CHANNEL or KVQP_KEY_PER_TOKEN                  */
    int32_t decode_splits;/* token-axis splits of decode attention; 0 = library chooses.
                             With per-head token counts the splits are equal token ranges
                             of the longest possible head, and a head uses as many as its
                             own tokens fill                                             */
    float sm_scale;       /* logit scale > 0, e.g. 1/sqrt(D) (Eq. (3) omits it)          */
    float outlier_threshold; /* tau; > 0 turns outlier filtering on (below), 0 = off     */
    int32_t decode_cache_hint; /* KVQP_CACHE_*: how kvqp_decode_attn's loads treat the
                             chip's memory-side cache (below); 0 = streamed            */
    int32_t outlier_overflow_cap; /* outlier filtering: entries of the overflow list of one
                             (batch, KV head) and tensor (below); >= 0                  */
} kvqp_cfg;

/*
 * decode_cache_hint: how kvqp_decode_attn's loads treat the chip's 256 MB
 * memory-side cache.  A decode step reads every layer's cache exactly once, and
 * between two steps the model's weights and activations pass through the chip,
 * so a cache is normally gone from there before it is read again; loads of such
 * data run faster when they go round that cache (non-temporal loads).
 *   KVQP_CACHE_AUTO    = KVQP_CACHE_STREAM: the case above.
 *   KVQP_CACHE_STREAM  every load non-temporal.
 *   KVQP_CACHE_KEEP    every load normal: for a caller that knows the cache
 *                      will still be resident when it is read again (the caches
 *                      of all layers of a step add up to well under 256 MB and
 *                      little else runs in between), or one that issues a call
 *                      per layer and wants the first layers' caches to stay.
 * Results do not depend on the hint.
 */
#define KVQP_CACHE_AUTO 0
#define KVQP_CACHE_STREAM 1
#define KVQP_CACHE_KEEP 2

/*
 * The compressed cache of one layer.  All eight buffers are device memory of
 * the sizes kvqp_cache_sizes reports, in this order.
 *
 * Token counts need not fill whole blocks or groups (Section 3 asks only for
 * s < n): below, R = n_kept rounded up to a multiple of 32 is the number of rows
 * the per-token arrays of one (batch, KV head) are laid out for, and rows past
 * n_kept hold zeros (code 0, scale 0, zero +0, no outliers).
 *
 * Key codes      k_codes  uint32 [batch, Hkv, R * D * bits / 32]
 *   Row-major [token][channel].  A 32-bit word holds E = 32/bits fields.
 *   Field p of the low half-word (bits [bits*p, bits*p + bits)) and field p of
 *   the high half-word (16 bits higher) hold two adjacent channels: channel d
 *   of token t is in word t*(D/E) + d/E, with r = d % E, p = r/2, half = r%2.
 *   At bits == 16 this is the plain little-endian half row.
 * Value codes    v_codes  uint32 [batch, Hkv, ceil(n_kept/SB) * 64 * (D/16) * wpt]
 *   Tile-transposed so that the P.V product can read it without a transpose.
 *   SB = 64 tokens at 2 bits, 32 otherwise; wpt = 4 at 16 bits, 2 at 8, else 1.
 *   Token t = SB*sb + 32*blk + 16*H + 4*kb + i  (H in {0,1}; kb, i in 0..3),
 *   channel d = 16*tile + n.  The low/high half-word pair is (H=0, H=1): two
 *   tokens 16 apart of the same channel.  For fixed (kb, d) the fields with
 *   running index run = 4*blk + i fill the half-words in order, E/2 per word:
 *   word-in-tile wl = run / (E/2), field p = run % (E/2).  With
 *   y = tile*wpt + wl the word sits at
 *     sb * (64*(D/16)*wpt) + ((y/4)*64 + kb*16 + n)*4 + y%4 .
 *   Tokens >= n_kept inside the last superblock hold zeros.
 * Key scale/zero k_scale, k_zero  half
 *   per channel: [batch, Hkv, ceil(n_kept/G), D] -- when G does not divide n_kept
 *   the last group holds the remaining n_kept mod G tokens (the same quantizer on
 *   fewer members);  per token: [batch, Hkv, R, D/G]
 * Value scale/zero v_scale, v_zero  half [batch, Hkv, R, D/G]
 *   (absent, size 0, at bits == 16)
 * Tail           tail_k, tail_v  half [batch, Hkv, tail_cap, D], row-major; the
 *   first tail_len rows are attended at full precision after the kept tokens.
 *   kvqp_compress writes the last W prompt rows there (Appendix B keeps the
 *   most recent tokens); a caller may append decoded tokens' K/V rows and
 *   raise tail_len up to tail_cap (the cache update of Eq. (2)).
 *
 * Quantizer, exactly (binary32, round-to-nearest-even, no fused multiply-add):
 *   z = min, m = max of the group (binary16 values, -0 orders below +0);
 *   r = float(m) - float(z);  s32 = r / float(2^bits - 1);  s = half(s32);
 *   s == 0  ->  all codes 0;  else inv = 1.0f / float(s),
 *   code = clamp(rint((float(x) - float(z)) * inv), 0, 2^bits - 1).
 * NaN inputs are not supported.
 *
 * Outlier filtering (Section 6.3, item (1); Appendix B: numbers whose absolute
 * value exceeds 6, about 1 %, are excluded from quantization).  With
 * cfg->outlier_threshold = tau > 0 (bits 2, 4, 8) every element of a kept
 * token's key row or value row with |x| > tau is an outlier, however many a
 * row has.  An outlier takes no part in its group's min / max and gets code 0;
 * a group left with no element stores scale 0, zero +0.  The outlier is kept
 * beside the codes as a 32-bit word: bits 31..8 the top 24 bits of the
 * binary32 difference float(x) - float(z), z the stored zero of the element's
 * group, bit 7 set, bits 6..0 the channel; it dequantizes to float(z) + that
 * difference (within 2^-15 of |x - z|, finer than a binary16 step of x).
 * Where the words are kept:
 *   k_out, v_out  uint32 [batch, Hkv, R, KVQP_OUTLIER_SLOTS]
 *     a row's first KVQP_OUTLIER_SLOTS outliers in ascending order of channel,
 *     unused slots 0;
 *   k_ovf, v_ovf  uint32 [batch, Hkv, S + 2 * cfg->outlier_overflow_cap],
 *     S = R/32 + 1 rounded up to a multiple of 4: per (batch, KV head)
 *     first the int32 prefix counts start[0 .. R/32] -- start[b] = number
 *     of list entries of the head's tokens before 32 b -- then the list: the
 *     outliers beyond their rows' slots as entries (word, token index in the
 *     head), in ascending (token, channel) order.  start[R/32] is the
 *     number of entries the head needs; entries beyond outlier_overflow_cap
 *     are not stored and those elements read as their group's zero, so a
 *     caller that sizes the list below n_kept * (D - KVQP_OUTLIER_SLOTS)
 *     compares that count (device memory) with its capacity.  Words of the
 *     list beyond the stored entries, and of the prefix array beyond
 *     start[R/32], are unspecified.
 *   (sizes from kvqp_outlier_sizes; all four NULL when filtering is off)
 */
#define KVQP_OUTLIER_SLOTS 4
typedef struct kvqp_cache {
    void *k_codes, *v_codes;
    void *k_scale, *k_zero;
    void *v_scale, *v_zero;
    void *tail_k, *tail_v;
    int32_t n_kept;   /* kept low-precision tokens; set by compress / quantize_selected */
    int32_t tail_len; /* valid tail rows                                                */
    int32_t tail_cap; /* allocated tail rows, >= window                                 */
    int32_t n_cap;    /* tokens the six packed buffers are laid out for: every "n_kept"
                         and "R" in the buffer shapes above is n_cap (the stride of the
                         [batch, Hkv] axes); 0 means n_kept, the compact layout of
                         kvqp_cache_sizes.  A larger n_cap (a multiple of 64 and of G,
                         sizes from kvqp_cache_sizes_cap) leaves room for
                         kvqp_append_tail.  Set by the caller, never changed.           */
    int32_t *head_n_kept; /* DEVICE int32 [batch * Hkv] or NULL.  Non-NULL marks a cache with
                         head-level token counts (kvqp_compress_ragged fills it): head h holds
                         head_n_kept[h] <= n_kept tokens at the start of its share of every
                         buffer, and n_kept is only the bound the counts stay under.       */
    void *k_out, *v_out;  /* outlier slots when cfg->outlier_threshold > 0, else unused (NULL) */
    void *k_ovf, *v_ovf;  /* overflow lists of the rows with more outliers than slots (the same) */
} kvqp_cache;

/* Bytes of the eight cache buffers (order of the struct) for n_kept =
 * min(budget, L - W) and the given tail capacity.  Host only. */
int kvqp_cache_sizes(const kvqp_cfg *cfg, int32_t tail_cap, size_t sizes_out[8]);

/* The same for buffers laid out for n_cap tokens per head (n_cap a multiple of 64 and of
 * group_size, >= 0); cfg->seq_len, window and budget are not read.  Host only. */
int kvqp_cache_sizes_cap(const kvqp_cfg *cfg, int32_t n_cap, int32_t tail_cap, size_t sizes_out[8]);

/* Bytes of k_out, v_out, k_ovf and v_ovf for buffers laid out for n_cap tokens per
 * head (n_cap = 0: for n_kept = min(budget, L - W)) and cfg->outlier_overflow_cap
 * list entries; all 0 when cfg->outlier_threshold is 0.  Host only. */
int kvqp_outlier_sizes(const kvqp_cfg *cfg, int32_t n_cap, size_t sizes_out[4]);

/* Workspace bytes needed by kvqp_compress and kvqp_decode_attn for this cfg
 * (either pointer may be NULL).  decode_bytes depends on batch, heads, bits,
 * decode_splits and outlier_threshold only: it serves a cache of any token
 * count, also one that kvqp_append_tail has grown.  Host only. */
int kvqp_workspace_bytes(const kvqp_cfg *cfg, size_t *compress_bytes, size_t *decode_bytes);

/*
 * Prefill-time compression of one layer (Section 3, "Quantized Pruning").
 *
 * Pruning rule (the paper uses an attention-score method from the literature
 * with the last 32 tokens retained, Section 4 / Appendix B, and gives no
 * further detail; this is the rule implemented):
 *   P = L - W.  Every query row of the last W positions, for every query head
 *   of a KV head's group, attends causally over keys 0..P+i with
 *   Softmax(sm_scale q k^T); vote[j], j < P, is the sum of those
 *   probabilities over the group's heads and the W rows; votes are max-pooled
 *   (stride 1, same length, window clipped at the ends); the n_kept highest
 *   pooled scores are kept, equal scores going to the lower position, and the
 *   survivors are stored in ascending position.
 *   Scores are evaluated in binary32 on the matrix cores; candidates whose
 *   pooled score lies within a relative 2e-5 of the cut are re-scored in
 *   binary64 before the cut is made.  The re-scoring holds up to 512 such
 *   candidates and the 2048 distinct positions under their pooling windows
 *   per head; a head with more (e.g. all keys identical) is cut by the
 *   binary32 scores and the position rule, and says so in unrefined_out.
 * The survivors are then quantized as described at kvqp_cache.
 *
 *   q_obs  half [batch, Hq, W, D]   queries of the last W prompt positions
 *   k, v   half [batch, Hkv, L, D]  full prompt keys / values
 *   cache  buffers filled; n_kept and tail_len (= W) set; tail_cap must be set
 *          by the caller and be >= W
 *   idx_out int32 [batch, Hkv, n_kept] ascending survivors, or NULL
 *   unrefined_out int32 [batch, Hkv] or NULL: per head 0 when every candidate
 *          near the cut was re-scored in binary64 (or none needed it), else
 *          the number of candidates near the cut that binary32 decided
 * Errors: INVALID_ARG on NULL/shape problems, UNSUPPORTED outside the
 * supported set, WORKSPACE, HIP.
 */
int kvqp_compress(const kvqp_cfg *cfg, const void *q_obs, const void *k, const void *v,
                  kvqp_cache *cache, int32_t *idx_out, int32_t *unrefined_out, void *workspace,
                  size_t workspace_bytes, void *hip_stream);

/*
 * Compression with a token count of its own for every KV head (Section 5, Q1, and
 * Table 1 evaluate head-level allocation, Ada-KV and HeadKV, which the paper
 * pairs with per-token key groups because the heads keep different numbers of
 * tokens, and PyramidKV, whose count varies by layer; Appendix B gives them a
 * window of 8).  The allocation rule itself is the caller's: this call takes
 * its result.  Scoring, the cut and the quantizer are those of kvqp_compress,
 * applied to head h with head_budget[h] in place of n_kept.
 *   head_budget  HOST int32 [batch * Hkv]; every entry >= 0 and
 *                <= min(cfg->budget, L - W).  Read before the call returns.
 *   cache        as for kvqp_compress with n_kept = min(cfg->budget, L - W) in
 *                every shape (or n_cap); head_n_kept must point to device memory
 *                and receives the counts (a copy enqueued on the stream);
 *                n_kept is set to the bound, tail_len to W.
 *   idx_out      int32 [batch, Hkv, n_kept] or NULL: the first head_budget[h]
 *                entries of head h are its survivors, the rest is unspecified.
 *   unrefined_out as for kvqp_compress.
 * kvqp_decode_attn reads such a cache through head_n_kept (tail_len must be
 * >= 1) and kvqp_append_tail_ragged extends it; kvqp_append_tail does not take
 * one (UNSUPPORTED), and kvqp_compress and kvqp_quantize_selected want
 * head_n_kept == NULL (INVALID_ARG).
 */
int kvqp_compress_ragged(const kvqp_cfg *cfg, const void *q_obs, const void *k, const void *v,
                         const int32_t *head_budget, kvqp_cache *cache, int32_t *idx_out,
                         int32_t *unrefined_out, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * The quantization half alone (Section 3 "KV Quantization" applied to given
 * survivors): idx int32 [batch, Hkv, n_kept] ascending positions < L - W
 * chosen by any pruning method; cfg->budget is ignored and n_kept is taken
 * from the argument.  Fills the cache exactly as kvqp_compress would for the
 * same survivors.  Needs no workspace.
 */
int kvqp_quantize_selected(const kvqp_cfg *cfg, const void *k, const void *v, const int32_t *idx,
                           int32_t n_kept, kvqp_cache *cache, void *hip_stream);

/*
 * The same with a count of its own per KV head (survivors chosen by a
 * head-level method of the caller's): idx int32 [batch, Hkv, n_kept], of which
 * head h uses its first head_count[h] entries; head_count is a HOST array
 * under the rules of kvqp_compress_ragged with n_kept as the bound, and
 * cache->head_n_kept receives it.
 */
int kvqp_quantize_selected_ragged(const kvqp_cfg *cfg, const void *k, const void *v, const int32_t *idx,
                                  int32_t n_kept, const int32_t *head_count, kvqp_cache *cache,
                                  void *hip_stream);

/*
 * One decode step of attention over the compressed cache (Section 3, Eq. (3)
 * on G' = Q(G) s + z): for every query head, softmax over the n_kept
 * dequantized tokens followed by tail_len full-precision rows, no mask.
 * Codes are expanded in registers; no dequantized copy is written.
 *   q   half [batch, Hq, D]
 *   out half [batch, Hq, D]   binary32 accumulation, rounded once at the end
 * cfg fields used: batch, heads, head_dim, bits, group_size, key_axis,
 * decode_splits, sm_scale, outlier_threshold, decode_cache_hint.
 * Reproducibility: the order in which partial sums meet depends on which wave takes
 * which 64-token chunk, so two runs may differ in the last bits of the binary32
 * accumulation (and, rarely, in the rounding of an output); kvqp_compress, by contrast,
 * is bit-for-bit reproducible (indices, codes, scales, zeros, tail).
 * Numerical range: the weights of the value product travel as binary16 numbers inside
 * the kernel, so a value group's scale should stay below 256 (a 2-bit group spanning
 * less than 768, a 4-bit group less than 3840); beyond that a weight can saturate at
 * the binary16 maximum and the output degrades (it stays finite).  Likewise the product
 * of a query element and its channel's key scale must stay inside the binary16 range
 * (|q| * scale < 65504: keys spanning tens of thousands at 2 bits would not).
 * n_kept + tail_len must be >= 1.  With head-level
 * counts (cache->head_n_kept non-NULL) head h attends its first
 * head_n_kept[h] tokens; the counts are read on the device, where a count
 * above n_kept is cut to n_kept.
 * Workspace: kvqp_workspace_bytes' decode_bytes, 16-byte aligned, prepared ONCE with
 * kvqp_decode_workspace_init before its first use.  It holds the partial results of
 * the token-axis splits and, at its head, one arrival counter per (batch, KV head)
 * that is zero between calls (the workgroup that merges a head puts it back).  Calls
 * that use different workspaces are independent and may overlap in time (several
 * streams, several graphs in flight); calls that share one workspace must not
 * overlap (calls issued on one stream never do).
 */
int kvqp_decode_attn(const kvqp_cfg *cfg, const void *q, const kvqp_cache *cache, void *out,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Prepares a decode workspace (the split merge of kvqp_decode_attn, Eq. (3) evaluated
 * in token ranges): zeroes its arrival counters with a small kernel enqueued on the
 * stream.  Needed once after allocation -- fresh device memory holds arbitrary bytes
 * -- and again only if a kvqp_decode_attn launch on this workspace did not run to
 * completion (device reset, aborted process).  cfg fields used: batch, n_kv_heads
 * (the counters of a larger batch * n_kv_heads cover a smaller one).
 * Errors: WORKSPACE when workspace is NULL or smaller than the counters.
 */
int kvqp_decode_workspace_init(const kvqp_cfg *cfg, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/*
 * kvqp_decode_attn for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same result, no workspace: the partial
 * results and arrival counters of the token-axis splits live in an array of
 * KVQP_STATIC_SCRATCH_BYTES that the library owns (static device storage, one
 * copy per GPU the library runs on, held until the process ends).  The call
 * allocates and frees nothing and never synchronises.
 *   - A launch whose splits need more than KVQP_STATIC_SCRATCH_BYTES (see
 *     kvqp_workspace_bytes' decode_bytes) returns KVQP_ERR_WORKSPACE and
 *     launches nothing: use kvqp_decode_attn.
 *   - Every such call on one GPU shares that GPU's array: calls that overlap
 *     in time on one GPU (two streams, two graphs in flight) race.  Calls on
 *     one stream never overlap.
 *   - The first call on a GPU looks the array's address up and zeroes its
 *     counters with a small kernel on the given stream.
 */
#define KVQP_STATIC_SCRATCH_BYTES (8u << 20)
int kvqp_decode_attn_static(const kvqp_cfg *cfg, const void *q, const kvqp_cache *cache, void *out,
                            void *hip_stream);

/*
 * Decode-time cache update (Section 3, Eq. (2): the new token's key and value
 * are concatenated to the cache; the paper's quantizer, KIVI, keeps the most
 * recent tokens in full precision and quantizes them group by group).  The
 * caller appends each decoded token's K/V row to the tail and raises tail_len;
 * this call moves the n_tokens OLDEST tail rows into the low-precision part:
 * they are quantized and packed exactly as kvqp_quantize_selected would have
 * done had they been survivors n_kept .. n_kept + n_tokens - 1, the remaining
 * tail rows move down, and n_kept / tail_len are updated.
 *   n_tokens  > 0, <= tail_len, and a multiple of q; n_kept must be a multiple
 *             of q too and n_kept + n_tokens <= n_cap, where q is 32, raised to
 *             64 for 2-bit caches and to a multiple of group_size for
 *             per-channel keys (whole key groups, whole value superblocks).
 * cfg fields used: batch, heads, head_dim, bits, group_size, key_axis.
 * Errors: INVALID_ARG when the counts do not fit the rules above.
 */
int kvqp_append_tail(const kvqp_cfg *cfg, kvqp_cache *cache, int32_t n_tokens, void *hip_stream);

/*
 * The same update for a cache with head-level counts (Section 3, Eq. (2) on a
 * cache filled by kvqp_compress_ragged): every head takes the n_tokens oldest
 * tail rows onto the end of ITS OWN packed part, so head h grows from
 * head_count[h] to head_count[h] + n_tokens tokens; the bound n_kept grows by
 * n_tokens and tail_len shrinks by it.
 *   head_count  HOST int32 [batch * Hkv]: the heads' CURRENT counts (the array
 *               given to kvqp_compress_ragged, plus earlier appends).  Every
 *               entry a multiple of q (as for kvqp_append_tail) and <= n_kept.
 *               Read before the call returns; cache->head_n_kept receives the
 *               new counts (a copy enqueued on the stream).  The quantizer
 *               takes a head's position from the device copy, cut to n_kept
 *               and rounded down to a multiple of q, so an array that differs
 *               from the device's misplaces tokens but never leaves the buffers.
 *   n_tokens    as for kvqp_append_tail, with n_kept + n_tokens <= n_cap.
 * Errors: INVALID_ARG as above, or when cache->head_n_kept is NULL.
 */
int kvqp_append_tail_ragged(const kvqp_cfg *cfg, kvqp_cache *cache, int32_t n_tokens,
                            const int32_t *head_count, void *hip_stream);

/* Static string for a return code. */
const char *kvqp_strerror(int code);

/* Library version, major*10000 + minor*100 + patch. */
int kvqp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVQP_H */
