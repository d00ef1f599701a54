/*
 * libqaq -- quality-adaptive quantization of an LLM KV cache and the decode-step
 * attention that reads it, for AMD MI355X (gfx950).
 *
 * Method: "QAQ: Quality Adaptive Quantization for LLM KV Cache" (arXiv 2403.04643).
 * Section / equation references below are to that paper.
 *
 * Conventions for every entry point
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host" pointers
 *     are ordinary host memory.  The library never frees or keeps caller tensors
 *     beyond the call, except the arena given to qaq_create, which it uses until
 *     qaq_destroy (and never frees).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue kernels on it and return; they do not synchronise, and after
 *     qaq_create they allocate nothing.  (qaq_create and qaq_stats do synchronise.)
 *   - Tensors are row-major with the head dimension D innermost.  fp16 is IEEE
 *     binary16.  All sequences of the batch have the same length unless
 *     qaq_set_shortfall says otherwise; a length argument is then the longest
 *     sequence's, and arrays are padded to it.
 *   - Return value: QAQ_OK (0) or a negative qaq_status.  Arguments are validated on
 *     the host without reading device memory; nothing crosses the ABI as an
 *     exception or abort.  qaq_last_error() gives a thread-local description.
 *   - Not checked: that inputs are finite, and that width arrays only hold members
 *     of the configured bit set.
 *   - Calls on one cache must be ordered by the caller (same stream, or events).
 */
#ifndef QAQ_H
#define QAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QAQ_OK = 0,
  QAQ_ERR_INVALID_ARG = -1,
  QAQ_ERR_CAPACITY = -2,     /* more tokens than max_tokens, or arena too small */
  QAQ_ERR_HIP = -3,          /* a HIP runtime call failed */
  QAQ_ERR_NEED_ORIGINAL = -4 /* reserved: widening without the unquantized copy is
                                refused per token and counted in qaq_stats, not failed */
} qaq_status;

typedef struct qaq_cache qaq_cache; /* opaque host-side descriptor */

enum { QAQ_WINDOW_FP32 = 0, QAQ_WINDOW_FP16 = 1, QAQ_WINDOW_BF16 = 2 };

typedef struct {
  int32_t batch;          /* B, number of sequences                                   */
  int32_t n_q_heads;      /* Hq, a multiple of n_kv_heads                             */
  int32_t n_kv_heads;     /* Hkv                                                      */
  int32_t head_dim;       /* D: 64 or 128                                             */
  int32_t max_tokens;     /* capacity per sequence (rounded up to a tile of 256)      */
  int32_t bit_set[5];     /* allowed code widths, ascending, a subset of {1,2,3,4,8}
                             (the paper's experiments: {2,3,4,8}; 1 is a variant)     */
  int32_t n_bits;         /* how many entries of bit_set are used (1..5)              */
  float   outlier_frac;   /* alpha, total over both ends (Section 4.2 "Outliers");
                             the paper's experiments use 0.01                        */
  int32_t n_outlier_per_side; /* <0: ceil(outlier_frac/2 * D); 0: none; at most 4     */
  int32_t window;         /* n of the attention window (Section 3.2); 1..8; paper: 5  */
  int32_t window_store;   /* how the window keeps its score rows: QAQ_WINDOW_FP32, or
                             (variants) QAQ_WINDOW_FP16 / QAQ_WINDOW_BF16: rounded to
                             nearest even when they are stored -- the predicted score is
                             the maximum of the stored values, the current step's
                             included                                                 */
  double  sigma_s_max;    /* bound on the std of a score   (Section 4.1, key rule)    */
  double  sigma_x_max;    /* bound on the std of an output (Section 4.1, value rule)  */
  const float* qnorm2;    /* host [n_kv_heads]: statistic of sum_d Q_d^2 used by the key
                             rule (the paper takes the upper-10% quantile), with the
                             query already carrying the softmax's 1/sqrt(D), i.e.
                             quantile(|q|^2) / D.  Copied by qaq_create.              */
  const float* outlier_thresholds; /* NULL: the count rule above.  Else (variant, Section 4.2
                             "Outliers" read literally) host [2 (K, V)][n_kv_heads][2 (lo, hi)],
                             lo <= hi, copied by qaq_create: the outliers of a token are its
                             values above hi or below lo, so their number varies per token;
                             a token keeps at most n_outlier_per_side per end (1..4; the
                             largest above hi, the smallest below lo), the others widen its
                             [min,max].  The side store is then variable-length: per token an
                             offset and a count into a per-tile pool of (channel, value).   */
} qaq_config;

typedef struct {
  int64_t tokens;            /* cached positions per sequence                         */
  int64_t hist_k[5];         /* token-heads per width, in the order {2,3,4,8,1}       */
  int64_t hist_v[5];
  int64_t code_bytes;        /* sum over token-heads of D*(bK+bV)/8 (Section 2.1:
                                memory "calculated by the quantized bit")             */
  int64_t layout_code_bytes; /* bytes the device layout actually reads for codes      */
  int64_t meta_bytes;        /* min/max, order bytes, outlier side store              */
  int64_t fp16_bytes;        /* the same tokens as an fp16 cache                      */
  int64_t refused_upgrades;  /* widenings asked for without an unquantized copy       */
  int64_t served_upgrades;   /* widenings done from the unquantized copy (each one reads
                                one fp16 token vector of it), since qaq_create           */
  int64_t update_handovers;  /* tile sides (of 2 * B * Hkv * tiles) that the last
                                qaq_decode_update rebuilt with the general kernel instead
                                of its decode-step kernel (too many tokens moved at once,
                                or a code region had to move with tokens in it)          */
} qaq_stats_t;

/* Bytes of device memory the cache needs for this configuration (worst case: every
 * token at the widest code).  0 if the configuration is invalid. */
size_t qaq_arena_bytes(const qaq_config* cfg);

/* Creates an empty cache inside `dev_arena` (at least qaq_arena_bytes, 256-byte
 * aligned).  Clears the arena's bookkeeping on the default stream and waits for it. */
int qaq_create(const qaq_config* cfg, void* dev_arena, size_t arena_bytes, qaq_cache** out);
int qaq_destroy(qaq_cache* c);

/* Forget all tokens and the score window (host bookkeeping only); the sequences have one
 * length again (see qaq_set_shortfall). */
int qaq_reset(qaq_cache* c);

/* Number of cached positions of the longest sequence (of every sequence, unless
 * qaq_set_shortfall made them differ). */
int qaq_length(const qaq_cache* c, int32_t* host_len);

/* Number of cached positions of every sequence: host_len int32 [batch]. */
int qaq_lengths(const qaq_cache* c, int32_t* host_len);

/* Sequences of different lengths (Section 5.1 evaluates one prompt at a time; a served batch
 * mixes prompt lengths, and the rules of Section 4.1 depend on each sequence's own token count T).
 * Declares, for an EMPTY cache with an empty window, that sequence b will always be
 * host_shortfall[b] tokens shorter than the longest one.  From then on every length that the
 * caller passes or reads (n_new of the first append, T of qaq_prefill_window, qaq_length, the
 * strides of bit, score and original-copy arrays) is the longest sequence's, and sequence b
 * has max(length - host_shortfall[b], 0) tokens: of a [.., length, ..] input or output only
 * its first that-many positions are read or written (the rest is padding and is left alone),
 * its thresholds tau_K(T, h) and c_V(T) take its own T, its softmax runs over its own tokens, and
 * in a score row with a new token that token's score sits right after its own cached tokens.
 * Every later append and decode step adds the same number of tokens to all sequences.
 *   host_shortfall  int32 [batch], >= 0, at least one 0, all < max_tokens; all 0 = one length
 * The first append must be longer than the largest shortfall (no sequence stays empty), and
 * a prompt must leave the shortest sequence at least n_rows tokens in qaq_prefill_window.
 * Limits: batch <= 64 and batch * n_kv_heads <= 256 when any shortfall is positive (the
 * per-sequence thresholds travel as kernel arguments).  QAQ_ERR_INVALID_ARG if the cache is not
 * empty or a limit is exceeded. */
int qaq_set_shortfall(qaq_cache* c, const int32_t* host_shortfall);

/* Change the two hyper-parameters of Section 4.1 between calls. */
int qaq_set_sigmas(qaq_cache* c, double sigma_s_max, double sigma_x_max);

/* The fp32 thresholds qaq_select_bits compares against when T tokens are attended:
 * tau_k[h] = 2*sqrt(3)*sigma_K(T, h) with sigma_K^2 = log(T^3/(T-1)*sigma_Smax^2 + 1)/qnorm2[h]
 * (last display of "Key cache quantization"), and c_v = 2*sqrt(3)*sigma_Xmax/sqrt(T)
 * (display of "Value cache quantization" combined with the bit formula of "Determining
 * quantization bits").  Computed in double, rounded once.  host_tau_k: [n_kv_heads]. */
int qaq_thresholds(const qaq_cache* c, int32_t T, float* host_tau_k, float* host_c_v);

/* Section 4.2 "Outliers" + Section 4.1 "Determining quantization bits": append n_new
 * tokens per sequence.  For every token vector the n_o largest and n_o smallest
 * entries go to the fp16 side store, [min,max] is taken over the rest, and all D
 * entries are coded with 2^B equal segments.
 *   dev_k, dev_v       fp16 [B, Hkv, n_new, D]
 *   dev_k_bits/v_bits  uint8 [B, Hkv, n_new] widths, or NULL = widest of the bit set
 * QAQ_ERR_CAPACITY if the cache would exceed max_tokens. */
int qaq_quantize_append(qaq_cache* c, const void* dev_k, const void* dev_v, int32_t n_new,
                        const uint8_t* dev_k_bits, const uint8_t* dev_v_bits, void* stream);

/* Section 4.1 bit rules + Section 4.2 "Attention score prediction": record one row of
 * attention scores in the window and compute the width of every cached token.
 *   dev_scores  fp32 [B, Hq, T] normalised scores of the last decode step over the T
 *               cached tokens (T = qaq_length), or NULL = use the window as it is.
 *               For grouped queries the maximum over the heads of a KV head is kept.
 *   dev_k_bits, dev_v_bits  out, uint8 [B, Hkv, T].
 * The predicted score of a token is the maximum over the last `window` rows that
 * cover it.  Widths: the smallest b of the bit set with range_K <= 2^b*tau_k, resp.
 * range_V * score <= 2^b*c_v (the printed ceil(log2(.)) written as comparisons),
 * the widest if none qualifies. */
int qaq_select_bits(qaq_cache* c, const float* dev_scores, uint8_t* dev_k_bits,
                    uint8_t* dev_v_bits, void* stream);

/* Section 4.2 "Integration in text generation process": move every cached token to
 * the requested width.  Narrowing drops low code bits in place.  Widening re-encodes
 * from the caller's unquantized copy with the stored [min,max] and outlier set.
 *   dev_k_bits, dev_v_bits  uint8 [B, Hkv, T] (either may be NULL = leave that side)
 *   dev_k_orig, dev_v_orig  fp16 [B, Hkv, orig_tokens, D] unquantized copies (the first T
 *                           rows of each head are used; orig_tokens >= T lets the caller
 *                           keep them in a buffer sized for the whole generation), or
 *                           NULL: tokens asked to widen keep their width and are counted. */
int qaq_requantize(qaq_cache* c, const uint8_t* dev_k_bits, const uint8_t* dev_v_bits,
                   const void* dev_k_orig, const void* dev_v_orig, int32_t orig_tokens,
                   void* stream);

/* Section 2.1 (prompt encoding) with Section 4.2 "Attention score prediction": when generation
 * starts, the scores each prompt token received in the last n steps are the last n rows of
 * the prompt's causal score matrix.  Computes those rows from the unquantized keys (a token
 * attends to itself and to the tokens before it; row i belongs to prompt position
 * T - n_rows + i and covers T - n_rows + i + 1 tokens) and makes them the window.  The cache
 * must be empty; follow with qaq_quantize_append_selected (or qaq_quantize_append and
 * qaq_select_bits(NULL)).
 *   dev_q_last      fp16 [B, Hq, n_rows, D], queries of the last n_rows prompt positions,
 *                   1 <= n_rows <= min(window, T), 16-byte aligned
 *   dev_k           fp16 [B, Hkv, T, D], 16-byte aligned
 *   dev_scores_out  fp32 [n_rows][B, Hq, T], required (it is also the kernels' working
 *                   buffer); entries of a row past its length are 0 */
int qaq_prefill_window(qaq_cache* c, const void* dev_q_last, int32_t n_rows, const void* dev_k, int32_t T,
                       float* dev_scores_out, void* stream);

/* Section 4.2 (outliers, then the quantizer of Section 4.1) at the widths of Section 4.1's
 * rules: appends n_new tokens, each at the width the key rule resp. the value rule gives for
 * its range, the window as it stands (a token no row covers has predicted score 0) and
 * T = tokens after the append.  Same result as qaq_quantize_append at the widest width +
 * qaq_select_bits(NULL) + qaq_requantize restricted to the new tokens; cached tokens are not
 * touched.
 *   dev_k, dev_v            fp16 [B, Hkv, n_new, D], 16-byte aligned
 *   dev_k_bits, dev_v_bits  out, uint8 [B, Hkv, n_new], or NULL */
int qaq_quantize_append_selected(qaq_cache* c, const void* dev_k, const void* dev_v, int32_t n_new,
                                 uint8_t* dev_k_bits, uint8_t* dev_v_bits, void* stream);

/* Section 4.2 "Integration in text generation process", the part of one decode step that
 * follows the attention, in one pass over the cache: record this step's scores in the
 * window, append the new token, compute the width of every token (the new one included) by
 * the bit rules, and move every token to its width.  Same result as qaq_quantize_append of
 * the new token (at the widest width) + qaq_select_bits(dev_scores) + qaq_requantize.
 *   dev_scores  fp32 [B, Hq, T+1] normalised scores of this step, the new token last
 *               (what qaq_decode_attention emits when it is given the new token)
 *   dev_k_new, dev_v_new    fp16 [B, Hkv, D], 16-byte aligned
 *   dev_k_orig, dev_v_orig  fp16 [B, Hkv, orig_tokens, D] unquantized copies of the T cached
 *                           tokens (orig_tokens >= T+1), or NULL as for qaq_requantize.  The
 *                           call writes the new token into row T of each ("copy the
 *                           unquantized new KV" of the same passage) and reads the rows of
 *                           the tokens that widen.  Any memory the device can address
 *                           serves: HBM, or host memory from qaq_host_alloc (then these two
 *                           accesses are the transfers between CPU and GPU the passage
 *                           speaks of, made by the kernel itself, row by row).
 *   dev_k_bits, dev_v_bits  out, uint8 [B, Hkv, T+1], or NULL
 * Returns QAQ_ERR_CAPACITY and changes nothing if the token does not fit. */
int qaq_decode_update(qaq_cache* c, const float* dev_scores, const void* dev_k_new, const void* dev_v_new,
                      void* dev_k_orig, void* dev_v_orig, int32_t orig_tokens,
                      uint8_t* dev_k_bits, uint8_t* dev_v_bits, void* stream);

/* Section 4.2 "Integration": the unquantized copies may live in CPU memory.  Allocates
 * `bytes` of page-locked host memory that the device can address and returns both views of
 * it: *host_ptr for the CPU (owned by the caller until qaq_host_free), *dev_ptr for the
 * dev_*_orig arguments of qaq_requantize and qaq_decode_update.  The contents are undefined. */
int qaq_host_alloc(size_t bytes, void** host_ptr, void** dev_ptr);
int qaq_host_free(void* host_ptr);

/* Section 2.1 attention over the quantized cache for one new query per head:
 * S = softmax(q K^^T / sqrt(D)), X = S V^, with K^, V^ the midpoint reconstruction and
 * outlier channels at their stored fp16 value.  If dev_k_new/dev_v_new are given, that
 * token takes part unquantized as position T (Section 4.2: the new token "combined
 * with the quantized KV cache of previous tokens"); it is not appended.
 *   dev_q       fp16 [B, Hq, D]
 *   dev_k_new, dev_v_new  fp16 [B, Hkv, D], both or neither
 *   dev_out     [B, Hq, D], fp32 if out_is_fp32 else fp16
 *   dev_scores_out  fp32 [B, Hq, T(+1)] normalised scores, or NULL
 * QAQ_ERR_INVALID_ARG if the cache is empty and no new token is given. */
int qaq_decode_attention(qaq_cache* c, const void* dev_q, const void* dev_k_new,
                         const void* dev_v_new, void* dev_out, int32_t out_is_fp32,
                         float* dev_scores_out, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace at the moment of the
 * call (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * qaq_decode_attention with the same arguments, results and errors, except that where a
 * head's tiles are scanned by more than four workgroups (long contexts with few heads: the
 * scan kernel is then followed by a merge kernel) the partial results (max, sum, output per
 * part, fp32) go to a file-scope device array of the library instead of the cache's arena.
 * That array has qaq_static_scratch_limit() bytes (1 MiB; every GPU the library runs on
 * holds one copy until the process ends) and needs B*Hq*parts*(D+4)*4 of them.  The library
 * cuts a call into at most four parts per compute unit (1024 on MI355X: 528 KiB at D = 128)
 * unless a part would then hold more than 64 tiles of 256 tokens; QAQ_ERR_CAPACITY, nothing
 * launched, if such a shape needs more than the array has.  The call itself allocates nothing and calls no allocating routine.  All calls on
 * one GPU share the array (nothing in it has to start at zero: every entry a call reads it
 * has written before), so two such calls that overlap on one GPU -- different streams,
 * different caches -- race; order them. */
int qaq_decode_attention_static(qaq_cache* c, const void* dev_q, const void* dev_k_new,
                                const void* dev_v_new, void* dev_out, int32_t out_is_fp32,
                                float* dev_scores_out, void* stream);
size_t qaq_static_scratch_limit(void);

/* Midpoint reconstruction of positions [t0, t1) with outliers restored exactly
 * (Section 4.1 / 4.2), rounded to fp16.  dev_k_out/dev_v_out: fp16 [B, Hkv, t1-t0, D],
 * either may be NULL. */
int qaq_dequantize(qaq_cache* c, int32_t t0, int32_t t1, void* dev_k_out, void* dev_v_out,
                   void* stream);

/* Layout-independent view of one side (side 0 = keys, 1 = values) for tests and
 * export, by position:
 *   dev_bits   uint8 [B, Hkv, T]
 *   dev_minmax fp16  [B, Hkv, T, 2]
 *   dev_oidx   uint8 [B, Hkv, T, 2*n_o] outlier channels, ascending
 *   dev_oval   fp16  [B, Hkv, T, 2*n_o]
 *   dev_codes  uint8 [B, Hkv, T, D]: the first D*B/8 bytes of a row are the token's
 *              codes as a little-endian bit string (channel d at bits [d*B,(d+1)*B)),
 *              the rest of the row is zero.
 * Any output pointer may be NULL. */
int qaq_export_canonical(qaq_cache* c, int32_t side, uint8_t* dev_bits, void* dev_minmax,
                         uint8_t* dev_oidx, void* dev_oval, uint8_t* dev_codes, void* stream);

/* Width histogram and byte accounting.  Runs a small kernel on `stream` and waits. */
int qaq_stats(qaq_cache* c, qaq_stats_t* host_out, void* stream);

/* Number of outliers kept per end of a token vector for this configuration. */
int qaq_outliers_per_side(const qaq_config* cfg);

const char* qaq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QAQ_H */
