/*
 * rkv - RotateKV's 2-bit KV-cache hot path for AMD MI355X (gfx950), C ABI.
 *
 * The library implements the write half and the read half of RotateKV (arXiv 2501.16383):
 *   write  (Sec. 4.1, 4.2, 4.4; Eq. 6-9): grouped-head Walsh-Hadamard rotation of pre-RoPE keys,
 *          calibrated channel reorder, per-token asymmetric 2-bit quantization in blocks of 128
 *          with a scale and an integer zero-point per block (fp16 + fp16, or FP8 + INT8 as in
 *          the quantization settings of Sec. 5.1: rkv_config.meta_format), attention-sink tokens
 *          kept in fp16 (Sec. 4.3);
 *   read   (decoding phase, Eq. 4-5; the online steps of Sec. 4.4 undone):
 *          dequantize, undo reorder and rotation, RoPE, softmax(q.K^T/sqrt(d)).V.
 *
 * General rules
 *   - Every pointer named dev_* is DEVICE memory owned by the caller; host_* is host memory.
 *     The library never allocates or frees device memory: the cache lives in a block the caller
 *     hands to rkv_cache_create, work space comes in through dev_scratch.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Unless stated
 *     otherwise a call only enqueues work on that stream and returns without synchronising.
 *   - Every call returns RKV_OK (0) or a negative error code; nothing is thrown across the ABI.
 *     On RKV_EHIP the HIP error is left readable through hipGetLastError.
 *   - One cache object holds one layer.  All sequences of a cache have the same length unless
 *     rkv_quantize_append_ragged has given them lengths of their own.
 *   - Tensors are dense, row-major, in the index order written next to each argument.
 *     A token's keys/values are [n_kv_heads][head_dim] (head-major), E = n_kv_heads*head_dim.
 *   - Keys are given and stored PRE-RoPE; RoPE is applied inside rkv_decode_attention to the
 *     query (at q_pos) and to every cached key (at its 0-based token index).
 */
#ifndef RKV_H_
#define RKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RKV_OK         0
#define RKV_EINVAL    (-1)  /* null pointer, unsupported shape or option, size too small          */
#define RKV_ECAPACITY (-2)  /* append past max_tokens                                            */
#define RKV_EPERM     (-3)  /* reorder indices are not a permutation or leave their perm_span    */
#define RKV_EHIP      (-4)  /* a HIP call or kernel launch failed                                */
#define RKV_ESTATE    (-5)  /* call not valid in the cache's current state (e.g. empty cache)    */
#define RKV_ESCRATCH  (-6)  /* rkv_decode_attention_static: built-in work space too small        */

typedef struct rkv_config {
  int32_t batch;        /* sequences per cache, >= 1                                             */
  int32_t n_q_heads;    /* query heads; multiple of n_kv_heads (GQA: query head h reads KV head  */
                        /* h / (n_q_heads / n_kv_heads))                                          */
  int32_t n_kv_heads;
  int32_t head_dim;     /* 128                                                                   */
  int32_t max_tokens;   /* capacity per sequence, 1..65536                                       */
  int32_t max_sinks;    /* fp16 sink rows kept per sequence (0..64)                              */
  int32_t rot_heads;    /* consecutive KV heads rotated together (Sec. 4.2): 1, 2, 4 or 8;       */
                        /* must divide n_kv_heads                                                */
  int32_t quant_group;  /* channels per quantization block: 128 (Sec. 5.1 quantization settings), */
                        /* 64 or 32 (Table tab:quantgrani)                                       */
  int32_t bits;         /* bits per code: 2 (the headline setting), 3 or 4 (Table tab:ablation). */
                        /* 3- and 4-bit codes in groups of 128 run on the matrix-core kernels    */
                        /* like 2-bit ones (the bits above the low two as a second plane);       */
                        /* groups of 64 / 32 have variants of the matrix-core kernels for every  */
                        /* code width, either metadata format and every reorder (rot_heads 2, 4) */
  int32_t perm_span;    /* reorder indices stay inside blocks of this many channels:            */
                        /* head_dim, rot_heads*head_dim, or n_kv_heads*head_dim (Alg. 1 as       */
                        /* printed sorts the whole row).  The append kernel for a reorder across */
                        /* rotation groups holds U = max(perm_span, rot_heads*head_dim) channels */
                        /* of 16 tokens in LDS: 24 U bytes (30 U with 3-bit, 32 U with 4-bit     */
                        /* codes) must not exceed 160 KB, else RKV_EINVAL from rkv_query_sizes   */
                        /* and rkv_cache_create (whole-row reorder: at most 53 KV heads, 40 with */
                        /* 4-bit codes).  Not so where every reorder has a matrix-core append    */
                        /* kernel (quant_group 128, rot_heads 2 or 4, v_rotate 0,                */
                        /* keys_rotated 0): up to 127 KV heads                                    */
  int32_t rope_style;   /* 0: channel j pairs with j+64; 1: channel 2j pairs with 2j+1          */
  int32_t v_rotate;     /* 0: values are quantized as given (the caller has folded the value    */
                        /* rotation of Sec. 4.4 into its weights); 1: the library applies a      */
                        /* per-head Hadamard before quantizing and undoes it on the output       */
  float   rope_theta;   /* RoPE base, e.g. 10000 or 500000                                       */
  float   clip_ratio;   /* 1.0 (Eq. 8-9 with no clipping)                                        */
  int32_t keys_rotated; /* 0: keys arrive in the original basis and are rotated and reordered    */
                        /* here; 1: they come from a projection with rotation and reorder folded */
                        /* in (Sec. 4.2; rkv_fold_rotation) and already are what enters Eq. 6.   */
                        /* Needs rot_heads 2 or 4, perm_span = head_dim, v_rotate = 0.  A        */
                        /* retained sink row is brought back to the original basis and rounded   */
                        /* to fp16                                                               */
  int32_t meta_format;  /* storage of each block's scale and zero-point (Eq. 8-9):               */
                        /* 0: fp16 + fp16, 2.25 bits per element with the codes;                 */
                        /* 1: FP8 + INT8 (Sec. 5.1 quantization settings), 2.125 bits: the scale */
                        /* is rounded UP to the next FP8 E4M3 number (at most 448) and is the    */
                        /* one Eq. 6 divides by, so 3 steps still cover the block; zero-points   */
                        /* are clamped to -128..127 (+-2048 with format 0)                       */
} rkv_config;

typedef struct rkv_cache rkv_cache;   /* opaque host object */

/* Bytes of device memory a cache needs (cache_bytes, for rkv_cache_create) and bytes of work
 * space rkv_decode_attention / rkv_calibrate_perm need (scratch_bytes).  Either out-pointer may
 * be NULL.  RKV_EINVAL if cfg is unsupported. */
int rkv_query_sizes(const rkv_config* cfg, size_t* cache_bytes, size_t* scratch_bytes);

/* Bind a cache to caller-owned device memory (256-byte aligned, >= cache_bytes).  Zero-fills the
 * block, writes the identity reorder and the RoPE angle table on `stream`.  *out is a small host
 * object; free it with rkv_cache_destroy (which never touches dev_mem). */
int rkv_cache_create(const rkv_config* cfg, void* dev_mem, size_t bytes, void* stream, rkv_cache** out);
void rkv_cache_destroy(rkv_cache* cache);

/* Forget all tokens and sinks (length 0); keeps the reorder indices. */
int rkv_cache_reset(rkv_cache* cache, void* stream);

/* Tokens currently cached per sequence (host-side count; of the longest sequence once lengths
 * differ), or RKV_EINVAL. */
int rkv_cache_length(const rkv_cache* cache);

/* The same per sequence: host_lengths [batch] int32 (host memory). */
int rkv_cache_lengths(const rkv_cache* cache, int32_t* host_lengths);

/* Shorten sequences: sequence b keeps its first host_new_lengths[b] tokens (0 <= new <= current
 * length, else RKV_EINVAL and nothing changes); retained sink rows at or behind the new end are
 * dropped.  This is the roll-back after a multi-token step whose later tokens were rejected
 * (speculative decoding with rkv_decode_attention_multi); the slots are reused by later appends.
 * If the new lengths differ the cache continues with per-sequence lengths, under the conditions
 * of rkv_quantize_append_ragged.
 *   host_new_lengths  [batch] int32 in host memory; read before the call returns */
int rkv_cache_truncate(rkv_cache* cache, const int32_t* host_new_lengths, void* stream);

/* Calibration for reordering indices (Alg. 1): rotate the calibration keys with the grouped-head
 * Hadamard, sum every channel over all tokens (signed, float64), and sort channel indices by that
 * sum - ascending, stable, inside each perm_span block.
 *   dev_k_cal      [n_tok][n_kv_heads][head_dim] fp16, pre-RoPE
 *   dev_perm_out   [E] int32: reordered channel i takes rotated channel perm[i]
 *   dev_scratch    >= scratch_bytes of rkv_query_sizes
 * cfg->batch, max_tokens and max_sinks are ignored. */
int rkv_calibrate_perm(const rkv_config* cfg, const void* dev_k_cal, int32_t n_tok,
                       int32_t* dev_perm_out, void* dev_scratch, void* stream);

/* Offline folding of the key rotation and reorder into a projection (Sec. 4.2, Sec. 4.4): for a
 * matrix with the E key channels along its rows' last axis (keys = x . W), every row is rotated by
 * the grouped-head Hadamard and reordered, so that x . W' = reorder(rotate(x . W)).
 *   dev_w, dev_w_out  [rows][E] fp32 (may be the same buffer)
 *   dev_perm          [E] int32 reorder indices, or NULL for none
 * Only n_kv_heads, head_dim and rot_heads of cfg are used (rot_heads = 1 and no perm fold the value
 * rotation).  RKV_EINVAL if E * 4 bytes exceed the LDS of a compute unit. */
int rkv_fold_rotation(const rkv_config* cfg, const float* dev_w, int32_t rows, const int32_t* dev_perm, float* dev_w_out,
                      void* stream);

/* Install reorder indices (Sec. 4.1).  Only valid on an empty cache.  Copies the indices to the
 * host to validate them (synchronises `stream`): RKV_EPERM if they are not a permutation of
 * 0..E-1 or move a channel out of its perm_span block. */
int rkv_set_perm(rkv_cache* cache, const int32_t* dev_perm, void* stream);

/* Attention-sink identification (Sec. 4.3, Fig. 3): the k tokens of every sequence with the most
 * massive activations in a caller-chosen activation tensor (the paper uses the output of the
 * previous decoder block).  A token's score is its largest |activation|; ties go to the lower token
 * index; indices come back in ascending order.
 *   dev_x         [batch][n_tok][width] fp16, width a multiple of 8
 *   dev_idx_out   [batch][k] int32, 1 <= k <= min(64, n_tok)
 *   dev_mask_out  [batch][n_tok] uint8 or NULL: 1 at the chosen tokens, 0 elsewhere - the form
 *                 rkv_quantize_append takes as dev_sink_mask
 *   dev_scratch   >= batch * n_tok * 4 bytes */
int rkv_select_sinks(const void* dev_x, int32_t batch, int32_t n_tok, int32_t width, int32_t k, int32_t* dev_idx_out,
                     uint8_t* dev_mask_out, void* dev_scratch, void* stream);

/* Write half: compress n_new tokens per sequence and append them at the current length.
 *   dev_k, dev_v    [batch][n_new][n_kv_heads][head_dim] fp16, keys pre-RoPE
 *   dev_sink_mask   [batch][n_new] uint8 or NULL; a non-zero entry marks an attention-sink token
 *                   (Sec. 4.3) whose original fp16 rows are kept.  While a sequence already holds
 *                   max_sinks sinks, further marked tokens are treated as ordinary tokens.
 * Works for one token (decode step) or many (prefill).  RKV_ECAPACITY past max_tokens. */
int rkv_quantize_append(rkv_cache* cache, const void* dev_k, const void* dev_v, int32_t n_new,
                        const uint8_t* dev_sink_mask, void* stream);

/* The same for sequences of different lengths (a batch of prompts, sequences that join a running
 * batch): sequence b appends the first host_n_new[b] of its n_new_max rows at its own length.
 * From then on every sequence has its own length: appends go to each sequence's own end, decode
 * attention reads each sequence's own tokens (default query position: its own last token), and
 * a sequence of length 0 makes decode return RKV_ESTATE.
 *   dev_k, dev_v    [batch][n_new_max][n_kv_heads][head_dim] fp16; rows beyond host_n_new[b] are not read
 *   host_n_new      [batch] int32 in host memory, 0 <= host_n_new[b] <= n_new_max; read before the call returns
 *   dev_sink_mask   [batch][n_new_max] uint8 or NULL
 * Needs a configuration the matrix-core append kernel covers (a reorder inside the rotation groups -
 * or anywhere in the row -, rot_heads 2 or 4, v_rotate 0),
 * else RKV_EINVAL; RKV_ECAPACITY if any sequence would pass
 * max_tokens (nothing is appended then).  rkv_import_codes returns RKV_ESTATE on such a cache;
 * the export and dequantize views cover rkv_cache_length tokens for every sequence, and what they
 * show past a sequence's own length is unspecified. */
int rkv_quantize_append_ragged(rkv_cache* cache, const void* dev_k, const void* dev_v, int32_t n_new_max,
                               const int32_t* host_n_new, const uint8_t* dev_sink_mask, void* stream);

/* Read half: one decode step of attention over the whole cache (Eq. 5).
 *   dev_q      [batch][n_q_heads][head_dim] fp16, pre-RoPE
 *   dev_q_pos  [batch] int32 position of the query token, or NULL for (length - 1)
 *   dev_out    [batch][n_q_heads][head_dim] fp32
 *   dev_lse    [batch][n_q_heads] fp32 log-sum-exp of the scaled scores, or NULL
 *   dev_scratch >= scratch_bytes of rkv_query_sizes; calls sharing a scratch block must be
 *              ordered on one stream.
 * RKV_ESTATE on an empty cache. */
int rkv_decode_attention(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos,
                         float* dev_out, float* dev_lse, void* dev_scratch, void* stream);

/* rkv_decode_attention for callers that cannot allocate or hand over a work space: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The prepared queries and
 * the split-K partials go to a work space built into the library (a device array of
 * RKV_STATIC_SCRATCH_BYTES, one copy per GPU, held until the process ends) instead of dev_scratch;
 * the call allocates and frees nothing.  Same arguments otherwise, same kernels, same results bit
 * for bit.  RKV_ESCRATCH - and nothing enqueued - if this call needs more than the built-in space:
 * 2560 bytes per (sequence, query head) plus 528 bytes per (sequence, query head, chunk of 256
 * cached tokens; of 128 on the general kernel), e.g. 7 MB for batch 16 x 40 heads x 4096 tokens.
 * With a reorder that crosses blocks of 128 (inside the rotation groups or over the whole row), or
 * groups of 64 / 32, on the matrix-core path the scores pass through the work space as well: the partials then count the chunks of max_tokens, and 4 bytes
 * per (sequence, query head, token slot of max_tokens rounded up to 256) come on top.
 * All calls on one GPU share that GPU's array and it keeps the last call's contents (nothing in
 * it needs clearing: every partial a call reads it has written first): calls that overlap on one
 * GPU - different streams, different caches - race; order them on one stream.  The device that
 * was current at rkv_cache_create must be current. */
#define RKV_STATIC_SCRATCH_BYTES (24u << 20)
int rkv_decode_attention_static(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos,
                                float* dev_out, float* dev_lse, void* stream);

/* The same, with the token being decoded attended in full precision (the decoding procedure that
 * concatenates the new key and value to the dequantized cache before they are quantized): the
 * token is not in the cache yet; its fp16 key (pre-RoPE) and value take part as an exact row at
 * position `length`, and dev_q_pos == NULL means `length`.  Call rkv_quantize_append for the token
 * afterwards.  Works on an empty cache (the first decode step).
 *   dev_k_cur, dev_v_cur  [batch][n_kv_heads][head_dim] fp16 */
int rkv_decode_attention_with_current(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos,
                                      const void* dev_k_cur, const void* dev_v_cur, float* dev_out,
                                      float* dev_lse, void* dev_scratch, void* stream);

/* One decode step in one call: rkv_quantize_append of one token per sequence (dev_k, dev_v
 * [batch][1][n_kv_heads][head_dim] fp16, no sink mask) followed by rkv_decode_attention with the
 * same remaining arguments - and the same results, bit for bit.  Where the matrix-core kernels
 * cover the configuration the token's compression and the query's preparation share one kernel
 * launch, which shortens the step by a few microseconds per layer; elsewhere the two calls are
 * made one after the other.  Error codes as for the two calls. */
int rkv_decode_step(rkv_cache* cache, const void* dev_k, const void* dev_v, const void* dev_q, const int32_t* dev_q_pos,
                    float* dev_out, float* dev_lse, void* dev_scratch, void* stream);

/* Several query tokens per sequence in one call (Eq. 5 with the causal mask): the tokens of a
 * multi-token step - verification of drafted tokens, a prefill continued in pieces - are appended
 * first and then read the cache together, so that the cache streams from memory once for all of
 * them.  Query i of sequence b sits at position dev_q_pos[b][i] (its RoPE angle) and attends the
 * cached tokens at positions <= min(dev_q_pos[b][i], length - 1), retained sink rows included.
 *   dev_q      [batch][n_queries][n_q_heads][head_dim] fp16, pre-RoPE
 *   dev_q_pos  [batch][n_queries] int32, required, every entry >= 0 (a query that sees no token
 *              has no defined output)
 *   n_queries  1 .. RKV_MAX_QUERIES
 *   dev_out    [batch][n_queries][n_q_heads][head_dim] fp32
 *   dev_lse    [batch][n_queries][n_q_heads] fp32, or NULL
 *   dev_scratch >= n_queries * scratch_bytes of rkv_query_sizes
 * Runs on the plain matrix-core decode kernel where the configuration has it (reorder inside
 * blocks of 128, rot_heads 2 or 4, groups of 128).  The matrix-core variants that take their
 * scores from the scores kernel (groups of 64 / 32, reorders across blocks) serve at most 8
 * (query token, query head) pairs per KV head, and so does the general kernel, which takes what
 * is left: RKV_EINVAL beyond that, or when rkv_set_decode_path(2) forces a matrix-core kernel the
 * configuration does not have for this many query tokens; RKV_ESTATE on an empty cache. */
#define RKV_MAX_QUERIES 64
int rkv_decode_attention_multi(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos, int32_t n_queries,
                               float* dev_out, float* dev_lse, void* dev_scratch, void* stream);

/* Choose the decode kernel: 0 = automatic (default), 1 = force the general kernel (any supported
 * configuration, vector ALU), 2 = force the matrix-core kernel (RKV_EINVAL at the next decode if
 * the configuration is outside what it covers: a reorder across rotation groups, rot_heads 1 or
 * 8; several query tokens
 * per step with a reorder across blocks of 128 or with quant_group 64 or 32 only up to 8 (query
 * token, query head) pairs per KV head).
 * 3 = measurement only: the matrix-core kernel with the cache stream (codes and metadata of keys
 * and values) replaced by values made up in registers, i.e. the time its arithmetic takes when no
 * byte of the cache has to arrive - the ceiling the vector and matrix units set.  Outputs are
 * meaningless.  Plain configurations only (2-bit codes, fp16 metadata, reorder inside blocks of
 * 128, one query head per KV head), else RKV_EINVAL at the next decode. */
int rkv_set_decode_path(rkv_cache* cache, int32_t path);

/* Which kernel the cache's configuration and installed reorder take (no device work): the decode
 * kernel of rkv_decode_attention / rkv_decode_step (n_queries = 0) or of
 * rkv_decode_attention_multi (n_queries >= 1), the append kernel of rkv_quantize_append.  A
 * caller - or a test - that counts on the matrix-core kernels can assert it instead of finding
 * out from the timing.  Returns one of the RKV_KERNEL_* values, or RKV_EINVAL where the call
 * itself would (rkv_set_decode_path(2) outside the matrix-core kernels' coverage, several query
 * tokens beyond what the general kernel serves). */
#define RKV_KERNEL_GENERAL    1  /* vector-ALU kernels: any supported configuration                  */
#define RKV_KERNEL_SHUFFLE    2  /* append only: FWHT in registers (v_rotate = 1, reorder in blocks)  */
#define RKV_KERNEL_MFMA       3  /* matrix-core kernels: reorder inside blocks of 128, rot_heads 2, 4 */
#define RKV_KERNEL_MFMA_CROSS 4  /* their variant for a reorder across blocks inside rotation groups  */
                                 /* (decode: scores by the scores kernel, the rest by the matrix-core one) */
#define RKV_KERNEL_MFMA_SUB   5  /* their variant for quant_group 64 / 32 (decode: scores by the      */
                                 /* scores kernel of the whole-row path, the rest by the matrix-core one) */
#define RKV_KERNEL_MFMA_ROW   6  /* a reorder over the whole row.  Decode: scores by a kernel of their */
                                 /* own (fp16 matrix products), the rest by the matrix-core one; append: */
                                 /* keys by a kernel that sees whole token rows (rot_heads 2 or 4;       */
                                 /* wider codes: the scores kernel runs once per plane of code bits,     */
                                 /* rows of up to 63 blocks; groups of 64 / 32: once per share of at     */
                                 /* most 40 of the row's blocks)                                         */
int rkv_decode_kernel_of(const rkv_cache* cache, int32_t n_queries);
int rkv_append_kernel_of(const rkv_cache* cache);

/* Measurement hook: ev_start / ev_stop are hipEvent_t handles (as void*) or NULL.  While set,
 * every rkv_decode_attention on this cache records ev_start immediately before and ev_stop
 * immediately after its main (cache-streaming) kernel, on the call's stream; likewise
 * rkv_quantize_append around its quantize kernel.  Pass NULLs to clear. */
int rkv_set_profile_events(rkv_cache* cache, void* ev_start, void* ev_stop);

/* ---- test support: exact views of what the cache stores ------------------------------------- */

/* Reconstructed keys and values (Eq. 7, inverse reorder, inverse rotation), original basis, keys
 * pre-RoPE, fp32 [batch][length][n_kv_heads][head_dim].  Sink rows are NOT substituted.
 * Either pointer may be NULL. */
int rkv_dequantize(rkv_cache* cache, float* dev_k_hat, float* dev_v_hat, void* stream);

/* The logical code array in canonical bytes, independent of the physical layout:
 *   dev_k_codes, dev_v_codes  [batch][length][E/4] uint8: byte j of a token holds reordered
 *                             channels 4j..4j+3, channel 4j+r in bits [2r, 2r+1]; with 3- or
 *                             4-bit codes [batch][length][E/2]: byte j holds channel 2j in its
 *                             low and channel 2j+1 in its high nibble
 *   dev_k_scale, dev_k_zero, dev_v_scale, dev_v_zero   [batch][length][E/quant_group] fp32
 * Any pointer may be NULL. */
int rkv_export_codes(rkv_cache* cache, uint8_t* dev_k_codes, float* dev_k_scale, float* dev_k_zero,
                     uint8_t* dev_v_codes, float* dev_v_scale, float* dev_v_zero, void* stream);

/* Overwrite the cache contents with n_tokens tokens given in the same canonical form (scale and
 * zero must be exactly representable in fp16); sets length = n_tokens, keeps sinks and perm. */
int rkv_import_codes(rkv_cache* cache, int32_t n_tokens, const uint8_t* dev_k_codes,
                     const float* dev_k_scale, const float* dev_k_zero, const uint8_t* dev_v_codes,
                     const float* dev_v_scale, const float* dev_v_zero, void* stream);

/* The sink store: dev_count [batch] int32, dev_pos [batch][max_sinks] int32 (token index, -1 if
 * unused), dev_k / dev_v [batch][max_sinks][E] fp16.  Any pointer may be NULL. */
int rkv_export_sinks(rkv_cache* cache, int32_t* dev_count, int32_t* dev_pos, void* dev_k, void* dev_v,
                     void* stream);

/* Where the physical layout keeps a code (host-only arithmetic, no device access): the index of
 * the 32-bit word inside the K-code (is_v = 0) or V-code (is_v = 1) region of a cache built from
 * cfg, and the bit position of the 2-bit code of sequence b, token t, ROTATED channel c (0..E-1,
 * i.e. before the reorder; of the low two bits of a wider code).  Also returns the number of words of the region in *n_words (may be
 * NULL).  Used to test that the layout is a bijection. */
int rkv_layout_locate(const rkv_config* cfg, int32_t is_v, int32_t b, int32_t t, int32_t c,
                      size_t* word_index, int32_t* bit_shift, size_t* n_words);

const char* rkv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* RKV_H_ */
