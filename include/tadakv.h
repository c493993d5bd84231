/*
 * tadakv.h -- C ABI of the MI355X-native TaDA KV-cache hot path (arxiv 2506.04642).
 *
 * What the library does
 *   kv_quant_append : Algorithm 1, step 8 (KVCache.update) together with the compression that
 *                     steps 3 and 5 produce: mean-centring (Sec. 3.1, Eq. 1-2), deviation
 *                     (Sec. 3.2, Eq. 3-4), group quantisation of the deviations to the layer's
 *                     bit width with 16-bit scale / zero metadata (Sec. 3 memory formula; the
 *                     S and M outputs of Algorithm 1), bit-packing, and the raw buffer of recent
 *                     "residual" tokens (Sec. 3.3, Eq. 9-10).
 *   kv_decode_attn  : Algorithm 1, step 9 (TaDAFlashAttn): softmax attention of one decode query
 *                     per sequence over the whole cache (Eq. 5-6), reconstructing keys and values
 *                     from mean + quantised deviation inside the kernel (Eq. 7-8), split over the
 *                     sequence with a log-sum-exp merge (flash decoding, App. A).
 *   per-layer bits  : one bit width in {2,4,8} (or 16 = stored raw) per layer for keys and for
 *                     values (Sec. 3.3 "Searching for quantization precision", App. B); the map is
 *                     an input here, the search that produces it is not part of this library.
 *   around these    : kv_rope_quant_append (Algorithm 1 step 5: the rotary embedding fused into the
 *                     key append), kv_append_decode_attn (steps 8-9 in one call), kv_dequant (Eq. 7-8
 *                     as tensors), sequences of different lengths, paged placement of the blocks
 *                     (kv_cache_set_block_table), idle slots (kv_cache_set_active).
 *
 * Conventions
 *   - Every function returns KV_OK (0) or a negative kv_status.  Nothing throws or aborts.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device memory of the
 *     GPU that is current when the call is made.  The library never allocates or frees device
 *     memory and never synchronises: work is enqueued on the given hipStream_t (passed as void*,
 *     NULL = the default stream) and ordered by it.
 *   - All arguments are validated on the host before anything is enqueued; on an argument error
 *     nothing has been enqueued and the cache is unchanged.  KV_E_HIP (the runtime refused a launch:
 *     kv_last_hip_error tells why) can come after earlier launches of the same call were enqueued:
 *     the layer's contents are then undefined and the layer should be reset.
 *   - Sequence lengths are tracked on the host, per sequence.  The batch-wide calls move all
 *     sequences together; kv_quant_append_seq / kv_cache_reset_seq let one sequence join or leave
 *     (a new request taking over a slot of the batch: Sec. 3.3's buffer and blocks are per sequence),
 *     after which the lengths differ and the decode kernels take each sequence's own counts.
 *     Caches of more than 256 sequences must keep their lengths equal.
 *   - The calls enqueue kernels only, so they may be recorded into a HIP graph for a fixed cache
 *     state.  The first use of a kernel variant in a process asks the runtime for its occupancy
 *     (and, for two quantiser variants, raises its LDS limit): make one ordinary call of each kind
 *     before recording.
 *   - One cache must be used by one thread at a time.
 *   - head_dim must be 128.
 *
 * Preconditions on the data (device memory cannot be validated by the host; outside them the
 * results are unspecified, never an out-of-range access): every input element is finite, and every
 * mean, group minimum and group range / (2^bits - 1) has magnitude below 65504 -- scale, zero and
 * mean are stored as binary16 (for binary16 inputs this always holds; bfloat16 inputs must stay
 * within about +-3e4).  Queries above 65504 in magnitude lose the cross-head mean's term.
 *
 * Error model
 *   - Cache contents (codes, scale, zero, mean, raw rows): a function of the inputs alone, the same
 *     bits on every run and for every way of cutting a sequence into append calls; |x - x^| <=
 *     scale / 2 per element (+ binary32 rounding), x^ = mean + (zero + scale * code) (Eq. 7-8).
 *   - Attention output against exact arithmetic on x^ (Eq. 5-6): the vector-ALU kernels accumulate
 *     in binary32 throughout: error <= 2e-3 absolute for any input within the preconditions whose
 *     outputs stay below about 1e3 in magnitude (relative 1e-6).  The matrix-core kernels form the
 *     products of codes exactly (int8 x int8 -> int32) and carry the small operands, q * key scale
 *     per block and softmax weight * value scale per 64-token chunk, as 23-bit fixed point relative
 *     to the largest of them in the block / chunk: error <= 1.6e-5 * R absolute, R = the largest
 *     range (max - min of the deviations) of a quantisation group in the layer, plus the binary32
 *     level of the other path; i.e. <= 2e-3 up to R = 128 (activations of the kind the paper
 *     quantises have R < 30: measured <= 1e-6), and 4.9e-3 on outputs of +-300 when a planted value
 *     of 300 sets R.
 *   - Repeated calls on the same state return the same bits (no atomics, fixed summation orders).
 */
#ifndef TADAKV_H
#define TADAKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KV_OK = 0,
    KV_E_NULL = -1,       /* a required pointer is NULL */
    KV_E_BAD_CONFIG = -2, /* shape / group / dtype / mode outside what is supported */
    KV_E_BAD_BITS = -3,   /* a layer's bit width is not one of 2, 4, 8, 16 */
    KV_E_BAD_LAYER = -4,  /* layer index out of range */
    KV_E_CAPACITY = -5,   /* append would exceed max_tokens */
    KV_E_WORKSPACE = -6,  /* workspace NULL or smaller than kv_workspace_bytes */
    KV_E_ALIGN = -7,      /* a device pointer or stride is not aligned as required */
    KV_E_HIP = -8,        /* a kernel launch failed (hipGetLastError) */
    KV_E_EMPTY = -9,      /* attention over a cache that holds no token */
    KV_E_UNSUPPORTED = -10 /* valid configuration whose GPU path is not built yet */
} kv_status;

typedef enum { KV_F16 = 0, KV_BF16 = 1 } kv_dtype;

/* Which axis the mean is taken over before the deviation is quantised.
 *   KV_MEAN_CHANNEL_BLOCK : per (kv head, channel) over each block of group_tokens tokens;
 *                           stored as head_dim binary16 values per (sequence, kv head, block).
 *   KV_MEAN_CROSS_HEAD    : over the kv heads, per (token, channel): Eq. 1-2 of the paper;
 *                           stored as one binary16 row per (sequence, token), shared by all heads.
 *   KV_MEAN_NONE          : no centring (plain group quantisation). */
typedef enum { KV_MEAN_CHANNEL_BLOCK = 0, KV_MEAN_CROSS_HEAD = 1, KV_MEAN_NONE = 2 } kv_mean_mode;

typedef struct {
    int32_t n_layers;
    int32_t batch;          /* sequences (slots); their lengths are tracked one by one */
    int32_t n_q_heads;      /* multiple of n_kv_heads; query head i reads kv head i / (Hq/Hkv) */
    int32_t n_kv_heads;
    int32_t head_dim;       /* 128 */
    int32_t max_tokens;     /* capacity per sequence, multiple of group_tokens */
    int32_t group_tokens;   /* G : tokens per key group = tokens per flushed block: 32, 64 or 128 */
    int32_t group_channels; /* Gc: channels per value group: 32, 64 or 128 */
    int32_t resid_cap;      /* R : raw tokens buffered before a flush; positive multiple of G */
    int32_t dtype;          /* kv_dtype of k, v, q inputs and of the raw residual */
    int32_t mean_mode;      /* kv_mean_mode */
    const uint8_t *k_bits;  /* host, [n_layers], each 2, 4, 8 or 16 */
    const uint8_t *v_bits;  /* host, [n_layers]; the paper uses the same width for both */
    int32_t pool_blocks;    /* 0: dense placement, every sequence owns its max_tokens/G block slots.
                               > 0: paged placement, a layer buffer holds pool_blocks block slots which
                               the sequences share through a block table (kv_cache_set_block_table) */
} kv_config;                /* copied by kv_cache_create; the caller keeps its arrays */

/* Byte offsets inside one layer's device buffer (see kv_cache_describe).
 * Layer buffer = records [batch*n_kv_heads][max_tokens/G] of rec_bytes each
 *              | cross-head mean plane [batch][max_tokens/G][2 (K,V)][G][head_dim] binary16
 *                (KV_MEAN_CROSS_HEAD only)
 *              | raw key residual [batch*n_kv_heads][R][head_dim] | raw value residual, same shape.
 * Paged placement (pool_blocks > 0): records [pool_blocks][n_kv_heads] of rec_bytes each (a block slot
 * holds one block of G tokens of every kv head of one sequence) | cross-head mean plane
 * [pool_blocks][2][G][head_dim] | the residual buffers as above.
 * Record (one sequence, one kv head, one block of G tokens), offsets relative to the record:
 *   k_codes | k_scale[head_dim] | k_zero[head_dim] | k_mean[head_dim]
 *   | v_codes | v_meta[G][head_dim/Gc]{scale,zero} | v_mean[head_dim]
 * all metadata binary16; the mean fields exist only for KV_MEAN_CHANNEL_BLOCK; a 16-bit side
 * stores its G x head_dim raw rows in the codes field and has no metadata.  Absent fields are -1.
 * Codes are stored as 16 x 16 tiles (keys: token x channel; values: channel x token): a tile row's
 * 16 codes take 2*bits bytes, i.e. bits/2 32-bit words of 32/bits codes; inside a word, code number
 * 4f + y is field f (bits [bits*f, bits*f + bits)) of byte y.  A 16-byte piece holds the same row
 * of 8/bits tiles; 16 pieces (rows 0..15) are consecutive.  Key pieces: one channel tile at 8 bits
 * (pieces ordered by token tile, tile parity, tile pair), channel tiles (2j, 2j+1) at 4 bits, and
 * those two tiles for two consecutive token tiles at 2 bits.  Value pieces: 8/bits consecutive
 * channel tiles of one 16-token tile. */
typedef struct {
    int32_t k_bits, v_bits;
    int64_t rec_bytes;
    int64_t k_codes, k_scale, k_zero, k_mean;
    int64_t v_codes, v_meta, v_mean;
    int64_t xmean_off, k_resid_off, v_resid_off;
    int64_t layer_bytes;
} kv_layer_layout;

typedef struct kv_cache kv_cache; /* opaque host-side descriptor */

/* Size of layer `layer`'s device buffer for this configuration.  cfg, bytes: host. */
kv_status kv_cache_bytes(const kv_config *cfg, int32_t layer, size_t *bytes);

/* Size of the workspace kv_decode_attn needs for any length up to max_tokens: the per-split partial
 * results, and, with KV_MEAN_CROSS_HEAD, float arrays of about 2 * batch * n_q_heads * max_tokens
 * elements through which the dense mean terms pass (the queries' products with the key mean of
 * every token, the softmax weights for the value mean) plus batch * n_q_heads * ranges * head_dim
 * for the value mean's share of the output per token range (ranges <= 768 / batch, at most 256). */
kv_status kv_workspace_bytes(const kv_config *cfg, size_t *bytes);

/* Which sequences the batch-wide calls act on (a serving loop whose slots are not all busy).
 *   active : host, [n] bytes, n == batch; non-zero = active.  NULL: all sequences (the initial state).
 * Until changed again: kv_quant_append, kv_rope_quant_append and kv_append_decode_attn(_split) give
 * tokens only to the active sequences (the input rows of the others are not read), and the decode
 * calls treat the others as empty for the call: their output rows are zeros and their part of the
 * cache is not read.  Lengths and contents of the sequences that are not active stay as they are;
 * the per-sequence calls (kv_quant_append_seq, kv_cache_reset_seq, kv_cache_len_seq) ignore the
 * setting.  Host call, copied, nothing is enqueued.  Limits as for sequences of different lengths. */
kv_status kv_cache_set_active(kv_cache *cache, const uint8_t *active, int32_t n);

/* Paged placement (caches created with pool_blocks > 0): where the blocks of the sequences live.
 *   table_dev : device, [batch][stride] int32; entry (b, j) is the block slot, 0 <= slot < pool_blocks,
 *               of logical block j (tokens j*G .. j*G + G - 1) of sequence b, for every layer alike.
 *               The caller owns the array and hands out the slots: a slot belongs to at most one live
 *               block (entries outside the range are clamped into it, so a stale entry cannot make a
 *               kernel leave the buffer).  The kernels read the entries when they run, in stream
 *               order: the array may be updated between calls on the same stream, and must hold an
 *               entry for every block a call touches (blocks below a sequence's length, and the
 *               blocks an append is about to fill).
 *   stride    : entries per sequence, at least max_tokens / G.
 * Host call, nothing is enqueued.  Until a table is set, appends and decodes of a paged cache return
 * KV_E_BAD_CONFIG.  KV_E_BAD_CONFIG also for a cache with dense placement. */
kv_status kv_cache_set_block_table(kv_cache *cache, const int32_t *table_dev, int32_t stride);

/* Build the host descriptor.  layer_dev_ptrs: host array of n_layers device pointers, each at
 * least kv_cache_bytes(layer) long and 256-byte aligned; the caller owns them and must keep them
 * alive until kv_cache_destroy.  No device work is enqueued.  All lengths start at 0. */
kv_status kv_cache_create(const kv_config *cfg, void *const *layer_dev_ptrs, kv_cache **out);

/* Free the host descriptor (never the device buffers). */
kv_status kv_cache_destroy(kv_cache *cache);

/* Forget the contents of one layer (layer < 0: all layers).  Host bookkeeping only. */
kv_status kv_cache_reset(kv_cache *cache, int32_t layer);

/* Forget the contents of one sequence in one layer (layer < 0: all layers): its slot is free for
 * a new request.  Host bookkeeping only.  KV_E_BAD_CONFIG for a sequence index out of range. */
kv_status kv_cache_reset_seq(kv_cache *cache, int32_t layer, int32_t seq);

/* Current lengths of a layer: tokens in packed blocks, tokens in the raw residual.
 * kv_cache_len answers for the whole batch and returns KV_E_UNSUPPORTED while the sequences differ. */
kv_status kv_cache_len(const kv_cache *cache, int32_t layer, int32_t *packed, int32_t *resid);
kv_status kv_cache_len_seq(const kv_cache *cache, int32_t layer, int32_t seq, int32_t *packed, int32_t *resid);

/* Offsets of a layer's buffer, so raw bytes can be compared with an independent packer. */
kv_status kv_cache_describe(const kv_cache *cache, int32_t layer, kv_layer_layout *out);

/* Append n_new tokens to every sequence of `layer`.
 *   k_new, v_new : device, 16-bit elements of cfg.dtype, logical shape [batch, n_new, n_kv_heads,
 *                  head_dim]; element (b,t,h,c) at index b*stride_b + t*stride_t + h*stride_h + c
 *                  (strides in elements; rows of head_dim are contiguous; every row 16-byte aligned).
 *                  Keys are post-RoPE.  The buffers may be reused once the stream has passed the call.
 * Semantics are those of n_new single-token appends: tokens enter the raw residual; whenever it
 * holds R tokens all R are compressed as R/G blocks and the residual restarts empty.
 * n_new == 0 is a no-op.  KV_E_CAPACITY if packed + resid + n_new > max_tokens. */
kv_status kv_quant_append(kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                          int32_t n_new, int64_t stride_b, int64_t stride_t, int64_t stride_h,
                          void *stream);

/* kv_quant_append for ONE sequence of the batch (a request's prompt entering its slot; NEXT to the
 * uniform-length workloads of the paper this is what serving needs).  k_new, v_new: rows of that
 * sequence only, element (t,h,c) at t*stride_t + h*stride_h + c.  Same semantics and errors as
 * kv_quant_append; KV_E_BAD_CONFIG for a sequence index out of range. */
kv_status kv_quant_append_seq(kv_cache *cache, int32_t layer, int32_t seq, const void *k_new, const void *v_new,
                              int32_t n_new, int64_t stride_t, int64_t stride_h, void *stream);

/* kv_quant_append with the rotary position embedding of the keys fused in (Algorithm 1 step 5,
 * "RoPECompress"; Sec. 3.4 and App. A: the rotation is the last computation before the cache
 * update, so the two are one kernel and the rotated keys never make a round trip through memory).
 *   k_pre    : device, keys BEFORE the rotation; shape, strides and alignment as k_new above
 *   rope_cos, rope_sin : device, float32 [n_new, head_dim/2], contiguous, 16-byte aligned: cosine and sine of the
 *              angle of (token t of this call, channel pair i).  The caller owns the schedule
 *              (positions, base, scaling); the tables may be reused once the stream has passed.
 *   pairing  : which channels form pair i (kv_rope_pairing)
 * Pair (a, b) becomes (x_a cos - x_b sin, x_b cos + x_a sin), evaluated in binary32 with one
 * rounding per operation and then rounded (nearest even) to cfg.dtype; from there on the call is
 * kv_quant_append of the rotated keys, bit for bit.  Values are not rotated.
 * Errors as kv_quant_append; KV_E_NULL for a missing table, KV_E_BAD_CONFIG for a bad pairing. */
typedef enum {
    KV_ROPE_HALF = 0,        /* pair i = channels (i, i + head_dim/2)  */
    KV_ROPE_INTERLEAVED = 1  /* pair i = channels (2i, 2i + 1)         */
} kv_rope_pairing;
kv_status kv_rope_quant_append(kv_cache *cache, int32_t layer, const void *k_pre, const void *v_new,
                               int32_t n_new, int64_t stride_b, int64_t stride_t, int64_t stride_h,
                               const float *rope_cos, const float *rope_sin, int32_t pairing,
                               void *stream);

/* Algorithm 1 steps 3 and 8 in one call ("CompressV(X, W_V)"; Sec. 3.4 and App. A "Compressing value
 * activations": the values' linear projection is fused with their mean-centring and quantisation, so
 * the projected values never make a round trip through memory), with the keys appended as by
 * kv_quant_append (or, with tables, as by kv_rope_quant_append: step 5).
 *   k_new   : device, keys [batch, n_new, n_kv_heads, head_dim], element (b,t,h,c) at
 *             b*k_stride_b + t*k_stride_t + h*k_stride_h + c (elements; rows 16-byte aligned);
 *             post-RoPE if rope_cos == rope_sin == NULL, else pre-RoPE
 *   x       : device, the layer input [batch, n_new, model_dim], 16-bit cfg.dtype, element (b,t,k) at
 *             b*x_stride_b + t*x_stride_t + k (rows contiguous and 16-byte aligned)
 *   w_v     : device, value projection weights [n_kv_heads * head_dim, model_dim], cfg.dtype, contiguous:
 *             one row per output channel (a linear layer's weight); channel o of the projection is
 *             channel o % head_dim of kv head o / head_dim
 *   model_dim : positive multiple of 64
 *   rope_cos, rope_sin, pairing : as kv_rope_quant_append, or both NULL
 *   v_proj  : device or NULL.  If given, [batch, n_new, n_kv_heads, head_dim] cfg.dtype, contiguous,
 *             16-byte aligned: receives the projected values as the kernels rounded them (for
 *             inspection and tests; production callers pass NULL and the tensor never exists)
 * The projected value V[b,t,o] = sum_k x[b,t,k] * w_v[o,k] is accumulated in binary32 on the matrix
 * cores (ascending k in steps of 32, the same chain for every token whichever kernel serves it, so the
 * result does not depend on how a sequence is cut into calls) and rounded to nearest even to
 * cfg.dtype: a 16-bit tensor, as it is when the projection is a step of its own.  It differs from the
 * exactly rounded dot product by at most one unit in the last place of cfg.dtype in all but
 * cancelling sums (error <= 2^-24 * sum_k |x w| + half a unit).  From there on the call is
 * kv_quant_append of (k_new, V), bit for bit.
 * Whole blocks made of this call's tokens are compressed in the projection kernel's epilogue; tokens
 * that stay in the raw residual buffer (and the ones that complete a block begun by an earlier call)
 * are stored there as rounded rows.  Served formats: group_tokens == 32, k_bits == v_bits in
 * {2, 4, 8}, KV_MEAN_CHANNEL_BLOCK or KV_MEAN_NONE; others return KV_E_UNSUPPORTED (project, then
 * kv_quant_append).  Other errors as kv_quant_append.  Sequences that are not active are skipped. */
kv_status kv_compressv_append(kv_cache *cache, int32_t layer, const void *k_new, int64_t k_stride_b,
                              int64_t k_stride_t, int64_t k_stride_h, const void *x, int64_t x_stride_b,
                              int64_t x_stride_t, const void *w_v, int32_t model_dim, int32_t n_new,
                              const float *rope_cos, const float *rope_sin, int32_t pairing, void *v_proj,
                              void *stream);

/* One decode step of attention for `layer` over all tokens currently cached (packed + residual).
 *   q    : device, [batch, n_q_heads, head_dim], 16-bit cfg.dtype, contiguous, post-RoPE
 *   out  : device, [batch, n_q_heads, head_dim] float32, contiguous
 *   workspace : device, at least kv_workspace_bytes, 256-byte aligned; contents are scratch.
 * Scores are scaled by 1/sqrt(head_dim).  KV_E_EMPTY if the layer holds no token at all; a sequence
 * without tokens next to others that have some gets zeros. */
kv_status kv_decode_attn(const kv_cache *cache, int32_t layer, const void *q, float *out,
                         void *workspace, size_t workspace_bytes, void *stream);

/* The two halves of kv_decode_attn, exposed so that a profiler can bracket them separately:
 * _split writes per-split partial (max, sum, output) into the workspace, _merge combines them
 * into `out`.  Calling _split then _merge with the same arguments equals kv_decode_attn. */
kv_status kv_decode_attn_split(const kv_cache *cache, int32_t layer, const void *q,
                               void *workspace, size_t workspace_bytes, void *stream);
kv_status kv_decode_attn_merge(const kv_cache *cache, int32_t layer, float *out,
                               const void *workspace, size_t workspace_bytes, void *stream);

/* As kv_decode_attn_merge, with the output narrowed (round to nearest even) to the cache's 16-bit
 * input type, for callers whose next layer takes 16-bit activations (the attention output O of
 * Algorithm 1 step 9 feeds a 16-bit projection): split (or the append-and-split call) first, then this.
 *   out16 : device, [batch, n_q_heads, head_dim] of kv_config.dtype, contiguous, 16-byte aligned */
kv_status kv_decode_attn_merge16(const kv_cache *cache, int32_t layer, void *out16,
                                 const void *workspace, size_t workspace_bytes, void *stream);

/* Reconstruction of a layer's contents (Eq. 7-8): x^ = mean + (zero + scale * code), evaluated in
 * binary32 in that order with one rounding per operation; tokens that are still raw (the residual
 * buffer, 16-bit layers) are widened.  Not on the decode path, which never forms x^; for callers
 * that need the tensors (a prefill kernel of their own, error measurements).
 *   k_out, v_out : device, [batch, t_cap, n_kv_heads, head_dim] binary32, 16-byte aligned; either may
 *                  be NULL.  Token t of sequence b is written for t < its length, the rest is left alone.
 *   t_cap        : tokens per sequence in the outputs; KV_E_CAPACITY if a sequence is longer.
 * KV_E_EMPTY if the layer holds no token.  Sequences that are not active (kv_cache_set_active) are
 * skipped. */
kv_status kv_dequant(const kv_cache *cache, int32_t layer, float *k_out, float *v_out, int32_t t_cap, void *stream);

/* One step of the decode loop in a single call (Algorithm 1 steps 8-9, KVCache.update followed by
 * TaDAFlashAttn): append ONE new token per sequence, then attend over the whole cache including it.
 * Equals kv_quant_append(n_new = 1) followed by kv_decode_attn, bit for bit; where the layer is
 * served by the matrix-core kernel and the token does not complete a block, the attention kernel
 * itself reads the new rows and stores them in the residual buffer, which saves a launch.
 *   k_new, v_new : device, element (b,h,c) at b*stride_b + h*stride_h + c (post-RoPE keys)
 *   other arguments as kv_decode_attn.  Errors of both calls apply; on error nothing is enqueued
 *   and the cache is unchanged.
 * _split is the first half, to be followed by kv_decode_attn_merge (as kv_decode_attn_split). */
kv_status kv_append_decode_attn(kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                                int64_t stride_b, int64_t stride_h, const void *q, float *out,
                                void *workspace, size_t workspace_bytes, void *stream);
kv_status kv_append_decode_attn_split(kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                                      int64_t stride_b, int64_t stride_h, const void *q,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* Number of sequence splits kv_decode_attn uses for `layer` at its current length. */
kv_status kv_decode_splits(const kv_cache *cache, int32_t layer, int32_t *n_splits);

/* Bytes kv_decode_attn must read and write for `layer` at its current length: packed codes,
 * scale / zero / mean metadata, raw residual rows, q in, out.  Excludes the split workspace. */
kv_status kv_decode_bytes(const kv_cache *cache, int32_t layer, size_t *bytes);

/* Select the decode kernel family: 0 = automatic (fastest available for the layer),
 * 1 = portable vector-ALU kernels, 2 = matrix-core (MFMA) kernels where supported.
 * The matrix-core kernels serve layers with k_bits == v_bits in {2, 4, 8}, group_tokens ==
 * group_channels in {32, 64, 128} -- and, except with KV_MEAN_CROSS_HEAD, any pair of these
 * sizes, and with groups of 32 / 32 under dense placement also k_bits != v_bits (both in {2, 4, 8})
 * -- and up to 8 query heads per kv head (with KV_MEAN_CROSS_HEAD:
 * at most 64 query heads); with path 2 a decode of any other layer returns KV_E_UNSUPPORTED.  The
 * vector-ALU kernels serve every format (about twenty times slower: use kv_decode_path_used to see
 * which family a layer gets).  Returns KV_E_BAD_CONFIG for other values.  Affects later calls on
 * this cache only. */
kv_status kv_set_decode_path(kv_cache *cache, int32_t path);

/* Which kernel family a decode call of `layer` would run on in the cache's present state:
 * *path = 1 (vector-ALU kernels) or 2 (matrix-core kernels).  A layer whose format the matrix-core
 * kernels do not take (different widths for keys and values with other groups than 32 / 32 or with a
 * block table, group_tokens != group_channels with KV_MEAN_CROSS_HEAD, a 16-bit layer) is served by the vector-ALU kernels under the automatic choice, at a small fraction
 * of the rate: this call makes that visible.  Errors as kv_decode_splits. */
kv_status kv_decode_path_used(const kv_cache *cache, int32_t layer, int32_t *path);

/* Force the number of sequence splits of later decode calls on this cache (clamped to the number
 * of blocks); 0 restores the automatic choice.  The workspace must then hold
 * batch * n_q_heads * n_splits * 132 floats (with KV_MEAN_CROSS_HEAD on the matrix-core kernels: the
 * dense mean arrays behind them as well), which may exceed kv_workspace_bytes: ask
 * kv_decode_workspace_need; a decode call with less returns KV_E_WORKSPACE.
 * KV_E_BAD_CONFIG if n_splits < 0 or > 256. */
kv_status kv_set_decode_splits(kv_cache *cache, int32_t n_splits);

/* Workspace bytes a decode call of `layer` needs in the cache's present state (lengths, kernel
 * family, forced split count); never more than kv_workspace_bytes unless a split count is forced. */
kv_status kv_decode_workspace_need(const kv_cache *cache, int32_t layer, size_t *bytes);

/* kv_decode_attn for callers that cannot allocate or carry a workspace (code under HIP graph
 * capture, serving loops and harnesses that forbid allocation): the per-split partial results go
 * through an array of KV_STATIC_WORKSPACE_BYTES that lives in the library's device image (each GPU
 * the library runs on holds its own copy until the process ends).  Same kernels, same results bit
 * for bit, same errors as kv_decode_attn; KV_E_WORKSPACE if the call needs more than the array holds
 * (kv_decode_workspace_need tells; the cross-head mean's dense arrays at long contexts do not fit).
 * The call allocates and frees nothing.  Every call on a GPU uses that GPU's one array, whose
 * contents are scratch (each call writes all it later reads): calls that overlap on one GPU, on
 * different streams or from different caches, race -- keep them on one stream or order them. */
#define KV_STATIC_WORKSPACE_BYTES (8u << 20)
kv_status kv_decode_attn_static(const kv_cache *cache, int32_t layer, const void *q, float *out, void *stream);

/* ---- Decode steps on device-resident lengths (Algorithm 1 steps 8-9 for serving loops that replay a
 * recorded step).  The entry points above take the lengths of the sequences from the host-side
 * descriptor and put them into their kernels' arguments, so a call recorded into a HIP graph is
 * right for one state of the cache only.  Here the kernels take them from device memory and advance
 * them themselves: one recorded call (per layer) replays step after step while the cache grows,
 * compressing a sequence's raw tokens whenever the step's token fills its buffer (Sec. 3.3).
 *   kv_dev_lengths_bytes       : size of the lengths array for a configuration (cfg, bytes: host).
 *   kv_cache_lengths_to_device : dev_lengths (device, that many bytes, 16-byte aligned, owned by the
 *       caller, kept by the cache until the next such call) receives the lengths the descriptor holds
 *       now, by an asynchronous copy on `stream` from memory the cache keeps alive -- call it
 *       outside graph capture, after the prompts have been appended, and again after any other call
 *       that changes lengths (appends, resets).
 *   kv_decode_step_dev : as kv_append_decode_attn -- one token per sequence appended, then attention
 *       over everything cached -- with the same results, bit for bit at the same split count; enqueues three kernels (store the
 *       token, write the lengths after the step and compress the raw buffers that the token filled,
 *       none on most steps; attention; merge, which also makes the new lengths current) and does NOT change
 *       the descriptor's lengths.  A sequence that has no room for the token keeps its state and
 *       attends over what it has.  The launch shapes (split count) are planned from the
 *       descriptor's lengths: re-record after a few hundred steps to keep them near the best.
 *   kv_cache_advance : the descriptor catches up with n_steps such steps of `layer` (-1: every
 *       layer), so that the other entry points see the cache as it is; host only.
 * Served: group_tokens == group_channels in {32, 64, 128}, k_bits == v_bits in {2, 4, 8}, dense or
 * paged placement (the block table must already hold the slots of the blocks that replayed steps will
 * fill), all sequences active, layers on the matrix-core kernels, every mean mode --
 * KV_MEAN_CROSS_HEAD (Eq. 1-2) with a multiple of 4 kv heads (four kernels then: the mean rows of a
 * block that is about to be compressed come first);
 * otherwise KV_E_UNSUPPORTED.  KV_E_BAD_CONFIG before kv_cache_lengths_to_device.  Other errors as
 * kv_append_decode_attn. */
kv_status kv_dev_lengths_bytes(const kv_config *cfg, size_t *bytes);
kv_status kv_cache_lengths_to_device(kv_cache *cache, void *dev_lengths, void *stream);
kv_status kv_decode_step_dev(const kv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                             int64_t stride_b, int64_t stride_h, const void *q, float *out,
                             void *workspace, size_t workspace_bytes, void *stream);
kv_status kv_cache_advance(kv_cache *cache, int32_t layer, int32_t n_steps);

/* Measurement aid, not part of the method: one read-only pass over `bytes` bytes at `buf` (device,
 * 16-byte aligned; whole 16-byte pieces are read) with 16-byte loads, one workgroup per contiguous
 * 64 KiB -- the rate the memory system delivers to a kernel that does nothing else,
 * which the benchmark reports beside the published HBM peak as the measured ceiling of the decode
 * kernels (they are bound by reading the packed cache, App. A).  sink8: device, 8 bytes, or NULL
 * (written only if the data folds to one particular value; its content is meaningless).
 * KV_E_BAD_CONFIG for fewer than 16 bytes. */
kv_status kv_stream_read_probe(const void *buf, size_t bytes, void *sink8, void *stream);

/* Measurement aid, not part of the method: the calling thread's next launch of the matrix-core split
 * kernel (kv_decode_attn_split, kv_append_decode_attn_split and the calls built on them) records the
 * kernel's own begin and end into the two HIP events (hipEvent_t, created with timing enabled; host
 * handles), so that hipEventElapsedTime between them is the kernel's execution time as a profiler's
 * kernel trace reports it -- events recorded on the stream before and after the call also count the
 * dispatch gaps on either side (1 - 2 us).  One-shot: that launch clears the request; (NULL, NULL)
 * cancels it; one of the two NULL: KV_E_NULL.  The vector-ALU kernels ignore it. */
kv_status kv_time_next_split(void *begin_event, void *end_event);

const char *kv_strerror(kv_status s);

/* Text of the HIP error behind the calling thread's most recent KV_E_HIP ("no error" if none). */
const char *kv_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TADAKV_H */
