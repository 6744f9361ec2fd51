/*
 * skvq.h -- C ABI of the MI355X (gfx950) SKVQ hot path.
 *
 * SKVQ (arXiv 2405.06219) keeps the last W tokens of a KV cache in fp16 and
 * stores every older token as low-bit codes: channels are reordered by an
 * offline permutation, then each group of G reordered channels of a token is
 * quantized with clipped dynamic asymmetric quantization (Section 3.1, Eq. 2;
 * Section 3.2; Algorithm 1).  This library is that cache's data path for one
 * attention layer on one GPU:
 *
 *   skvq_prefill_attention  the prompt's own causal attention on the full-precision K and V
 *   skvq_prefill_quantize   bulk-quantize a prompt, keep its last W tokens fp16
 *   skvq_quantize_append    one decode step: the token leaving the window is
 *                           quantized, the new token enters the window
 *   skvq_decode_attention   one query token attends over packed + fp16 tokens
 *
 * Conventions
 *  - C99, plain pointers and sizes.  Pointers marked HOST are read during the
 *    call only.  Pointers marked DEVICE are HIP device memory that the caller
 *    owns (allocates, keeps alive until the stream has drained, frees).
 *  - Work is enqueued on the caller's hipStream_t (passed as void*, NULL = the
 *    default stream) and the call returns without synchronising.  The token
 *    counters live on the host and advance when a call is enqueued.
 *  - Every function returns a skvq_status (0 = ok, negative = error).  On
 *    error nothing is enqueued and no state changes.
 *  - Calls on one skvq_cache must not overlap (one stream, or ordered streams).
 *  - Inputs must be finite fp16; the result for inf/nan input is unspecified.
 *
 * Numerics contract: codes and (scale, zero) are a pure function of the
 * inputs -- each fp32 operation of Eq. 2 is a single IEEE round-to-nearest
 * operation in a fixed order (listed at skvq_prefill_quantize).  Attention
 * outputs are computed with fp32 accumulation.
 */
#ifndef SKVQ_H
#define SKVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct skvq_cache skvq_cache; /* opaque host object */

typedef enum {
  SKVQ_OK = 0,
  SKVQ_ERR_INVALID_ARG = -1, /* NULL pointer, bad shape, non-permutation, alpha outside (0,1] */
  SKVQ_ERR_UNSUPPORTED = -2, /* a bit-width / head_dim / group size this build has no kernel for */
  SKVQ_ERR_CAPACITY = -3,    /* the packed region (max_quant_tokens) would overflow */
  SKVQ_ERR_STATE = -4,       /* e.g. attention over an empty cache, a rewind by skvq_set_state */
  SKVQ_ERR_HIP = -5          /* a HIP runtime call failed; see skvq_last_error */
} skvq_status;

/* Code widths; the value is the number of levels (Abstract: 2-bit keys, 1.5-bit values;
 * Table 1 also runs 4-bit keys and values). */
typedef enum {
  SKVQ_BITS_4 = 16,  /* sixteen levels, codes 0..15 */
  SKVQ_BITS_3 = 8,   /* eight levels, codes 0..7; keys and values together only */
  SKVQ_BITS_2 = 4,   /* four levels, codes 0..3 */
  SKVQ_BITS_1P5 = 3  /* three levels, codes 0..2 (this build's reading of "1.5-bit") */
} skvq_bits;

/* Storage of (scale, zero): Section 4.1 keeps them in FP8 (E4M3); Section 4.3 also counts
 * fp16.  The rounded values are the ones the codes are computed with. */
typedef enum {
  SKVQ_META_F32 = 0,
  SKVQ_META_F16 = 1,
  SKVQ_META_FP8_E4M3 = 2 /* bias 7, largest finite value 448, saturating */
} skvq_meta_format;

/* Most packed rows per sequence: the kernels count packed tokens in 32-bit integers. */
#define SKVQ_MAX_QUANT_TOKENS 2147483583LL /* 2^31 - 1 - 64 */

/* Parameters of Algorithm 1: window W, group size G; Prologue outputs P_k, P_v, clipping. */
typedef struct {
  int32_t batch;        /* B >= 1; all sequences of a batch have the same length          */
  int32_t n_q_heads;    /* Hq, a multiple of n_kv_heads with Hq/Hk <= 8                   */
  int32_t n_kv_heads;   /* Hk                                                             */
  int32_t head_dim;     /* D, must be 128                                                 */
  int32_t group_size;   /* G in {32, 64, 128}: consecutive REORDERED channels of a token;
                           with group_bounds, the AVERAGE group size (D/G groups)         */
  int32_t k_bits;       /* skvq_bits; keys: SKVQ_BITS_2, SKVQ_BITS_3 or SKVQ_BITS_4       */
  int32_t v_bits;       /* skvq_bits; values: SKVQ_BITS_1P5, _2, _3 or _4; SKVQ_BITS_3
                           only together with 3-bit keys (SKVQ_ERR_UNSUPPORTED else)      */
  int32_t window;       /* W >= 1 most recent tokens stay fp16 (Section 3.2)              */
  int32_t n_sink;       /* S >= 0: fp16 rows for tokens that the filter rules of Section 3.2 /
                           Algorithm 1 keep in full precision; the built-in rule keeps the
                           first S tokens (attention sinks) for ever; 0 = off             */
  int32_t meta_format;  /* skvq_meta_format                                              */
  int64_t max_quant_tokens; /* Tcap: rows of the packed region per sequence, >= 1 and at
                           most SKVQ_MAX_QUANT_TOKENS (SKVQ_ERR_UNSUPPORTED beyond)       */
  const int32_t *perm_k; /* HOST [Hk][D]: reordered position p takes channel perm[h][p]   */
  const int32_t *perm_v; /* HOST [Hk][D]  (each row a permutation of 0..D-1)              */
  const float *clip_k;   /* HOST [Hk][D/G]: alpha in (0,1] per (kv head, group), Eq. 2    */
  const float *clip_v;   /* HOST [Hk][D/G]                                                */
  float sm_scale;        /* softmax scale; 0 selects 1/sqrt(D)                            */
  int32_t max_new_tokens; /* most query tokens per sequence that skvq_decode_attention_multi will be
                           given (sizes the workspace); 0 or 1: single-token decode only; at most
                           SKVQ_MAX_NEW_TOKENS                                            */
  const int32_t *group_bounds; /* HOST [Hk][D/G + 1] or NULL.  NULL: uniform groups of G positions.
                           Else (Section 4.1: clustering the channels gives groups of unequal
                           size, G being their average): group g of kv head h covers the
                           reordered positions [bounds[h][g], bounds[h][g+1]), bounds[h][0] = 0
                           < ... < bounds[h][D/G] = D, every boundary a multiple of 16
                           (SKVQ_ERR_UNSUPPORTED otherwise).  A head's boundaries serve its
                           keys and its values.                                           */
} skvq_config;

/* DEVICE buffers of one layer's cache; byte sizes come from skvq_sizes(), in this order.
 *   k_codes   u8  [B][Hk][Tcap][32 | 48 | 64]  row t, 2-bit: code of position p in byte p/4,
 *             bits 2(p%4).. ; 4-bit: in byte p/2, bits 4(p%2).. ; 3-bit: bytes 0..31 hold the
 *             low two bits as a 2-bit row, bytes 32..47 four dwords of top bits: position p in
 *             dword p/32 at bit 16((p%16)/8) + KSIG[(p%32)/16][p%8],
 *             KSIG = {{0,2,1,3,4,6,8,5},{7,9,10,12,11,13,15,14}}
 *   v_codes   u8  [B][Hk][ceil(Tcap/32)][832 | 1024 | 1536 | 2048]   blocks of 32 tokens, token-minor:
 *             token slot s=t%32 -> kb=s/8, i=s%8 ; position p -> n=p/16, j=p%16 ; unit u=16kb+j
 *             2-bit  : unit = 16 B little-endian, code(n,i) at bit 32(n/2)+16(i%2)+8(n%2)+2(i/2)
 *             3-level: unit = 13 B little-endian, field n = bits [13n,13n+13) = sum_i code(n,i)*3^i
 *             4-bit  : unit = 32 B little-endian, code(n,i) at bit 32n+16(i%2)+4(i/2)
 *             3-bit  : unit = 24 B: bytes 0..15 the low two bits as a 2-bit unit, bytes 16..23
 *                      two dwords of top bits: code(n,i) in dword n/4 at bit
 *                      16(i%2) + VTAU[n%4][i/2], VTAU = {{0,2,4,12},{1,3,5,13},{6,8,10,14},{7,9,11,15}}
 *             a block is zero-filled when its first token is stored
 *   k_meta    [B][Hk][Tcap][D/G][2]      (scale, zero) of Eq. 2, zero = alpha*min, each an
 *   v_meta    [B][Hk][Tcap][D/G][2]      fp32, fp16 or FP8 E4M3 value (meta_format)
 *   k_win     f16 [B][Hk][W+S][D]        rows 0..W-1: the ring, token number a (0-based) sits
 *   v_win     f16 [B][Hk][W+S][D]        in slot a % W; row W+a: sink token a, once it has
 *                                        left the window
 *   workspace f32 [B][max(max_new_tokens,1)][Hq][SKVQ_MAX_SPLITS+1][132]  split partials of skvq_decode_attention
 *             (running max, sum of weights, two pads, 128 weighted value sums); scratch: any
 *             content is fine before a call and nothing in it survives one
 * All seven must be 16-byte aligned. */
typedef struct {
  void *k_codes, *v_codes, *k_meta, *v_meta, *k_win, *v_win, *workspace;
} skvq_buffers;

/* Byte size of each skvq_buffers member, in declaration order.  Pure host arithmetic.
 * Returns SKVQ_OK or the error skvq_create would give for this config. */
int skvq_sizes(const skvq_config *cfg, size_t bytes[7]);

/* Checks cfg (shapes, bit-widths, permutation rows, alpha range).  Pure host code. */
int skvq_validate_config(const skvq_config *cfg);

/* Creates the host object, copies perm/clip (and small constant tables) to the current
 * HIP device, synchronously.  The cache starts empty.  bufs are borrowed, never freed. */
int skvq_create(const skvq_config *cfg, const skvq_buffers *bufs, skvq_cache **out);

/* Frees what skvq_create allocated (never the caller's buffers).  NULL is allowed. */
void skvq_destroy(skvq_cache *cache);

/* Where token a of T cached tokens lives: the last min(T,W) tokens are in the ring; of the
 * older ones, token a < S is sink row a (fp16, bit for bit) and token a >= S is packed row
 * a - S.
 *
 * Section 3.2 prefill phase / Algorithm 1 with l = len(prompt), quantization part only.
 * k, v: DEVICE fp16 [B][Hk][T][D], original channel order, T >= 0.  Resets the cache, then
 * every token goes to its place as above.  Per (token, kv head, group g) of a packed row,
 * with xp[p] = x[perm[p]]:
 *   mn,mx = min,max xp (a zero of either sign counts as +0); lo = alpha_g*mn; hi = alpha_g*mx;
 *   scale = stored((hi-lo)/(levels-1)); zero = stored(lo)   (round to nearest even into
 *   meta_format, FP8 saturating at +-448; the identity for fp32); inv = scale>0 ? 1/scale : 0;
 *   code = clamp(rint((xp-zero)*inv), 0, levels-1), ties to even.
 * SKVQ_ERR_CAPACITY if T-W-S > Tcap. */
int skvq_prefill_quantize(skvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                          void *hip_stream);

/* The filter rules of Section 3.2 / Algorithm 1 ("for filter in F": tokens that a filter selects
 * keep full precision when they slide out of the window) as the caller's own decisions.  The
 * cache has n_sink rows of fp16 storage for kept tokens; the attention-sink rule of the entry
 * points without "_filtered" fills them with the first n_sink tokens.  Here the caller decides
 * token by token: a kept token takes the next free fp16 row (the j-th kept token row W + j of
 * k_win / v_win), every other token the next packed row, both in token order.  Attention reads
 * kept rows like window rows.  A cache may be driven with either set of entry points (the
 * sink rule then means: keep token a if a < n_sink and a row is free).
 *
 * skvq_prefill_quantize_filtered: as skvq_prefill_quantize; keep: HOST array, one byte per token
 * older than the window (tokens 0 .. n_tokens - W - 1), nonzero = keep; NULL = the sink rule.
 * SKVQ_ERR_CAPACITY if more than n_sink tokens are kept or the others exceed Tcap;
 * SKVQ_ERR_UNSUPPORTED for n_tokens >= 2^31 with a mask.  Copies the kept tokens' numbers to
 * the device on the stream and waits for that copy (at most n_sink integers) before it returns.
 *
 * skvq_quantize_append_filtered: as skvq_quantize_append; keep_leaving != 0 keeps the token that
 * leaves the window in this step (ignored while the window is not full).  SKVQ_ERR_CAPACITY if
 * no fp16 row (or no packed row) is free; the cache is unchanged then. */
int skvq_prefill_quantize_filtered(skvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                                   const uint8_t *keep, void *hip_stream);
int skvq_quantize_append_filtered(skvq_cache *cache, const void *k_new, const void *v_new,
                                  int32_t keep_leaving, void *hip_stream);

/* Section 3.2 prefill phase, first step (the prompt attends over its own keys and values before
 * any of them is quantized; Algorithm 1 with h = 0, l = len(prompt)): causal softmax attention of the prompt on
 * the fp16 inputs, original channel order, fp32 accumulation: query t of head hq sees keys
 * 0..t of kv head hq / (Hq/Hk); scale sm_scale.  Reads only the cache's configuration; the cache
 * contents and counters are untouched (call skvq_prefill_quantize on the same k, v afterwards).
 * q: DEVICE fp16 [B][Hq][T][D]; k, v: DEVICE fp16 [B][Hk][T][D]; out_f32: DEVICE fp32
 * [B][Hq][T][D]; out_f16: DEVICE fp16 [B][Hq][T][D] or NULL.  All 16-byte aligned, T >= 1. */
int skvq_prefill_attention(skvq_cache *cache, const void *q, const void *k, const void *v,
                           int64_t n_tokens, void *out_f32, void *out_f16, void *hip_stream);

/* The whole prefill phase of Section 3.2 as one call: skvq_prefill_attention on q, k, v, then
 * skvq_prefill_quantize of the same k, v (sink rule), on the same stream; arguments, results
 * and errors as those two (a prompt that does not fit is refused before anything is launched).
 * The two stay separate launches: the attention streams every K/V tile once per block of 256
 * queries, the quantizer once in all, so a merged kernel would save one pass out of hundreds. */
int skvq_prefill_attention_quantize(skvq_cache *cache, const void *q, const void *k, const void *v,
                                    int64_t n_tokens, void *out_f32, void *out_f16, void *hip_stream);

/* Section 3.2 decode phase: with T tokens cached, if T >= W the token T-W (ring slot T % W)
 * leaves the window: it is copied to sink row T-W if T-W < S, else quantized into packed row
 * T-W-S by the same arithmetic; then the new token is written to slot T % W.
 * k_new, v_new: DEVICE fp16 [B][Hk][D].  SKVQ_ERR_CAPACITY if row T-W-S >= Tcap. */
int skvq_quantize_append(skvq_cache *cache, const void *k_new, const void *v_new,
                         void *hip_stream);

/* Eq. 1 for one query token per sequence (Algorithm 1 with l = 1, attention part):
 * scores of packed rows are (reordered query) . (dequantized reordered key), scores of sink
 * and ring tokens use the original order; one softmax (scale sm_scale, no mask) over all T tokens;
 * output = weighted sum of dequantized values, returned in ORIGINAL channel order.
 * q: DEVICE fp16 [B][Hq][D].  out_f32: DEVICE fp32 [B][Hq][D].  out_f16: DEVICE fp16
 * [B][Hq][D] or NULL.  Query head hq reads kv head hq / (Hq/Hk).  The sequence is split
 * into chunks that are merged by their running max and sum (online softmax).
 * SKVQ_ERR_STATE if the cache is empty. */
int skvq_decode_attention(skvq_cache *cache, const void *q, void *out_f32, void *out_f16,
                          void *hip_stream);
/* skvq_decode_attention for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and
 * the same results, but the split partials go to a fixed array inside the library's device image
 * (SKVQ_STATIC_MAX_ROWS * (SKVQ_MAX_SPLITS + 1) * 132 floats = 4.4 MB per GPU, held until the
 * process ends) instead of skvq_buffers.workspace, and the call makes no hipMalloc / hipFree or any
 * allocating library call.  The array's address on the cache's device is looked up once, in
 * skvq_create.  SKVQ_ERR_UNSUPPORTED if batch * n_q_heads > SKVQ_STATIC_MAX_ROWS (nothing is
 * launched); SKVQ_ERR_HIP if that lookup had failed.  Every cache on one GPU shares the array:
 * calls of this entry point that overlap on one GPU (different streams) race -- keep them on one
 * stream or order the streams.  Nothing in the array has to start at zero (every partial that the
 * merge reads is written by the same call first), so it is never cleared. */
#define SKVQ_STATIC_MAX_ROWS 64
int skvq_decode_attention_static(skvq_cache *cache, const void *q, void *out_f32, void *out_f16,
                                 void *hip_stream);

/* One decode step of Algorithm 1 with l = 1 as a single call: skvq_quantize_append(k_new, v_new)
 * followed by skvq_decode_attention(q), same arguments, same results in the cache and in the
 * outputs, same errors.  When a kv head has at most four query heads, its packed rows are split
 * into at least four chunks (long caches, few sequences) and the token that leaves the window
 * is packed (not kept as a sink), both run as one launch: the workgroup that reads the
 * last packed rows quantizes the leaving token itself before it reads them, and the new token's
 * fp16 row is taken from k_new / v_new; otherwise the two kernels are launched one after the
 * other.  k_new and v_new must stay valid until the call has finished on the stream. */
int skvq_append_decode_attention(skvq_cache *cache, const void *k_new, const void *v_new, const void *q,
                                 void *out_f32, void *out_f16, void *hip_stream);


/* Section 3.1 / Algorithm 1 Prologue, get_permutation_matrix (channels whose value
 * distributions look alike are put into the same group by KMeans over a per-channel feature),
 * in two steps.  Offline routines: they allocate and free their own scratch and synchronise.
 *
 * skvq_calibrate_channel_stats: x: DEVICE fp16 [B][Hk][T][D] calibration keys (or values);
 * stats: HOST [Hk][D][2] = (min, max) of every channel over all B*T tokens.
 *
 * skvq_calibrate_reorder: pure host code.  Per kv head, KMeans over the channels' (min, max)
 * into D/G clusters (the paper names neither feature nor start; this build's): channels
 * ordered by range max-min (ties: channel index), initial centroid j = mean feature of the j-th
 * run of G channels in that order; Lloyd iterations in fp64 (nearest centroid by squared
 * Euclidean distance, ties: the lowest cluster; an empty cluster keeps its centroid) until no
 * channel moves, at most max_iter; clusters listed by the range of their centroid, ascending,
 * the channels of a cluster by their own range, ascending (ties: index).
 * perm: HOST out [Hk][D] (reordered position p takes channel perm[h][p]); bounds: HOST out
 * [Hk][D/G + 1], the clusters as groups, boundaries rounded to the nearest multiple of
 * `granularity` with every group keeping at least `granularity` positions (pass 16 to use them
 * as skvq_config.group_bounds).  group_size must be a multiple of granularity. */
int skvq_calibrate_channel_stats(const void *x, int32_t batch, int32_t n_kv_heads, int64_t n_tokens,
                                 float *stats, void *hip_stream);
int skvq_calibrate_reorder(const float *stats, int32_t n_kv_heads, int32_t group_size,
                           int32_t granularity, int32_t max_iter, int32_t *perm, int32_t *bounds);

/* Replaces the clip scales alpha of Eq. 2.  clip_k, clip_v: HOST [Hk][D/G], each in (0,1].
 * Ordered after the work already enqueued on hip_stream; synchronises that stream.  Rows
 * already packed keep the codes they were given. */
int skvq_set_clip(skvq_cache *cache, const float *clip_k, const float *clip_v, void *hip_stream);

/* Eq. 3 (Section 3.1; Algorithm 1 Prologue, get_group_clipping): chooses the clip scales that
 * minimise the squared error of the attention output after quantization, on calibration data.
 * The search (the paper leaves it open) is one pass of coordinate descent over the candidate
 * grid `alphas` (HOST [n_alphas], each in (0,1]), starting from the cache's current scales:
 * keys first, then values; group by group; every candidate is tried with the other groups at
 * their current choice; each kv head keeps the candidate with the smallest error summed over
 * its query heads, the queries, the batch and the channels (ties: the earliest candidate).
 * One evaluation = skvq_prefill_quantize of the calibration tokens + one
 * skvq_decode_attention per calibration query, compared with o_ref.
 * k, v: DEVICE fp16 [B][Hk][T][D]; q: DEVICE fp16 [n_queries][B][Hq][D]; o_ref: DEVICE fp32
 * [n_queries][B][Hq][D], the full-precision attention outputs of the queries over all T tokens
 * (e.g. from a cache whose window holds all T tokens).  clip_k_out, clip_v_out: HOST
 * [Hk][D/G]; loss_out: HOST double [Hk] (summed squared error at the result) or NULL.
 * Offline routine: allocates and frees device scratch, synchronises hip_stream repeatedly.
 * Afterwards the cache uses the new scales; its contents are the calibration tokens as the
 * LAST candidate quantized them: call skvq_prefill_quantize before using it.
 * SKVQ_ERR_CAPACITY if T-W-S > Tcap; on any error the cache keeps its old scales. */
int skvq_calibrate_clip(skvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                        const void *q, int32_t n_queries, const void *o_ref, const float *alphas,
                        int32_t n_alphas, float *clip_k_out, float *clip_v_out, double *loss_out,
                        void *hip_stream);

/* Algorithm 1 with l = n_new > 1 on a non-empty cache (several query tokens per sequence in one
 * call, e.g. to verify speculated tokens): the last n_new cached tokens are the new ones (append
 * them first; they must all still be in the fp16 window: n_new <= min(T, W)); query token j
 * attends over the cached tokens 0 .. T - n_new + j, each in the form it is stored in now.
 * q: DEVICE fp16 [B][n_new][Hq][D]; out_f32: DEVICE fp32 [B][n_new][Hq][D]; out_f16 likewise or
 * NULL.  n_new = 1 is skvq_decode_attention.  The packed cache is read once per four
 * (query token, query head) rows of a kv head.
 * SKVQ_ERR_INVALID_ARG if n_new > max_new_tokens or n_new exceeds the tokens in the window. */
#define SKVQ_MAX_NEW_TOKENS 64
int skvq_decode_attention_multi(skvq_cache *cache, const void *q, int32_t n_new, void *out_f32,
                                void *out_f16, void *hip_stream);

/* Host counters: tokens cached, of which packed, of which in the ring (the rest, at most S,
 * are the kept tokens' fp16 rows).  Any may be NULL. */
int skvq_get_state(const skvq_cache *cache, int64_t *n_tokens, int64_t *n_quant, int32_t *n_win);

/* Adopts a cache that was filled elsewhere: declares that the buffers hold a valid cache of
 * n_tokens tokens laid out by the sink rule (the first min(n_tokens - W, S) tokens kept), e.g.
 * copied from the buffers of another cache of the same configuration.  The count only moves
 * forward: a cache cannot be rewound (the ring rows of the tokens that would come back have
 * been overwritten, and an append assumes that the slots after its own in a V unit are still
 * zero), so n_tokens below the current count is refused with SKVQ_ERR_STATE and nothing changes;
 * skvq_prefill_quantize (also with n_tokens = 0) starts over.  SKVQ_ERR_CAPACITY if it cannot fit. */
int skvq_set_state(skvq_cache *cache, int64_t n_tokens);

/* Number of sequence chunks of the packed region per kv head used by
 * skvq_decode_attention; 0 (default) lets the library choose.  At most SKVQ_MAX_SPLITS. */
#define SKVQ_MAX_SPLITS 128
int skvq_set_num_splits(skvq_cache *cache, int32_t n_splits);

/* Measurement yardstick, no part of the method (for benchmarks that price the decode path against
 * what the device can read): a kernel that only reads `bytes` bytes (a multiple of 16) from src
 * (DEVICE, 16-byte aligned) once, with grid-strided streaming 16-byte loads, eight workgroups of 256
 * threads per compute unit (the fastest shape of a sweep), on hip_stream, asynchronously.  sink:
 * DEVICE, 4 bytes, written only if the XOR of all words read equals a magic number (so that the
 * loads cannot be dropped). */
int skvq_read_yardstick(const void *src, size_t bytes, void *sink, void *hip_stream);

/* Second yardstick, for the prefill quantizer (which reads the prompt's fp16 K and V and writes about a
 * seventh of that): a kernel that reads ratio * write_bytes bytes from src once and writes write_bytes
 * bytes to dst, computing nothing -- 4 KB piece g of dst becomes the XOR of the 4 KB pieces g * ratio ..
 * g * ratio + ratio - 1 of src (16-byte word by word).  src, dst: DEVICE, 16-byte aligned, not
 * overlapping; write_bytes: a multiple of 4096, below 2^43; ratio: 1..8.  One workgroup of 256 threads per
 * 4 KB written, streaming loads and stores, on hip_stream, asynchronously. */
int skvq_read_write_yardstick(const void *src, void *dst, size_t write_bytes, int32_t ratio, void *hip_stream);

/* Static description of a status code; the cache's last HIP error text (owned by cache). */
const char *skvq_status_string(int status);
const char *skvq_last_error(const skvq_cache *cache);

#ifdef __cplusplus
}
#endif
#endif /* SKVQ_H */
