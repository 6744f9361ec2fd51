/*
 * SKVQ CPU oracle: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-purpose reference of the SKVQ hot path (arXiv
 * 2405.06219): clipped dynamic group quantization with channel reorder
 * (Section 3.1, Eq. 2; Algorithm 1 clipping_quant), the sliding fp16 window
 * (Section 3.2) with the attention-sink filter rule (Section 3.2, "filter
 * rules"; Algorithm 1 body), and one decode-step attention over the
 * mixed-precision cache (Eq. 1; Algorithm 1 body with l = 1).
 *
 * Nothing in the product (the HIP library and its Python binding) may
 * include, link or call this; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg do.  It shares no code with the HIP path.
 *
 * All pointers are HOST pointers.  fp16 values travel as raw uint16_t bits.
 *
 * Pins (tests marked "not gpu"): every function below is pinned to something
 * outside this file -- hand-derived values of Eq. 2, the scale/2 error bound,
 * lossless round trips, exact textbook attention (a library routine) on the
 * window-only and lossless cases, permutation invariance of Eq. 1, the
 * paper's printed average-bit figures; prefill attention: the library's
 * causal attention and a closed form.  The one thing with no external pin is
 * the meaning of "1.5-bit": the paper never defines it; three-level codes are
 * this build's reading ("parity with the authors' 1.5-bit numbers: unpinned").
 */
#ifndef SKVQ_ORACLE_H
#define SKVQ_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKVQ_REF_HEAD_DIM 128
#define SKVQ_REF_VBLOCK_TOKENS 32

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim must be 128      */
  int32_t group_size;                             /* G, divides head_dim (with
                                                     group_bounds: the average
                                                     group size)               */
  int32_t k_levels, v_levels;                     /* 16 = 4-bit, 8 = 3-bit, 4 = 2-bit, 3 = "1.5-bit" (keys: 16, 8 or 4) */
  int32_t window;                                 /* W >= 1                    */
  int32_t n_sink;                                 /* S >= 0: tokens 0..S-1 are
                                                     never quantized           */
  int32_t meta_format;                            /* storage of (scale, zero):
                                                     0 fp32, 1 fp16, 2 FP8 E4M3 */
  int64_t max_quant_tokens;                       /* rows in the packed region */
  const int32_t *perm_k, *perm_v;                 /* [Hk][D] gather index      */
  const float *clip_k, *clip_v;                   /* [Hk][D/G] alpha           */
  float sm_scale;                                 /* softmax scale             */
  const int32_t *group_bounds;                    /* NULL = uniform groups; else
                                                     [Hk][D/G + 1]: per kv head
                                                     ascending entries 0 .. D,
                                                     group g covers the
                                                     reordered positions
                                                     [bounds[g], bounds[g+1])  */
} skvq_ref_config;

typedef struct {
  uint8_t *k_codes;  /* [B][Hk][Tcap][32, 48 or 64: 2-, 3-, 4-bit]             */
  uint8_t *v_codes;  /* [B][Hk][ceil(Tcap/32)][832, 1024, 1536 or 2048]        */
  void *k_meta;      /* [B][Hk][Tcap][D/G][2] = (scale, zero), 4, 2 or 1 byte  */
  void *v_meta;      /* each (meta_format)                                     */
  uint16_t *k_win;   /* fp16 bits [B][Hk][W+S][D]: rows 0..W-1 are the ring    */
  uint16_t *v_win;   /* (token a in slot a % W), row W+a keeps sink token a    */
} skvq_ref_buffers;

/* fp16 <-> fp32 helpers (exact widening; round-to-nearest-even narrowing). */
float skvq_ref_half_to_float(uint16_t h);
uint16_t skvq_ref_float_to_half(float f);

/* FP8 E4M3 (the 8-bit format Section 4.1 stores scale and zero in: 1 sign, 4
 * exponent bits with bias 7, 3 mantissa bits, no infinities, largest finite
 * value 448, 0x7f/0xff = NaN).  Narrowing rounds to nearest, ties to even, and
 * saturates at +-448. */
uint8_t skvq_ref_float_to_e4m3(float f);
float skvq_ref_e4m3_to_float(uint8_t b);

/* A (scale, zero) value as it reads back from storage in the given format. */
float skvq_ref_round_meta(float x, int meta_format);

/* Eq. 2 for one group of n already-reordered values: codes[n], scale, zero.
 * levels = 2^N (or 3).  Every fp32 operation is a separately rounded IEEE
 * operation, in this order:
 *   mn, mx = min, max (a zero of either sign becomes +0)
 *   lo = alpha*mn ; hi = alpha*mx ; h = (hi-lo)/(levels-1)
 *   scale = stored(h) ; zero = stored(lo)      (identity for fp32 storage:
 *           the codes are computed with the values that decoding will read)
 *   inv = scale > 0 ? 1/scale : 0
 *   code = clamp(rint((x-zero)*inv), 0, levels-1)   (ties to even)           */
void skvq_ref_encode_group(const float *xp, int n, float alpha, int levels, int meta_format,
                           uint8_t *codes, float *scale, float *zero);

/* Storage accounting in the paper's style: average bits per cached element
 * = code bits + 2 * meta_bits / group_size (Section 4.3, breakdown paragraph). */
double skvq_ref_avg_bits(double code_bits, int meta_bits, int group_size);

/* Byte sizes of the six cache buffers for this build's formats. */
void skvq_ref_sizes(const skvq_ref_config *cfg, size_t bytes[6]);

/* Packed-format accessors (the format is stated in the .c file). */
int skvq_ref_k_get(const uint8_t *k_row, int levels, int p);
void skvq_ref_k_put(uint8_t *k_row, int levels, int p, int code);
int skvq_ref_v_get(const uint8_t *v_block, int levels, int t_in_block, int p);
void skvq_ref_v_put(uint8_t *v_block, int levels, int t_in_block, int p, int code);

/* Where token a of T cached tokens lives (Section 3.2): the last min(T, W)
 * tokens are in the fp16 ring; of the older ones, tokens a < S (the attention
 * sinks that the filter rule keeps in full precision) sit in sink row a and
 * token a >= S is packed row a - S.
 *
 * Prefill (Section 3.2, phase 1): every token older than the window goes to
 * its place as above (reordered, quantized and packed, or copied bit for bit
 * if it is a sink); the last min(T, W) tokens are copied bit for bit into the
 * ring.  k, v: fp16 bits [B][Hk][T][D], original channel order.  Returns 0,
 * or -3 if T-W-S exceeds max_quant_tokens.  *n_tokens = T.                  */
int skvq_ref_prefill_quantize(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                              const uint16_t *k, const uint16_t *v, int64_t T,
                              int64_t *n_tokens);

/* Decode (Section 3.2, phase 2): the token that slides out of the window
 * (number n_tokens-W) goes to its place as above, then the new token takes
 * its ring slot.
 * k_new, v_new: fp16 bits [B][Hk][D].  *n_tokens is advanced by one.        */
int skvq_ref_quantize_append(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                             const uint16_t *k_new, const uint16_t *v_new,
                             int64_t *n_tokens);

/* One decode-step attention (Eq. 1 with the standard 1/sqrt(d)-style scale):
 * dequantize every packed row in fp64, score against the reordered query,
 * score the sink and ring tokens in original order, one softmax over all,
 * weighted sum of dequantized values scattered back to original channel
 * order.  q: fp16 bits [B][Hq][D]; out_f32: [B][Hq][D]; out_f16 may be NULL.
 * Returns 0, or -4 if the cache is empty.                                    */
int skvq_ref_decode_attention(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                              int64_t n_tokens, const uint16_t *q, float *out_f32,
                              uint16_t *out_f16);

/* The same three steps with the filter rules of Section 3.2 / Algorithm 1 ("for filter in F")
 * given as a mask over the tokens that have left the window: keep[a] != 0 keeps token a in full
 * precision.  The kept tokens take the rows W, W+1, ... of the fp16 buffers in token order
 * (at most S = n_sink of them: -3 beyond), the others the packed rows 0, 1, ... in token
 * order.  keep == NULL is the attention-sink rule (a < S), i.e. the functions above.
 * prefill: keep covers tokens 0 .. T-W-1.  append: keep covers tokens 0 .. n_tokens-W (the last
 * entry is the decision for the token that leaves now).  decode: keep covers 0 .. T-W-1;
 * n_new query tokens as in skvq_ref_decode_attention_multi.                              */
int skvq_ref_prefill_quantize_filtered(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                                       const uint16_t *k, const uint16_t *v, int64_t T,
                                       const uint8_t *keep, int64_t *n_tokens);
int skvq_ref_quantize_append_filtered(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                                      const uint16_t *k_new, const uint16_t *v_new,
                                      const uint8_t *keep, int64_t *n_tokens);
int skvq_ref_decode_attention_filtered(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                                       int64_t n_tokens, const uint8_t *keep, const uint16_t *q,
                                       int n_new, float *out_f32, uint16_t *out_f16);

/* Several query tokens at once (Algorithm 1 with l = n_new > 1 on a non-empty
 * cache): the last n_new cached tokens are the new ones (they have been
 * appended, and all still sit in the fp16 window: n_new <= min(T, W)); query
 * token j attends over the cached tokens 0 .. T - n_new + j, each in the form
 * it is stored in now.  q: fp16 bits [B][n_new][Hq][D]; out: [B][n_new][Hq][D].
 * Returns -1 if n_new is out of range.                                       */
int skvq_ref_decode_attention_multi(const skvq_ref_config *cfg, const skvq_ref_buffers *buf,
                                    int64_t n_tokens, const uint16_t *q, int n_new,
                                    float *out_f32, uint16_t *out_f16);

/* Prefill attention (Section 3.2, phase 1; Algorithm 1 with h = 0 and
 * l = len(prompt)): the attention of the prompt itself is computed on the
 * full-precision K and V, before anything is quantized.  Plain causal softmax
 * attention in fp64: query t of head hq sees keys 0..t of kv head hq/(Hq/Hk).
 * q: fp16 bits [B][Hq][T][D]; k, v: [B][Hk][T][D]; out_f32: [B][Hq][T][D].   */
int skvq_ref_prefill_attention(const skvq_ref_config *cfg, const uint16_t *q, const uint16_t *k,
                               const uint16_t *v, int64_t T, float *out_f32);
/* The same for chosen rows only (prompts too long to compute whole): row i of
 * out_f32 [n_rows][D] is query rows[3i+2] of sequence rows[3i], query head
 * rows[3i+1].  Returns -1 for an index out of range.                          */
int skvq_ref_prefill_attention_rows(const skvq_ref_config *cfg, const uint16_t *q, const uint16_t *k,
                                    const uint16_t *v, int64_t T, const int64_t *rows, int64_t n_rows,
                                    float *out_f32);

/* Clip calibration (Eq. 3; Algorithm 1 Prologue, get_group_clipping): one pass
 * of coordinate descent over the candidate grid `alphas` (keys, then values;
 * group by group; per kv head the candidate with the smallest squared error of
 * the attention outputs against o_ref; ties: the earliest candidate), starting
 * from cfg's clips.  k, v: calibration tokens [B][Hk][T][D]; q: [n_queries]
 * [B][Hq][D], each attending over all T tokens; o_ref: their full-precision
 * outputs [n_queries][B][Hq][D].  clip_k_out, clip_v_out: [Hk][D/G];
 * loss_out: [Hk] final summed squared error, or NULL.  buf is scratch (it ends
 * up holding the last evaluation's cache).  n_kv_heads <= 1024.              */
int skvq_ref_calibrate_clip(const skvq_ref_config *cfg, const skvq_ref_buffers *buf, const uint16_t *k,
                            const uint16_t *v, int64_t T, const uint16_t *q, int n_queries,
                            const float *o_ref, const float *alphas, int n_alphas, float *clip_k_out,
                            float *clip_v_out, double *loss_out);

/* Channel reorder (Section 3.1; Algorithm 1 Prologue, get_permutation_matrix).
 * skvq_ref_channel_stats: stats[Hk][D][2] = (min, max) of every channel of
 * x (fp16 bits [B][Hk][T][D]) over all tokens.
 * skvq_ref_calibrate_reorder: KMeans over the channels' (min, max) into D/G
 * clusters per kv head (the steps are listed in the .c file); perm[Hk][D]:
 * reordered position p takes channel perm[h][p]; bounds[Hk][D/G + 1]: the
 * clusters as groups, boundaries at multiples of `granularity`.              */
void skvq_ref_channel_stats(const uint16_t *x, int B, int Hk, int64_t T, float *stats);
int skvq_ref_calibrate_reorder(const float *stats, int Hk, int group_size, int granularity,
                               int max_iter, int32_t *perm, int32_t *bounds);

/* Number of OpenMP threads the decode/prefill loops will use. */
int skvq_ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
