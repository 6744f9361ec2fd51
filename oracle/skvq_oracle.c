/*
 * SKVQ CPU oracle: TEST INFRASTRUCTURE ONLY (see skvq_oracle.h).
 *
 * Build: gcc -O2 -std=c11 -fPIC -shared -fopenmp -ffp-contract=off
 *        (no -ffast-math: the encoder's fp32 operations must each round once).
 *
 * Packed formats (the paper gives none; these are this build's):
 *
 *  K codes, one row per (token, kv head).  2-bit: 32 bytes, the code of
 *  reordered position p sits in byte p/4 at bits [2*(p%4), 2*(p%4)+2).
 *  4-bit: 64 bytes, position p in byte p/2 at bits [4*(p%2), 4*(p%2)+4).
 *  3-bit: 48 bytes in two planes.  Bytes 0..31 hold the low two bits of every
 *  code exactly as a 2-bit row does.  Bytes 32..47 are four little-endian
 *  dwords; dword p/32 holds the top bit of position p at bit
 *  16*((p%16)/8) + KSIG[(p%32)/16][p%8]  (table below; the order is the one
 *  the GPU kernel unpacks with the fewest shifts).
 *
 *  V codes, one block per 32 consecutive tokens of a kv head, stored so that
 *  the codes of CONSECUTIVE TOKENS of one channel are neighbours (the value
 *  product sums over tokens).  Token slot s = t % 32 splits as kb = s / 8,
 *  i = s % 8; position p splits as n = p / 16, j = p % 16.  The block holds 64
 *  units, unit u = 16*kb + j, each covering 8 tokens x 8 positions.
 *    2-bit : unit = 16 bytes read as a 128-bit little-endian string; code
 *            (n, i) sits at bit 32*(n/2) + 16*(i%2) + 8*(n%2) + 2*(i/2).
 *    3-level: unit = 13 bytes read as a 104-bit little-endian string; field n
 *            is bits [13n, 13n+13) and holds sum_i code(n, i) * 3^i  (< 6561).
 *    4-bit : unit = 32 bytes read as a 256-bit little-endian string; code
 *            (n, i) sits at bit 32*n + 16*(i%2) + 4*(i/2).
 *    3-bit : unit = 24 bytes; bytes 0..15 hold the low two bits of every code
 *            exactly as the 2-bit unit does; bytes 16..23 are two dwords,
 *            dword n/4 holds the top bit of code (n, i) at bit
 *            16*(i%2) + VTAU[n%4][i/2].
 *  A block is zero-filled when its first token arrives, so slots of tokens
 *  that do not exist yet read as code 0.
 *
 *  Meta: (scale, zero) pairs, [token][group], as fp32, fp16 or FP8 E4M3.
 */
#include "skvq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define D SKVQ_REF_HEAD_DIM
#define VBT SKVQ_REF_VBLOCK_TOKENS

/* ---------------------------------------------------------------- fp16 --- */

float skvq_ref_half_to_float(uint16_t h) {
  int sign = (h >> 15) & 1, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0)
    v = ldexp((double)m, -24);
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = ldexp((double)(m + 1024), e - 25);
  return (float)(sign ? -v : v); /* every fp16 value is exact in fp32 */
}

uint16_t skvq_ref_float_to_half(float f) {
  if (isnan(f)) return 0x7e00;
  uint16_t sign = signbit(f) ? 0x8000 : 0;
  double a = fabs((double)f);
  if (a >= 65520.0) return sign | 0x7c00; /* rounds to infinity */
  if (a < ldexp(1.0, -14)) {              /* subnormal range: spacing 2^-24 */
    double r = nearbyint(ldexp(a, 24));   /* ties to even */
    return sign | (uint16_t)r;            /* r == 1024 lands on the first normal */
  }
  int e;
  double fr = frexp(a, &e);                /* a = fr * 2^e, fr in [0.5, 1) */
  double r = nearbyint(ldexp(fr, 11));     /* 11 significant bits, in [1024, 2048] */
  if (r == 2048.0) {
    r = 1024.0;
    e += 1;
  }
  int be = e - 1 + 15;
  return sign | (uint16_t)(be << 10) | (uint16_t)((int)r - 1024);
}

/* ----------------------------------------------------------- FP8 E4M3 --- */

float skvq_ref_e4m3_to_float(uint8_t b) {
  int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0)
    v = ldexp((double)m, -9); /* subnormal: m/8 * 2^-6 */
  else
    v = ldexp((double)(8 + m), e - 10); /* (1 + m/8) * 2^(e-7) */
  return (float)(sign ? -v : v);
}

uint8_t skvq_ref_float_to_e4m3(float f) {
  if (isnan(f)) return 0x7f;
  uint8_t sign = signbit(f) ? 0x80 : 0;
  double a = fabs((double)f);
  if (a >= 448.0) return sign | 0x7e; /* saturate at the largest finite value */
  if (a < ldexp(1.0, -6)) {           /* subnormal range: spacing 2^-9 */
    double r = nearbyint(ldexp(a, 9)); /* ties to even; r == 8 lands on the first normal */
    return sign | (uint8_t)r;
  }
  int e;
  double fr = frexp(a, &e);            /* a = fr * 2^e, fr in [0.5, 1) */
  double r = nearbyint(ldexp(fr, 4));  /* 4 significant bits, in [8, 16] */
  if (r == 16.0) {
    r = 8.0;
    e += 1;
  }
  int be = e - 1 + 7;
  uint8_t out = (uint8_t)((be << 3) | ((int)r - 8));
  if (out > 0x7e) out = 0x7e; /* rounding up from just below 448 stays at 448 */
  return sign | out;
}

float skvq_ref_round_meta(float x, int fmt) {
  if (fmt == 1) return skvq_ref_half_to_float(skvq_ref_float_to_half(x));
  if (fmt == 2) return skvq_ref_e4m3_to_float(skvq_ref_float_to_e4m3(x));
  return x;
}

static size_t meta_bytes(int fmt) { return fmt == 2 ? 1 : fmt == 1 ? 2 : 4; }

static void meta_store(void *base, size_t idx, float x, int fmt) {
  if (fmt == 2)
    ((uint8_t *)base)[idx] = skvq_ref_float_to_e4m3(x);
  else if (fmt == 1)
    ((uint16_t *)base)[idx] = skvq_ref_float_to_half(x);
  else
    ((float *)base)[idx] = x;
}

static float meta_load(const void *base, size_t idx, int fmt) {
  if (fmt == 2) return skvq_ref_e4m3_to_float(((const uint8_t *)base)[idx]);
  if (fmt == 1) return skvq_ref_half_to_float(((const uint16_t *)base)[idx]);
  return ((const float *)base)[idx];
}

/* ------------------------------------------------------------- encoder --- */

void skvq_ref_encode_group(const float *xp, int n, float alpha, int levels, int meta_format,
                           uint8_t *codes, float *scale, float *zero) {
  float mn = xp[0], mx = xp[0];
  for (int p = 1; p < n; ++p) {
    if (xp[p] < mn) mn = xp[p];
    if (xp[p] > mx) mx = xp[p];
  }
  if (mn == 0.0f) mn = 0.0f; /* -0 -> +0, so that the stored zero has one bit pattern */
  if (mx == 0.0f) mx = 0.0f;
  float top = (float)(levels - 1);
  float lo = alpha * mn;
  float hi = alpha * mx;
  float h = (hi - lo) / top;
  /* the values decoding will read back: the codes are computed with these */
  h = skvq_ref_round_meta(h, meta_format);
  lo = skvq_ref_round_meta(lo, meta_format);
  float inv = h > 0.0f ? 1.0f / h : 0.0f;
  for (int p = 0; p < n; ++p) {
    float t = (xp[p] - lo) * inv;
    float r = nearbyintf(t);
    if (r < 0.0f) r = 0.0f;
    if (r > top) r = top;
    codes[p] = (uint8_t)r;
  }
  *scale = h;
  *zero = lo;
}

double skvq_ref_avg_bits(double code_bits, int meta_bits, int group_size) {
  return code_bits + 2.0 * (double)meta_bits / (double)group_size;
}

/* -------------------------------------------------------------- format --- */

static size_t v_block_bytes(int levels) {
  return levels == 3 ? 832 : levels == 16 ? 2048 : levels == 8 ? 1536 : 1024;
}
static size_t k_row_bytes(int levels) { return levels == 16 ? 64 : levels == 8 ? 48 : 32; }

/* Bit positions of the top-bit planes of the 3-bit formats (see the format statement). */
static const int KSIG[2][8] = {{0, 2, 1, 3, 4, 6, 8, 5}, {7, 9, 10, 12, 11, 13, 15, 14}};
static const int VTAU[4][4] = {{0, 2, 4, 12}, {1, 3, 5, 13}, {6, 8, 10, 14}, {7, 9, 11, 15}};
static int k3_top_bit(int p) { return 256 + 32 * (p / 32) + 16 * ((p % 16) / 8) + KSIG[(p % 32) / 16][p % 8]; }
static int v3_top_bit(int n, int i) { return 128 + 32 * (n / 4) + 16 * (i % 2) + VTAU[n % 4][i / 2]; }

void skvq_ref_sizes(const skvq_ref_config *c, size_t bytes[6]) {
  size_t heads = (size_t)c->batch * c->n_kv_heads;
  size_t tcap = (size_t)c->max_quant_tokens;
  size_t ng = (size_t)(c->head_dim / c->group_size);
  bytes[0] = heads * tcap * k_row_bytes(c->k_levels);
  bytes[1] = heads * ((tcap + VBT - 1) / VBT) * v_block_bytes(c->v_levels);
  bytes[2] = heads * tcap * ng * 2 * meta_bytes(c->meta_format);
  bytes[3] = bytes[2];
  bytes[4] = heads * (size_t)(c->window + c->n_sink) * D * 2;
  bytes[5] = bytes[4];
}

/* little-endian bit strings */
static unsigned bits_get(const uint8_t *s, int bit, int width) {
  unsigned v = 0;
  for (int k = 0; k < width; ++k) v |= (unsigned)((s[(bit + k) >> 3] >> ((bit + k) & 7)) & 1) << k;
  return v;
}

static void bits_put(uint8_t *s, int bit, int width, unsigned v) {
  for (int k = 0; k < width; ++k) {
    uint8_t m = (uint8_t)(1u << ((bit + k) & 7));
    if ((v >> k) & 1)
      s[(bit + k) >> 3] |= m;
    else
      s[(bit + k) >> 3] &= (uint8_t)~m;
  }
}

int skvq_ref_k_get(const uint8_t *row, int levels, int p) {
  if (levels == 16) return (row[p >> 1] >> (4 * (p & 1))) & 15;
  int lo = (row[p >> 2] >> (2 * (p & 3))) & 3;
  if (levels == 8) return lo + 4 * (int)bits_get(row, k3_top_bit(p), 1);
  return lo;
}

void skvq_ref_k_put(uint8_t *row, int levels, int p, int code) {
  if (levels == 16) {
    int sh = 4 * (p & 1);
    row[p >> 1] = (uint8_t)((row[p >> 1] & ~(15 << sh)) | (code << sh));
    return;
  }
  int sh = 2 * (p & 3);
  row[p >> 2] = (uint8_t)((row[p >> 2] & ~(3 << sh)) | ((code & 3) << sh));
  if (levels == 8) bits_put(row, k3_top_bit(p), 1, (unsigned)code >> 2);
}

static const unsigned POW3[8] = {1, 3, 9, 27, 81, 243, 729, 2187};

int skvq_ref_v_get(const uint8_t *block, int levels, int s, int p) {
  int kb = s / 8, i = s % 8, n = p / 16, j = p % 16;
  int u = 16 * kb + j;
  if (levels == 3) {
    unsigned f = bits_get(block + 13 * u, 13 * n, 13);
    return (int)((f / POW3[i]) % 3);
  }
  if (levels == 16) return (int)bits_get(block + 32 * u, 32 * n + 16 * (i % 2) + 4 * (i / 2), 4);
  if (levels == 8)
    return (int)bits_get(block + 24 * u, 32 * (n / 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i / 2), 2) +
           4 * (int)bits_get(block + 24 * u, v3_top_bit(n, i), 1);
  return (int)bits_get(block + 16 * u, 32 * (n / 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i / 2), 2);
}

void skvq_ref_v_put(uint8_t *block, int levels, int s, int p, int code) {
  int kb = s / 8, i = s % 8, n = p / 16, j = p % 16;
  int u = 16 * kb + j;
  if (levels == 3) {
    unsigned f = bits_get(block + 13 * u, 13 * n, 13);
    unsigned old = (f / POW3[i]) % 3;
    f = f - old * POW3[i] + (unsigned)code * POW3[i];
    bits_put(block + 13 * u, 13 * n, 13, f);
  } else if (levels == 16) {
    bits_put(block + 32 * u, 32 * n + 16 * (i % 2) + 4 * (i / 2), 4, (unsigned)code);
  } else if (levels == 8) {
    bits_put(block + 24 * u, 32 * (n / 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i / 2), 2, (unsigned)code & 3);
    bits_put(block + 24 * u, v3_top_bit(n, i), 1, (unsigned)code >> 2);
  } else {
    bits_put(block + 16 * u, 32 * (n / 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i / 2), 2,
             (unsigned)code);
  }
}

/* --------------------------------------------------- quantize one token --- */

/* Group g covers the reordered positions [group_lo(g), group_lo(g+1)): g*G when
 * the groups are uniform, else the caller's boundaries (Section 4.1: clustering
 * the channels gives groups of unequal size; G is then their average). */
static int group_lo(const skvq_ref_config *c, int hk, int g) {
  int ng = D / c->group_size;
  return c->group_bounds ? c->group_bounds[hk * (ng + 1) + g] : g * c->group_size;
}
static int group_of(const skvq_ref_config *c, int hk, int p) {
  int g = 0;
  while (p >= group_lo(c, hk, g + 1)) ++g;
  return g;
}

/* x: fp16 bits [D] of one (token, kv head), original channel order.
 * Gathers through perm (out[p] = in[perm[p]]), encodes each group, returns
 * codes[D] in reordered order and meta[D/G][2]. */
static void encode_token(const skvq_ref_config *c, int hk, const uint16_t *x, const int32_t *perm,
                         const float *alpha, int levels, uint8_t *codes, float *meta) {
  float xp[D];
  for (int p = 0; p < D; ++p) xp[p] = skvq_ref_half_to_float(x[perm[p]]);
  for (int g = 0; g < D / c->group_size; ++g) {
    int lo = group_lo(c, hk, g), hi = group_lo(c, hk, g + 1);
    skvq_ref_encode_group(xp + lo, hi - lo, alpha[g], levels, c->meta_format, codes + lo,
                          &meta[2 * g], &meta[2 * g + 1]);
  }
}

/* Quantize token (b, hk) and store it as packed row t. */
static void store_quantized(const skvq_ref_config *c, const skvq_ref_buffers *buf, int b, int hk,
                            int64_t t, const uint16_t *kx, const uint16_t *vx) {
  int G = c->group_size, ng = D / G;
  size_t head = (size_t)b * c->n_kv_heads + hk;
  size_t tcap = (size_t)c->max_quant_tokens;
  uint8_t codes[D];
  float meta[2 * D];

  int fmt = c->meta_format;
  encode_token(c, hk, kx, c->perm_k + hk * D, c->clip_k + hk * ng, c->k_levels, codes, meta);
  uint8_t *krow = buf->k_codes + (head * tcap + (size_t)t) * k_row_bytes(c->k_levels);
  memset(krow, 0, k_row_bytes(c->k_levels));
  for (int p = 0; p < D; ++p) skvq_ref_k_put(krow, c->k_levels, p, codes[p]);
  for (int x = 0; x < 2 * ng; ++x)
    meta_store(buf->k_meta, (head * tcap + (size_t)t) * ng * 2 + x, meta[x], fmt);

  encode_token(c, hk, vx, c->perm_v + hk * D, c->clip_v + hk * ng, c->v_levels, codes, meta);
  size_t nblk = (tcap + VBT - 1) / VBT, bb = v_block_bytes(c->v_levels);
  uint8_t *blk = buf->v_codes + (head * nblk + (size_t)(t / VBT)) * bb;
  if (t % VBT == 0) memset(blk, 0, bb);
  for (int p = 0; p < D; ++p) skvq_ref_v_put(blk, c->v_levels, (int)(t % VBT), p, codes[p]);
  for (int x = 0; x < 2 * ng; ++x)
    meta_store(buf->v_meta, (head * tcap + (size_t)t) * ng * 2 + x, meta[x], fmt);
}

static int check_config(const skvq_ref_config *c) {
  if (c->head_dim != D || c->group_size <= 0 || D % c->group_size) return -1;
  if ((c->k_levels != 4 && c->k_levels != 8 && c->k_levels != 16) ||
      (c->v_levels != 4 && c->v_levels != 3 && c->v_levels != 8 && c->v_levels != 16))
    return -2;
  if (c->n_kv_heads <= 0 || c->n_q_heads % c->n_kv_heads || c->window < 1 || c->batch < 1 ||
      c->n_sink < 0 || c->meta_format < 0 || c->meta_format > 2)
    return -1;
  if (c->group_bounds) { /* per kv head: 0 = b_0 < b_1 < ... < b_ng = D */
    int ng = D / c->group_size;
    for (int h = 0; h < c->n_kv_heads; ++h) {
      const int32_t *gb = c->group_bounds + h * (ng + 1);
      if (gb[0] != 0 || gb[ng] != D) return -1;
      for (int g = 0; g < ng; ++g)
        if (gb[g + 1] <= gb[g]) return -1;
    }
  }
  return 0;
}

/* The filter rules of Algorithm 1 as a mask over the tokens that have left the window: keep[a]
 * != 0 keeps token a in full precision.  keep == NULL is the attention-sink rule, a < S.  The
 * kept tokens take the rows W, W+1, ... of the fp16 buffers in token order, the others the
 * packed rows 0, 1, ... in token order. */
static int token_kept(const skvq_ref_config *c, const uint8_t *keep, int64_t a) {
  return keep ? keep[a] != 0 : a < c->n_sink;
}
/* number of kept tokens among 0 .. a-1 */
static int64_t kept_before(const skvq_ref_config *c, const uint8_t *keep, int64_t a) {
  int64_t n = 0;
  for (int64_t x = 0; x < a; ++x) n += token_kept(c, keep, x);
  return n;
}

int skvq_ref_prefill_quantize_filtered(const skvq_ref_config *c, const skvq_ref_buffers *buf,
                                       const uint16_t *k, const uint16_t *v, int64_t T,
                                       const uint8_t *keep, int64_t *n_tokens) {
  int rc = check_config(c);
  if (rc) return rc;
  if (T < 0) return -1;
  int64_t W = c->window, S = c->n_sink, first_win = T > W ? T - W : 0;
  int64_t n_kept = kept_before(c, keep, first_win);
  if (n_kept > S || first_win - n_kept > c->max_quant_tokens) return -3;
  int heads = c->batch * c->n_kv_heads;
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < heads; ++bh) {
    int b = bh / c->n_kv_heads, hk = bh % c->n_kv_heads;
    const uint16_t *kh = k + (size_t)bh * (size_t)T * D;
    const uint16_t *vh = v + (size_t)bh * (size_t)T * D;
    uint16_t *kw = buf->k_win + (size_t)bh * (size_t)(W + S) * D;
    uint16_t *vw = buf->v_win + (size_t)bh * (size_t)(W + S) * D;
    int64_t nk = 0; /* kept so far */
    for (int64_t a = 0; a < first_win; ++a) {
      if (token_kept(c, keep, a)) { /* a filter rule keeps the token in full precision */
        memcpy(kw + (size_t)(W + nk) * D, kh + a * D, D * 2);
        memcpy(vw + (size_t)(W + nk) * D, vh + a * D, D * 2);
        ++nk;
      } else {
        store_quantized(c, buf, b, hk, a - nk, kh + a * D, vh + a * D);
      }
    }
    for (int64_t a = first_win; a < T; ++a) {
      memcpy(kw + (size_t)(a % W) * D, kh + a * D, D * 2);
      memcpy(vw + (size_t)(a % W) * D, vh + a * D, D * 2);
    }
  }
  *n_tokens = T;
  return 0;
}

int skvq_ref_prefill_quantize(const skvq_ref_config *c, const skvq_ref_buffers *buf,
                              const uint16_t *k, const uint16_t *v, int64_t T,
                              int64_t *n_tokens) {
  return skvq_ref_prefill_quantize_filtered(c, buf, k, v, T, NULL, n_tokens);
}

int skvq_ref_quantize_append_filtered(const skvq_ref_config *c, const skvq_ref_buffers *buf,
                                      const uint16_t *k_new, const uint16_t *v_new,
                                      const uint8_t *keep, int64_t *n_tokens) {
  int rc = check_config(c);
  if (rc) return rc;
  int64_t T = *n_tokens, W = c->window, S = c->n_sink;
  int64_t a = T - W; /* the token that leaves the window, if a >= 0 */
  int64_t nk = a >= 0 ? kept_before(c, keep, a) : 0;
  int keeps = a >= 0 && token_kept(c, keep, a);
  if (a >= 0 && (keeps ? nk >= S : a - nk >= c->max_quant_tokens)) return -3;
  for (int b = 0; b < c->batch; ++b)
    for (int hk = 0; hk < c->n_kv_heads; ++hk) {
      size_t bh = (size_t)b * c->n_kv_heads + hk;
      uint16_t *kw = buf->k_win + bh * (size_t)(W + S) * D;
      uint16_t *vw = buf->v_win + bh * (size_t)(W + S) * D;
      size_t slot = (size_t)(T % W);
      if (a >= 0) { /* the slot holds token T-W, which now leaves the window */
        if (keeps) {
          memcpy(kw + (size_t)(W + nk) * D, kw + slot * D, D * 2);
          memcpy(vw + (size_t)(W + nk) * D, vw + slot * D, D * 2);
        } else {
          store_quantized(c, buf, b, hk, a - nk, kw + slot * D, vw + slot * D);
        }
      }
      memcpy(kw + slot * D, k_new + bh * D, D * 2);
      memcpy(vw + slot * D, v_new + bh * D, D * 2);
    }
  *n_tokens = T + 1;
  return 0;
}

int skvq_ref_quantize_append(const skvq_ref_config *c, const skvq_ref_buffers *buf,
                             const uint16_t *k_new, const uint16_t *v_new, int64_t *n_tokens) {
  return skvq_ref_quantize_append_filtered(c, buf, k_new, v_new, NULL, n_tokens);
}

/* ---------------------------------------------------- decode attention --- */

/* Attention of n_new query tokens per sequence, the last n_new cached tokens being theirs
 * (Algorithm 1 with l = n_new): query token j sees the cached tokens 0 .. T - n_new + j.
 * q, out: [B][n_new][Hq][D]. */
static int decode_rows(const skvq_ref_config *c, const skvq_ref_buffers *buf, int64_t T, const uint8_t *keep,
                       const uint16_t *q, int n_new, float *out_f32, uint16_t *out_f16) {
  int rc = check_config(c);
  if (rc) return rc;
  if (T <= 0) return -4;
  int64_t W = c->window, S = c->n_sink, first_win = T > W ? T - W : 0;
  if (n_new < 1 || n_new > T - first_win) return -1; /* the new tokens are all in the window */
  /* where each token older than the window lives: its row of the fp16 buffers (kept) or its
   * packed row */
  int64_t *fp_row = (int64_t *)malloc(sizeof(int64_t) * (size_t)(first_win + 1));
  int64_t *packed_row = (int64_t *)malloc(sizeof(int64_t) * (size_t)(first_win + 1));
  if (!fp_row || !packed_row) {
    free(fp_row);
    free(packed_row);
    return -5;
  }
  {
    int64_t nk = 0;
    for (int64_t a = 0; a < first_win; ++a) {
      int kept = token_kept(c, keep, a);
      fp_row[a] = kept ? W + nk : -1;
      packed_row[a] = kept ? -1 : a - nk;
      nk += kept;
    }
    if (nk > S) {
      free(fp_row);
      free(packed_row);
      return -1;
    }
  }
  int G = c->group_size, ng = D / G, rep = c->n_q_heads / c->n_kv_heads;
  size_t tcap = (size_t)c->max_quant_tokens, nblk = (tcap + VBT - 1) / VBT;
  size_t bb = v_block_bytes(c->v_levels);
  int nqh = c->batch * n_new * c->n_q_heads;
  int fail = 0;

#pragma omp parallel for schedule(dynamic, 1)
  for (int bq = 0; bq < nqh; ++bq) {
    int hq = bq % c->n_q_heads, j = (bq / c->n_q_heads) % n_new, b = bq / (c->n_q_heads * n_new), hk = hq / rep;
    int64_t Tv = T - n_new + j + 1; /* tokens this query sees */
    size_t head = (size_t)b * c->n_kv_heads + hk;
    const int32_t *pk = c->perm_k + hk * D, *pv = c->perm_v + hk * D;
    double qf[D], acc[D];
    int gof[D]; /* group of reordered position p */
    for (int p = 0; p < D; ++p) gof[p] = group_of(c, hk, p);
    for (int ch = 0; ch < D; ++ch) qf[ch] = skvq_ref_half_to_float(q[(size_t)bq * D + ch]);
    double *s = (double *)malloc(sizeof(double) * (size_t)T);
    if (!s) {
      fail = 1;
      continue;
    }
    const uint16_t *kwin = buf->k_win + head * (size_t)(W + S) * D;
    const uint16_t *vwin = buf->v_win + head * (size_t)(W + S) * D;
    /* scores of packed rows: reordered query . dequantized reordered key */
    for (int64_t a = 0; a < first_win; ++a) {
      if (packed_row[a] < 0) continue;
      size_t t = (size_t)packed_row[a];
      const uint8_t *row = buf->k_codes + (head * tcap + t) * k_row_bytes(c->k_levels);
      size_t mi = (head * tcap + t) * ng * 2;
      double dot = 0.0;
      for (int p = 0; p < D; ++p) {
        double kd = (double)skvq_ref_k_get(row, c->k_levels, p) *
                        (double)meta_load(buf->k_meta, mi + 2 * gof[p], c->meta_format) +
                    (double)meta_load(buf->k_meta, mi + 2 * gof[p] + 1, c->meta_format);
        dot += qf[pk[p]] * kd;
      }
      s[a] = (double)c->sm_scale * dot;
    }
    /* scores of kept and ring tokens, original channel order */
    for (int64_t a = 0; a < Tv; ++a) {
      if (a < first_win && fp_row[a] < 0) continue;
      const uint16_t *kw = kwin + (size_t)(a < first_win ? fp_row[a] : a % W) * D;
      double dot = 0.0;
      for (int ch = 0; ch < D; ++ch) dot += qf[ch] * (double)skvq_ref_half_to_float(kw[ch]);
      s[a] = (double)c->sm_scale * dot;
    }
    double m = s[0];
    for (int64_t t = 1; t < Tv; ++t)
      if (s[t] > m) m = s[t];
    double denom = 0.0;
    for (int ch = 0; ch < D; ++ch) acc[ch] = 0.0;
    for (int64_t a = 0; a < first_win; ++a) {
      if (packed_row[a] < 0) continue;
      double w = exp(s[a] - m);
      denom += w;
      size_t t = (size_t)packed_row[a];
      const uint8_t *blk = buf->v_codes + (head * nblk + t / VBT) * bb;
      size_t mi = (head * tcap + t) * ng * 2;
      for (int p = 0; p < D; ++p) {
        double vd = (double)skvq_ref_v_get(blk, c->v_levels, (int)(t % VBT), p) *
                        (double)meta_load(buf->v_meta, mi + 2 * gof[p], c->meta_format) +
                    (double)meta_load(buf->v_meta, mi + 2 * gof[p] + 1, c->meta_format);
        acc[pv[p]] += w * vd;
      }
    }
    for (int64_t a = 0; a < Tv; ++a) {
      if (a < first_win && fp_row[a] < 0) continue;
      double w = exp(s[a] - m);
      denom += w;
      const uint16_t *vw = vwin + (size_t)(a < first_win ? fp_row[a] : a % W) * D;
      for (int ch = 0; ch < D; ++ch) acc[ch] += w * (double)skvq_ref_half_to_float(vw[ch]);
    }
    for (int ch = 0; ch < D; ++ch) {
      float o = (float)(acc[ch] / denom);
      out_f32[(size_t)bq * D + ch] = o;
      if (out_f16) out_f16[(size_t)bq * D + ch] = skvq_ref_float_to_half(o);
    }
    free(s);
  }
  free(fp_row);
  free(packed_row);
  return fail ? -5 : 0;
}

int skvq_ref_decode_attention(const skvq_ref_config *c, const skvq_ref_buffers *buf,
                              int64_t T, const uint16_t *q, float *out_f32, uint16_t *out_f16) {
  return decode_rows(c, buf, T, NULL, q, 1, out_f32, out_f16);
}

int skvq_ref_decode_attention_filtered(const skvq_ref_config *c, const skvq_ref_buffers *buf, int64_t T,
                                       const uint8_t *keep, const uint16_t *q, int n_new, float *out_f32,
                                       uint16_t *out_f16) {
  return decode_rows(c, buf, T, keep, q, n_new, out_f32, out_f16);
}

int skvq_ref_decode_attention_multi(const skvq_ref_config *c, const skvq_ref_buffers *buf,
                                    int64_t T, const uint16_t *q, int n_new, float *out_f32,
                                    uint16_t *out_f16) {
  return decode_rows(c, buf, T, NULL, q, n_new, out_f32, out_f16);
}

/* ---------------------------------------------------- prefill attention --- */

/* Section 3.2, prefill phase: "compute attention using full-precision KV
 * cache" -- Algorithm 1 with h = 0, l = len(prompt): plain causal softmax
 * attention on the fp16 inputs, original channel order (Eq. 1 with identity
 * permutations), query t seeing keys 0..t. */
/* One row of the prompt's attention: query `t` of (sequence b, query head hq) over keys 0..t.
 * Returns nonzero when memory runs out. */
static int prefill_attention_row(const skvq_ref_config *c, const uint16_t *q, const uint16_t *k,
                                 const uint16_t *v, int64_t T, int b, int hq, int64_t t, float *out_row) {
  int hk = hq / (c->n_q_heads / c->n_kv_heads);
  const uint16_t *qr = q + (((size_t)b * c->n_q_heads + hq) * (size_t)T + (size_t)t) * D;
  const uint16_t *kh = k + ((size_t)b * c->n_kv_heads + hk) * (size_t)T * D;
  const uint16_t *vh = v + ((size_t)b * c->n_kv_heads + hk) * (size_t)T * D;
  double qf[D], acc[D];
  for (int ch = 0; ch < D; ++ch) qf[ch] = skvq_ref_half_to_float(qr[ch]);
  double *s = (double *)malloc(sizeof(double) * (size_t)(t + 1));
  if (!s) return 1;
  double m = -INFINITY;
  for (int64_t a = 0; a <= t; ++a) {
    double dot = 0.0;
    for (int ch = 0; ch < D; ++ch) dot += qf[ch] * (double)skvq_ref_half_to_float(kh[(size_t)a * D + ch]);
    s[a] = (double)c->sm_scale * dot;
    if (s[a] > m) m = s[a];
  }
  double denom = 0.0;
  for (int ch = 0; ch < D; ++ch) acc[ch] = 0.0;
  for (int64_t a = 0; a <= t; ++a) {
    double w = exp(s[a] - m);
    denom += w;
    for (int ch = 0; ch < D; ++ch) acc[ch] += w * (double)skvq_ref_half_to_float(vh[(size_t)a * D + ch]);
  }
  for (int ch = 0; ch < D; ++ch) out_row[ch] = (float)(acc[ch] / denom);
  free(s);
  return 0;
}

int skvq_ref_prefill_attention(const skvq_ref_config *c, const uint16_t *q, const uint16_t *k,
                               const uint16_t *v, int64_t T, float *out_f32) {
  int rc = check_config(c);
  if (rc) return rc;
  if (T < 0) return -1;
  int64_t rows = (int64_t)c->batch * c->n_q_heads * T;
  int fail = 0;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t row = 0; row < rows; ++row) {
    int64_t t = row % T, bq = row / T;
    int b = (int)(bq / c->n_q_heads), hq = (int)(bq % c->n_q_heads);
    if (prefill_attention_row(c, q, k, v, T, b, hq, t, out_f32 + (size_t)row * D)) fail = 1;
  }
  return fail ? -5 : 0;
}

/* The same for chosen rows only (for prompts too long to compute whole): row i is query
 * rows[3 i + 2] of (sequence rows[3 i], query head rows[3 i + 1]); out_f32 [n_rows][D]. */
int skvq_ref_prefill_attention_rows(const skvq_ref_config *c, const uint16_t *q, const uint16_t *k,
                                    const uint16_t *v, int64_t T, const int64_t *rows, int64_t n_rows,
                                    float *out_f32) {
  int rc = check_config(c);
  if (rc) return rc;
  if (T < 0 || n_rows < 0) return -1;
  for (int64_t i = 0; i < n_rows; ++i)
    if (rows[3 * i] < 0 || rows[3 * i] >= c->batch || rows[3 * i + 1] < 0 || rows[3 * i + 1] >= c->n_q_heads ||
        rows[3 * i + 2] < 0 || rows[3 * i + 2] >= T)
      return -1;
  int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_rows; ++i)
    if (prefill_attention_row(c, q, k, v, T, (int)rows[3 * i], (int)rows[3 * i + 1], rows[3 * i + 2],
                              out_f32 + (size_t)i * D))
      fail = 1;
  return fail ? -5 : 0;
}

/* ------------------------------------------------------ clip calibration --- */

/* Eq. 3 (Section 3.1; Algorithm 1 Prologue, get_group_clipping): the clip scale
 * of a group is the one that minimises the squared error of the attention
 * output after quantizing the cache, on calibration data.  The paper leaves the
 * search itself open; this build's is one pass of coordinate descent over a
 * caller-given grid: keys first, then values; group by group; every candidate is
 * tried with the other groups at their current choice; each kv head keeps the
 * candidate with the smallest error summed over its query heads, the queries,
 * the batch and the channels (ties: the earliest candidate).  An evaluation is
 * a prefill-quantize of the calibration tokens followed by one decode attention
 * per calibration query, compared with o_ref, the full-precision outputs. */
int skvq_ref_calibrate_clip(const skvq_ref_config *c, const skvq_ref_buffers *buf, const uint16_t *k,
                            const uint16_t *v, int64_t T, const uint16_t *q, int n_queries,
                            const float *o_ref, const float *alphas, int n_alphas, float *clip_k_out,
                            float *clip_v_out, double *loss_out) {
  int rc = check_config(c);
  if (rc) return rc;
  if (T < 1 || n_queries < 1 || n_alphas < 1 || c->n_kv_heads > 1024) return -1;
  int ng = D / c->group_size, hk_n = c->n_kv_heads, rep = c->n_q_heads / hk_n;
  size_t out_n = (size_t)c->batch * c->n_q_heads * D;
  float *out = (float *)malloc(sizeof(float) * out_n);
  double *err = (double *)malloc(sizeof(double) * (size_t)n_alphas * hk_n);
  if (!out || !err) {
    free(out);
    free(err);
    return -5;
  }
  for (int x = 0; x < hk_n * ng; ++x) clip_k_out[x] = c->clip_k[x], clip_v_out[x] = c->clip_v[x];
  skvq_ref_config cc = *c;
  cc.clip_k = clip_k_out;
  cc.clip_v = clip_v_out;
  for (int which = 0; which < 2 && !rc; ++which) {
    float *clip = which ? clip_v_out : clip_k_out;
    for (int g = 0; g < ng && !rc; ++g) {
      float saved[1024];
      for (int h = 0; h < hk_n; ++h) saved[h] = clip[h * ng + g];
      for (int a = 0; a < n_alphas && !rc; ++a) {
        for (int h = 0; h < hk_n; ++h) clip[h * ng + g] = alphas[a], err[(size_t)a * hk_n + h] = 0.0;
        int64_t n = 0;
        rc = skvq_ref_prefill_quantize(&cc, buf, k, v, T, &n);
        for (int i = 0; i < n_queries && !rc; ++i) {
          rc = skvq_ref_decode_attention(&cc, buf, n, q + (size_t)i * out_n, out, NULL);
          for (size_t x = 0; x < out_n && !rc; ++x) {
            int hq = (int)((x / D) % (size_t)c->n_q_heads);
            double d = (double)out[x] - (double)o_ref[(size_t)i * out_n + x];
            err[(size_t)a * hk_n + hq / rep] += d * d;
          }
        }
      }
      for (int h = 0; h < hk_n && !rc; ++h) {
        int best = 0;
        for (int a = 1; a < n_alphas; ++a)
          if (err[(size_t)a * hk_n + h] < err[(size_t)best * hk_n + h]) best = a;
        clip[h * ng + g] = alphas[best];
        if (loss_out) loss_out[h] = err[(size_t)best * hk_n + h];
      }
      if (rc)
        for (int h = 0; h < hk_n; ++h) clip[h * ng + g] = saved[h];
    }
  }
  free(out);
  free(err);
  return rc;
}

/* ------------------------------------------------------ channel reorder --- */

/* Per (kv head, channel): minimum and maximum over all B*T calibration tokens. */
void skvq_ref_channel_stats(const uint16_t *x, int B, int Hk, int64_t T, float *stats) {
  for (int h = 0; h < Hk; ++h)
    for (int ch = 0; ch < D; ++ch) {
      float mn = INFINITY, mx = -INFINITY;
      for (int b = 0; b < B; ++b)
        for (int64_t t = 0; t < T; ++t) {
          float f = skvq_ref_half_to_float(x[(((size_t)b * Hk + h) * (size_t)T + (size_t)t) * D + ch]);
          if (f < mn) mn = f;
          if (f > mx) mx = f;
        }
      stats[((size_t)h * D + ch) * 2] = mn;
      stats[((size_t)h * D + ch) * 2 + 1] = mx;
    }
}

/* Section 3.1 (channels with similar value distributions are clustered into one
 * group by KMeans over a per-channel feature; Algorithm 1 Prologue,
 * get_permutation_matrix).  The paper names
 * neither the feature nor the initialisation; this build's reading, per kv head:
 *   feature of a channel = (min, max) over the calibration tokens;
 *   k = D/G clusters; channels ordered by range max-min (ties: channel index),
 *   initial centroid j = mean feature of the j-th run of G channels in that order;
 *   Lloyd iterations in fp64 (nearest centroid by squared Euclidean distance, ties:
 *   the lowest cluster; an empty cluster keeps its centroid) until no channel
 *   moves, at most max_iter;
 *   clusters are listed by the range of their centroid, ascending (ties: index),
 *   the channels of a cluster by their own range, ascending (ties: index):
 *   perm[p] = channel at reordered position p; the groups are the clusters, their
 *   boundaries rounded to multiples of `granularity` (nearest; every group keeps
 *   at least `granularity` positions), which moves the channels next to a
 *   boundary into the neighbouring group. */
int skvq_ref_calibrate_reorder(const float *stats, int Hk, int group_size, int granularity,
                               int max_iter, int32_t *perm, int32_t *bounds) {
  if (group_size <= 0 || D % group_size || granularity < 1 || group_size % granularity || max_iter < 0)
    return -1;
  int ng = D / group_size;
  for (int h = 0; h < Hk; ++h) {
    const float *f = stats + (size_t)h * D * 2;
    double rng[D];
    int order[D], label[D];
    for (int ch = 0; ch < D; ++ch) rng[ch] = (double)f[2 * ch + 1] - (double)f[2 * ch], order[ch] = ch;
    for (int i = 1; i < D; ++i) { /* insertion sort by (range, channel) */
      int o = order[i], j = i;
      while (j > 0 && rng[order[j - 1]] > rng[o]) order[j] = order[j - 1], --j;
      order[j] = o;
    }
    double cmin[D], cmax[D];
    for (int j = 0; j < ng; ++j) {
      double a = 0.0, b = 0.0;
      for (int i = 0; i < group_size; ++i) {
        a += (double)f[2 * order[j * group_size + i]];
        b += (double)f[2 * order[j * group_size + i] + 1];
      }
      cmin[j] = a / group_size, cmax[j] = b / group_size;
    }
    for (int ch = 0; ch < D; ++ch) label[ch] = -1;
    for (int it = 0; it <= max_iter; ++it) {
      int moved = 0;
      for (int ch = 0; ch < D; ++ch) {
        int best = 0;
        double bd = 0.0;
        for (int j = 0; j < ng; ++j) {
          double da = (double)f[2 * ch] - cmin[j], db = (double)f[2 * ch + 1] - cmax[j];
          double d = da * da + db * db;
          if (j == 0 || d < bd) best = j, bd = d;
        }
        if (best != label[ch]) label[ch] = best, moved = 1;
      }
      if (!moved || it == max_iter) break;
      for (int j = 0; j < ng; ++j) {
        double a = 0.0, b = 0.0;
        int n = 0;
        for (int ch = 0; ch < D; ++ch)
          if (label[ch] == j) a += (double)f[2 * ch], b += (double)f[2 * ch + 1], ++n;
        if (n) cmin[j] = a / n, cmax[j] = b / n;
      }
    }
    /* clusters by centroid range */
    int corder[D];
    for (int j = 0; j < ng; ++j) corder[j] = j;
    for (int i = 1; i < ng; ++i) {
      int o = corder[i], j = i;
      while (j > 0 && cmax[corder[j - 1]] - cmin[corder[j - 1]] > cmax[o] - cmin[o]) corder[j] = corder[j - 1], --j;
      corder[j] = o;
    }
    int32_t *pm = perm + (size_t)h * D, *gb = bounds + (size_t)h * (ng + 1);
    int p = 0;
    gb[0] = 0;
    for (int jj = 0; jj < ng; ++jj) {
      for (int i = 0; i < D; ++i) /* `order` is by (range, channel) already */
        if (label[order[i]] == corder[jj]) pm[p++] = order[i];
      gb[jj + 1] = p;
    }
    /* boundaries to multiples of the granularity, every group at least that large */
    for (int j = 1; j < ng; ++j) {
      int b = ((2 * gb[j] + granularity) / (2 * granularity)) * granularity; /* nearest, halves up */
      int lo = gb[j - 1] + granularity, hi = D - (ng - j) * granularity;
      gb[j] = b < lo ? lo : b > hi ? hi : b;
    }
  }
  return 0;
}

int skvq_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
