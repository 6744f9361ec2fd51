// Host side of libskvq: argument checking, size arithmetic, token counters and kernel
// launches.  See include/skvq.h for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "skvq_internal.h"

using namespace skvq;

// Split partials of skvq_decode_attention_static: device memory that exists from load time, so that
// the call itself allocates nothing.  One copy per GPU, shared by every cache on that GPU; the name
// below is only a host-side handle, the device address comes from hipGetSymbolAddress (per device).
// (File scope, not an unnamed namespace: the runtime finds the device copy by the symbol's name.)
constexpr size_t kStaticScratchFloats =
    (size_t)SKVQ_STATIC_MAX_ROWS * (SKVQ_MAX_SPLITS + 1) * skvq::kPartialStride;
static __device__ __align__(256) float scratch[kStaticScratchFloats];

struct skvq_cache {
  float *static_scratch = nullptr;  // this cache's device's copy of `scratch` (looked up at creation)
  int device = -1;                  // the HIP device that was current at creation
  Layout L;
  long long n_tokens = 0;
  long long n_kept = 0;  // tokens older than the window that the filter rules keep in fp16 (<= L.S)
  int *dev_kept_ids = nullptr;  // device [S]: their token numbers (written by a prefill with a mask)
  int forced_splits = 0;
  int max_new = 1;  // query tokens per sequence the workspace was sized for
  int n_cus = 256;
  void *dev_consts = nullptr;  // one allocation: perm_k, perm_v, clip_k, clip_v
  std::vector<float> clip_k, clip_v;  // host copies of the clip scales [Hk][NG]
  std::string last_error;
};

namespace {

int check_config(const skvq_config *c) {
  if (!c) return SKVQ_ERR_INVALID_ARG;
  if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->window < 1 || c->n_sink < 0 ||
      c->max_quant_tokens < 1)
    return SKVQ_ERR_INVALID_ARG;
  if (c->n_q_heads % c->n_kv_heads) return SKVQ_ERR_INVALID_ARG;
  if (c->head_dim != kD) return SKVQ_ERR_UNSUPPORTED;
  if (c->n_q_heads / c->n_kv_heads > 8) return SKVQ_ERR_UNSUPPORTED;
  if (c->group_size != 32 && c->group_size != 64 && c->group_size != 128)
    return SKVQ_ERR_UNSUPPORTED;
  if (c->k_bits != SKVQ_BITS_2 && c->k_bits != SKVQ_BITS_3 && c->k_bits != SKVQ_BITS_4) return SKVQ_ERR_UNSUPPORTED;
  if (c->v_bits != SKVQ_BITS_2 && c->v_bits != SKVQ_BITS_1P5 && c->v_bits != SKVQ_BITS_3 && c->v_bits != SKVQ_BITS_4)
    return SKVQ_ERR_UNSUPPORTED;
  // 3-bit keys go with 3-bit values (the one 3-bit setting of Table 1)
  if ((c->k_bits == SKVQ_BITS_3) != (c->v_bits == SKVQ_BITS_3)) return SKVQ_ERR_UNSUPPORTED;
  if (c->meta_format != SKVQ_META_F32 && c->meta_format != SKVQ_META_F16 &&
      c->meta_format != SKVQ_META_FP8_E4M3)
    return SKVQ_ERR_UNSUPPORTED;
  if (!(c->sm_scale >= 0.0f) || !std::isfinite(c->sm_scale)) return SKVQ_ERR_INVALID_ARG;
  if (c->max_new_tokens < 0 || c->max_new_tokens > SKVQ_MAX_NEW_TOKENS) return SKVQ_ERR_INVALID_ARG;
  if ((long long)c->window > (1ll << 20) || c->n_sink > (1 << 20)) return SKVQ_ERR_INVALID_ARG;
  // the kernels hold packed token numbers (and a tile's 64 tokens past the last one) in 32-bit integers
  if (c->max_quant_tokens > SKVQ_MAX_QUANT_TOKENS) return SKVQ_ERR_UNSUPPORTED;
  if (!c->perm_k || !c->perm_v || !c->clip_k || !c->clip_v) return SKVQ_ERR_INVALID_ARG;
  const int ng = kD / c->group_size;
  if (c->group_bounds) {
    for (int h = 0; h < c->n_kv_heads; ++h) {
      const int32_t *gb = c->group_bounds + (size_t)h * (ng + 1);
      if (gb[0] != 0 || gb[ng] != kD) return SKVQ_ERR_INVALID_ARG;
      for (int g = 0; g < ng; ++g)
        if (gb[g + 1] <= gb[g]) return SKVQ_ERR_INVALID_ARG;
    }
    for (int x = 0; x < c->n_kv_heads * (ng + 1); ++x)
      if (c->group_bounds[x] % 16) return SKVQ_ERR_UNSUPPORTED;
  }
  for (int which = 0; which < 2; ++which) {
    const int32_t *perm = which ? c->perm_v : c->perm_k;
    const float *clip = which ? c->clip_v : c->clip_k;
    for (int h = 0; h < c->n_kv_heads; ++h) {
      bool seen[kD] = {false};
      for (int p = 0; p < kD; ++p) {
        int32_t ch = perm[h * kD + p];
        if (ch < 0 || ch >= kD || seen[ch]) return SKVQ_ERR_INVALID_ARG;
        seen[ch] = true;
      }
      for (int g = 0; g < ng; ++g) {
        float a = clip[h * ng + g];
        if (!(a > 0.0f && a <= 1.0f)) return SKVQ_ERR_INVALID_ARG;
      }
    }
  }
  return SKVQ_OK;
}

void compute_sizes(const skvq_config *c, size_t bytes[7]) {
  const size_t heads = (size_t)c->batch * c->n_kv_heads;
  const size_t tcap = (size_t)c->max_quant_tokens;
  const size_t ng = kD / c->group_size;
  const size_t vb = v_block_bytes_of(c->v_bits);  // skvq_bits values are level counts
  bytes[0] = heads * tcap * k_row_bytes_of(c->k_bits);
  bytes[1] = heads * ((tcap + kVBlock - 1) / kVBlock) * vb;
  const size_t es = c->meta_format == SKVQ_META_FP8_E4M3 ? 1 : c->meta_format == SKVQ_META_F16 ? 2 : 4;
  bytes[2] = heads * tcap * ng * 2 * es;
  bytes[3] = bytes[2];
  bytes[4] = heads * ((size_t)c->window + (size_t)c->n_sink) * kD * sizeof(__half);
  bytes[5] = bytes[4];
  // one partial per (sequence, query head, split); the ring is one more split
  const size_t max_new = c->max_new_tokens > 0 ? (size_t)c->max_new_tokens : 1;
  bytes[6] = (size_t)c->batch * max_new * c->n_q_heads * (SKVQ_MAX_SPLITS + 1) * kPartialStride * sizeof(float);
}

int fail_hip(skvq_cache *c, hipError_t e, const char *what) {
  c->last_error = std::string(what) + ": " + hipGetErrorString(e);
  return SKVQ_ERR_HIP;
}

// where the cached tokens are now
Counts counts_now(const skvq_cache *c) { return counts_with(c->n_tokens, c->L.W, c->n_kept); }
// the sink rule's decision for token a when it leaves the window
bool sink_rule_keeps(const skvq_cache *c, long long a) { return a < c->L.S && c->n_kept < c->L.S; }

// One append with the filter rules' decision for the token that leaves the window (if any).
int append_with(skvq_cache *c, const void *k_new, const void *v_new, bool keep, hipStream_t s, const char *what) {
  const long long T = c->n_tokens;
  const bool leaves = T >= c->L.W;
  const Counts n = counts_now(c);
  if (leaves && (keep ? c->n_kept >= c->L.S : n.n_quant >= c->L.Tcap)) return SKVQ_ERR_CAPACITY;
  hipError_t e = launch_append(c->L, (const __half *)k_new, (const __half *)v_new, T,
                               leaves && keep ? (int)c->n_kept : -1, n.n_quant, s);
  if (e != hipSuccess) return fail_hip(c, e, what);
  c->n_tokens = T + 1;
  if (leaves && keep) ++c->n_kept;
  return SKVQ_OK;
}

int choose_splits(const skvq_cache *c, long long n_quant, int n_new = 1) {
  if (n_quant <= 0) return 0;
  const long long tiles = (n_quant + 63) / 64;  // a split is a whole number of 64-token tiles
  long long s;
  if (c->forced_splits > 0) {
    s = c->forced_splits;
  } else {
    // one workgroup per compute unit over all (sequence, kv head) pairs, but every wavefront of
    // a workgroup should have at least two tiles
    const long long heads = (long long)c->L.B * c->L.Hk * decode_passes(c->L.R * n_new);
    s = c->n_cus / heads;
    const long long cap = tiles / (2 * kMfmaWavesPerGroup);
    if (s > cap) s = cap;
  }
  if (s > SKVQ_MAX_SPLITS) s = SKVQ_MAX_SPLITS;
  if (s > tiles) s = tiles;
  if (s < 1) s = 1;
  return (int)s;
}

}  // namespace

extern "C" {

int skvq_validate_config(const skvq_config *cfg) { return check_config(cfg); }

int skvq_sizes(const skvq_config *cfg, size_t bytes[7]) {
  if (!bytes) return SKVQ_ERR_INVALID_ARG;
  // sizes do not depend on perm/clip; allow them to be absent here
  if (!cfg) return SKVQ_ERR_INVALID_ARG;
  skvq_config tmp = *cfg;
  std::vector<int32_t> ident;
  std::vector<float> ones;
  if (!tmp.perm_k || !tmp.perm_v || !tmp.clip_k || !tmp.clip_v) {
    if (tmp.n_kv_heads < 1 || tmp.n_kv_heads > (1 << 20)) return SKVQ_ERR_INVALID_ARG;
    ident.resize((size_t)tmp.n_kv_heads * kD);
    for (size_t i = 0; i < ident.size(); ++i) ident[i] = (int32_t)(i % kD);
    ones.assign((size_t)tmp.n_kv_heads * 4, 1.0f);
    if (!tmp.perm_k) tmp.perm_k = ident.data();
    if (!tmp.perm_v) tmp.perm_v = ident.data();
    if (!tmp.clip_k) tmp.clip_k = ones.data();
    if (!tmp.clip_v) tmp.clip_v = ones.data();
  }
  int rc = check_config(&tmp);
  if (rc != SKVQ_OK) return rc;
  compute_sizes(&tmp, bytes);
  return SKVQ_OK;
}

int skvq_create(const skvq_config *cfg, const skvq_buffers *bufs, skvq_cache **out) {
  if (!out) return SKVQ_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != SKVQ_OK) return rc;
  if (!bufs) return SKVQ_ERR_INVALID_ARG;
  const void *ptrs[7] = {bufs->k_codes, bufs->v_codes, bufs->k_meta, bufs->v_meta,
                         bufs->k_win,   bufs->v_win,   bufs->workspace};
  for (const void *p : ptrs)
    if (!p || ((uintptr_t)p & 15)) return SKVQ_ERR_INVALID_ARG;

  skvq_cache *c = new (std::nothrow) skvq_cache();
  if (!c) return SKVQ_ERR_HIP;
  Layout &L = c->L;
  L.B = cfg->batch;
  L.Hq = cfg->n_q_heads;
  L.Hk = cfg->n_kv_heads;
  L.R = L.Hq / L.Hk;
  L.G = cfg->group_size;
  L.NG = kD / L.G;
  L.uneq = 0;
  std::vector<unsigned> gmaps((size_t)L.Hk, 0u);
  for (int h = 0; h < L.Hk; ++h)
    for (int n = 0; n < 8; ++n) {  // group of positions 16n .. 16n+15 of kv head h
      int g = 16 * n / L.G;
      if (cfg->group_bounds) {
        const int32_t *gb = cfg->group_bounds + (size_t)h * (L.NG + 1);
        g = 0;
        while (16 * n >= gb[g + 1]) ++g;
        if (g != 16 * n / L.G) L.uneq = 1;
      }
      gmaps[h] |= (unsigned)g << (4 * n);
    }
  c->max_new = cfg->max_new_tokens > 0 ? cfg->max_new_tokens : 1;
  L.W = cfg->window;
  L.S = cfg->n_sink;
  L.meta_fmt = cfg->meta_format;
  L.k_levels = cfg->k_bits;
  L.k_row_bytes = k_row_bytes_of(L.k_levels);
  L.v_levels = cfg->v_bits;
  L.v_block_bytes = v_block_bytes_of(L.v_levels);
  L.Tcap = cfg->max_quant_tokens;
  L.n_vblocks = (L.Tcap + kVBlock - 1) / kVBlock;
  L.sm_scale = cfg->sm_scale > 0.0f ? cfg->sm_scale : 1.0f / std::sqrt((float)kD);
  if (cfg->sm_scale == 0.0f) L.sm_scale = 1.0f / std::sqrt((float)kD);
  L.k_codes = (uint8_t *)bufs->k_codes;
  L.v_codes = (uint8_t *)bufs->v_codes;
  L.k_meta = bufs->k_meta;
  L.v_meta = bufs->v_meta;
  L.k_win = (__half *)bufs->k_win;
  L.v_win = (__half *)bufs->v_win;
  L.workspace = (float *)bufs->workspace;

  // constants: [perm_k | perm_v | clip_k | clip_v | gmaps | kept token numbers], one allocation
  const size_t n_perm = (size_t)L.Hk * kD, n_clip = (size_t)L.Hk * L.NG;
  const size_t off_pv = n_perm * 4, off_ck = off_pv + n_perm * 4;
  const size_t off_cv = off_ck + ((n_clip * 4 + 15) & ~(size_t)15);
  const size_t off_gm = off_cv + ((n_clip * 4 + 15) & ~(size_t)15);
  const size_t off_ids = off_gm + (((size_t)L.Hk * 4 + 15) & ~(size_t)15);
  const size_t total = off_ids + (((size_t)L.S * 4 + 15) & ~(size_t)15);
  std::vector<uint8_t> host(total, 0);
  std::memcpy(host.data(), cfg->perm_k, n_perm * 4);
  std::memcpy(host.data() + off_pv, cfg->perm_v, n_perm * 4);
  std::memcpy(host.data() + off_ck, cfg->clip_k, n_clip * 4);
  std::memcpy(host.data() + off_cv, cfg->clip_v, n_clip * 4);
  std::memcpy(host.data() + off_gm, gmaps.data(), (size_t)L.Hk * 4);

  hipError_t e = hipMalloc(&c->dev_consts, total);
  if (e != hipSuccess) {
    delete c;
    return SKVQ_ERR_HIP;
  }
  e = hipMemcpy(c->dev_consts, host.data(), total, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(c->dev_consts);
    delete c;
    return SKVQ_ERR_HIP;
  }
  c->clip_k.assign(cfg->clip_k, cfg->clip_k + n_clip);
  c->clip_v.assign(cfg->clip_v, cfg->clip_v + n_clip);
  uint8_t *d = (uint8_t *)c->dev_consts;
  L.perm_k = (const int *)d;
  L.perm_v = (const int *)(d + off_pv);
  L.clip_k = (const float *)(d + off_ck);
  L.clip_v = (const float *)(d + off_cv);
  L.gmaps = (const unsigned *)(d + off_gm);
  c->dev_kept_ids = (int *)(d + off_ids);

  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
      prop.multiProcessorCount > 0)
    c->n_cus = prop.multiProcessorCount;
  // the static scratch array's address on this device (each GPU has its own copy at its own address)
  c->device = dev;
  void *sp = nullptr;
  e = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
  if (e == hipSuccess) {
    c->static_scratch = (float *)sp;
  } else {
    c->static_scratch = nullptr;  // skvq_decode_attention_static reports it; the other calls do not need it
    c->last_error = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
    (void)hipGetLastError();
  }
  *out = c;
  return SKVQ_OK;
}

void skvq_destroy(skvq_cache *c) {
  if (!c) return;
  if (c->dev_consts) (void)hipFree(c->dev_consts);
  delete c;
}

int skvq_prefill_quantize(skvq_cache *c, const void *k, const void *v, int64_t T, void *stream) {
  return skvq_prefill_quantize_filtered(c, k, v, T, nullptr, stream);
}

int skvq_prefill_quantize_filtered(skvq_cache *c, const void *k, const void *v, int64_t T, const uint8_t *keep,
                                   void *stream) {
  if (!c) return SKVQ_ERR_INVALID_ARG;
  if (T < 0 || (T > 0 && (!k || !v))) return SKVQ_ERR_INVALID_ARG;
  const long long left = T > c->L.W ? T - c->L.W : 0;  // tokens older than the window
  long long n_kept;
  const int *ids = nullptr;
  if (keep) {
    if (T > 0x7fffffffll) return SKVQ_ERR_UNSUPPORTED;
    std::vector<int> list;
    for (long long a = 0; a < left; ++a)
      if (keep[a]) {
        if ((long long)list.size() >= c->L.S) return SKVQ_ERR_CAPACITY;
        list.push_back((int)a);
      }
    n_kept = (long long)list.size();
    if (n_kept > 0) {
      // On the caller's stream (an earlier prefill on it may still be reading the previous list), and
      // waited for: the host list is gone when this function returns.
      hipError_t e = hipMemcpyAsync(c->dev_kept_ids, list.data(), list.size() * sizeof(int), hipMemcpyHostToDevice,
                                    (hipStream_t)stream);
      if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
      if (e != hipSuccess) return fail_hip(c, e, "skvq_prefill_quantize_filtered copy of the kept tokens");
      ids = c->dev_kept_ids;
    }
  } else {
    n_kept = left < c->L.S ? left : c->L.S;
  }
  if (left - n_kept > c->L.Tcap) return SKVQ_ERR_CAPACITY;
  if (T > 0) {
    hipError_t e = launch_prefill(c->L, (const __half *)k, (const __half *)v, T, n_kept, ids, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(c, e, "skvq_prefill_quantize launch");
  }
  c->n_tokens = T;
  c->n_kept = n_kept;
  return SKVQ_OK;
}

int skvq_prefill_attention(skvq_cache *c, const void *q, const void *k, const void *v, int64_t T, void *out_f32,
                           void *out_f16, void *stream) {
  if (!c || !q || !k || !v || !out_f32 || T < 1) return SKVQ_ERR_INVALID_ARG;
  const void *ptrs[5] = {q, k, v, out_f32, out_f16};
  for (const void *p : ptrs)
    if ((uintptr_t)p & 15) return SKVQ_ERR_INVALID_ARG;
  hipError_t e = launch_prefill_attention(c->L, (const __half *)q, (const __half *)k, (const __half *)v,
                                          (float *)out_f32, (__half *)out_f16, T, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e, "skvq_prefill_attention launch");
  return SKVQ_OK;
}

// Writes the host copies of the clip scales to the device, ordered in `stream`, and waits.
static int upload_clips(skvq_cache *c, hipStream_t stream) {
  const size_t bytes = c->clip_k.size() * sizeof(float);
  hipError_t e = hipMemcpyAsync(const_cast<float *>(c->L.clip_k), c->clip_k.data(), bytes, hipMemcpyHostToDevice, stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(const_cast<float *>(c->L.clip_v), c->clip_v.data(), bytes, hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  return e == hipSuccess ? SKVQ_OK : fail_hip(c, e, "clip scale upload");
}

int skvq_prefill_attention_quantize(skvq_cache *c, const void *q, const void *k, const void *v, int64_t T,
                                    void *out_f32, void *out_f16, void *stream) {
  // refuse before anything is launched what the second step would refuse
  if (!c || T < 1) return SKVQ_ERR_INVALID_ARG;
  const long long left = T > c->L.W ? T - c->L.W : 0;
  if (left - (left < c->L.S ? left : c->L.S) > c->L.Tcap) return SKVQ_ERR_CAPACITY;
  const int rc = skvq_prefill_attention(c, q, k, v, T, out_f32, out_f16, stream);
  if (rc != SKVQ_OK) return rc;
  return skvq_prefill_quantize(c, k, v, T, stream);
}

int skvq_calibrate_channel_stats(const void *x, int32_t batch, int32_t n_kv_heads, int64_t T, float *stats,
                                 void *stream_) {
  if (!x || !stats || batch < 1 || n_kv_heads < 1 || T < 1 || ((uintptr_t)x & 15) || batch > 65535 ||
      n_kv_heads > 65535 || T > (1ll << 40))
    return SKVQ_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const long long heads = (long long)batch * n_kv_heads;
  long long chunks = 4096 / heads;  // about 4096 workgroups over all heads, at least 64 rows each
  if (chunks > (T + 63) / 64) chunks = (T + 63) / 64;
  if (chunks < 1) chunks = 1;
  const size_t n_part = (size_t)heads * chunks * kD * 2;
  float *d_part = nullptr;
  if (hipMalloc(&d_part, n_part * sizeof(float)) != hipSuccess) return SKVQ_ERR_HIP;
  std::vector<float> part(n_part);
  hipError_t e = launch_channel_stats((const __half *)x, d_part, batch, n_kv_heads, T, (int)chunks, stream);
  if (e == hipSuccess) e = hipMemcpyAsync(part.data(), d_part, n_part * sizeof(float), hipMemcpyDeviceToHost, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  (void)hipFree(d_part);
  if (e != hipSuccess) return SKVQ_ERR_HIP;
  for (int h = 0; h < n_kv_heads; ++h)
    for (int ch = 0; ch < kD; ++ch) {
      float mn = INFINITY, mx = -INFINITY;
      for (int b = 0; b < batch; ++b)
        for (long long k = 0; k < chunks; ++k) {
          const float *p = &part[((((size_t)b * n_kv_heads + h) * chunks + k) * kD + ch) * 2];
          mn = p[0] < mn ? p[0] : mn;
          mx = p[1] > mx ? p[1] : mx;
        }
      stats[((size_t)h * kD + ch) * 2] = mn;
      stats[((size_t)h * kD + ch) * 2 + 1] = mx;
    }
  return SKVQ_OK;
}

int skvq_calibrate_reorder(const float *stats, int32_t n_kv_heads, int32_t group_size, int32_t granularity,
                           int32_t max_iter, int32_t *perm, int32_t *bounds) {
  if (!stats || !perm || !bounds || n_kv_heads < 1 || max_iter < 0 || granularity < 1) return SKVQ_ERR_INVALID_ARG;
  if (group_size != 32 && group_size != 64 && group_size != 128) return SKVQ_ERR_UNSUPPORTED;
  if (group_size % granularity) return SKVQ_ERR_INVALID_ARG;
  for (size_t x = 0; x < (size_t)n_kv_heads * kD * 2; ++x)
    if (!std::isfinite(stats[x])) return SKVQ_ERR_INVALID_ARG;
  return reorder_channels(stats, n_kv_heads, group_size, granularity, max_iter, perm, bounds) ? SKVQ_ERR_INVALID_ARG
                                                                                               : SKVQ_OK;
}

int skvq_set_clip(skvq_cache *c, const float *clip_k, const float *clip_v, void *stream) {
  if (!c || !clip_k || !clip_v) return SKVQ_ERR_INVALID_ARG;
  const size_t n = c->clip_k.size();
  for (size_t x = 0; x < n; ++x)
    if (!(clip_k[x] > 0.0f && clip_k[x] <= 1.0f) || !(clip_v[x] > 0.0f && clip_v[x] <= 1.0f)) return SKVQ_ERR_INVALID_ARG;
  c->clip_k.assign(clip_k, clip_k + n);
  c->clip_v.assign(clip_v, clip_v + n);
  return upload_clips(c, (hipStream_t)stream);
}

int skvq_calibrate_clip(skvq_cache *c, const void *k, const void *v, int64_t T, const void *q, int32_t n_queries,
                        const void *o_ref, const float *alphas, int32_t n_alphas, float *clip_k_out,
                        float *clip_v_out, double *loss_out, void *stream_) {
  if (!c || !k || !v || !q || !o_ref || !alphas || !clip_k_out || !clip_v_out || T < 1 || n_queries < 1 ||
      n_alphas < 1 || n_queries > (1 << 20) || n_alphas > (1 << 16))
    return SKVQ_ERR_INVALID_ARG;
  for (int a = 0; a < n_alphas; ++a)
    if (!(alphas[a] > 0.0f && alphas[a] <= 1.0f)) return SKVQ_ERR_INVALID_ARG;
  const Layout &L = c->L;
  if (counts_of(T, L.W, L.S).n_quant > L.Tcap) return SKVQ_ERR_CAPACITY;
  hipStream_t stream = (hipStream_t)stream_;
  const size_t out_n = (size_t)L.B * L.Hq * kD, slots = (size_t)L.B * L.Hk;
  const size_t err_n = (size_t)n_alphas * n_queries * slots;
  float *d_out = nullptr, *d_err = nullptr;
  hipError_t e = hipMalloc(&d_out, out_n * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&d_err, err_n * sizeof(float));
  if (e != hipSuccess) {
    (void)hipFree(d_out);
    return fail_hip(c, e, "skvq_calibrate_clip allocation");
  }
  std::vector<float> h_err(err_n);
  const std::vector<float> start_k = c->clip_k, start_v = c->clip_v;
  const Counts cnt = counts_of(T, L.W, L.S);
  const int n_splits = choose_splits(c, cnt.n_quant);
  int rc = SKVQ_OK;
  for (int which = 0; which < 2 && rc == SKVQ_OK; ++which) {
    std::vector<float> &clip = which ? c->clip_v : c->clip_k;
    for (int g = 0; g < L.NG && rc == SKVQ_OK; ++g) {
      for (int a = 0; a < n_alphas && rc == SKVQ_OK; ++a) {
        for (int h = 0; h < L.Hk; ++h) clip[(size_t)h * L.NG + g] = alphas[a];
        rc = upload_clips(c, stream);
        if (rc != SKVQ_OK) break;
        e = launch_prefill(L, (const __half *)k, (const __half *)v, T, cnt.n_sink, nullptr, stream);
        for (int i = 0; i < n_queries && e == hipSuccess; ++i) {
          e = launch_decode(L, (const __half *)q + (size_t)i * out_n, d_out, nullptr, T, cnt.n_sink, n_splits, 1, stream);
          if (e == hipSuccess)
            e = launch_sqerr(L, d_out, (const float *)o_ref + (size_t)i * out_n,
                             d_err + ((size_t)a * n_queries + i) * slots, stream);
        }
        if (e != hipSuccess) rc = fail_hip(c, e, "skvq_calibrate_clip launch");
      }
      if (rc != SKVQ_OK) break;
      e = hipMemcpyAsync(h_err.data(), d_err, err_n * sizeof(float), hipMemcpyDeviceToHost, stream);
      if (e == hipSuccess) e = hipStreamSynchronize(stream);
      if (e != hipSuccess) {
        rc = fail_hip(c, e, "skvq_calibrate_clip read-back");
        break;
      }
      for (int h = 0; h < L.Hk; ++h) {  // per kv head: the candidate with the smallest error, the earliest on ties
        int best = 0;
        double best_err = 0.0;
        for (int a = 0; a < n_alphas; ++a) {
          double s = 0.0;
          for (int i = 0; i < n_queries; ++i)
            for (int b = 0; b < L.B; ++b) s += (double)h_err[((size_t)a * n_queries + i) * slots + (size_t)b * L.Hk + h];
          if (a == 0 || s < best_err) best = a, best_err = s;
        }
        clip[(size_t)h * L.NG + g] = alphas[best];
        if (loss_out) loss_out[h] = best_err;
      }
    }
  }
  (void)hipFree(d_out);
  (void)hipFree(d_err);
  if (rc != SKVQ_OK) {  // leave the cache's clip scales as they were
    c->clip_k = start_k;
    c->clip_v = start_v;
    (void)upload_clips(c, stream);
    return rc;
  }
  rc = upload_clips(c, stream);
  if (rc != SKVQ_OK) return rc;
  std::memcpy(clip_k_out, c->clip_k.data(), c->clip_k.size() * sizeof(float));
  std::memcpy(clip_v_out, c->clip_v.data(), c->clip_v.size() * sizeof(float));
  c->n_tokens = T;  // the buffers hold the calibration tokens as the last candidate quantized them
  c->n_kept = cnt.n_sink;
  return SKVQ_OK;
}

int skvq_quantize_append(skvq_cache *c, const void *k_new, const void *v_new, void *stream) {
  if (!c || !k_new || !v_new) return SKVQ_ERR_INVALID_ARG;
  return append_with(c, k_new, v_new, sink_rule_keeps(c, c->n_tokens - c->L.W), (hipStream_t)stream,
                     "skvq_quantize_append launch");
}

int skvq_quantize_append_filtered(skvq_cache *c, const void *k_new, const void *v_new, int32_t keep_leaving,
                                  void *stream) {
  if (!c || !k_new || !v_new) return SKVQ_ERR_INVALID_ARG;
  return append_with(c, k_new, v_new, keep_leaving != 0, (hipStream_t)stream, "skvq_quantize_append_filtered launch");
}

int skvq_decode_attention(skvq_cache *c, const void *q, void *out_f32, void *out_f16, void *stream) {
  if (!c || !q || !out_f32) return SKVQ_ERR_INVALID_ARG;
  if (c->n_tokens <= 0) return SKVQ_ERR_STATE;
  hipError_t e = launch_decode(c->L, (const __half *)q, (float *)out_f32, (__half *)out_f16, c->n_tokens, c->n_kept,
                               choose_splits(c, counts_now(c).n_quant), 1, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e, "skvq_decode_attention launch");
  return SKVQ_OK;
}

int skvq_decode_attention_static(skvq_cache *c, const void *q, void *out_f32, void *out_f16, void *stream) {
  if (!c || !q || !out_f32) return SKVQ_ERR_INVALID_ARG;
  if (c->n_tokens <= 0) return SKVQ_ERR_STATE;
  if ((long long)c->L.B * c->L.Hq > SKVQ_STATIC_MAX_ROWS) {
    c->last_error = "skvq_decode_attention_static: batch * n_q_heads exceeds SKVQ_STATIC_MAX_ROWS";
    return SKVQ_ERR_UNSUPPORTED;
  }
  if (!c->static_scratch) return SKVQ_ERR_HIP;  // the lookup at creation failed; last_error says why
  Layout L = c->L;
  L.workspace = c->static_scratch;  // the kernels take it as they take the caller's workspace
  hipError_t e = launch_decode(L, (const __half *)q, (float *)out_f32, (__half *)out_f16, c->n_tokens, c->n_kept,
                               choose_splits(c, counts_now(c).n_quant), 1, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e, "skvq_decode_attention_static launch");
  return SKVQ_OK;
}

int skvq_append_decode_attention(skvq_cache *c, const void *k_new, const void *v_new, const void *q, void *out_f32,
                                 void *out_f16, void *stream) {
  if (!c || !k_new || !v_new || !q || !out_f32) return SKVQ_ERR_INVALID_ARG;
  const long long T = c->n_tokens;
  const bool leaves = T >= c->L.W, keep = leaves && sink_rule_keeps(c, T - c->L.W);
  const Counts now = counts_now(c);
  const long long nq = now.n_quant + (leaves && !keep ? 1 : 0);  // packed rows after the step
  if (nq > c->L.Tcap) return SKVQ_ERR_CAPACITY;
  hipStream_t s = (hipStream_t)stream;
  const int n_splits = choose_splits(c, nq);
  // One launch pays when few workgroups do the append (one per kv head, of n_splits): with one or
  // two chunks per kv head every (other) workgroup would wait for its own append, which costs more
  // than the separate launch (measured at 16 sequences x 32 heads x 32k tokens: 240 against 236 us).
  if (append_fusable(c->L, T + 1, keep) && n_splits >= kMinSplitsForOneLaunch) {
    hipError_t e = launch_decode(c->L, (const __half *)q, (float *)out_f32, (__half *)out_f16, T + 1, c->n_kept,
                                 n_splits, 1, s, (const __half *)k_new, (const __half *)v_new);
    if (e != hipSuccess) return fail_hip(c, e, "skvq_append_decode_attention launch");
    c->n_tokens = T + 1;
    return SKVQ_OK;
  }
  const int rc = append_with(c, k_new, v_new, keep, s, "skvq_append_decode_attention launch (append)");
  if (rc != SKVQ_OK) return rc;
  hipError_t e = launch_decode(c->L, (const __half *)q, (float *)out_f32, (__half *)out_f16, T + 1, c->n_kept,
                               n_splits, 1, s);
  if (e != hipSuccess) return fail_hip(c, e, "skvq_append_decode_attention launch (decode)");
  return SKVQ_OK;
}

int skvq_decode_attention_multi(skvq_cache *c, const void *q, int32_t n_new, void *out_f32, void *out_f16,
                                void *stream) {
  if (!c || !q || !out_f32 || n_new < 1) return SKVQ_ERR_INVALID_ARG;
  if (c->n_tokens <= 0) return SKVQ_ERR_STATE;
  const Counts n = counts_now(c);
  if (n_new > c->max_new || n_new > n.n_win) return SKVQ_ERR_INVALID_ARG;
  hipError_t e = launch_decode(c->L, (const __half *)q, (float *)out_f32, (__half *)out_f16, c->n_tokens, c->n_kept,
                               choose_splits(c, n.n_quant, n_new), n_new, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e, "skvq_decode_attention_multi launch");
  return SKVQ_OK;
}

int skvq_get_state(const skvq_cache *c, int64_t *n_tokens, int64_t *n_quant, int32_t *n_win) {
  if (!c) return SKVQ_ERR_INVALID_ARG;
  const Counts n = counts_now(c);
  if (n_tokens) *n_tokens = c->n_tokens;
  if (n_quant) *n_quant = n.n_quant;
  if (n_win) *n_win = (int32_t)n.n_win;
  return SKVQ_OK;
}

int skvq_set_state(skvq_cache *c, int64_t n_tokens) {
  if (!c || n_tokens < 0) return SKVQ_ERR_INVALID_ARG;
  if (n_tokens < c->n_tokens) return SKVQ_ERR_STATE;  // no rewind: ring rows and V unit tails are gone
  const Counts n = counts_of(n_tokens, c->L.W, c->L.S);  // (the sink rule)
  if (n.n_quant > c->L.Tcap) return SKVQ_ERR_CAPACITY;
  c->n_tokens = n_tokens;
  c->n_kept = n.n_sink;
  return SKVQ_OK;
}

int skvq_set_num_splits(skvq_cache *c, int32_t n) {
  if (!c || n < 0 || n > SKVQ_MAX_SPLITS) return SKVQ_ERR_INVALID_ARG;
  c->forced_splits = n;
  return SKVQ_OK;
}

const char *skvq_status_string(int s) {
  switch (s) {
    case SKVQ_OK: return "ok";
    case SKVQ_ERR_INVALID_ARG: return "invalid argument";
    case SKVQ_ERR_UNSUPPORTED: return "unsupported configuration";
    case SKVQ_ERR_CAPACITY: return "packed region full";
    case SKVQ_ERR_STATE: return "invalid state (empty cache, or a rewind)";
    case SKVQ_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char *skvq_last_error(const skvq_cache *c) { return c ? c->last_error.c_str() : ""; }

}  // extern "C"
