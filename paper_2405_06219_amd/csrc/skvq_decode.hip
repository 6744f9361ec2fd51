// Decode attention over the mixed-precision cache (Eq. 1; Algorithm 1 with l = 1) for gfx950.
//
// The packed region of every (sequence, kv head) is cut into n_splits chunks of whole 64-token
// tiles; one workgroup per chunk keeps a running (max, sum, weighted value sum) per query
// head of the GQA group (online softmax) and writes one partial.  The fp16 ring is one more
// chunk.  A merge kernel combines the partials, and returns the result in original channel
// order.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "skvq_internal.h"
#include "skvq_meta.h"

namespace skvq {

namespace {

constexpr int kMaxR = 8;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// code of reordered position p of the token in slot s of a V block
__device__ __forceinline__ unsigned v_code(const uint8_t *blk, int levels, int s, int p) {
  const int kb = s >> 3, i = s & 7, n = p >> 4, j = p & 15, u = 16 * kb + j;
  if (levels == 4) {
    const unsigned w = reinterpret_cast<const unsigned *>(blk + 16 * u)[n >> 1];
    return (w >> (16 * (i & 1) + 8 * (n & 1) + 2 * (i >> 1))) & 3u;
  }
  const uint8_t *unit = blk + 13 * u;
  const int bit = 13 * n, byte = bit >> 3;
  unsigned w = unit[byte] | (unit[byte + 1] << 8);
  if (byte + 2 < 13) w |= unit[byte + 2] << 16;
  unsigned f = (w >> (bit & 7)) & 0x1fffu;
  for (int q = 0; q < i; ++q) f /= 3;
  return f % 3;
}

// ---------------------------------------------------------------------------------------
// Generic chunk kernel: any group size, any GQA ratio up to 8.  Plain vector arithmetic;
// thread = token for the scores, thread = reordered position for the value sum.
// grid (n_splits + 1, Hk, B); the last x index is the fp16 ring.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void decode_generic_kernel(Layout L, const __half *__restrict__ q,
                                                             long long T, long long nq, int n_sink,
                                                             int n_splits, long long tiles_per_split,
                                                             int sp_base) {
  __shared__ float qs[kMaxR][kD];     // query in the order the chunk's keys use, times sm_scale*log2(e)
  __shared__ float qsum[kMaxR][4];    // its per-group sums
  __shared__ float pr[kMaxR][256];    // softmax numerators of the current tile
  __shared__ float red[kMaxR][4];
  __shared__ float accs[kMaxR][kD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sp = blockIdx.x + sp_base, hk = blockIdx.y, b = blockIdx.z;
  const bool ring = sp == n_splits;
  const long long head = (long long)b * L.Hk + hk;
  const int R = L.R, G = L.G, NG = L.NG;
  // fp16 tokens in token order: n_sink sink rows (rows W.. of the ring buffers), then the window
  const long long n_fp = T - nq, first_win = nq + n_sink;
  const long long win_rows = (long long)L.W + L.S;
  auto fp_row = [&](long long u) { return u < n_sink ? L.W + u : (first_win + (u - n_sink)) % L.W; };
  const float c = L.sm_scale * kLog2e;

  for (int x = tid; x < R * kD; x += 256) {
    const int r = x / kD, p = x % kD;
    const int ch = ring ? p : L.perm_k[hk * kD + p];
    qs[r][p] = c * __half2float(q[((long long)b * L.Hq + hk * R + r) * kD + ch]);
  }
  __syncthreads();
  if (tid < R * NG) {
    const int r = tid / NG, g = tid % NG;
    float s = 0.f;
    for (int p = g * G; p < (g + 1) * G; ++p) s += qs[r][p];
    qsum[r][g] = s;
  }
  __syncthreads();

  long long t_begin, t_end;
  if (ring) {
    t_begin = 0;
    t_end = n_fp;
  } else {
    t_begin = (long long)sp * tiles_per_split * 64;
    t_end = t_begin + tiles_per_split * 64;
    if (t_end > nq) t_end = nq;
    if (t_begin > t_end) t_begin = t_end;
  }

  float m[kMaxR], l[kMaxR], acc[kMaxR];
  for (int r = 0; r < kMaxR; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.f;
    acc[r] = 0.f;
  }
  const int p_own = tid & 127, half_id = tid >> 7;  // value phase: position, and which half of the tile
  const int g_own = p_own / G;

  for (long long tile = t_begin; tile < t_end; tile += 256) {
    const long long t = tile + tid;
    const bool valid = t < t_end;
    float s[kMaxR];
    for (int r = 0; r < kMaxR; ++r) s[r] = -INFINITY;
    if (valid) {
      if (ring) {
        const __half *row = L.k_win + (head * win_rows + fp_row(t)) * kD;
        for (int r = 0; r < R; ++r) s[r] = 0.f;
        for (int ch = 0; ch < kD; ++ch) {
          const float kv = __half2float(row[ch]);
          for (int r = 0; r < R; ++r) s[r] += qs[r][ch] * kv;
        }
      } else {
        const unsigned *row = reinterpret_cast<const unsigned *>(L.k_codes + (head * L.Tcap + t) * (kD / 4));
        const long long meta0 = (head * L.Tcap + t) * NG;
        for (int r = 0; r < R; ++r) s[r] = 0.f;
        for (int g = 0; g < NG; ++g) {
          float dot[kMaxR];
          for (int r = 0; r < R; ++r) dot[r] = 0.f;
          for (int p = g * G; p < (g + 1) * G; ++p) {
            const float code = (float)((row[p >> 4] >> (2 * (p & 15))) & 3u);
            for (int r = 0; r < R; ++r) dot[r] += qs[r][p] * code;
          }
          const float2 mz = meta_load_pair(L.k_meta, meta0 + g, L.meta_fmt);
          for (int r = 0; r < R; ++r) s[r] += mz.x * dot[r] + mz.y * qsum[r][g];
        }
      }
    }
    // tile maximum and new running maximum per query head
    for (int r = 0; r < R; ++r) {
      const float wm = wave_max(s[r]);
      if (lane == 0) red[r][wave] = wm;
    }
    __syncthreads();
    float scale_old[kMaxR];
    for (int r = 0; r < R; ++r) {
      const float tm = fmaxf(fmaxf(red[r][0], red[r][1]), fmaxf(red[r][2], red[r][3]));
      const float mn = fmaxf(m[r], tm);
      scale_old[r] = exp2f(m[r] - mn);  // m = -inf on the first tile gives 0
      m[r] = mn;
      const float pv = valid ? exp2f(s[r] - mn) : 0.f;
      pr[r][tid] = pv;
      s[r] = pv;
    }
    __syncthreads();
    for (int r = 0; r < R; ++r) {
      const float ws = wave_sum(s[r]);
      if (lane == 0) red[r][wave] = ws;
    }
    __syncthreads();
    for (int r = 0; r < R; ++r) {
      l[r] = l[r] * scale_old[r] + (red[r][0] + red[r][1] + red[r][2] + red[r][3]);
      acc[r] *= scale_old[r];
    }
    // weighted value sum: this thread owns position p_own over one half of the tile
    const int n_in_tile = (int)((t_end - tile) < 256 ? (t_end - tile) : 256);
    for (int k = half_id * 128; k < half_id * 128 + 128 && k < n_in_tile; ++k) {
      const long long tt = tile + k;
      float val;
      if (ring) {
        val = __half2float(L.v_win[(head * win_rows + fp_row(tt)) * kD + p_own]);
      } else {
        const uint8_t *blk = L.v_codes + (head * L.n_vblocks + tt / kVBlock) * L.v_block_bytes;
        const float2 mz = meta_load_pair(L.v_meta, (head * L.Tcap + tt) * NG + g_own, L.meta_fmt);
        val = (float)v_code(blk, L.v_levels, (int)(tt % kVBlock), p_own) * mz.x + mz.y;
      }
      for (int r = 0; r < R; ++r) acc[r] += pr[r][k] * val;
    }
    __syncthreads();
  }

  // fold the two halves, write the partial in ORIGINAL channel order
  if (half_id == 1)
    for (int r = 0; r < R; ++r) accs[r][p_own] = acc[r];
  __syncthreads();
  if (half_id == 0) {
    const int ch = ring ? p_own : L.perm_v[hk * kD + p_own];
    for (int r = 0; r < R; ++r) {
      float *part = L.workspace + (((long long)b * L.Hq + hk * R + r) * (SKVQ_MAX_SPLITS + 1) + sp) * kPartialStride;
      part[4 + ch] = acc[r] + accs[r][p_own];
      if (p_own == 0) {
        part[0] = m[r];
        part[1] = l[r];
      }
    }
  }
}

// Combines the chunk partials of one (sequence, query head): out = sum_i acc_i 2^(m_i - m*) /
// sum_i l_i 2^(m_i - m*).  Partials hold base-2 exponents.  grid (Hq, B), 1024 threads:
// wavefront 0 turns the (m_i, l_i) into weights, thread (channel, slice) adds every eighth
// partial.
__global__ __launch_bounds__(1024) void merge_kernel(Layout L, float *__restrict__ out_f32,
                                                     __half *__restrict__ out_f16, int n_all) {
  __shared__ float wts[SKVQ_MAX_SPLITS + 1];
  __shared__ float den_s;
  __shared__ float red[8][kD];
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const float *base = L.workspace + ((long long)b * L.Hq + hq) * (SKVQ_MAX_SPLITS + 1) * kPartialStride;
  const int ch = tid & 127, sl = tid >> 7;
  // the first 32 partials' values are requested before their weights are known: one round trip
  float pre[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = sl + 8 * k;
    pre[k] = i < n_all ? base[(long long)i * kPartialStride + 4 + ch] : 0.f;
  }
  if (tid < 64) {
    float mi[3], li[3], mstar = -INFINITY;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int i = tid + 64 * k;
      mi[k] = -INFINITY, li[k] = 0.f;
      if (i < n_all) {
        const float2 ml = *reinterpret_cast<const float2 *>(base + (long long)i * kPartialStride);
        mi[k] = ml.x, li[k] = ml.y;
      }
      if (li[k] > 0.f) mstar = fmaxf(mstar, mi[k]);
    }
    mstar = wave_max(mstar);
    float den = 0.f;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int i = tid + 64 * k;
      const float w = li[k] > 0.f ? exp2f(mi[k] - mstar) : 0.f;
      if (i < n_all) wts[i] = w;
      den += w * li[k];
    }
    den = wave_sum(den);
    if (tid == 0) den_s = den;
  }
  __syncthreads();
  float num = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = sl + 8 * k;
    if (i < n_all && wts[i] > 0.f) num = fmaf(wts[i], pre[k], num);
  }
  for (int i = sl + 32; i < n_all; i += 8) {
    const float w = wts[i];
    if (w > 0.f) num = fmaf(w, base[(long long)i * kPartialStride + 4 + ch], num);
  }
  red[sl][ch] = num;
  __syncthreads();
  if (tid < kD) {
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) tot += red[k][tid];
    const float o = tot / den_s;
    const long long idx = ((long long)b * L.Hq + hq) * kD + tid;
    out_f32[idx] = o;
    if (out_f16) out_f16[idx] = __float2half_rn(o);
  }
}

}  // namespace

hipError_t launch_decode(const Layout &L, const __half *q, float *out_f32, __half *out_f16, long long T,
                         int n_splits, hipStream_t s) {
  const Counts n = counts_of(T, L.W, L.S);
  const long long nq = n.n_quant;
  if (L.Hk > 65535 || L.B > 65535 || L.Hq > 65535) return hipErrorInvalidValue;
  if (n_splits > SKVQ_MAX_SPLITS || (nq > 0 && n_splits < 1)) return hipErrorInvalidValue;
  if (nq == 0) n_splits = 0;
  const long long tiles = (nq + 63) / 64;
  const long long tps = n_splits ? (tiles + n_splits - 1) / n_splits : 0;
  hipError_t e;
  int n_parts;
  if (decode_mfma_supported(L)) {
    if (n_splits < 1) n_splits = 1;
    e = launch_decode_mfma(L, q, T, nq, (int)n.n_sink, n_splits, s);
    if (e != hipSuccess) return e;
    n_parts = n_splits;  // the ring is folded into the chunks' partials
  } else {
    hipLaunchKernelGGL(decode_generic_kernel, dim3(n_splits + 1, L.Hk, L.B), dim3(256), 0, s, L, q, T, nq,
                       (int)n.n_sink, n_splits, tps, 0);
    n_parts = n_splits + 1;
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(merge_kernel, dim3(L.Hq, L.B), dim3(1024), 0, s, L, out_f32, out_f16, n_parts);
  return hipGetLastError();
}

}  // namespace skvq
