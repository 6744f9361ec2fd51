// Merge of the split partials of skvq_decode_attention (Eq. 1; Algorithm 1 with l = 1) for
// gfx950, and the launcher of one decode call.
//
// The packed region of every (sequence, kv head) is cut into n_splits chunks of whole 64-token
// tiles; the chunk kernel (skvq_decode_mfma.hip) keeps a running (max, sum, weighted value sum)
// per query head (online softmax) and writes one partial per chunk, in original channel order.
// A kv head read as one chunk has its output written by the chunk kernel; several chunks' partials
// are combined by the merge kernel below.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "skvq_internal.h"

namespace skvq {

namespace {

__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
  return v;
}


// Combines the chunk partials of one (sequence, query head): out = sum_i acc_i 2^(m_i - m*) /
// sum_i l_i 2^(m_i - m*).  Partials hold base-2 exponents.  grid (Hq, B), 1024 threads:
// wavefront 0 turns the (m_i, l_i) into weights, thread (channel, slice) adds every eighth
// partial.
__global__ __launch_bounds__(1024) void merge_kernel(Layout L, float *__restrict__ out_f32,
                                                     __half *__restrict__ out_f16, int n_all, int n_heads) {
  __shared__ float wts[SKVQ_MAX_SPLITS + 1];
  __shared__ float den_s;
  __shared__ float red[8][kD];
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  // n_heads = query tokens x query heads per sequence; hq counts (token, head) pairs
  const float *base = L.workspace + ((long long)b * n_heads + hq) * (SKVQ_MAX_SPLITS + 1) * kPartialStride;
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
    const long long idx = ((long long)b * n_heads + hq) * kD + tid;
    out_f32[idx] = o;
    if (out_f16) out_f16[idx] = __float2half_rn(o);
  }
}

}  // namespace

hipError_t launch_decode(const Layout &L, const __half *q, float *out_f32, __half *out_f16, long long T,
                         long long n_kept, int n_splits, int n_new, hipStream_t s, const __half *k_new,
                         const __half *v_new) {
  const Counts n = counts_with(T, L.W, n_kept);
  if (n_kept < 0 || n_kept > L.S || n.n_quant < 0 || n.n_quant > L.Tcap) return hipErrorInvalidValue;
  if (L.Hk > 65535 || L.B > 65535 || (long long)L.Hq * n_new > 65535) return hipErrorInvalidValue;
  if (n_new < 1 || n_new > n.n_win) return hipErrorInvalidValue;  // the new tokens are all in the window
  if (n_splits > SKVQ_MAX_SPLITS || (n.n_quant > 0 && n_splits < 1)) return hipErrorInvalidValue;
  if (n_splits < 1) n_splits = 1;  // nothing packed yet: one chunk, fp16 tokens only
  if (k_new && (n_new != 1 || !append_fusable(L, T, false))) return hipErrorInvalidValue;
  // (with the new token taken along: the leaving token's packed row is the last one)
  const long long te = k_new && T - 1 >= L.W ? n.n_quant - 1 : -1;
  MergeOut mo;
  mo.out_f32 = out_f32;
  mo.out_f16 = out_f16;
  mo.mode = n_splits == 1 ? kMergeDirect : kMergeSeparate;
  hipError_t e = launch_decode_mfma(L, q, T, n.n_quant, (int)n.n_sink, n_splits, n_new, k_new, v_new, te, mo, s);
  if (e != hipSuccess || mo.mode != kMergeSeparate) return e;
  // the fp16 tokens are folded into the chunks' partials
  hipLaunchKernelGGL(merge_kernel, dim3(L.Hq * n_new, L.B), dim3(1024), 0, s, L, out_f32, out_f16, n_splits,
                     L.Hq * n_new);
  return hipGetLastError();
}

}  // namespace skvq
