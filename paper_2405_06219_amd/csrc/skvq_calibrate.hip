// Kernel of the clip calibration (Eq. 3; Algorithm 1 Prologue, get_group_clipping): the squared
// error of one decode call's outputs against the full-precision outputs, per (sequence, kv head).
// The search itself is host code (skvq_calibrate_clip in skvq_api.hip) that runs the
// prefill-quantize and decode kernels once per candidate.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "skvq_internal.h"

namespace skvq {
namespace {

// grid (Hk, B), 256 threads: err[b * Hk + hk] = sum over the kv head's query heads and channels
// of (out - ref)^2, summed in a fixed order (the result does not depend on scheduling).
__global__ __launch_bounds__(256) void sqerr_kernel(const float *__restrict__ out, const float *__restrict__ ref,
                                                    float *__restrict__ err, int Hq, int Hk) {
  __shared__ float part[256];
  const int hk = blockIdx.x, b = blockIdx.y, R = Hq / Hk, tid = threadIdx.x;
  const size_t base = ((size_t)b * Hq + (size_t)hk * R) * kD;
  float s = 0.f;
  for (int x = tid; x < R * kD; x += 256) {
    const float d = out[base + x] - ref[base + x];
    s = fmaf(d, d, s);
  }
  part[tid] = s;
  __syncthreads();
  for (int off = 128; off; off >>= 1) {
    if (tid < off) part[tid] += part[tid + off];
    __syncthreads();
  }
  if (tid == 0) err[(size_t)b * Hk + hk] = part[0];
}

}  // namespace

hipError_t launch_sqerr(const Layout &L, const float *out, const float *ref, float *err, hipStream_t s) {
  if (L.Hk > 65535 || L.B > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(sqerr_kernel, dim3(L.Hk, L.B), dim3(256), 0, s, out, ref, err, L.Hq, L.Hk);
  return hipGetLastError();
}

}  // namespace skvq

// ---------------------------------------------------------------------------------------
// Channel reorder (Section 3.1; Algorithm 1 Prologue, get_permutation_matrix): per-channel
// (min, max) of the calibration tokens on the GPU; the clustering over them is host code
// (skvq_reorder.hip).
// ---------------------------------------------------------------------------------------
namespace skvq {
namespace {

typedef unsigned uint4_t __attribute__((ext_vector_type(4)));

// grid (chunks, Hk, B), 256 threads.  A wavefront reads four rows per load (lane = row l/16,
// channels 8 (l%16) .. +7) and keeps their minima and maxima; the rows of the chunk are dealt to
// the four wavefronts.  part[((b*Hk + hk)*chunks + chunk)][D][2] (fp32).
__global__ __launch_bounds__(256) void channel_stats_kernel(const __half *__restrict__ x, float *__restrict__ part,
                                                            long long T, int Hk, long long rows_per_chunk) {
  __shared__ float red[4][kD][2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const long long head = (long long)b * Hk + hk;
  const uint4_t *src = reinterpret_cast<const uint4_t *>(x + head * T * kD);
  const long long t0 = chunk * rows_per_chunk, t1 = t0 + rows_per_chunk < T ? t0 + rows_per_chunk : T;
  float mn[8], mx[8];  // channels 8 (lane%16) + e
#pragma unroll
  for (int e = 0; e < 8; ++e) mn[e] = INFINITY, mx[e] = -INFINITY;
  for (long long t = t0 + 4 * wave + (lane >> 4); t < t1; t += 16) {
    const uint4_t v = src[t * 16 + (lane & 15)];
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const __half2 h2 = __builtin_bit_cast(__half2, w[j]);
      const float lo = __low2float(h2), hi = __high2float(h2);
      mn[2 * j] = fminf(mn[2 * j], lo), mx[2 * j] = fmaxf(mx[2 * j], lo);
      mn[2 * j + 1] = fminf(mn[2 * j + 1], hi), mx[2 * j + 1] = fmaxf(mx[2 * j + 1], hi);
    }
  }
  // the four rows of a load sit 16 lanes apart
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int off = 16; off < 64; off <<= 1) {
      mn[e] = fminf(mn[e], __shfl_xor(mn[e], off));
      mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], off));
    }
  if (lane < 16) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      red[wave][8 * lane + e][0] = mn[e];
      red[wave][8 * lane + e][1] = mx[e];
    }
  }
  __syncthreads();
  if (threadIdx.x < kD) {
    const int ch = threadIdx.x;
    const float a = fminf(fminf(red[0][ch][0], red[1][ch][0]), fminf(red[2][ch][0], red[3][ch][0]));
    const float c = fmaxf(fmaxf(red[0][ch][1], red[1][ch][1]), fmaxf(red[2][ch][1], red[3][ch][1]));
    float *dst = part + ((head * gridDim.x + chunk) * kD + ch) * 2;
    dst[0] = a;
    dst[1] = c;
  }
}

}  // namespace

hipError_t launch_channel_stats(const __half *x, float *part, int B, int Hk, long long T, int chunks,
                                hipStream_t s) {
  if (B < 1 || Hk < 1 || T < 1 || chunks < 1 || Hk > 65535 || B > 65535) return hipErrorInvalidValue;
  const long long rows = (T + chunks - 1) / chunks;
  hipLaunchKernelGGL(channel_stats_kernel, dim3(chunks, Hk, B), dim3(256), 0, s, x, part, T, Hk, rows);
  return hipGetLastError();
}

}  // namespace skvq
