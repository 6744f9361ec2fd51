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
// (min, max) of the calibration tokens on the GPU, KMeans over them on the host.
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

// KMeans over the channels' (min, max), per kv head; see skvq_calibrate_reorder in skvq.h for
// the steps.  Host code, fp64, every operation rounded once (this file is compiled without
// contraction).
int reorder_channels(const float *stats, int Hk, int G, int gran, int max_iter, int32_t *perm, int32_t *bounds) {
  const int ng = kD / G;
  for (int h = 0; h < Hk; ++h) {
    const float *f = stats + (size_t)h * kD * 2;
    double range[kD], cmin[kD], cmax[kD];
    int order[kD], label[kD];
    for (int ch = 0; ch < kD; ++ch) range[ch] = (double)f[2 * ch + 1] - (double)f[2 * ch], order[ch] = ch, label[ch] = -1;
    for (int i = 1; i < kD; ++i) {  // stable insertion sort: by range, then by channel
      const int o = order[i];
      int j = i;
      for (; j > 0 && range[order[j - 1]] > range[o]; --j) order[j] = order[j - 1];
      order[j] = o;
    }
    for (int j = 0; j < ng; ++j) {  // start: the mean feature of every run of G channels in that order
      double a = 0.0, b = 0.0;
      for (int i = 0; i < G; ++i) a += (double)f[2 * order[j * G + i]], b += (double)f[2 * order[j * G + i] + 1];
      cmin[j] = a / G, cmax[j] = b / G;
    }
    for (int it = 0;; ++it) {
      bool moved = false;
      for (int ch = 0; ch < kD; ++ch) {
        int best = 0;
        double best_d = 0.0;
        for (int j = 0; j < ng; ++j) {
          const double da = (double)f[2 * ch] - cmin[j], db = (double)f[2 * ch + 1] - cmax[j];
          const double d = da * da + db * db;
          if (j == 0 || d < best_d) best = j, best_d = d;
        }
        if (best != label[ch]) label[ch] = best, moved = true;
      }
      if (!moved || it == max_iter) break;
      for (int j = 0; j < ng; ++j) {
        double a = 0.0, b = 0.0;
        int n = 0;
        for (int ch = 0; ch < kD; ++ch)
          if (label[ch] == j) a += (double)f[2 * ch], b += (double)f[2 * ch + 1], ++n;
        if (n) cmin[j] = a / n, cmax[j] = b / n;  // an empty cluster keeps its centroid
      }
    }
    int corder[kD];
    for (int j = 0; j < ng; ++j) corder[j] = j;
    for (int i = 1; i < ng; ++i) {  // clusters by the range of their centroid
      const int o = corder[i];
      int j = i;
      for (; j > 0 && cmax[corder[j - 1]] - cmin[corder[j - 1]] > cmax[o] - cmin[o]; --j) corder[j] = corder[j - 1];
      corder[j] = o;
    }
    int32_t *pm = perm + (size_t)h * kD, *gb = bounds + (size_t)h * (ng + 1);
    int p = 0;
    gb[0] = 0;
    for (int jj = 0; jj < ng; ++jj) {
      for (int i = 0; i < kD; ++i)
        if (label[order[i]] == corder[jj]) pm[p++] = order[i];
      gb[jj + 1] = p;
    }
    for (int j = 1; j < ng; ++j) {  // boundaries to the nearest multiple of gran, groups of at least gran
      const int b = ((2 * gb[j] + gran) / (2 * gran)) * gran;
      const int lo = gb[j - 1] + gran, hi = kD - (ng - j) * gran;
      gb[j] = b < lo ? lo : b > hi ? hi : b;
    }
  }
  return 0;
}

}  // namespace skvq
