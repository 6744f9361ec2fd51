// Kernel of the clip calibration (Eq. 3; Algorithm 1 Prologue, get_group_clipping): the squared
// error of one decode call's outputs against the full-precision outputs, per (sequence, kv head).
// The search itself is host code (skvq_calibrate_clip in skvq_api.hip) that runs the
// prefill-quantize and decode kernels once per candidate.
#include <hip/hip_runtime.h>

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
