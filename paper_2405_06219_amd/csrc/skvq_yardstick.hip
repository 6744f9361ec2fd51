// Measurement yardstick of the library (no part of the method): a kernel that only reads.  The
// decode path is bound by how fast the packed cache can be read from HBM; this gives the time that
// reading the same number of bytes, and nothing else, takes on the device at hand, in the launch
// shape of the decode kernel (one workgroup of 512 threads per compute unit, contiguous slices,
// 16-byte loads, several in flight per lane).
#include <hip/hip_runtime.h>

#include "skvq_internal.h"

namespace skvq {
namespace {

typedef unsigned uint4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512) void read_yardstick_kernel(const uint4_t *__restrict__ src, size_t n16,
                                                             unsigned *__restrict__ sink) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t begin = blockIdx.x * per, end = begin + per < n16 ? begin + per : n16;
  unsigned acc = 0;
  size_t i = begin + threadIdx.x;
  for (; i + 3 * 512 < end; i += 4 * 512) {  // four loads in flight per lane
    const uint4_t a = src[i], b = src[i + 512], c = src[i + 1024], d = src[i + 1536];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < end; i += 512) {
    const uint4_t a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x5ca1ab1eu) sink[0] = acc;  // (keeps the loads alive; practically never taken)
}

}  // namespace
}  // namespace skvq

extern "C" int skvq_read_yardstick(const void *src, size_t bytes, void *sink, void *stream) {
  if (!src || !sink || bytes == 0 || (bytes & 15) || ((uintptr_t)src & 15)) return SKVQ_ERR_INVALID_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return SKVQ_ERR_HIP;
  hipLaunchKernelGGL(skvq::read_yardstick_kernel, dim3(cus), dim3(512), 0, (hipStream_t)stream,
                     (const skvq::uint4_t *)src, bytes / 16, (unsigned *)sink);
  return hipGetLastError() == hipSuccess ? SKVQ_OK : SKVQ_ERR_HIP;
}
