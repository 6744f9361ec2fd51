// Measurement yardstick of the library (no part of the method): a kernel that only reads.  The
// decode path is bound by how fast the packed cache can be read from HBM; this gives the time that
// reading the same number of bytes, and nothing else, takes on the device at hand, in the launch
// shape that a sweep found fastest for it: eight workgroups of 256 threads per compute unit,
// grid-strided streaming 16-byte loads (consecutive workgroups read consecutive 4 KB pieces).
// Measured for 78 MB slices / 2.5 GB: 12.2 us / 354 us (6.4 / 7.1 TB/s); the same with plain loads
// 12.9 / 391 us; 1 to 4 workgroups per compute unit with 4 to 32 loads per thread in flight 13.1 to
// 14.7 / 362 to 476 us; each workgroup of 512 threads its own contiguous slice, the decode kernel's
// pattern, 13.1 us.
#include <hip/hip_runtime.h>

#include "skvq_internal.h"

namespace skvq {
namespace {

typedef unsigned uint4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void read_yardstick_kernel(const uint4_t *__restrict__ src, size_t n16,
                                                             unsigned *__restrict__ sink) {
  // grid-strided: consecutive workgroups read consecutive 4 KB pieces
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += stride) {
    const uint4_t a = __builtin_nontemporal_load(src + i);
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
  hipLaunchKernelGGL(skvq::read_yardstick_kernel, dim3(8 * cus), dim3(256), 0, (hipStream_t)stream,
                     (const skvq::uint4_t *)src, bytes / 16, (unsigned *)sink);
  return hipGetLastError() == hipSuccess ? SKVQ_OK : SKVQ_ERR_HIP;
}
