// Measurement yardsticks of the library (no part of the method): a kernel that only reads, and one
// that reads and writes in the prefill quantizer's proportion.  The
// decode path is bound by how fast the packed cache can be read from HBM; this gives the time that
// reading the same number of bytes, and nothing else, takes on the device at hand, in the launch
// shape that a sweep found fastest for it: eight workgroups of 256 threads per compute unit,
// grid-strided streaming 16-byte loads (consecutive workgroups read consecutive 4 KB pieces).
// Measured for 78 MB slices / 2.5 GB: 12.2 us / 354 us (6.4 / 7.1 TB/s); the same with plain loads
// 12.9 / 391 us; 1 to 4 workgroups per compute unit with 4 to 32 loads per thread in flight 13.1 to
// 14.7 / 362 to 476 us; each workgroup of 512 threads its own contiguous slice, the decode kernel's
// pattern, 13.1 us.
//
// The prefill quantizer reads the prompt's fp16 K and V once and writes about a seventh of that as
// packed codes; reads and writes that share the memory system run slower than reads alone.  The
// read/write kernel moves the same mix and computes nothing: a workgroup of 256 threads makes one
// trip, `ratio` streaming 16-byte loads per thread (each a contiguous 4 KB piece per workgroup) and
// one streaming 16-byte store of their XOR -- the fastest shape of a sweep.  Measured for 537 MB
// read + 77 MB written / 8.6 GB + 1.2 GB: 101 us / 1.74 ms (6.0 / 5.65 TB/s); grid-strided with
// fewer, longer-lived workgroups 5.3 to 5.8 / 4.7 to 5.3 TB/s; plain instead of streaming stores or
// loads 5 to 10 % less.
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

constexpr int kMaxRatio = 8;

template <int RATIO>
__global__ __launch_bounds__(256) void read_write_yardstick_kernel(const uint4_t *__restrict__ src,
                                                                   uint4_t *__restrict__ dst) {
  // workgroup g reads the RATIO 4 KB pieces from piece g * RATIO on and writes 4 KB piece g
  const uint4_t *from = src + ((size_t)blockIdx.x * RATIO) * 256 + threadIdx.x;
  uint4_t a[RATIO];
#pragma unroll
  for (int j = 0; j < RATIO; ++j) a[j] = __builtin_nontemporal_load(from + (size_t)j * 256);
  uint4_t acc = a[0];
#pragma unroll
  for (int j = 1; j < RATIO; ++j) acc ^= a[j];
  __builtin_nontemporal_store(acc, dst + (size_t)blockIdx.x * 256 + threadIdx.x);
}

}  // namespace
}  // namespace skvq

extern "C" int skvq_read_write_yardstick(const void *src, void *dst, size_t write_bytes, int32_t ratio, void *stream) {
  if (!src || !dst || write_bytes == 0 || (write_bytes & 4095) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15) ||
      ratio < 1 || ratio > skvq::kMaxRatio || write_bytes / 4096 > 0x7fffffffull)
    return SKVQ_ERR_INVALID_ARG;
  const dim3 grid((unsigned)(write_bytes / 4096)), block(256);
#define SKVQ_RW(R)                                                                                             \
  case R:                                                                                                      \
    hipLaunchKernelGGL(skvq::read_write_yardstick_kernel<R>, grid, block, 0, (hipStream_t)stream,               \
                       (const skvq::uint4_t *)src, (skvq::uint4_t *)dst);                                        \
    break
  switch (ratio) {
    SKVQ_RW(1); SKVQ_RW(2); SKVQ_RW(3); SKVQ_RW(4); SKVQ_RW(5); SKVQ_RW(6); SKVQ_RW(7); SKVQ_RW(8);
  }
#undef SKVQ_RW
  return hipGetLastError() == hipSuccess ? SKVQ_OK : SKVQ_ERR_HIP;
}

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
