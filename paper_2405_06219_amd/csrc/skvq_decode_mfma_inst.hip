// One (K format, V format) pair of the matrix-core decode kernels: compiled once per pair with
// -DSKVQ_KL=<key levels> -DSKVQ_VL=<value levels> (the pairs are listed in build.py and in the
// dispatcher, skvq_decode_mfma.hip).
#include "skvq_decode_mfma_kernel.h"

#if !defined(SKVQ_KL) || !defined(SKVQ_VL)
#error "compile with -DSKVQ_KL=4|8|16 -DSKVQ_VL=3|4|8|16"
#endif

namespace skvq {
template hipError_t launch_decode_mfma_fmt<SKVQ_KL, SKVQ_VL>(const Layout &, const __half *, long long, long long,
                                                             int, int, int, const __half *, const __half *, long long,
                                                             MergeOut, hipStream_t);
}  // namespace skvq
