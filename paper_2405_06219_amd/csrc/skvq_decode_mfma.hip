// Dispatcher of the matrix-core decode kernels over the (K format, V format) pairs; each pair's
// kernels are compiled in a translation unit of their own (skvq_decode_mfma_inst.hip).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "skvq_internal.h"

namespace skvq {

template <int KL, int VL>
hipError_t launch_decode_mfma_fmt(const Layout &L, const __half *q, long long T, long long nq, int n_sink,
                                  int n_splits, int n_new, const __half *knew, const __half *vnew, long long te,
                                  MergeOut mo, hipStream_t s);
#define SKVQ_FMT(KL, VL)                                                                              \
  extern template hipError_t launch_decode_mfma_fmt<KL, VL>(const Layout &, const __half *, long long, \
                                                            long long, int, int, int, const __half *, const __half *,    \
                                                            long long, MergeOut, hipStream_t);
SKVQ_FMT(4, 3) SKVQ_FMT(4, 4) SKVQ_FMT(4, 16) SKVQ_FMT(8, 8) SKVQ_FMT(16, 3) SKVQ_FMT(16, 4) SKVQ_FMT(16, 16)
#undef SKVQ_FMT

hipError_t launch_decode_mfma(const Layout &L, const __half *q, long long T, long long nq, int n_sink,
                              int n_splits, int n_new, const __half *knew, const __half *vnew, long long te,
                              MergeOut mo, hipStream_t s) {
  const int fmt = L.k_levels * 100 + L.v_levels;
  switch (fmt) {
    case 403: return launch_decode_mfma_fmt<4, 3>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    case 404: return launch_decode_mfma_fmt<4, 4>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    case 416: return launch_decode_mfma_fmt<4, 16>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    case 808: return launch_decode_mfma_fmt<8, 8>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    case 1603: return launch_decode_mfma_fmt<16, 3>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    case 1604: return launch_decode_mfma_fmt<16, 4>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    case 1616: return launch_decode_mfma_fmt<16, 16>(L, q, T, nq, n_sink, n_splits, n_new, knew, vnew, te, mo, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace skvq
