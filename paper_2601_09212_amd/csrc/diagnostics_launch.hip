// Per-position terms of Theorem 2 (alpha_i, beta_i): launch code of diag_kernel / diag_combine_kernel.
#include "diagnostics_kernels.h"

namespace csd {

template <int DT, bool XF, bool AL>
static hipError_t launch_diag_local_typed(const KArgs& a, bool ver, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  constexpr int kA = AL ? kAligned : kUnaligned;
  const int64_t pairs = int64_t(a.B) * a.L;
  if (!ver)
    return launch("diag_kernel (one chunk)", diag_kernel<DT, XF, kA, kT / 2, true>, dim3((unsigned)pairs), dim3(512), stream, a);
  // with the verify call's statistics: B more workgroups take the bonus rows
  const int64_t groups = pairs + (a.has_bonus ? a.B : 0);
  return launch("diag_kernel (with the verify call's statistics)", diag_kernel<DT, XF, kA, kT / 2, true, true>,
                dim3((unsigned)groups), dim3(512), stream, a);
}

template <int DT, bool XF, bool AL>
static hipError_t launch_diag_chunks_typed(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  constexpr int kA = AL ? kAligned : kUnaligned;
  const int64_t pairs = int64_t(a.B) * a.L;
  // this pass is the last reader of the logits: beyond what the caches hold, nontemporal loads
  const double bytes = double(pairs) * 2.0 * a.V * Vec<DT>::kES * (a.tu ? 2 : 1);
  const dim3 gridd((unsigned)(pairs * a.nchunks));
  hipError_t e;
  if (AL && bytes > 128e6)
    e = launch("diag_kernel", diag_kernel<DT, XF, AL ? kAlignedStream : kUnaligned, kT / 2, false>, gridd, dim3(kThreads), stream, a);
  else
    e = launch("diag_kernel", diag_kernel<DT, XF, kA, kT / 2, false>, gridd, dim3(kThreads), stream, a);
  if (e != hipSuccess) return e;
  return launch("diag_combine_kernel", diag_combine_kernel, dim3((unsigned)((pairs + kThreads - 1) / kThreads)),
                dim3(kThreads), stream, a);
}

#define CSD_DISPATCH(FN, ...)                                                                              \
  do {                                                                                                     \
    if (dtype == kDtBF16) {                                                                                \
      if (xf) return a.aligned ? FN<kDtBF16, true, true>(__VA_ARGS__) : FN<kDtBF16, true, false>(__VA_ARGS__);   \
      return a.aligned ? FN<kDtBF16, false, true>(__VA_ARGS__) : FN<kDtBF16, false, false>(__VA_ARGS__);   \
    }                                                                                                      \
    if (xf) return a.aligned ? FN<kDtF32, true, true>(__VA_ARGS__) : FN<kDtF32, true, false>(__VA_ARGS__); \
    return a.aligned ? FN<kDtF32, false, true>(__VA_ARGS__) : FN<kDtF32, false, false>(__VA_ARGS__);       \
  } while (0)

hipError_t launch_diag_local(const KArgs& a, int dtype, bool xf, bool ver, hipStream_t stream) {
  CSD_DISPATCH(launch_diag_local_typed, a, ver, stream);
}

hipError_t launch_diag_chunks(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  CSD_DISPATCH(launch_diag_chunks_typed, a, stream);
}

#undef CSD_DISPATCH

}  // namespace csd
