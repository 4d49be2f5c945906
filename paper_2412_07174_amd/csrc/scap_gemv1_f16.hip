// Instantiations of the one-token GEMV kernel for f16 weights.
#include "scap_gemv1b.hpp"

namespace scap {
template int launch_gemv1_wdt<kF16>(const Gemv1Args&, int, int, hipStream_t);
template int launch_gemv1_block<kF16, kFuseSwiglu>(const Gemv1Args&, hipStream_t);
template int launch_gemv1_block<kF16, kFuseList>(const Gemv1Args&, hipStream_t);
template int launch_gemv1b_wdt<kF16>(const Gemv1bArgs&, hipStream_t);
template int launch_gemv1b_block_wdt<kF16>(const Gemv1bArgs&, int, hipStream_t);
}  // namespace scap
