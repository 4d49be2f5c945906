// Instantiations of the one-token GEMV kernel for bf16 weights.
#include "scap_gemv1b.hpp"

namespace scap {
template int launch_gemv1_wdt<kBF16>(const Gemv1Args&, int, int, hipStream_t);
template int launch_gemv1_block<kBF16, kFuseSwiglu>(const Gemv1Args&, hipStream_t);
template int launch_gemv1_block<kBF16, kFuseList>(const Gemv1Args&, hipStream_t);
template int launch_gemv1b_wdt<kBF16>(const Gemv1bArgs&, hipStream_t);
template int launch_gemv1b_block_wdt<kBF16>(const Gemv1bArgs&, int, hipStream_t);
}  // namespace scap
