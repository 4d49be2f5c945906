// Instantiations of the one-token GEMV kernel for i8 weights.
#include "scap_gemv1b.hpp"

namespace scap {
template int launch_gemv1_wdt<kI8>(const Gemv1Args&, int, int, hipStream_t);
template int launch_gemv1_wdt<kI8Half>(const Gemv1Args&, int, int, hipStream_t);
template int launch_gemv1_block<kI8, kFuseSwiglu>(const Gemv1Args&, hipStream_t);
template int launch_gemv1_block<kI8, kFuseList>(const Gemv1Args&, hipStream_t);
template int launch_gemv1_block<kI8Half, kFuseSwiglu>(const Gemv1Args&, hipStream_t);
template int launch_gemv1_block<kI8Half, kFuseList>(const Gemv1Args&, hipStream_t);
template int launch_gemv1b_wdt<kI8>(const Gemv1bArgs&, hipStream_t);
template int launch_gemv1b_wdt<kI8Half>(const Gemv1bArgs&, hipStream_t);
template int launch_gemv1b_block_wdt<kI8>(const Gemv1bArgs&, int, hipStream_t);
template int launch_gemv1b_block_wdt<kI8Half>(const Gemv1bArgs&, int, hipStream_t);
}  // namespace scap
