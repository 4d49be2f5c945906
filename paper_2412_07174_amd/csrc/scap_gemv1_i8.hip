// Instantiations of the one-token GEMV kernel for i8 weights.
#include "scap_gemv1.hpp"

namespace scap {
template int launch_gemv1_wdt<kI8>(const Gemv1Args&, int, int, hipStream_t);
template int launch_gemv1_wdt<kI8Half>(const Gemv1Args&, int, int, hipStream_t);
}  // namespace scap
