// Instantiations of the one-token GEMV kernel for bf16 weights.
#include "scap_gemv1.hpp"

namespace scap {
template int launch_gemv1_wdt<kBF16>(const Gemv1Args&, int, int, hipStream_t);
}  // namespace scap
