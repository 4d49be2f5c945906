// Instantiations of the column-gathered GEMV kernel for bf16 weights.
#include "scap_gemv_launch.hpp"

namespace scap {
template int launch_wdt<kBF16>(const GemvArgs&, int, int, int, int, hipStream_t);
}  // namespace scap
