// Instantiations of the column-gathered GEMV kernel for f16 weights.
#include "scap_gemv_launch.hpp"

namespace scap {
template int launch_wdt<kF16>(const GemvArgs&, int, int, int, int, hipStream_t);
}  // namespace scap
