// Instantiations of the column-gathered GEMV kernel for i8 weights.
#include "scap_gemv_launch.hpp"

namespace scap {
template int launch_wdt<kI8>(const GemvArgs&, int, int, int, int, hipStream_t);
}  // namespace scap
