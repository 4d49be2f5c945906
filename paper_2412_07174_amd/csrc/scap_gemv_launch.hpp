// The GEMV kernel and its table of instantiations (waves x rows in flight x token slots x lanes per row)
// for one weight dtype.  Included by one translation unit per dtype.
#pragma once

#include "scap_gemv_body.hpp"

namespace scap {

template <int WDT, int WAVES, int UNROLL, int BT, int LPR>
__global__ __launch_bounds__(WAVES * kWave) void gemv_kernel(const GemvArgs a) {
    gemv_body<WDT, WAVES, UNROLL, BT, LPR, kFusePlain>(a);
}

template <int WDT, int WAVES, int UNROLL, int BT, int LPR>
static int launch_one(const GemvArgs& a, hipStream_t stream) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    const size_t lds = lds_bytes(a.Kc, BT, (size_t)WAVES * kWave * (ELEMS > 4 ? ELEMS : 4) * 4);
    if (lds > 64 * 1024) return SCAP_ERR_CONFIG;
    const dim3 grid((unsigned)(a.S * a.T));
    const dim3 block(WAVES * kWave);
    hipLaunchKernelGGL((gemv_kernel<WDT, WAVES, UNROLL, BT, LPR>), grid, block, lds, stream, a);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

template <int WDT, int WAVES, int UNROLL>
static int launch_lpr(const GemvArgs& a, int lpr, hipStream_t stream) {
    switch (lpr) {
        case 64: return launch_one<WDT, WAVES, UNROLL, 1, 64>(a, stream);
        case 32: return launch_one<WDT, WAVES, UNROLL, 1, 32>(a, stream);
    }
    return SCAP_ERR_CONFIG;
}

template <int WDT, int BT>
static int launch_bt(const GemvArgs& a, int waves, int unroll, int lpr, hipStream_t stream) {
    if constexpr (BT == 1) {
#define SCAP_CASE(WV, UN) \
    if (waves == WV && unroll == UN) return launch_lpr<WDT, WV, UN>(a, lpr, stream);
        SCAP_CASE(4, 4) SCAP_CASE(4, 8) SCAP_CASE(4, 16)
        SCAP_CASE(8, 4) SCAP_CASE(8, 8) SCAP_CASE(8, 16)
        SCAP_CASE(16, 4) SCAP_CASE(16, 8) SCAP_CASE(16, 16)
#undef SCAP_CASE
        return SCAP_ERR_CONFIG;
    } else if constexpr (BT <= 4) {
        if (waves == 8 && unroll == 8 && lpr == 64) return launch_one<WDT, 8, 8, BT, 64>(a, stream);
        if (waves == 8 && unroll == 8 && lpr == 32) return launch_one<WDT, 8, 8, BT, 32>(a, stream);
        return SCAP_ERR_CONFIG;
    } else {
        if (waves == 8 && unroll == 4 && lpr == 64) return launch_one<WDT, 8, 4, BT, 64>(a, stream);
        return SCAP_ERR_CONFIG;
    }
}

template <int WDT>
int launch_wdt(const GemvArgs& a, int bt, int waves, int unroll, int lpr, hipStream_t stream) {
    switch (bt) {
        case 1: return launch_bt<WDT, 1>(a, waves, unroll, lpr, stream);
        case 2: return launch_bt<WDT, 2>(a, waves, unroll, lpr, stream);
        case 4: return launch_bt<WDT, 4>(a, waves, unroll, lpr, stream);
        case 8: return launch_bt<WDT, 8>(a, waves, unroll, lpr, stream);
        case 16: return launch_bt<WDT, 16>(a, waves, unroll, lpr, stream);
    }
    return SCAP_ERR_SHAPE;
}

}  // namespace scap
