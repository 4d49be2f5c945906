// Launch of the one-token GEMV kernel (scap_gemv1.hpp): K split, argument block, dispatch by weight type.
#include "scap_gemv1.hpp"

namespace scap {

extern template int launch_gemv1_wdt<kF16>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1_wdt<kBF16>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1_wdt<kI8>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1_wdt<kI8Half>(const Gemv1Args&, int, int, hipStream_t);

// One token through a K x N layer (sparse, dense or bias-folding mode).  Returns a scap_status, or
// kG1NotApplicable when the shape needs more than 2048 channels per workgroup (the caller then takes the
// general kernel).  cfg: rows_per_group and unroll are honoured, flags bit 0 forces device-scope loads.
int launch_gemv1(const GemvArgs& g, int wdt, const scap_launch_cfg* cfg, hipStream_t stream) {
    if (g.B != 1) return kG1NotApplicable;
    // int8 weights: 16 bytes per lane (1024-column tiles) unless that leaves at most 4 tiles -- then 8 bytes per
    // lane, twice the tiles and half the K splits (14336 x 4096 int8: 18.8 -> ?? us dense)
    const bool i8_half = wdt == kI8 && g.N <= 4 * 1024;
    const int elems = wdt == kI8 && !i8_half ? 16 : 8;
    const int tile = kWave * elems;
    int kc = 0, unroll = 0, flags = 0, waves = 8;
    if (cfg) {
        if (cfg->rows_per_group) kc = cfg->rows_per_group;
        if (cfg->unroll) unroll = cfg->unroll;
        if (cfg->waves_per_group) waves = cfg->waves_per_group;
        flags = cfg->flags;
        if (kc < 0 || (kc % 8) != 0) return SCAP_ERR_CONFIG;  // whole octets of channels per workgroup
        if (kc > kG1MaxChunks * kG1Chunk) return kG1NotApplicable;
    }
    GemvArgs p = g;
    // LDS: header, the eight wavefronts' sums, then 8 bytes per listed channel
    const size_t lds_budget = 64 * 1024 - (size_t)waves * tile * 4 - 64 + (kHdrBytes - kG1HdrBytes);
    // Rows per workgroup in multiples of 64, unless the input is so short that 64-row pieces would leave compute
    // units without a workgroup (1024 x 4096: 16 splits x 8 tiles; with 32-row pieces 8.5 -> 6.5 us dense)
    p.T = (p.N + tile - 1) / tile;
    const int granule = ((int64_t)((p.K + kWave - 1) / kWave) * p.T < 256) ? 8 : kWave;
    const int rc = plan_splits(p, tile, 1, kc, cfg && cfg->rows_per_group, lds_budget, granule);
    if (rc != SCAP_OK) return rc == SCAP_ERR_SHAPE ? kG1NotApplicable : rc;
    if (p.Kc > kG1MaxChunks * kG1Chunk) return kG1NotApplicable;

    // rows in flight per wavefront: 4 x 1 KB (16-byte lanes), 8 x 512 bytes (8-byte lanes)
    if (unroll == 0) unroll = i8_half ? 8 : 4;
    Gemv1Args a{};
    a.W = g.W;
    a.x = g.x;
    a.col_scale = g.col_scale;
    a.bias = g.bias;
    a.y = g.y;
    a.partial = g.partial;
    a.counters = g.counters;
    a.idx_out = g.idx_out;
    a.nnz_out = g.nnz_out;
    a.union_nnz_out = g.union_nnz_out;
    a.seg_cnt = g.seg_cnt;
    a.K = g.K;
    a.N = g.N;
    a.Kc = p.Kc;
    a.S = p.S;
    a.T = p.T;
    a.mode = g.mode;
    a.xdt = g.xdt;
    a.flags = flags;
    a.m = g.m;
    a.tau = g.tau;
    switch (wdt) {
        case kF16: return launch_gemv1_wdt<kF16>(a, waves, unroll, stream);
        case kBF16: return launch_gemv1_wdt<kBF16>(a, waves, unroll, stream);
        case kI8: return i8_half ? launch_gemv1_wdt<kI8Half>(a, waves, unroll, stream) : launch_gemv1_wdt<kI8>(a, waves, unroll, stream);
    }
    return SCAP_ERR_DTYPE;
}

}  // namespace scap
