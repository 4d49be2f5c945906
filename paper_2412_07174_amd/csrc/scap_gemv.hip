// Column-gathered GEMV for a centred, thresholded input (SCAP Alg. 3; Eq. 2, 3, 6), gfx950.
//
// One launch does the whole layer.  The K input channels are cut into S ranges of Kc channels and the
// N output columns into T tiles of one 16-byte vector per lane (512 columns for 16-bit weights, 1024
// for int8).  Workgroup (split, tile):
//   1. centre + threshold its Kc inputs, ballot/prefix-sum the kept channels of every token into an
//      ascending list in LDS (channel index + centred value per token; a channel kept by any token of
//      the batch is in the list, tokens that pruned it carry 0) -- pruned rows are never addressed;
//   2. its wavefronts take list entries round-robin, so the rows a workgroup has to read are spread
//      evenly whatever the mask looks like; each lane streams 16 bytes of a row and keeps fp32 sums;
//   3. the wavefronts' sums are added through LDS and stored as one split-K partial;
//   4. the last workgroup to arrive at a tile (device-scope counter) adds the S partials in split order
//      -- a fixed order, so y is bit-reproducible -- plus the fused bias, and resets the counter.
// The last arrival of tile 0 also closes the gaps between the per-split index lists that the splits
// left in idx_out, and writes nnz_out.
#include "scap_gemv_body.hpp"

namespace scap {

// ---------------------------------------------------------------------------------------------- launch
int plan_splits(GemvArgs& a, int tile, int floats_per_entry, int kc, bool kc_forced, size_t lds_budget, int granule) {
    a.T = (int)((a.N + tile - 1) / tile);
    if (a.T > kMaxTiles) return SCAP_ERR_SHAPE;
    // bounds from the workspace (at most kMaxSplits splits and partial_capacity floats per token) and from
    // LDS (the kept-channel list of one workgroup must fit)
    const size_t tile_cols = (size_t)a.T * tile;
    size_t s_cap = partial_capacity(a.N) / tile_cols;
    if (s_cap > (size_t)kMaxSplits) s_cap = kMaxSplits;
    if (s_cap < 1) s_cap = 1;
    const int kc_lds = (int)((lds_budget - kHdrBytes) / (4 * (1 + floats_per_entry)) / kWave * kWave);
    if (kc == 0) {
        // Rows per workgroup, a multiple of `granule`.  Workgroups are spread over the 256 compute units, so the
        // launch takes about as long as the busiest unit: ceil(workgroups / 256) workgroups, each costing
        // its kc rows plus a fixed part (prologue, reduction, hand-over) worth about kFixedRows rows.
        // Slightly more than 256 workgroups is the worst case (on 4096 x 28672, 280 workgroups of 832 rows
        // took 50.8 us, 224 of 1024 rows 38.2 us); more splits than needed only lengthen the final
        // reduction, so ties go to the larger kc.
        // Candidates: for every split count the smallest kc (a multiple of `granule`) that gives it; any other
        // kc with the same split count only costs more.
        constexpr int kFixedRows = 128;
        long best_cost = -1;
        const long s_max = (long)((a.K + granule - 1) / granule);
        for (long sp = 1; sp <= s_max && (size_t)sp <= s_cap; ++sp) {
            const int c = (int)align_up((size_t)((a.K + sp - 1) / sp), (size_t)granule);
            if (c > kc_lds) continue;
            const long splits = (a.K + c - 1) / c;
            const long cost = ((splits * a.T + 255) / 256) * (c + kFixedRows);
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                kc = c;
            }
        }
        if (kc == 0) return SCAP_ERR_SHAPE;
    }
    int s = (a.K + kc - 1) / kc;
    if ((size_t)s > s_cap) {
        if (kc_forced) return SCAP_ERR_CONFIG;
        kc = (int)align_up((size_t)((a.K + s_cap - 1) / s_cap), kWave);
        s = (a.K + kc - 1) / kc;
    }
    if (kc > kc_lds) {
        if (kc_forced) return SCAP_ERR_CONFIG;
        kc = kc_lds;
        s = (a.K + kc - 1) / kc;
        if ((size_t)s > s_cap) return SCAP_ERR_SHAPE;
    }
    a.Kc = kc;
    a.S = s;
    return SCAP_OK;
}

// launch_wdt<WDT> picks the instantiation for a token count and launch shape; one translation unit per
// weight dtype (scap_gemv_f16.hip, scap_gemv_bf16.hip, scap_gemv_i8.hip) so that they compile side by side.
template <int WDT>
int launch_wdt(const GemvArgs& a, int bt, int waves, int unroll, int lpr, hipStream_t stream);
extern template int launch_wdt<kF16>(const GemvArgs&, int, int, int, int, hipStream_t);
extern template int launch_wdt<kBF16>(const GemvArgs&, int, int, int, int, hipStream_t);
extern template int launch_wdt<kI8>(const GemvArgs&, int, int, int, int, hipStream_t);

int launch_gemv(const GemvArgs& a_in, int wdt, const scap_launch_cfg* cfg, hipStream_t stream) {
    GemvArgs a = a_in;
    int bt = 1;
    while (bt < a.B) bt <<= 1;
    if (bt > SCAP_MAX_TOKENS) return SCAP_ERR_SHAPE;

    // y += result: a property of the one-token kernel alone.  Anything that would take another kernel is refused
    // rather than run with the wrong meaning.
    if (cfg && (cfg->flags & SCAP_CFG_ACCUMULATE)) {
        if (a.B != 1 || a.mode == kModeFold || (cfg->flags & SCAP_CFG_GENERAL_KERNEL) ||
            (cfg->waves_per_group && cfg->waves_per_group != 8 && cfg->waves_per_group != 4) ||
            (cfg->lanes_per_row && cfg->lanes_per_row != 64))
            return SCAP_ERR_CONFIG;
        const int rc = launch_gemv1(a, wdt, cfg, stream);
        return rc == kG1NotApplicable ? SCAP_ERR_CONFIG : rc;
    }

    // Several tokens: the gathered rows form a dense sub-GEMM -> matrix cores (bf16 and int8 weights from 2
    // tokens; fp16 weights from 5, on the single-launch kernel only).
    // lanes_per_row = 16 asks for the single-launch matrix-core kernel (its lane layout), 1 for the
    // two-launch form whose lists live in the workspace, 64 or 32 for the vector kernel.  By default the
    // single-launch kernel runs from kMfmaAutoTokens (bf16) / kMfmaAutoTokensI8 (int8) tokens on, the
    // two-launch form when the input is too long for LDS-sized pieces, the vector kernel otherwise.
    const int lanes = cfg ? cfg->lanes_per_row : 0;
    const bool mfma_ok = a.mode != kModeFold &&
                         ((a.B >= kMfmaMinTokens && (wdt == kBF16 || wdt == kI8)) || (a.B > 4 && wdt == kF16));
    if ((lanes == 16 || lanes == 1) && !mfma_ok) return SCAP_ERR_CONFIG;
    if (lanes == 1 && wdt == kF16) return SCAP_ERR_CONFIG;
    if (lanes == 16) {
        const int rc = launch_gemm_inline(a, wdt, cfg, stream);
        return rc == SCAP_ERR_SHAPE ? SCAP_ERR_CONFIG : rc;
    }
    if (lanes == 1) return launch_gemm_mfma(a, wdt, cfg, stream);
    // 2 tokens: the two-token form of the one-token kernel, unless the caller asks for a launch shape or the
    // general kernels.  Measured against them (dense / 90 % sparse, us), with the fixed-point hand-over: 14336 x 4096
    // bf16 22.56 / 9.26 against 24.36 / 10.94, int8 14.68 / 8.53 against 17.60 / 10.60, 4096 x 4096 bf16 10.41 / 7.01
    // against 12.82 / 7.59, 4096 x 14336 bf16 21.58 / 8.71 against 22.96 / 9.98.  With partial sums handed over
    // instead (layers too wide for the fixed-point words) wide 16-bit layers were faster on the general kernel
    // (23.26 / 10.20 against 23.01 / 9.97): those keep it.
    // 3-4 tokens, 16-bit weights: its four-slot form (fixed-point hand-over only).  Measured against the kernels below
    // (dense / 50 / 90 %, us): 4 tokens 4096 x 14336 bf16 24.4 / 23.0 / 13.4 against 26.1 / 24.9 / 14.8, 4096 x 6144
    // 15.2 / 14.5 / 10.5 against 18.1 / 17.2 / 12.4, 14336 x 4096 25.5 / 24.6 / 14.9 against 24.7 / 25.5 / 15.6 -- so a
    // dense call with a long input into a narrow layer stays on the staged-tile kernel.  int8 weights in 8-byte lanes
    // (N <= 4096; wider int8 layers do not fit and fall through to the matrix cores): 14336 x 4096, 4 tokens,
    // 19.7 / 17.7 / 12.9 at 50 / 70 / 90 % against 19.9 / 18.3 / 14.0, 3 tokens 18.1 / 15.8 / 11.9 against 19.1 / 17.0 / 12.9.
    const bool four_slots = (a.B == 3 || a.B == 4) &&
                            !(a.mode == kModeDense && (int64_t)a.K >= 2 * (int64_t)a.N);
    if ((a.B == 2 || four_slots) && lanes == 0 &&
        (wdt == kI8 || a.N <= 8192 || 2 * (int64_t)a.N <= (int64_t)kFxCols) &&
        !(cfg && ((cfg->flags & SCAP_CFG_GENERAL_KERNEL) || cfg->waves_per_group || cfg->rows_per_group || cfg->unroll))) {
        const int rc = launch_gemv1b(a, wdt, cfg ? cfg->flags : 0, stream);
        if (rc != kG1NotApplicable) return rc;
    }
    // 3-4 tokens in the 16-slot staged-tile kernel: faster than the 4-slot forms for int8 weights unless the layer
    // is very wide (its narrow tiles repeat the prologue), and than the vector kernel for a long input into a
    // narrow bf16 layer (14336 x 4096, 4 tokens: 28.7 -> 27.3 us dense, 22.2 -> 20.0 at 90 %).
    if (mfma_ok && lanes == 0 && a.B >= 3 && a.B <= 4 && a.K % 8 == 0 &&
        ((wdt == kI8 && (int64_t)a.N <= 4 * (int64_t)a.K) || (wdt == kBF16 && (int64_t)a.K >= 2 * (int64_t)a.N))) {
        const int rc = launch_gemm_inline(a, wdt, cfg, stream, true);
        if (rc != SCAP_ERR_SHAPE) return rc;
    }
    const bool mfma_auto = mfma_ok && lanes == 0 && a.B >= (wdt == kI8 ? kMfmaAutoTokensI8 : kMfmaAutoTokens);
    if (mfma_auto) {
        // one launch; the two-launch form takes over where the input is too long for LDS-sized pieces
        int rc = launch_gemm_inline(a, wdt, cfg, stream);
        if (rc == SCAP_ERR_SHAPE && wdt != kF16) rc = launch_gemm_mfma(a, wdt, cfg, stream);
        // more narrow tiles than there are arrival counters: the vector kernel's tiles are four times wider
        if (rc != SCAP_ERR_SHAPE) return rc;
    }

    // One token: the one-token kernel, unless the caller asks for another workgroup shape or the general kernel.
    if (a.B == 1 && !(cfg && ((cfg->flags & SCAP_CFG_GENERAL_KERNEL) || (cfg->waves_per_group && cfg->waves_per_group != 8 && cfg->waves_per_group != 4) ||
                              (cfg->lanes_per_row && cfg->lanes_per_row != 64)))) {
        const int rc = launch_gemv1(a, wdt, cfg, stream);
        if (rc != kG1NotApplicable) return rc;
    }

    int waves = 8, unroll = (bt <= 4) ? 8 : 4, kc = 0, lpr = 64;
    if (cfg) {
        if (cfg->waves_per_group) waves = cfg->waves_per_group;
        if (cfg->unroll) unroll = cfg->unroll;
        if (cfg->rows_per_group) kc = cfg->rows_per_group;
        if (cfg->lanes_per_row) lpr = cfg->lanes_per_row;
        if (kc < 0 || (kc % kWave) != 0) return SCAP_ERR_CONFIG;
        if (lpr != 64 && lpr != 32) return SCAP_ERR_CONFIG;  // 16 and 1 were handled above
    }
    const int elems = (wdt == kI8) ? 16 : 8;
    // Few column tiles mean many K splits, and the tile's last arrival has to pull all their partial sums
    // through one compute unit: with at most 4 full-width tiles (int8 weights and N = 4096, say) half-width
    // tiles halve that (measured on 14336 x 4096 int8: 20.0 -> 18.4 us dense, 10.1 -> 8.1 us at 90 %).
    // With 2-4 tokens the partial sums are 2-4 times larger, and half-width tiles also pay off at 8 full-width
    // tiles when the input is short (4096 x 4096 bf16, 4 tokens: 16.2 -> 14.5 us dense, 12.7 -> 10.3 at 90 %;
    // 14336 x 4096 int8, 2 tokens: 22.4 -> 19.6); with a long input or a wide layer they lose.
    if (!(cfg && cfg->lanes_per_row) && bt <= 4) {
        const int full_tiles = (a.N + 64 * elems - 1) / (64 * elems);
        if (full_tiles <= 4 || (bt > 1 && full_tiles <= 8 && a.K <= 8192)) lpr = 32;
    }
    // (The vector kernel would take any multiple of 8 rows per workgroup -- 11008 rows as 32 x 344 instead of
    // 29 x 384 -- but that measured faster only at medium sparsity and slower dense and on small layers.)
    const int rc = plan_splits(a, lpr * elems, bt, kc, cfg && cfg->rows_per_group);
    if (rc != SCAP_OK) {
        // a batch's kept-channel list of a very long input does not fit the vector kernel's LDS; the
        // matrix-core path keeps its lists in the workspace
        if (rc == SCAP_ERR_SHAPE && mfma_ok && lanes == 0 && !(cfg && cfg->rows_per_group)) {
            const int rc2 = launch_gemm_inline(a_in, wdt, cfg, stream);
            return (rc2 == SCAP_ERR_SHAPE && wdt != kF16) ? launch_gemm_mfma(a_in, wdt, cfg, stream) : rc2;
        }
        return (rc == SCAP_ERR_SHAPE && cfg && cfg->lanes_per_row) ? SCAP_ERR_CONFIG : rc;
    }
    a.Kl = a.Kc;
    a.Sl = a.S;

    switch (wdt) {
        case kF16: return launch_wdt<kF16>(a, bt, waves, unroll, lpr, stream);
        case kBF16: return launch_wdt<kBF16>(a, bt, waves, unroll, lpr, stream);
        case kI8: return launch_wdt<kI8>(a, bt, waves, unroll, lpr, stream);
    }
    return SCAP_ERR_DTYPE;
}

// ---------------------------------------------------------------------------------------------- helpers
__global__ void fill_words_kernel(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

static int launch_fill_words(uint32_t* p, size_t n, uint32_t v, hipStream_t stream) {
    if (n == 0) return SCAP_OK;
    size_t blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, n, v);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

int launch_zero_words(int32_t* p, size_t n, hipStream_t stream) {
    return launch_fill_words(reinterpret_cast<uint32_t*>(p), n, 0u, stream);
}

int launch_workspace_init(void* workspace, size_t bytes, hipStream_t stream) {
    // the fixed header holds the arrival counters, calibration scratch and segment counts
    const size_t head = bytes < kOffPartial ? bytes : kOffPartial;
    return launch_fill_words(static_cast<uint32_t*>(workspace), head / 4, 0u, stream);
}

// Streaming read of `nvec` 16-byte vectors with the same non-temporal loads the GEMV uses for weights (the
// fastest way found to read HBM on this part); a per-workgroup checksum keeps the loads alive.
constexpr int kProbeGroups = 2048;
__global__ __launch_bounds__(512) void read_probe_kernel(const uint4* __restrict__ src, size_t nvec, uint32_t* out) {
    __shared__ uint32_t sh[8];
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 7 * stride < nvec; i += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = load_weights16(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < nvec; i += stride) {
        const uint4 v = load_weights16(src + i);
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    acc = (uint32_t)wave_sum((int)acc);
    if (lane_id() == 0) sh[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < 8; ++w) t += sh[w];
        out[blockIdx.x] = t;
    }
}

int launch_read_probe(const void* src, size_t bytes, uint32_t* out, hipStream_t stream) {
    const size_t nvec = bytes / 16;
    hipLaunchKernelGGL(read_probe_kernel, dim3(kProbeGroups), dim3(512), 0, stream, reinterpret_cast<const uint4*>(src),
                       nvec, out);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

}  // namespace scap
