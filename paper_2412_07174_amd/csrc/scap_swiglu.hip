// Fused SwiGLU feed-forward block (SCAP Appendix B, Alg. 2, each scap_fc in the centred form of Alg. 3), gfx950.
//
// Two launches of the column-gathered GEMV body:
//   1. gate|up: the weights of the gate and up projections are interleaved in groups of 4 columns, so that
//      the workgroup that finishes a column tile holds matching gate and up pre-activations.  It forms
//      z = silu(gate) * up, applies the next layer's centring and threshold, and writes the kept channels of
//      each 64-channel segment, compacted, with their centred values.  Neither the pre-activations nor z
//      make a round trip through memory, and no separate activation kernel runs.
//   2. down: its prologue copies those lists into LDS (one memory latency: counts and entry slots are
//      loaded together) instead of loading, centring, thresholding and compacting an input vector.
#include "scap_gemv_body.hpp"

namespace scap {

constexpr int kBlockWaves = 8;
constexpr int kBlockUnroll = 8;
constexpr int kMaxListRows = 4096;  // input channels of one down workgroup: 64 segments of 64

template <int WDT, int BT>
__global__ __launch_bounds__(kBlockWaves* kWave) void swiglu_up_kernel(const GemvArgs a) {
    gemv_body<WDT, kBlockWaves, kBlockUnroll, BT, kWave, kFuseSwiglu>(a);
}

template <int WDT, int BT, int LPR>
__global__ __launch_bounds__(kBlockWaves* kWave) void swiglu_down_kernel(const GemvArgs a) {
    gemv_body<WDT, kBlockWaves, kBlockUnroll, BT, LPR, kFuseList>(a);
}

// wdt, flags: for blocks of 2-4 tokens, whose launches run on the two- / four-slot kernel where that applies (unless the
// caller asks for the general kernels)
template <int WDT, int BT>
static int launch_block(GemvArgs up, GemvArgs dn, int wdt, int flags, hipStream_t stream) {
    const GemvArgs up_in = up, dn_in = dn;
    const bool two = (BT == 2 || BT == 4) && up.B >= 2 && !(flags & SCAP_CFG_GENERAL_KERNEL);
    const bool up_two = two && swiglu_block2_part_applies(up_in, dn_in, wdt, 0);
    const bool dn_two = two && swiglu_block2_part_applies(up_in, dn_in, wdt, 1);
    constexpr int TILE = kWave * Vec<WDT>::kElems;
    constexpr int NT = kBlockWaves * kWave;
    constexpr size_t RED = (size_t)(kBlockWaves * TILE > NT * 4 ? kBlockWaves * TILE : NT * 4);

    int rc = plan_splits(up, TILE, BT, 0, false);
    if (rc != SCAP_OK) return rc;
    up.Kl = up.Kc;
    up.Sl = up.S;
    const size_t lds_up = lds_bytes(up.Kc, BT, (RED + (size_t)BT * TILE) * 4);

    // few full-width tiles of output: half-width tiles, by the rule of the plain launch
    const int full_tiles = (dn.N + TILE - 1) / TILE;
    const bool half = full_tiles <= 4 || (BT > 1 && full_tiles <= 8 && dn.K <= 8192);
    const int dn_tile = half ? TILE / 2 : TILE;
    rc = plan_splits(dn, dn_tile, BT, 0, false);
    if (rc == SCAP_OK && dn.Kc > kMaxListRows) rc = plan_splits(dn, dn_tile, BT, kMaxListRows, false);
    if (rc != SCAP_OK) return rc;
    if (dn.Kc > kMaxListRows || dn.Kc % kWave != 0) return SCAP_ERR_SHAPE;
    dn.Kl = kWave;
    dn.Sl = (dn.K + kWave - 1) / kWave;
    size_t lds_dn = lds_bytes(dn.Kc, BT, RED * 4);
    const size_t tables = kHdrBytes + (size_t)dn.Sl * 4;  // offsets of every segment (tile 0's last arrival)
    if (lds_dn < tables) lds_dn = tables;
    if (lds_up > 64 * 1024 || lds_dn > 64 * 1024) return SCAP_ERR_SHAPE;

    if (up_two) {
        rc = launch_swiglu_block2_part(up_in, dn_in, wdt, 0, stream);
        if (rc != SCAP_OK) return rc;
    } else {
        hipLaunchKernelGGL((swiglu_up_kernel<WDT, BT>), dim3((unsigned)(up.S * up.T)), dim3(NT), lds_up, stream, up);
        if (hipGetLastError() != hipSuccess) return SCAP_ERR_HIP;
    }
    if (dn_two) return launch_swiglu_block2_part(up_in, dn_in, wdt, 1, stream);
    if (half) {
        hipLaunchKernelGGL((swiglu_down_kernel<WDT, BT, kWave / 2>), dim3((unsigned)(dn.S * dn.T)), dim3(NT), lds_dn,
                           stream, dn);
        return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
    }
    hipLaunchKernelGGL((swiglu_down_kernel<WDT, BT, kWave>), dim3((unsigned)(dn.S * dn.T)), dim3(NT), lds_dn, stream, dn);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

template <int WDT>
static int launch_block_wdt(const GemvArgs& up, const GemvArgs& down, int flags, hipStream_t stream) {
    if (up.B == 1) return launch_block<WDT, 1>(up, down, WDT, flags, stream);
    if (up.B == 2) return launch_block<WDT, 2>(up, down, WDT, flags, stream);
    if (up.B <= kBlockVectorTokens) return launch_block<WDT, 4>(up, down, WDT, flags, stream);
    return SCAP_ERR_UNIMPL;
}

// flags1: launch flags -- partial sums / parked slices for the one-token form; SCAP_CFG_GENERAL_KERNEL keeps a
// two-token block on the general kernels
int launch_swiglu_block(const GemvArgs& up, const GemvArgs& down, int wdt, hipStream_t stream, int flags1) {
    // Matrix cores: more than 4 tokens, and int8 from 3 tokens on, where the vector kernel is bound by its
    // per-element converts.  Their lists use 4 or 16 token slots, like the vector kernel's for
    // 3-4 tokens, so the choice only has to be the same for both launches.
    if (up.B == 1 && !(flags1 & SCAP_CFG_GENERAL_KERNEL)) {  // the one-token kernel with the gating epilogue / the list prologue
        const int rc = launch_swiglu_block1(up, down, wdt, flags1 & (SCAP_CFG_PARTIAL_SUMS | SCAP_CFG_PARK_SLICES),
                                            flags1 & SCAP_CFG_PARTIAL_SUMS, stream);
        if (rc != kG1NotApplicable) return rc;
    }
    const bool matrix = up.B > kBlockVectorTokens || (wdt == kI8 && up.B >= 3);
    if (matrix) {
        const int rc = launch_swiglu_block_inline(up, down, wdt, stream);
        if (rc != SCAP_ERR_SHAPE || up.B > kBlockVectorTokens) return rc == SCAP_ERR_SHAPE ? SCAP_ERR_UNIMPL : rc;
    }
    switch (wdt) {
        case kF16: return launch_block_wdt<kF16>(up, down, flags1, stream);
        case kBF16: return launch_block_wdt<kBF16>(up, down, flags1, stream);
        case kI8: return launch_block_wdt<kI8>(up, down, flags1, stream);
    }
    return SCAP_ERR_DTYPE;
}

// ---------------------------------------------------------------------------------------------- packing
// out[r][8j + 0..3] = gate[r][4j + 0..3], out[r][8j + 4..7] = up[r][4j + 0..3]; UNIT = 4 elements
template <typename UNIT>
__global__ void pack_gate_up_kernel(const UNIT* __restrict__ gate, const UNIT* __restrict__ up, size_t units,
                                    UNIT* __restrict__ out) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < 2 * units; i += (size_t)gridDim.x * blockDim.x)
        out[i] = (i & 1) ? up[i >> 1] : gate[i >> 1];
}

int launch_pack_gate_up(const void* gate, const void* up, int64_t rows, int64_t F, int elem_bytes, void* out,
                        hipStream_t stream) {
    const size_t units = (size_t)rows * (size_t)(F / 4);  // 4-element groups per source; group i of a row-major
                                                          // [rows, F/4] array goes to group 2i (gate) / 2i+1 (up)
    if (units == 0) return SCAP_OK;
    size_t blocks = (2 * units + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    const dim3 grid((unsigned)blocks), block(256);
    switch (elem_bytes) {
        case 1:
            hipLaunchKernelGGL(pack_gate_up_kernel<uint32_t>, grid, block, 0, stream, static_cast<const uint32_t*>(gate),
                               static_cast<const uint32_t*>(up), units, static_cast<uint32_t*>(out));
            break;
        case 2:
            hipLaunchKernelGGL(pack_gate_up_kernel<uint2>, grid, block, 0, stream, static_cast<const uint2*>(gate),
                               static_cast<const uint2*>(up), units, static_cast<uint2*>(out));
            break;
        case 4:
            hipLaunchKernelGGL(pack_gate_up_kernel<uint4>, grid, block, 0, stream, static_cast<const uint4*>(gate),
                               static_cast<const uint4*>(up), units, static_cast<uint4*>(out));
            break;
        default: return SCAP_ERR_DTYPE;
    }
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

}  // namespace scap
