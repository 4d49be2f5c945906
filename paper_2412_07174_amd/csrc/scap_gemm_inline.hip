// Batched sparse FC on the matrix cores in ONE launch (gfx950 MFMA), bf16 or int8 weights, 2..16 tokens.
//
// Workgroup (K split, column tile of 16 lanes x 16 bytes) centres, thresholds and compacts its Kc input
// channels of every token into LDS exactly as the one-token kernel does (SCAP Alg. 3 steps 1-2; per-token
// masks, the union of the masks decides which rows are read, Appendix C), then walks the list in 16-row
// blocks: channel indices and centred values come out of LDS, the weight rows stream from HBM, and the
// products run on the matrix cores (operand layout: scap_mfma_parts.hpp).  gfx950 gives a workgroup up to
// 160 KB of LDS, which holds the list of ~2300 channels for 16 tokens (index + 16 centred values each), so
// the separate union launch of scap_gemm_mfma.hip, its kernel boundary and its lists in memory are not
// needed; that form remains for inputs too long to split into LDS-sized pieces.
//
// The column tile is narrow (128 columns for bf16, 256 for int8), so the prologue is repeated by more
// workgroups than in the vector kernel; it is loads from L2 and a few hundred ALU operations per thread
// and costs less than the kernel boundary it replaces.
#include <atomic>

#include "scap_mfma_parts.hpp"

namespace scap {

constexpr size_t kInlineLdsBudget = 160 * 1024;
constexpr int kInlineWaves = 8;
// chunks of 64 channels a wavefront compacts from registers: 5 x 16 or 8 x 4 values per lane
constexpr int inline_max_chunks(int bt) { return bt == 16 ? 5 : 8; }

constexpr int kTreeFloats = 32 * 1024 / 4;  // LDS floats of the reduction tree (and of the final reduction)

// FUSE (kFusePlain / kFuseSwiglu / kFuseList) as in the vector kernel: where the inputs come from and what the
// tile's last arrival does with the finished columns (the two launches of the fused SwiGLU block, Alg. 2).
template <int WDT, int BT, int FUSE>
__global__ __launch_bounds__(kInlineWaves* kWave) void gemm_inline_kernel(const GemvArgs a) {
    constexpr int WAVES = kInlineWaves;
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr int TILE = 16 * ELEMS;

    extern __shared__ uint4 smem_raw[];
    Lds L = carve_lds<WAVES, BT>(reinterpret_cast<char*>(smem_raw), a.Kc);
    if constexpr (FUSE == kFuseSwiglu) L.fin = L.red + kTreeFloats;  // behind both uses of the reduction buffer
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;

    // constants of the column group this thread finishes if its workgroup is the tile's last arrival
    const ColConst mine = load_col_const<WDT, TILE>(a, tile, tid % (TILE / 4));

    // ------------------------------------------------------------------ 1. centre, threshold, compact
    int cnt;
    if constexpr (FUSE == kFuseList)
        cnt = gather_lists<WAVES, BT>(a, split, L);
    else
        cnt = compact_inputs_wide<WAVES, BT, inline_max_chunks(BT)>(a, tile, split, L);
    const int n_blocks = (cnt + kMfmaBlock - 1) / kMfmaBlock;

    // ------------------------------------------------------------------ 2. stream the kept rows
    const int cg = lane & 15;  // column group (B/C index n); also the token whose values this lane supplies (A index m)
    const int kg = lane >> 4;  // row group: list rows 4*kg .. 4*kg+3 of a block
    const int col0 = tile * TILE + cg * ELEMS;
    const uint32_t lane_off = (col0 < a.N) ? (uint32_t)col0 * Vec<WDT>::kBytes : 0u;
    const uint32_t row_bytes = (uint32_t)a.N * Vec<WDT>::kBytes;
    const char* wbase = reinterpret_cast<const char*>(a.W);
    const int tok = cg < BT ? cg : BT - 1;  // token slots past BT carry zeros (read slot BT-1, discard)
    const float* d_tok = L.d + tok * a.Kc;

    f32x4_t acc[ELEMS];
#pragma unroll
    for (int e = 0; e < ELEMS; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Three stages per wavefront: list entries of block n+2 come out of LDS while the weight rows of block
    // n+1 are in flight and the MFMAs of block n run.  No branch anywhere: a slot past the end of the list
    // reads LDS at a clamped position and weight row 0, and is zeroed by a select.
    struct Entries {
        int4 rows;
        float4 d;
        int left;  // valid entries from this lane's first one on (<= 0: none)
    };
    struct Stage {
        uint4 r[4];
        float4 d;
    };
    auto entries = [&](int blk, Entries& en) {  // blk is wave-uniform and may lie past the end
        const int e0 = blk * kMfmaBlock + 4 * kg;
        const int e0c = min(e0, a.Kc - 4);
        en.left = cnt - e0;
        en.rows = *reinterpret_cast<const int4*>(L.idx + e0c);
        en.d = *reinterpret_cast<const float4*>(d_tok + e0c);
    };
    auto issue = [&](const Entries& en, Stage& st) {
        const int rj[4] = {en.rows.x, en.rows.y, en.rows.z, en.rows.w};
        const float dj[4] = {en.d.x, en.d.y, en.d.z, en.d.w};
        float dm[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool ok = j < en.left;
            const uint32_t row = ok ? (uint32_t)rj[j] : 0u;
            const uint4 v = load_weights16(wbase + (uint64_t)row * row_bytes + lane_off);
            st.r[j] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
            dm[j] = (ok && cg < BT) ? dj[j] : 0.f;
        }
        st.d = make_float4(dm[0], dm[1], dm[2], dm[3]);
    };
    auto compute = [&](const Stage& st) {
        s16x4_t a_hi, a_lo;
        split_bf16x4(st.d, a_hi, a_lo);
        mfma_block<WDT>(acc, a_hi, a_lo, st.r);
    };

    Entries E0, E1;
    Stage A, Bs;
    entries(w, E0);
    entries(w + WAVES, E1);
    issue(E0, A);
    for (int blk = w; blk < n_blocks;) {
        entries(blk + 2 * WAVES, E0);
        issue(E1, Bs);
        compute(A);
        blk += WAVES;
        if (blk >= n_blocks) break;
        entries(blk + 2 * WAVES, E1);
        issue(E0, A);
        compute(Bs);
        blk += WAVES;
    }

    // ------------------------------------------------------------------ 3. add the wavefronts' sums
    const __amdgpu_buffer_rsrc_t pbuf = partial_buffer<TILE>(a);
    reduce_waves_and_emit<WDT, WAVES, FUSE>(a, pbuf, tile, split, acc, L.red, L.fin);  // starts with a barrier: the list is done with

    // ------------------------------------------------------------------ 4. last arrival finishes the tile
    finish_tile<WDT, WAVES, TILE, BT, FUSE>(a, pbuf, tile, L, mine);
}

template <int WDT, int BT, int FUSE>
static int launch_inline(const GemvArgs& a, size_t lds, hipStream_t stream) {
    if (lds > kInlineLdsBudget) return SCAP_ERR_SHAPE;
    if (lds > 64 * 1024) {
        // more dynamic LDS than the default limit: ask once per kernel and device
        constexpr int kMaxDevices = 64;
        static std::atomic<bool> asked[kMaxDevices];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SCAP_ERR_HIP;
        if (!asked[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_inline_kernel<WDT, BT, FUSE>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kInlineLdsBudget) != hipSuccess)
                return SCAP_ERR_HIP;
            asked[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL((gemm_inline_kernel<WDT, BT, FUSE>), dim3((unsigned)(a.S * a.T)), dim3(kInlineWaves * kWave), lds,
                       stream, a);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

template <int FUSE>
static int launch_inline_any(const GemvArgs& a, int wdt, int bt, size_t lds, hipStream_t stream) {
    if (wdt == kBF16) return bt == 4 ? launch_inline<kBF16, 4, FUSE>(a, lds, stream) : launch_inline<kBF16, 16, FUSE>(a, lds, stream);
    if (wdt == kI8) return bt == 4 ? launch_inline<kI8, 4, FUSE>(a, lds, stream) : launch_inline<kI8, 16, FUSE>(a, lds, stream);
    return SCAP_ERR_CONFIG;
}

// Plan one launch: token slots, rows per workgroup (bounded by LDS and, for the input prologue, by the
// registers that hold a wavefront's chunks), LDS bytes.
static int plan_inline(GemvArgs& a, int wdt, int kc, bool kc_forced, int fuse, int* bt_out, size_t* lds_out) {
    if (wdt != kBF16 && wdt != kI8) return SCAP_ERR_CONFIG;
    if (a.B < 1 || a.B > kMfmaTokens) return SCAP_ERR_CONFIG;
    const int bt = a.B <= 4 ? 4 : 16;
    const int tile_cols = wdt == kI8 ? 2 * kMfmaTile : kMfmaTile;
    size_t budget = kInlineLdsBudget;
    int kc_cap = kMaxSplits * kWave * 1024;  // no cap
    if (fuse == kFuseList) {
        kc_cap = 64 * kWave;  // gather_lists: at most 64 segments of 64 channels per workgroup
    } else {
        kc_cap = kInlineWaves * kWave * inline_max_chunks(bt);
    }
    const size_t by_cap = kHdrBytes + (size_t)kc_cap * 4 * (1 + bt);
    if (by_cap < budget) budget = by_cap;
    const int rc = plan_splits(a, tile_cols, bt, kc, kc_forced, budget);
    if (rc != SCAP_OK) return rc;
    if (a.Kc > kc_cap) return SCAP_ERR_SHAPE;
    size_t red = (size_t)kTreeFloats * 4;
    if (fuse == kFuseSwiglu) red += (size_t)bt * tile_cols * 4;
    *bt_out = bt;
    *lds_out = lds_bytes(a.Kc, bt, red);
    return SCAP_OK;
}

int launch_gemm_inline(const GemvArgs& a_in, int wdt, const scap_launch_cfg* cfg, hipStream_t stream) {
    GemvArgs a = a_in;
    if (a.B < kMfmaMinTokens) return SCAP_ERR_CONFIG;
    int kc = 0;
    if (cfg) {
        if (cfg->rows_per_group) kc = cfg->rows_per_group;
        if (kc < 0 || (kc % kWave) != 0) return SCAP_ERR_CONFIG;
        if (cfg->waves_per_group && cfg->waves_per_group != kInlineWaves) return SCAP_ERR_CONFIG;
    }
    int bt = 0;
    size_t lds = 0;
    const int rc = plan_inline(a, wdt, kc, kc != 0, kFusePlain, &bt, &lds);
    if (rc != SCAP_OK) return rc;
    a.Kl = a.Kc;
    a.Sl = a.S;
    return launch_inline_any<kFusePlain>(a, wdt, bt, lds, stream);
}

// The two launches of the fused SwiGLU block on the matrix cores (see scap_swiglu.hip for the vector form).
int launch_swiglu_block_inline(const GemvArgs& up_in, const GemvArgs& dn_in, int wdt, hipStream_t stream) {
    GemvArgs up = up_in, dn = dn_in;
    int bt_up = 0, bt_dn = 0;
    size_t lds_up = 0, lds_dn = 0;
    int rc = plan_inline(up, wdt, 0, false, kFuseSwiglu, &bt_up, &lds_up);
    if (rc != SCAP_OK) return rc;
    up.Kl = up.Kc;
    up.Sl = up.S;
    rc = plan_inline(dn, wdt, 0, false, kFuseList, &bt_dn, &lds_dn);
    if (rc != SCAP_OK) return rc;
    dn.Kl = kWave;
    dn.Sl = (dn.K + kWave - 1) / kWave;
    const size_t tables = kHdrBytes + (size_t)dn.Sl * 4;  // offsets of every segment (tile 0's last arrival)
    if (lds_dn < tables) lds_dn = tables;
    rc = launch_inline_any<kFuseSwiglu>(up, wdt, bt_up, lds_up, stream);
    if (rc != SCAP_OK) return rc;
    return launch_inline_any<kFuseList>(dn, wdt, bt_dn, lds_dn, stream);
}

}  // namespace scap
