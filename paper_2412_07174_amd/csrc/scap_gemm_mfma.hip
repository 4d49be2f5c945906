// Batched sparse FC on the matrix cores (gfx950 MFMA), bf16 or int8 weights, 2..16 tokens.
//
// With several tokens each token keeps its own mask (SCAP Eq. 2 is elementwise); the rows that have to be
// read are the union of the masks (Appendix C), and what multiplies them is a [tokens x kept-rows] matrix of
// centred values with zeros where a token pruned the channel -- a dense contraction, so it goes to MFMA:
//
//     Y[16 tokens, 16 columns] += D[16 tokens, 16 rows] * W[16 rows, 16 columns]     v_mfma_f32_16x16x16_bf16
//
// Two launches.  `batch_union_kernel` (one workgroup per K split) centres and thresholds the inputs of all
// tokens once and leaves the ascending union list of its split in the workspace (plus the per-token lists
// when the caller wants them).  Doing this inside every (split, column tile) workgroup, as the one-token
// kernel does, repeats 16 tokens' worth of work per tile and took longer than the GEMM itself.
// `gemm_mfma_kernel` (split, tile of 128 columns) then streams the listed rows; the centred values come
// from the list, stored per 16-entry block exactly as the MFMA wants them: lane l of a block finds its A
// operand (bf16 heads and tails of token l%16 at entries 4*(l/16)+0..3) in 16 contiguous bytes, a wavefront
// reads 1 KB in one instruction (gathering from x instead touches one cache line per token and row, and
// per-value loads from a plain [entry][token] array cost four instructions per block; both throttled the
// weight stream).
//
// Operand layout, bf16 head/tail split of the centred values and the int8 widening: see scap_mfma_parts.hpp.
// This two-launch form keeps its lists in the workspace, so the input length is not bounded by LDS; the
// single-launch form (scap_gemm_inline.hip) is preferred whenever a workgroup's list fits LDS.
#include "scap_mfma_parts.hpp"

namespace scap {

// ---------------------------------------------------------------------------------------------- launch 1
// Workgroup `seg` owns channels [seg*Kl, (seg+1)*Kl): one channel per thread and pass; the x values of all
// tokens are loaded together, the union of the keep tests is compacted with a ballot per wavefront and a
// scan over the wavefronts.  Segments are short (512 channels unless K is huge) so that the whole input is
// handled in one round of loads by many workgroups.
//   u_idx[seg*Kl ...]        ascending channels kept by at least one token
//   u_d as [block of 16 entries][lane 0..63][4 bf16 heads, 4 bf16 tails]: lane = 16*(entry%16/4) + token,
//                            value j = entry%4; 0 where the token pruned the channel or the list has ended
//   seg_cnt[B*Sl + seg]      their number;   seg_cnt[b*Sl + seg], idx_out: per-token lists on request
__global__ __launch_bounds__(kCompactWaves * kWave) void batch_union_kernel(const GemvArgs a) {
    constexpr int BT = kMfmaTokens;
    constexpr int NT = kCompactWaves * kWave;
    __shared__ int s_cnt[1 + BT][kCompactWaves];
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int seg = blockIdx.x;
    const int k0 = seg * a.Kl;
    const int kend = min(k0 + a.Kl, a.K);
    const bool per_token = a.nnz_out != nullptr || a.idx_out != nullptr;
    const bool want_idx = a.idx_out != nullptr;
    int32_t* __restrict__ out = a.u_idx + (int64_t)seg * a.Kl;
    // operand blocks of this segment: (Kl / 16) blocks of 64 lanes x 16 bytes
    uint4* __restrict__ out_a = reinterpret_cast<uint4*>(a.u_d) + (int64_t)seg * (a.Kl / kMfmaBlock) * kWave;
    __shared__ float s_val[NT][BT + 1];  // centred values of the entries placed in this pass (+1: no bank conflicts)

    int run_u = 0;
    int run_t[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) run_t[b] = 0;

    for (int p0 = k0; p0 < kend; p0 += NT) {
        const int k = p0 + tid;
        const bool valid = k < kend;
        uint32_t xb[BT];  // branch-free loads: slots past the batch or the end re-read a valid element, masked below
        const int kc_ = min(k, a.K - 1);
#pragma unroll
        for (int b = 0; b < BT; ++b) xb[b] = (uint32_t)a.x[(int64_t)min(b, a.B - 1) * a.K + kc_];
        uint32_t keepmask = 0;
        float dm[BT];  // centred value where the token keeps the channel, else 0
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const float xf = a.xdt == kBF16 ? bf16_bits_to_f32(xb[b]) : f16_bits_to_f32(xb[b]);
            const float d = (a.mode == kModeDense) ? xf : xf - a.m;  // one fp32 subtraction
            const bool keep = valid && b < a.B && (a.mode == kModeDense || fabsf(d) > a.tau);
            keepmask |= keep ? (1u << b) : 0u;
            dm[b] = keep ? d : 0.f;
        }
        const bool any = keepmask != 0;
        const uint64_t ub = __ballot(any);
        if (lane == 0) s_cnt[0][w] = __popcll(ub);
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const uint64_t tb = __ballot((keepmask >> b) & 1u);
                if (lane == 0) s_cnt[1 + b][w] = __popcll(tb);
            }
        }
        __syncthreads();
        int below = 0, total = 0;
#pragma unroll
        for (int i = 0; i < kCompactWaves; ++i) {
            const int v = s_cnt[0][i];
            if (i < w) below += v;
            total += v;
        }
        // This pass places entries [run_u, run_u + total) of the segment's list.  Their values go through
        // LDS so that whole operand blocks can be written; a block that straddles two passes is completed
        // by the later one, which re-reads the earlier entries' values from the block itself.
        const int first_blk = run_u / kMfmaBlock;
        const int carry = run_u - first_blk * kMfmaBlock;  // entries of the first block placed by earlier passes
        if (any) {
            const int pos = run_u + below + lanes_below(ub);
            out[pos] = k;
#pragma unroll
            for (int b = 0; b < BT; ++b) s_val[pos - run_u][b] = dm[b];
        }
        __syncthreads();
        const int n_items = ((carry + total + kMfmaBlock - 1) / kMfmaBlock) * kWave;  // (block, lane) pairs
        constexpr int kItemRounds = (NT / kMfmaBlock + 2) * kWave / NT + 1;  // covers carry + NT entries
#pragma unroll
        for (int q = 0; q < kItemRounds; ++q) {
            const int it = tid + q * NT;
            if (it >= n_items) break;
            const int blk = first_blk + it / kWave;
            const int l = it % kWave;
            const int tok = l & 15, kg = l >> 4;
            uint4 prev = make_uint4(0u, 0u, 0u, 0u);
            if (carry != 0) {  // only a segment longer than one pass can have a block that straddles passes
                if (it < kWave) prev = out_a[(int64_t)blk * kWave + l];
            }
            float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
            float* dv = &d.x;
            bool from_prev[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = (it / kWave) * kMfmaBlock + 4 * kg + j - carry;  // index into this pass's entries
                from_prev[j] = e < 0;
                if (e >= 0 && e < total) dv[j] = s_val[e][tok];
            }
            s16x4_t hi, lo;
            split_bf16x4(d, hi, lo);
            union { uint4 q4; short h[8]; } pk;
            pk.q4 = prev;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!from_prev[j]) {
                    pk.h[j] = hi[j];
                    pk.h[4 + j] = lo[j];
                }
            }
            out_a[(int64_t)blk * kWave + l] = pk.q4;
        }
        run_u += total;
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                int tbelow = 0, ttotal = 0;
                for (int i = 0; i < kCompactWaves; ++i) {
                    const int v = s_cnt[1 + b][i];
                    if (i < w) tbelow += v;
                    ttotal += v;
                }
                const uint64_t tb = __ballot((keepmask >> b) & 1u);
                if (want_idx && ((keepmask >> b) & 1u))
                    a.idx_out[(int64_t)b * a.K + k0 + run_t[b] + tbelow + lanes_below(tb)] = k;
                run_t[b] += ttotal;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        a.seg_cnt[a.B * a.Sl + seg] = run_u;
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b)
                if (b < a.B) a.seg_cnt[b * a.Sl + seg] = run_t[b];
        }
    }
}

// ---------------------------------------------------------------------------------------------- launch 2
template <int WDT, int WAVES, int UB>
__global__ __launch_bounds__(WAVES * kWave) void gemm_mfma_kernel(const GemvArgs a) {
    constexpr int BT = kMfmaTokens;
    constexpr int ELEMS = Vec<WDT>::kElems;  // columns in a lane's 16-byte load = MFMAs per block
    constexpr int TILE = 16 * ELEMS;

    extern __shared__ uint4 smem_raw[];
    const Lds L = carve_lds<WAVES, BT>(reinterpret_cast<char*>(smem_raw), 0);
    float* s_red = L.red;  // tree reduction buffer, then the final reduction's

    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;

    // The split covers list segments [seg0, seg1) written by the previous launch.  Their 16-row blocks are
    // numbered through: s_pre[i] = blocks before segment seg0+i.
    constexpr int kMaxSeg = 64;
    __shared__ int s_segcnt[kMaxSeg];
    __shared__ int s_pre[kMaxSeg + 1];
    const int per_split = a.Kc / a.Kl;
    const int seg0 = split * per_split;
    const int nseg = min(per_split, a.Sl - seg0);
    if (w == 0) {  // nseg <= 64: one wavefront loads the counts and scans the block numbers
        const int cnt = lane < nseg ? a.seg_cnt[a.B * a.Sl + seg0 + lane] : 0;
        const int blocks = (cnt + kMfmaBlock - 1) / kMfmaBlock;
        const int inc = wave_inclusive_scan(blocks);
        if (lane < nseg) {
            s_segcnt[lane] = cnt;
            s_pre[lane] = inc - blocks;
        }
        if (lane == kWave - 1) s_pre[nseg] = inc;
    }
    __syncthreads();
    const int n_blocks = uniform(s_pre[nseg]);

    const int cg = lane & 15;   // column group: columns ELEMS*cg .. +ELEMS-1 of the tile (B/C index n)
    const int kg = lane >> 4;   // row group: list rows 4*kg .. 4*kg+3 of a block (k of A and B); token group of C
    const int col0 = tile * TILE + cg * ELEMS;
    const uint32_t lane_off = (col0 < a.N) ? (uint32_t)col0 * Vec<WDT>::kBytes : 0u;
    const uint32_t row_bytes = (uint32_t)a.N * Vec<WDT>::kBytes;
    const char* wbase = reinterpret_cast<const char*>(a.W);

    // constants of the column group this thread finishes if its workgroup is the tile's last arrival
    const ColConst mine = load_col_const<WDT, TILE>(a, tile, tid % (TILE / 4));

    f32x4_t acc[ELEMS];
#pragma unroll
    for (int e = 0; e < ELEMS; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Block blk (wave-uniform) -> its four list entries for this lane's row group: the int4 of channel
    // indices, how many of them are valid (0..4), and where this lane's A operand of the block lies.
    // Blocks past the end give 0 valid entries.
    const uint4* const a_base = reinterpret_cast<const uint4*>(a.u_d);
    auto fetch = [&](int blk, int4& rows, const uint4*& aptr) -> int {
        rows = make_int4(0, 0, 0, 0);
        aptr = a_base + lane;  // any readable address; nothing is loaded through it (see issue())
        if (blk >= n_blocks) return -1;
        int i = 0;
        while (i + 1 < nseg && s_pre[i + 1] <= blk) ++i;  // nseg is small
        i = uniform(i);
        const int local = blk - s_pre[i];
        aptr = a_base + ((int64_t)(seg0 + i) * (a.Kl / kMfmaBlock) + local) * kWave + lane;
        const int left = s_segcnt[i] - local * kMfmaBlock - 4 * kg;  // entries from this lane's first one on
        if (left <= 0) return 0;
        const int64_t e = (int64_t)(seg0 + i) * a.Kl + local * kMfmaBlock + 4 * kg;  // this lane's first entry
        rows = *reinterpret_cast<const int4*>(a.u_idx + e);
        return left < 4 ? left : 4;
    };

    // Software pipeline, three deep: while the MFMAs of iteration `it` run, the row loads of `it+1` are in
    // flight and the list indices of `it+2` are being fetched.  An iteration is UB blocks per wavefront.
    struct IdxSet {
        int4 ix[UB];
        int nv[UB];
        const uint4* ap[UB];
    };
    struct Stage {
        uint4 r[UB][4];
        uint4 av[UB];  // A operand: 4 bf16 heads, 4 bf16 tails
    };
    auto fetch_set = [&](int it, IdxSet& I) {
#pragma unroll
        for (int u = 0; u < UB; ++u) I.nv[u] = fetch(w + (it * UB + u) * WAVES, I.ix[u], I.ap[u]);
    };
    auto issue = [&](const IdxSet& I, Stage& st) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int rows[4] = {I.ix[u].x, I.ix[u].y, I.ix[u].z, I.ix[u].w};
            // one 1 KB read per wavefront and block, issued without a branch; past the end of the list the
            // value read is replaced by zeros
            const uint4 av = *I.ap[u];
            const bool live = I.nv[u] >= 0;
            st.av[u] = make_uint4(live ? av.x : 0u, live ? av.y : 0u, live ? av.z : 0u, live ? av.w : 0u);
            // The row loads carry no branch either: a slot past the end of the list reads row 0 (a handful
            // of extra 256-byte reads per list segment) and is zeroed afterwards.
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool ok = j < I.nv[u];
                const uint32_t row = ok ? (uint32_t)rows[j] : 0u;
                const uint4 v = load_weights16(wbase + (uint64_t)row * row_bytes + lane_off);
                st.r[u][j] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
            }
        }
    };
    auto compute = [&](const Stage& st) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            union { uint32_t u32[2]; s16x4_t v; } ah, al;
            ah.u32[0] = st.av[u].x;
            ah.u32[1] = st.av[u].y;
            al.u32[0] = st.av[u].z;
            al.u32[1] = st.av[u].w;
            mfma_block<WDT>(acc, ah.v, al.v, st.r[u]);
        }
    };

    const int niter = (n_blocks > w) ? (n_blocks - w + WAVES * UB - 1) / (WAVES * UB) : 0;
    IdxSet I0, I1;
    Stage A, Bs;
    fetch_set(0, I0);
    fetch_set(1, I1);
    issue(I0, A);
    for (int it = 0; it < niter;) {
        fetch_set(it + 2, I0);
        issue(I1, Bs);
        compute(A);
        if (++it >= niter) break;
        fetch_set(it + 2, I1);
        issue(I0, A);
        compute(Bs);
        ++it;
    }

    // ------------------------------------------------------------------ add the wavefronts' sums
    const __amdgpu_buffer_rsrc_t pbuf = partial_buffer<TILE>(a);
    reduce_waves_and_emit<WDT, WAVES>(a, pbuf, tile, split, acc, s_red);

    finish_tile<WDT, WAVES, TILE, BT>(a, pbuf, tile, L, mine);
}

int launch_gemm_mfma(const GemvArgs& a_in, int wdt, const scap_launch_cfg* cfg, hipStream_t stream) {
    GemvArgs a = a_in;
    if (wdt != kBF16 && wdt != kI8) return SCAP_ERR_CONFIG;
    const int tile_cols = wdt == kI8 ? 2 * kMfmaTile : kMfmaTile;
    if (!a.u_idx || !a.u_d) return SCAP_ERR_WORKSPACE;
    int kc = 0, waves = 8, ub = 1;
    if (cfg) {
        if (cfg->rows_per_group) kc = cfg->rows_per_group;
        if (kc < 0 || (kc % kWave) != 0) return SCAP_ERR_CONFIG;
        if (cfg->waves_per_group) waves = cfg->waves_per_group;
        if (cfg->unroll) ub = cfg->unroll;  // 16-row blocks in flight per wavefront
    }
    // list segments: 512 channels each, longer only if K is so large that there would be more than 256
    a.Kl = 512;
    while (((int64_t)a.K + a.Kl - 1) / a.Kl > kMaxSplits) a.Kl *= 2;
    a.Sl = (a.K + a.Kl - 1) / a.Kl;
    if ((size_t)a.Sl * a.Kl > union_list_entries(a.K)) return SCAP_ERR_SHAPE;
    // K split of the GEMM: whole segments, at most 64 per workgroup; no list in LDS
    kc = (int)align_up((size_t)kc, (size_t)a.Kl);  // a requested split is rounded up to whole segments
    if (kc == 0) {
        // Segments per workgroup g: every workgroup gets the same number (an uneven last split leaves compute
        // units idle at the end), and the busiest compute unit -- ceil(workgroups / 256) workgroups of g
        // segments -- should have as little as possible; ties go to the larger g (fewer partial sums).
        const int tiles = (a.N + tile_cols - 1) / tile_cols;
        long best_cost = -1;
        int best_g = 1;
        for (int g = 1; g <= a.Sl && g <= 64; ++g) {
            const int splits = (a.Sl + g - 1) / g;
            const long cost = (((long)splits * tiles + 255) / 256) * g;
            if (best_cost < 0 || cost <= best_cost) {
                best_cost = cost;
                best_g = g;
            }
        }
        kc = best_g * a.Kl;
    }
    const int rc = plan_splits(a, tile_cols, 0, kc, cfg && cfg->rows_per_group);
    if (rc != SCAP_OK) return rc;
    a.Kc = (int)align_up((size_t)a.Kc, (size_t)a.Kl);
    if (a.Kc / a.Kl > 64) a.Kc = 64 * a.Kl;
    a.S = (a.K + a.Kc - 1) / a.Kc;
    if ((size_t)a.S * a.T * tile_cols > partial_capacity(a.N)) return SCAP_ERR_SHAPE;

    // Everything that can refuse the call comes before the first launch: the union kernel already writes the
    // caller's lists and counts.
    const bool instantiated = (wdt == kBF16 && (waves == 16 || waves == 8) && (ub == 1 || ub == 2 || ub == 4)) ||
                              (wdt == kI8 && waves == 8 && (ub == 1 || ub == 2));
    if (!instantiated) return SCAP_ERR_CONFIG;
    // tree reduction buffer: 32 KB (the final reduction needs less)
    const size_t lds = lds_bytes(0, 0, (size_t)32 * 1024);
    if (lds > 64 * 1024) return SCAP_ERR_CONFIG;

    hipLaunchKernelGGL(batch_union_kernel, dim3((unsigned)a.Sl), dim3(kCompactWaves * kWave), 0, stream, a);
    if (hipGetLastError() != hipSuccess) return SCAP_ERR_HIP;

    const dim3 grid((unsigned)(a.S * a.T));
    const dim3 block(waves * kWave);
#define SCAP_MFMA_CASE(WD, WV, UBV)                                                                 \
    if (wdt == WD && waves == WV && ub == UBV) {                                                     \
        hipLaunchKernelGGL((gemm_mfma_kernel<WD, WV, UBV>), grid, block, lds, stream, a);            \
        return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;                             \
    }
    SCAP_MFMA_CASE(kBF16, 16, 1) SCAP_MFMA_CASE(kBF16, 16, 2) SCAP_MFMA_CASE(kBF16, 16, 4)
    SCAP_MFMA_CASE(kBF16, 8, 1) SCAP_MFMA_CASE(kBF16, 8, 2) SCAP_MFMA_CASE(kBF16, 8, 4)
    SCAP_MFMA_CASE(kI8, 8, 1) SCAP_MFMA_CASE(kI8, 8, 2)
#undef SCAP_MFMA_CASE
    return SCAP_ERR_CONFIG;  // not reached: `instantiated` lists the same table
}

}  // namespace scap
