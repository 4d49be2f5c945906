// Batched sparse FC on the matrix cores in ONE launch (gfx950 MFMA): bf16 or int8 weights from 2 tokens, fp16
// weights from 5, up to 16 tokens.  Two kernels: gemm_inline_kernel (below) keeps per-token value lists in LDS;
// gemm_inline_raw_kernel (further down, the default whenever K is a multiple of 8 and 16 token slots are used)
// stages the raw input tile instead and forms the centred values when the MFMA operand is assembled.
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
#include <type_traits>

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
        split_operand<WDT>(st.d, a_hi, a_lo);
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
    reduce_waves_and_emit<WDT, WAVES, FUSE, WDT != kI8>(a, pbuf, tile, split, acc, L.red, L.fin);  // starts with a barrier: the list is done with

    // ------------------------------------------------------------------ 4. last arrival finishes the tile
    finish_tile<WDT, WAVES, TILE, BT, FUSE>(a, pbuf, tile, L, mine);
}

// ---------------------------------------------------------------------------------------------- staged-tile form
// 16 token slots, K a multiple of 8.  The prologue above costs ~10 us at 16 tokens: 80 two-byte loads per lane,
// ~10 ALU operations per input element and 16 four-byte LDS writes per kept channel, repeated by every column
// tile.  Here the workgroup's input tile is staged as it is (16-byte loads, 16-byte LDS writes), only the union
// list of channels is compacted, and the centred, thresholded value of (token, channel) is formed from the
// staged tile when the matrix-core operand is assembled, in the shadow of the weight stream.  Same arithmetic
// per element (one fp32 subtraction, strict compare), so masks and values are those of the other forms.
constexpr int kRawChunks = 5;  // chunks of 64 channels per wavefront (loads of all of them are in flight at once)
constexpr int kRawPad = 16;    // bytes between token rows of the staged tile: rows start 4 LDS banks apart

__host__ __device__ constexpr size_t raw_tile_bytes(int Kc) { return (size_t)kMfmaTokens * ((size_t)Kc * 2 + kRawPad); }

// bit o of an 8-bit value to bit 8*o (two 4-bit halves: the partial products of a half never share a bit)
__device__ __forceinline__ uint64_t spread_bits_to_bytes(uint32_t v) {
    const uint32_t lo = ((v & 15u) * 0x00204081u) & 0x01010101u;
    const uint32_t hi = ((v >> 4) * 0x00204081u) & 0x01010101u;
    return (uint64_t)lo | ((uint64_t)hi << 32);
}

// Input code (low 16 bits) to fp32 without a branch on the (uniform) activation type: both conversions, bit select.
__device__ __forceinline__ float act_code_to_f32(uint32_t code, uint32_t bf16_sel) {
    const uint32_t as_bf16 = code << 16;
    const uint32_t as_f16 = __float_as_uint(f16_bits_to_f32(code));
    return __uint_as_float((as_bf16 & bf16_sel) | (as_f16 & ~bf16_sel));
}

// One of the two 16-bit inputs of a word, activation type known at compile time.
template <bool BF16X>
__device__ __forceinline__ float word_half_to_f32(uint32_t wd, int half) {
    if constexpr (BF16X)
        return __uint_as_float(half ? (wd & 0xffff0000u) : (wd << 16));
    else
        return f16_bits_to_f32(half ? (wd >> 16) : (wd & 0xffffu));
}

// Stage the tile, build the ascending union list in L.idx.  Lane = (token group tg = lane % 8, octet o = lane / 8
// of 8 channels): it loads tokens tg and tg+8 of its octet and tests its 16 elements; the compare masks are
// scalar registers, so a channel's keep bits over all tokens are one byte of a mask and "kept by any token" is
// a nonzero-byte test.  Everything in the test is straight-line: the instruction count per element is what the
// prologue costs, repeated by every column tile.  Per-token lists and counts (column tile 0, on request) are
// read back from the staged tile with one channel per lane.  Returns the list length; ends with a barrier.
template <int WAVES, int MAXC, bool SUPERSET>
__device__ __forceinline__ int stage_inputs_and_list(const GemvArgs& a, int tile, int split, const Lds& L, char* xs,
                                                     uint32_t xrow) {
    constexpr int BT = kMfmaTokens;
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int k0 = split * a.Kc;
    const int kend = min(k0 + a.Kc, a.K);
    const bool per_token = tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr);
    const bool want_idx = tile == 0 && a.idx_out != nullptr;
    // dense mode as data, not as control flow: x - 0 is x, and every valid element is kept
    const bool dense = a.mode == kModeDense;
    const float m_eff = dense ? 0.f : a.m;
    const uint32_t bf16_sel = a.xdt == kBF16 ? 0xffffffffu : 0u;
    const uint32_t nan_pair = a.xdt == kBF16 ? 0x7fc07fc0u : 0x7e007e00u;  // two quiet NaNs: never above a threshold
    const int nchunk = (kend - k0 + kWave - 1) / kWave;
    const int cpw = (nchunk + WAVES - 1) / WAVES;
    const int c_begin = min(w * cpw, nchunk);
    const int c_end = min(c_begin + cpw, nchunk);
    const int tg = lane & 7, o = lane >> 3;

    // ---- all loads, branch-free (slots past the end re-read a valid octet)
    uint4 xv[MAXC][2];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int kb = min(k0 + (c_begin + j) * kWave + 8 * o, a.K - 8);
#pragma unroll
        for (int r = 0; r < 2; ++r)
            xv[j][r] = *reinterpret_cast<const uint4*>(a.x + (int64_t)min(tg + 8 * r, a.B - 1) * a.K + kb);
    }
    // ---- stage, test, union mask per chunk
    uint64_t um[MAXC];
    int ucount = 0;
    // The list only decides which rows are READ: what a token contributes is decided again, exactly, when the
    // operand is assembled.  So the list may be a superset of the union.  With many tokens the union is nearly
    // everything (Appendix C: 1 - s^B), and testing 16 tokens per channel to find that out is the larger part
    // of this prologue.  Each wavefront therefore tests its first chunk; if at most 2 of its 64 channels are
    // dropped by every token, it lists its other chunks whole (a few rows read for nothing against three
    // quarters of the tests).  Dense mode lists everything without a test (there that is the exact union).
    // The decision depends on the inputs only, so every column tile of a split takes the same one: the list,
    // and with it the order of every fp32 sum, never depends on which outputs the caller asked for.  When the
    // caller wants the size of the union, which has to be exact, column tile 0 also tests the chunks it lists
    // whole, for the count alone.
    const bool count_exactly = tile == 0 && a.union_nnz_out != nullptr;
    int ecount = 0;  // channels kept by at least one token among those tested (the exact union where all are)
    auto test_chunks = [&](auto bf16x) {
        constexpr bool BF16X = decltype(bf16x)::value;
        // stage chunk slot j and list all its channels (wave-uniform)
        auto list_whole = [&](int j) {
            const int c = c_begin + j;
            um[j] = 0;
            if (c < c_end) {
                const int nval = min((int)kWave, kend - (k0 + c * kWave));
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    if (r == 1 && a.B <= 8) break;
                    *reinterpret_cast<uint4*>(xs + (size_t)(tg + 8 * r) * xrow + (size_t)(c * kWave + 8 * o) * 2) = xv[j][r];
                }
                um[j] = nval >= kWave ? ~0ull : ((1ull << nval) - 1ull);
                ucount += nval;
            }
        };
        // stage chunk slot j and list the channels kept by at least one token
        auto test_slot = [&](int j) {
            const int c = c_begin + j;
            um[j] = 0;
            if (c < c_end) {  // wave-uniform
                const bool oct_ok = (k0 + c * kWave + 8 * o) < kend;  // K and Kc are multiples of 8: whole octets
                uint64_t kp[8];  // lane masks (bit tg + 8*o): channel 8*o+e kept by token tg or tg+8
                uint64_t any_ok = 0;
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    if (r == 1 && a.B <= 8) break;  // at most 8 tokens: the second token of every lane does not exist
                    const bool ok = oct_ok && (tg + 8 * r) < a.B;
                    any_ok |= __ballot(ok);
                    // an element that does not exist becomes a NaN: the strict compare drops it
                    uint4 v = xv[j][r];
                    v = make_uint4(ok ? v.x : nan_pair, ok ? v.y : nan_pair, ok ? v.z : nan_pair, ok ? v.w : nan_pair);
                    const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float dv = word_half_to_f32<BF16X>(wd[e >> 1], e & 1) - m_eff;  // one fp32 subtraction
                        const uint64_t kb = __ballot(fabsf(dv) > a.tau);                      // strict; NaN is pruned
                        kp[e] = r == 0 ? kb : (kp[e] | kb);
                    }
                    *reinterpret_cast<uint4*>(xs + (size_t)(tg + 8 * r) * xrow + (size_t)(c * kWave + 8 * o) * 2) = v;
                }
                const uint64_t dense_ok = dense ? any_ok : 0ull;  // dense mode keeps every element that exists
                uint64_t u = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // byte o of the mask holds the eight token groups: nonzero byte -> bit 8*o+7 -> bit 8*o+e
                    const uint64_t v = kp[e] | dense_ok;
                    const uint64_t nz = (((v & 0x7f7f7f7f7f7f7f7full) + 0x7f7f7f7f7f7f7f7full) | v) & 0x8080808080808080ull;
                    u |= nz >> (7 - e);
                }
                um[j] = u;  // bit i: channel i of the chunk is kept by some token
                ucount += __popcll(u);
                ecount += __popcll(u);
            }
        };
        if constexpr (SUPERSET) {
            if (dense) {  // every element that exists is kept: the list is all valid channels, exactly
#pragma unroll
                for (int j = 0; j < MAXC; ++j) list_whole(j);
                ecount = ucount;
                return;
            }
            test_slot(0);
            const int nval0 = c_begin < c_end ? min((int)kWave, kend - (k0 + c_begin * kWave)) : 0;
            if (__popcll(um[0]) + 2 >= nval0) {  // wave-uniform
                if (count_exactly) {
                    const int listed = ucount;
#pragma unroll
                    for (int j = 1; j < MAXC; ++j) test_slot(j);  // adds to ecount; the list is rebuilt below
                    ucount = listed;
                }
#pragma unroll
                for (int j = 1; j < MAXC; ++j) list_whole(j);
            } else {
#pragma unroll
                for (int j = 1; j < MAXC; ++j) test_slot(j);
            }
        } else {
#pragma unroll
            for (int j = 0; j < MAXC; ++j) test_slot(j);
        }
    };
    if (a.xdt == kBF16)
        test_chunks(std::true_type{});
    else
        test_chunks(std::false_type{});
    if (lane == 0) {
        L.hdr[w] = ucount;
        L.hdr[(2 + BT) * WAVES + w] = ecount;  // behind the per-token rows and the flag row
    }
    __syncthreads();  // counts published, tile staged

    // ---- per-token counts (column tile 0 on request): one channel per lane from the staged tile
    auto kept_by = [&](int j, int b) {
        const int c = min(c_begin + j, nchunk - 1);
        const int k = k0 + (c_begin + j) * kWave + lane;
        const bool valid = (c_begin + j) < c_end && k < kend && b < a.B;
        const uint32_t code = *reinterpret_cast<const uint16_t*>(xs + (size_t)min(b, a.B - 1) * xrow + (size_t)(c * kWave + lane) * 2);
        const float dv = act_code_to_f32(code, bf16_sel) - m_eff;
        return valid & (dense | (fabsf(dv) > a.tau));
    };
    if (per_token) {
        for (int b = 0; b < BT; ++b) {
            int tc = 0;
#pragma unroll
            for (int j = 0; j < MAXC; ++j) tc += __popcll(__ballot(kept_by(j, b)));
            if (lane == 0) L.hdr[(1 + b) * WAVES + w] = tc;
        }
        __syncthreads();
    }
    int ubase = 0, cnt = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        const int v = L.hdr[i];
        if (i < w) ubase += v;
        cnt += v;
    }
    cnt = uniform(cnt);
    ubase = uniform(ubase);
    // ---- place the union list
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        if ((um[j] >> lane) & 1ull) L.idx[ubase + lanes_below(um[j])] = k0 + (c_begin + j) * kWave + lane;
        ubase += __popcll(um[j]);
    }
    if (per_token) {
        for (int b = 0; b < BT; ++b) {
            int tbase = 0, ttotal = 0;
            for (int i = 0; i < WAVES; ++i) {
                const int v = L.hdr[(1 + b) * WAVES + i];
                if (i < w) tbase += v;
                ttotal += v;
            }
#pragma unroll
            for (int j = 0; j < MAXC; ++j) {
                const bool kb = kept_by(j, b);
                const uint64_t tb = __ballot(kb);
                if (want_idx && kb)
                    store_dev(&a.idx_out[(int64_t)b * a.K + k0 + tbase + lanes_below(tb)], k0 + (c_begin + j) * kWave + lane);
                tbase += __popcll(tb);
            }
            if (tid == 0 && b < a.B) store_dev(&a.seg_cnt[b * a.Sl + split], ttotal);
        }
    }
    if (tile == 0 && tid == 0) {  // size of the union: the list's length, or the exact count where the list is a superset
        int exact = 0;
        for (int i = 0; i < WAVES; ++i) exact += L.hdr[(2 + BT) * WAVES + i];
        store_dev(&a.seg_cnt[a.B * a.Sl + split], count_exactly ? exact : cnt);
    }
    __syncthreads();
    return cnt;
}

// X32: the 32-deep matrix instruction (bf16 / fp16 weights).  It needs 151 registers per lane against 109, i.e. one
// workgroup per compute unit instead of two, so launches of more than 256 workgroups keep the 16-deep form.
template <int WDT, int FUSE, bool X32>
__global__ __launch_bounds__(kInlineWaves* kWave) void gemm_inline_raw_kernel(const GemvArgs a) {
    constexpr int WAVES = kInlineWaves;
    constexpr int BT = kMfmaTokens;
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr int TILE = 16 * ELEMS;

    extern __shared__ uint4 smem_raw[];
    Lds L = carve_lds<WAVES, BT>(reinterpret_cast<char*>(smem_raw), a.Kc);
    if constexpr (FUSE == kFuseSwiglu) L.fin = L.red + kTreeFloats;
    char* xs = reinterpret_cast<char*>(L.idx + a.Kc);  // staged inputs [16][Kc * 2 + pad] in place of the value lists
    const uint32_t xrow = (uint32_t)a.Kc * 2 + kRawPad;
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;
    const int k0 = split * a.Kc;
    const bool dense = a.mode == kModeDense;
    const float m_eff = dense ? 0.f : a.m;  // dense mode: x - 0 is x
    const uint32_t bf16_sel = a.xdt == kBF16 ? 0xffffffffu : 0u;

    const ColConst mine = load_col_const<WDT, TILE>(a, tile, tid % (TILE / 4));

    // ------------------------------------------------------------------ 1. stage the inputs, list the union
    // int8 weights: 256-column tiles, so half as many workgroups repeat a split's prologue and a wavefront has
    // two chunks; listing supersets measured no gain there (and 0.14 us lost to the extra code)
    const int cnt = stage_inputs_and_list<WAVES, kRawChunks, WDT != kI8>(a, tile, split, L, xs, xrow);
    const int n_blocks = (cnt + kMfmaBlock - 1) / kMfmaBlock;

    // ------------------------------------------------------------------ 2. stream the kept rows
    const int cg = lane & 15;  // column group (B/C index n); also the token whose values this lane supplies (A index m)
    const int kg = lane >> 4;  // row group: list rows 4*kg .. 4*kg+3 of a block
    const int col0 = tile * TILE + cg * ELEMS;
    const uint32_t lane_off = (col0 < a.N) ? (uint32_t)col0 * Vec<WDT>::kBytes : 0u;
    const uint32_t row_bytes = (uint32_t)a.N * Vec<WDT>::kBytes;
    const char* wbase = reinterpret_cast<const char*>(a.W);
    const bool tok_ok = cg < a.B;  // token slots past B carry zeros
    const char* xs_tok = xs + (size_t)min(cg, a.B - 1) * xrow;

    f32x4_t acc[ELEMS];
#pragma unroll
    for (int e = 0; e < ELEMS; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Four stages per wavefront, no branch anywhere: list rows of block n+3 and staged inputs of block n+2 come
    // out of LDS while the weight rows of block n+1 are in flight and the MFMAs of block n run.  A slot past the
    // end of the list reads LDS at a clamped position and weight row 0, and is zeroed by a select.
    struct Rows {
        int4 rows;
        int left;  // valid entries from this lane's first one on (<= 0: none)
    };
    struct Entries {
        int4 rows;
        uint32_t code[4];
        int left;
    };
    struct Stage {
        uint4 r[4];
        float4 d;
    };
    auto rows_of = [&](int blk, Rows& rw) {  // blk is wave-uniform and may lie past the end
        const int e0 = blk * kMfmaBlock + 4 * kg;
        rw.left = cnt - e0;
        rw.rows = *reinterpret_cast<const int4*>(L.idx + min(e0, a.Kc - 4));
    };
    auto codes_of = [&](const Rows& rw, Entries& en) {
        const int rj[4] = {rw.rows.x, rw.rows.y, rw.rows.z, rw.rows.w};
        en.rows = rw.rows;
        en.left = rw.left;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ch = j < rw.left ? rj[j] - k0 : 0;  // list entries lie in [k0, k0 + Kc)
            en.code[j] = *reinterpret_cast<const uint16_t*>(xs_tok + (size_t)ch * 2);
        }
    };
    auto issue = [&](const Entries& en, Stage& st) {
        const int rj[4] = {en.rows.x, en.rows.y, en.rows.z, en.rows.w};
        float dm[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool ok = j < en.left;
            const uint32_t row = ok ? (uint32_t)rj[j] : 0u;
            const uint4 v = load_weights16(wbase + (uint64_t)row * row_bytes + lane_off);
            st.r[j] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
            const float dv = act_code_to_f32(en.code[j], bf16_sel) - m_eff;  // one fp32 subtraction
            const bool keep = ok & tok_ok & (dense | (fabsf(dv) > a.tau));    // strict; NaN is pruned
            dm[j] = keep ? dv : 0.f;
        }
        st.d = make_float4(dm[0], dm[1], dm[2], dm[3]);
    };
    if constexpr (!X32) {
        // (int8 weights always: with 16 columns per lane the 32-deep form needs 180 registers and measured slower,
        // 14336 x 4096, 16 tokens: 23.3 against 24.8 us)
        auto compute = [&](const Stage& st) {
            s16x4_t a_hi, a_lo;
            split_operand<WDT>(st.d, a_hi, a_lo);
            mfma_block<WDT>(acc, a_hi, a_lo, st.r);
        };
        Rows R;
        Entries E0, E1;
        Stage A, Bs;
        rows_of(w, R);
        codes_of(R, E0);
        rows_of(w + WAVES, R);
        codes_of(R, E1);
        rows_of(w + 2 * WAVES, R);
        issue(E0, A);
        for (int blk = w; blk < n_blocks;) {
            codes_of(R, E0);
            rows_of(blk + 3 * WAVES, R);
            issue(E1, Bs);
            compute(A);
            blk += WAVES;
            if (blk >= n_blocks) break;
            codes_of(R, E1);
            rows_of(blk + 3 * WAVES, R);
            issue(E0, A);
            compute(Bs);
            blk += WAVES;
        }
    } else {
        // The matrix instruction is 32 rows deep (gfx950's 16x16x32): a wavefront's blocks are taken two at a time,
        // block w + 2p*WAVES in k-slots 0-3 of every lane and block w + (2p+1)*WAVES in k-slots 4-7.  A pair whose
        // second block lies past the end of the list carries zeros there.
        struct Rows2 {
            Rows a, b;
        };
        struct Entries2 {
            Entries a, b;
        };
        struct Stage2 {
            Stage a, b;
        };
        auto rows2_of = [&](int pr, Rows2& rw) {
            rows_of(w + 2 * pr * WAVES, rw.a);
            rows_of(w + (2 * pr + 1) * WAVES, rw.b);
        };
        auto codes2_of = [&](const Rows2& rw, Entries2& en) {
            codes_of(rw.a, en.a);
            codes_of(rw.b, en.b);
        };
        auto issue2 = [&](const Entries2& en, Stage2& st) {
            issue(en.a, st.a);
            issue(en.b, st.b);
        };
        auto compute2 = [&](const Stage2& st) {
            s16x4_t a_hi[2], a_lo[2];
            split_operand<WDT>(st.a.d, a_hi[0], a_lo[0]);
            split_operand<WDT>(st.b.d, a_hi[1], a_lo[1]);
            const uint4 r8[8] = {st.a.r[0], st.a.r[1], st.a.r[2], st.a.r[3], st.b.r[0], st.b.r[1], st.b.r[2], st.b.r[3]};
            mfma_block32<WDT>(acc, a_hi, a_lo, r8);
        };
        const int n_mine = n_blocks > w ? (n_blocks - w + WAVES - 1) / WAVES : 0;  // blocks w, w + WAVES, ...
        const int n_pairs = (n_mine + 1) / 2;

        Rows2 R;
        Entries2 E0, E1;
        Stage2 A, Bs;
        rows2_of(0, R);
        codes2_of(R, E0);
        rows2_of(1, R);
        codes2_of(R, E1);
        rows2_of(2, R);
        issue2(E0, A);
        for (int pr = 0; pr < n_pairs;) {
            codes2_of(R, E0);
            rows2_of(pr + 3, R);
            issue2(E1, Bs);
            compute2(A);
            if (++pr >= n_pairs) break;
            codes2_of(R, E1);
            rows2_of(pr + 3, R);
            issue2(E0, A);
            compute2(Bs);
            ++pr;
        }

    }

    // ------------------------------------------------------------------ 3. add the wavefronts' sums
    const __amdgpu_buffer_rsrc_t pbuf = partial_buffer<TILE>(a);
    reduce_waves_and_emit<WDT, WAVES, FUSE, WDT != kI8>(a, pbuf, tile, split, acc, L.red, L.fin);  // starts with a barrier: the tile is done with

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

template <int WDT, int FUSE, bool X32>
static int launch_inline_raw(const GemvArgs& a, size_t lds, hipStream_t stream) {
    if (lds > kInlineLdsBudget) return SCAP_ERR_SHAPE;
    if (lds > 64 * 1024) {
        constexpr int kMaxDevices = 64;
        static std::atomic<bool> asked[kMaxDevices];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SCAP_ERR_HIP;
        if (!asked[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_inline_raw_kernel<WDT, FUSE, X32>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kInlineLdsBudget) != hipSuccess)
                return SCAP_ERR_HIP;
            asked[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL((gemm_inline_raw_kernel<WDT, FUSE, X32>), dim3((unsigned)(a.S * a.T)), dim3(kInlineWaves * kWave),
                       lds, stream, a);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

template <int WDT, int FUSE>
static int launch_inline_wdt(const GemvArgs& a, int bt, bool raw, size_t lds, hipStream_t stream) {
    if constexpr (FUSE != kFuseList) {
        if (raw) {
            if constexpr (WDT != kI8) {
                if ((long)a.S * a.T <= 256) return launch_inline_raw<WDT, FUSE, true>(a, lds, stream);
            }
            return launch_inline_raw<WDT, FUSE, false>(a, lds, stream);
        }
    }
    if constexpr (WDT == kF16)  // fp16 weights: 16 token slots only (2-4 tokens stay on the vector kernel)
        return launch_inline<WDT, 16, FUSE>(a, lds, stream);
    else
        return bt == 4 ? launch_inline<WDT, 4, FUSE>(a, lds, stream) : launch_inline<WDT, 16, FUSE>(a, lds, stream);
}

template <int FUSE>
static int launch_inline_any(const GemvArgs& a, int wdt, int bt, bool raw, size_t lds, hipStream_t stream) {
    if (wdt == kBF16) return launch_inline_wdt<kBF16, FUSE>(a, bt, raw, lds, stream);
    if (wdt == kF16) return bt == kMfmaTokens ? launch_inline_wdt<kF16, FUSE>(a, bt, raw, lds, stream) : SCAP_ERR_CONFIG;
    if (wdt == kI8) return launch_inline_wdt<kI8, FUSE>(a, bt, raw, lds, stream);
    return SCAP_ERR_CONFIG;
}

// Plan one launch: token slots, rows per workgroup (bounded by LDS and, for the input prologue, by the
// registers that hold a wavefront's chunks), LDS bytes.
static int plan_inline(GemvArgs& a, int wdt, int kc, bool kc_forced, int fuse, int* bt_out, size_t* lds_out,
                       bool* raw_out = nullptr, bool slots16 = false) {
    if (wdt != kBF16 && wdt != kI8 && wdt != kF16) return SCAP_ERR_CONFIG;
    if (a.B < 1 || a.B > kMfmaTokens) return SCAP_ERR_CONFIG;
    const int bt = (a.B <= 4 && !slots16) ? 4 : 16;
    if (wdt == kF16 && bt != kMfmaTokens) return SCAP_ERR_CONFIG;  // fp16: the 16-slot kernels only
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
    // staged-tile form: 16 token slots, whole octets of channels, 16-byte aligned token rows
    const bool raw = raw_out != nullptr && bt == kMfmaTokens && fuse != kFuseList && a.K >= 8 && (a.K % 8) == 0 &&
                     (reinterpret_cast<uintptr_t>(a.x) & 15u) == 0 && a.Kc <= kInlineWaves * kWave * kRawChunks;
    if (raw) {
        const size_t body = (size_t)a.Kc * 4 + raw_tile_bytes(a.Kc);
        *lds_out = kHdrBytes + (body > red ? body : red);
    }
    if (raw_out) *raw_out = raw;
    return SCAP_OK;
}

// slots16: run 2-4 tokens in the 16-slot kernels (the staged-tile form when the shape allows it)
int launch_gemm_inline(const GemvArgs& a_in, int wdt, const scap_launch_cfg* cfg, hipStream_t stream, bool slots16) {
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
    bool raw = false;
    const int rc = plan_inline(a, wdt, kc, kc != 0, kFusePlain, &bt, &lds, &raw, slots16);
    if (rc != SCAP_OK) return rc;
    a.Kl = a.Kc;
    a.Sl = a.S;
    return launch_inline_any<kFusePlain>(a, wdt, bt, raw, lds, stream);
}

// The two launches of the fused SwiGLU block on the matrix cores (see scap_swiglu.hip for the vector form).
int launch_swiglu_block_inline(const GemvArgs& up_in, const GemvArgs& dn_in, int wdt, hipStream_t stream) {
    GemvArgs up = up_in, dn = dn_in;
    int bt_up = 0, bt_dn = 0;
    size_t lds_up = 0, lds_dn = 0;
    bool raw_up = false;
    int rc = plan_inline(up, wdt, 0, false, kFuseSwiglu, &bt_up, &lds_up, &raw_up);
    if (rc != SCAP_OK) return rc;
    up.Kl = up.Kc;
    up.Sl = up.S;
    rc = plan_inline(dn, wdt, 0, false, kFuseList, &bt_dn, &lds_dn);
    if (rc != SCAP_OK) return rc;
    dn.Kl = kWave;
    dn.Sl = (dn.K + kWave - 1) / kWave;
    const size_t tables = kHdrBytes + (size_t)dn.Sl * 4;  // offsets of every segment (tile 0's last arrival)
    if (lds_dn < tables) lds_dn = tables;
    rc = launch_inline_any<kFuseSwiglu>(up, wdt, bt_up, raw_up, lds_up, stream);
    if (rc != SCAP_OK) return rc;
    return launch_inline_any<kFuseList>(dn, wdt, bt_dn, false, lds_dn, stream);
}

}  // namespace scap
