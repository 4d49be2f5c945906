// Two to four tokens through the structure of the one-token kernel (scap_gemv1.hpp): the rows read are the union of
// the tokens' masks (Appendix C), every row read once and multiplied into one accumulator set per token, a token that
// pruned the channel contributing a zero (Eq. 3 per token).  Same four stages -- every wavefront tests all of the
// workgroup's inputs and keeps every 8th union position, the ring of row loads, one barrier and the slice-wise
// reduction, the split-K hand-over (fixed point by default, else ticketed partial sums per (tile, slice)) -- with BT
// token slots.  Wavefront b of a tile-0 workgroup writes token b's ascending list; the last of its writers closes it.
// FUSE gives it the two halves of the fused SwiGLU block (Alg. 2) in the list format of the batched block kernels
// (scap_gemv_parts.hpp, "list input"): kFuseSwiglu (2 slots) -- the wavefront that finishes a (tile, slice) of the
// gate|up launch gates it (16-byte int8 lanes only: its slice is 128 columns = one 64-channel list segment) --, and
// kFuseList (2 or 4 slots) -- the down launch takes its channels and centred values from those segments instead of x.
// BT = 2 token slots, and 4 (3-4 tokens) for 16-bit weights and for plain calls with int8 weights in 8-byte lanes.
// With the partial-sum hand-over the kernel's fixed part grows with the token slots -- the last arrival of a tile
// pulls S x BT partial slices through one compute unit's L1 (14336 x 4096 bf16: 0.9 us for one token, 2.1 for two,
// 3.8 for four); the fixed-point hand-over has nothing to pull, and four slots run with it only.
#pragma once

#include <atomic>

#include "scap_gemv1.hpp"

namespace scap {

constexpr int kG1bWaves = 8;
constexpr int kG1bMaxLds = 128 * 1024;  // of gfx950's 160 KB per compute unit

// a wavefront's list in LDS: channel index and BT centred values per entry
template <int BT> struct G1bList;
template <> struct G1bList<2> {
    int4* e;
    static constexpr int kBytes = 16;
    __device__ __forceinline__ G1bList(char* base, int w, int slots) : e(reinterpret_cast<int4*>(base) + w * slots) {}
    __device__ __forceinline__ void put(int p, int idx, const float* d) const {
        e[p] = make_int4(idx, __float_as_int(d[0]), __float_as_int(d[1]), 0);
    }
    __device__ __forceinline__ void get(int p, int& idx, float* d) const {
        const int4 t = e[p];
        idx = t.x;
        d[0] = __int_as_float(t.y);
        d[1] = __int_as_float(t.z);
    }
};
template <> struct G1bList<4> {  // two 16-byte halves per entry
    int4* e;
    static constexpr int kBytes = 32;
    __device__ __forceinline__ G1bList(char* base, int w, int slots) : e(reinterpret_cast<int4*>(base) + 2 * w * slots) {}
    __device__ __forceinline__ void put(int p, int idx, const float* d) const {
        e[2 * p] = make_int4(idx, __float_as_int(d[0]), __float_as_int(d[1]), __float_as_int(d[2]));
        e[2 * p + 1] = make_int4(__float_as_int(d[3]), 0, 0, 0);
    }
    __device__ __forceinline__ void get(int p, int& idx, float* d) const {
        const int4 t = e[2 * p], u = e[2 * p + 1];
        idx = t.x;
        d[0] = __int_as_float(t.y);
        d[1] = __int_as_float(t.z);
        d[2] = __int_as_float(t.w);
        d[3] = __int_as_float(u.x);
    }
};
// list slots per wavefront: a multiple of 4, so that the 16-byte parts of the lists stay aligned
__host__ __device__ inline int g1b_slots(int Kc) { return (Kc / kG1bWaves + 4) & ~3; }

inline size_t gemv1b_lds_bytes(int tile_cols, int Kc, int bt) {
    return (size_t)kG1HdrBytes * bt + (size_t)kG1bWaves * bt * tile_cols * 4 + (size_t)kG1bWaves * g1b_slots(Kc) * (bt == 2 ? 16 : 32);
}

template <int WDT, int NCH, int BT, int FUSE = kFusePlain>
__global__ __launch_bounds__(kG1bWaves * kWave) void gemv1b_kernel(const uint16_t* x, const void* W, int K, int N, int Kc, int S,
                                                                int T, int B, int mode, int xdt, float m, float tau, int flags,
                                                                const float* bias, float* y, float* partial,
                                                                int32_t* counters, const uint16_t* col_scale,
                                                                int32_t* idx_out, int32_t* nnz_out, int32_t* union_nnz_out,
                                                                int32_t* seg_cnt, float m2, float tau2, float* z_out,
                                                                int32_t* zl_idx, float* zl_d, int32_t* zl_cnt, int F,
                                                                unsigned long long* fx_acc) {
    constexpr int WAVES = kG1bWaves;
    constexpr int UNROLL = WDT == kI8Half ? 8 : 4;
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr bool IS_I8 = WDT == kI8 || WDT == kI8Half;
    constexpr int TILE = kWave * ELEMS;
    constexpr int CPL = ELEMS / WAVES;  // columns per lane of a wavefront's slice
    constexpr int SLICE = kWave * CPL;
    static_assert(CPL == 1 || CPL == 2, "a slice is 4 or 8 bytes per lane");
    static_assert(BT == 2 || (BT == 4 && FUSE != kFuseSwiglu), "two token slots; four without the gating epilogue");
    static_assert(FUSE != kFuseSwiglu || CPL == 2, "the gating epilogue needs a slice of 128 columns: one 64-channel list segment");
    typedef SliceVec<CPL> slice_t;

    extern __shared__ uint4 smem_raw[];
    char* smem = reinterpret_cast<char*>(smem_raw);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = uniform(tid >> 6);
    // header: one block of split offsets and counts per token slot (the wavefront that closes token b's list uses block b)
    int* s_off = reinterpret_cast<int*>(smem + (w < BT ? w : 0) * kG1HdrBytes);
    int* s_cnt = s_off + kMaxSplits;
    float* s_red = reinterpret_cast<float*>(smem + BT * kG1HdrBytes);  // [WAVES][BT][TILE]
    const int slots = g1b_slots(Kc);
    const G1bList<BT> mylist(smem + BT * kG1HdrBytes + WAVES * BT * TILE * 4, w, slots);
    static_assert(G1bList<BT>::kBytes == (BT == 2 ? 16 : 32), "entry size assumed by gemv1b_lds_bytes");

    const int tile = blockIdx.x % T;
    const int split = blockIdx.x / T;
    const int k0 = split * Kc;
    const int kend = min(k0 + Kc, K);

    // ------------------------------------------------------------------ 1. inputs: every wavefront, all Kc, all tokens
    // (K is a multiple of 8 -- checked on the host --, so every token's row is 16-byte aligned and no octet is ragged)
    uint4 xv[BT][NCH];
    if constexpr (FUSE != kFuseList) {
#pragma unroll
        for (int b = 0; b < BT; ++b) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                xv[b][c] = make_uint4(0u, 0u, 0u, 0u);
                const int kb = k0 + c * kG1Chunk + 8 * lane;
                if (b < B && kb < kend) xv[b][c] = *reinterpret_cast<const uint4*>(x + (size_t)b * K + kb);
            }
        }
    }
    // Column c of this lane is fcol + c * CSTR: lanes side by side (every store and atomic of the hand-over then covers
    // 64 consecutive words), except under the gating epilogue, which pairs gate and up columns through neighbouring
    // lanes and keeps a lane's columns adjacent.
    constexpr int CSTR = FUSE == kFuseSwiglu ? 1 : kWave;
    constexpr int LSTR = FUSE == kFuseSwiglu ? CPL : 1;
    const int fcol = tile * TILE + w * SLICE + lane * LSTR;
    float cbias[CPL], cscale[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        cbias[c] = 0.f;
        cscale[c] = 1.f;
        if (fcol + c * CSTR < N) {
            if (bias) cbias[c] = bias[fcol + c * CSTR];
            if (IS_I8) cscale[c] = f16_bits_to_f32(col_scale[fcol + c * CSTR]);
        }
    }

    const bool want_lists = FUSE == kFusePlain && tile == 0 && w < B && (nnz_out != nullptr || union_nnz_out != nullptr);
    const float m_eff = mode == kModeSparse ? m : 0.f;
    const uint32_t keep_all = mode == kModeSparse ? 0u : 1u;
    int cnt = 0;   // union positions so far -- wave-uniform
    int lcnt = 0;  // kept channels of token w so far (tile 0, w < B)
    if constexpr (FUSE == kFuseList) {
        // The workgroup's channels are Kc / 64 list segments of the gated product (K = F here; Kc is a multiple of
        // 64).  Every entry slot of those segments and their counts are fetched together, whatever the counts will
        // say (one memory round trip; slots past a segment's count hold stale entries and are dropped below); lane l
        // takes the count of segment l, a prefix sum gives every entry its position in the workgroup's list.
        constexpr int ITS = 8 * NCH;  // Kc / 64 segments at most
        const int seg0 = k0 >> 6;
        const int nsegw = (kend - k0 + kWave - 1) >> 6;
        const int nsegs = (K + kWave - 1) >> 6;
        int eidx[ITS];
        float ed[ITS][BT];
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            eidx[it] = 0;
#pragma unroll
            for (int b = 0; b < BT; ++b) ed[it][b] = 0.f;
            if (it < nsegw) {
                const int64_t e = (int64_t)(seg0 + it) * kWave + lane;
                eidx[it] = zl_idx[e];
                typedef float dvec_t __attribute__((ext_vector_type(BT)));
                const dvec_t dv = *reinterpret_cast<const dvec_t*>(zl_d + e * BT);
#pragma unroll
                for (int b = 0; b < BT; ++b) ed[it][b] = dv[b];
            }
        }
        int c_l = lane < nsegw ? zl_cnt[seg0 + lane] : 0;
        c_l = min(max(c_l, 0), (int)kWave);  // keeps LDS writes in range whatever the memory holds
        const int inc = wave_inclusive_scan(c_l);
        const int off_l = inc - c_l;
        cnt = __shfl(inc, kWave - 1, kWave);
        int pos[ITS];
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int c_s = __shfl(c_l, it, kWave), o_s = __shfl(off_l, it, kWave);
            pos[it] = (it < nsegw && lane < c_s) ? o_s + lane : -1;
        }
#pragma unroll
        for (int it = 0; it < ITS; ++it)
            if (pos[it] >= 0 && (pos[it] & (WAVES - 1)) == w) mylist.put(pos[it] / WAVES, eidx[it], ed[it]);
        if (tile == 0 && w < B && (nnz_out != nullptr || idx_out != nullptr)) {
            // Token w's ascending list of kept channels: an entry is the token's where its centred value is non-zero
            // (kept means |d| > tau >= 0).  No gap closing: the entries of all earlier segments are counted in what
            // the first launch wrote.
            int before = 0;
            for (int s0 = 0; s0 < seg0; s0 += kWave) {
                const int sg = s0 + lane;
                before += sg < seg0 ? min(max(zl_cnt[(1 + w) * nsegs + sg], 0), (int)kWave) : 0;
            }
            before = wave_sum(before);
            int run = 0;
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                float dw = 0.f;  // token w's value of the entry
#pragma unroll
                for (int b = 0; b < BT; ++b)
                    if (w == b) dw = ed[it][b];
                const bool mine = pos[it] >= 0 && dw != 0.f;
                const uint64_t bal = __ballot(mine);
                if (mine && idx_out) idx_out[(int64_t)w * K + before + run + lanes_below(bal)] = eidx[it];
                run += __popcll(bal);
            }
            if (split == S - 1 && lane == 0 && nnz_out) nnz_out[w] = before + run;
        }
    } else {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if (k0 + c * kG1Chunk < kend) {  // wave-uniform
            const int kb = k0 + c * kG1Chunk + 8 * lane;
            const int nvalid = kend - kb;  // elements j < nvalid of this lane exist
            float dv[BT][8];
            uint32_t kbits[BT], any = 0;
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const uint32_t wd[4] = {xv[b][c].x, xv[b][c].y, xv[b][c].z, xv[b][c].w};
                float xf[8];
                if (xdt == kBF16) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) xf[j] = __uint_as_float((j & 1) ? (wd[j >> 1] & 0xFFFF0000u) : (wd[j >> 1] << 16));
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) xf[j] = f16_bits_to_f32((j & 1) ? (wd[j >> 1] >> 16) : (wd[j >> 1] & 0xFFFFu));
                }
                // sparse mode: d = x - m in one fp32 subtraction (Alg. 3 step 1), kept if |d| > tau, strictly (Eq. 2; NaN
                // is pruned).  Dense mode (Eq. 1): d = x - 0 = x, every channel that exists is kept.  Bit arithmetic
                // instead of && / ?: keeps this free of branches.
                uint32_t kb_b = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float d = xf[j] - m_eff;
                    const uint32_t keep = ((uint32_t)(fabsf(d) > tau) | keep_all) & (uint32_t)(j < nvalid) & (uint32_t)(b < B);
                    dv[b][j] = keep ? d : 0.f;
                    kb_b |= keep << j;
                }
                kbits[b] = kb_b;
                any |= kb_b;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool mine = (any >> j) & 1u;
                const uint64_t bal = __ballot(mine);
                const int pos = cnt + lanes_below(bal);
                if (mine && (pos & (WAVES - 1)) == w) {
                    float d[BT];
#pragma unroll
                    for (int b = 0; b < BT; ++b) d[b] = dv[b][j];
                    mylist.put(pos / WAVES, kb + j, d);
                }
                cnt += __popcll(bal);
            }
            if (want_lists) {
                uint32_t mybits = 0;
#pragma unroll
                for (int b = 0; b < BT; ++b)
                    if (w == b) mybits = kbits[b];
                const int mine = __popc(mybits);
                const int inc = wave_inclusive_scan(mine);
                if (idx_out) {
                    int64_t p = (int64_t)w * K + k0 + lcnt + inc - mine;
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if ((mybits >> j) & 1u) store_dev(&idx_out[p++], kb + j);
                }
                lcnt += __shfl(inc, kWave - 1, kWave);
            }
        }
    }
    }
    cnt = uniform(cnt);
    lcnt = uniform(lcnt);
    if (want_lists && lane == 0) {
        if (S == 1) {
            if (nnz_out) nnz_out[w] = lcnt;
            if (w == 0 && union_nnz_out) union_nnz_out[0] = cnt;
        } else {
            store_dev(&seg_cnt[(1 + w) * kMaxSplits + split], lcnt);
            if (w == 0) store_dev(&seg_cnt[split], cnt);
        }
    }
    __builtin_amdgcn_wave_barrier();  // the list is this wavefront's own: written above, read below, in order

    // ------------------------------------------------------------------ 2. stream the union's rows
    float acc[BT][ELEMS];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int j = 0; j < ELEMS; ++j) acc[b][j] = 0.f;
    const int col0 = tile * TILE + lane * ELEMS;
    const uint32_t lane_off = col0 < N ? (uint32_t)col0 * Vec<WDT>::kBytes : 0u;  // lanes past N re-read column 0
    const uint32_t row_bytes = (uint32_t)N * Vec<WDT>::kBytes;
    const char* wbase = reinterpret_cast<const char*>(W);
    const int n_w = cnt > w ? (cnt - w + WAVES - 1) / WAVES : 0;  // positions w, w + WAVES, ...

    for (int i0 = 0; i0 < n_w; i0 += kWave) {
        const int e = i0 + lane;
        int vidx = 0;
        float vd[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) vd[b] = 0.f;
        if (e < n_w) mylist.get(e, vidx, vd);
        const int nb = min((int)kWave, n_w - i0);
        auto row_load = [&](int i) {
            return load_row<WDT>(wbase, (uint32_t)__builtin_amdgcn_readlane(vidx, i), row_bytes, lane_off);
        };
        auto fma_rows = [&](const uint4& r, int i) {
#pragma unroll
            for (int b = 0; b < BT; ++b) fma_row<WDT>(acc[b], r, read_lane_f(vd[b], i));
        };
        uint4 r[UNROLL];
        if (nb < UNROLL) {
#pragma unroll
            for (int q = 0; q < UNROLL - 1; ++q)
                if (q < nb) r[q] = row_load(q);
#pragma unroll
            for (int q = 0; q < UNROLL - 1; ++q)
                if (q < nb) fma_rows(r[q], q);
        } else {
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) r[q] = row_load(q);
            int u = 0;
            for (; u + 2 * UNROLL <= nb; u += UNROLL) {
#pragma unroll
                for (int q = 0; q < UNROLL; ++q) {
                    fma_rows(r[q], u + q);
                    r[q] = row_load(u + UNROLL + q);
                    __builtin_amdgcn_sched_barrier(0);  // keep each load where it is: right behind the row it replaces
                }
            }
            // rows u .. u+UNROLL-1 are in flight; fewer than UNROLL further rows are left to issue
            const int rest = nb - u - UNROLL;
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                fma_rows(r[q], u + q);
                if (q < rest) r[q] = row_load(u + UNROLL + q);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int q = 0; q < UNROLL - 1; ++q)
                if (q < rest) fma_rows(r[q], u + UNROLL + q);
        }
    }

    // ------------------------------------------------------------------ 3. add the wavefronts' sums, slice by slice
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        float4* dst = reinterpret_cast<float4*>(s_red + (w * BT + b) * TILE + lane * ELEMS);
#pragma unroll
        for (int j = 0; j < ELEMS / 4; ++j) dst[j] = make_float4(acc[b][4 * j], acc[b][4 * j + 1], acc[b][4 * j + 2], acc[b][4 * j + 3]);
    }
    __syncthreads();
    slice_t sum[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) {
#pragma unroll
        for (int c = 0; c < CPL; ++c) sum[b].v[c] = 0.f;
#pragma unroll
        for (int i = 0; i < WAVES; ++i) {
#pragma unroll
            for (int c = 0; c < CPL; ++c) sum[b].v[c] += s_red[(i * BT + b) * TILE + w * SLICE + lane * LSTR + c * CSTR];
        }
    }

    // the finished slice of both tokens: scaled (int8), fused bias added (Eq. 6); y written through to memory, or gated
    auto finish = [&](const slice_t* s) {
        float p[BT][CPL];
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int c = 0; c < CPL; ++c) p[b][c] = (IS_I8 ? s[b].v[c] * cscale[c] : s[b].v[c]) + cbias[c];
        if constexpr (FUSE != kFuseSwiglu) {
#pragma unroll
            for (int b = 0; b < BT; ++b)
#pragma unroll
                for (int c = 0; c < CPL; ++c)
                    if (b < B && fcol + c * CSTR < N) store_dev(&y[(size_t)b * N + fcol + c * CSTR], p[b][c]);
        } else {
            // Columns come in groups of 8: 4 gate pre-activations, then the 4 matching up pre-activations; a lane holds
            // 2 adjacent columns, so lanes 0-1 of every 4 hold a group's gate columns and fetch their up partners from
            // 2 lanes further on.  z = silu(gate) * up (Alg. 2), centred and thresholded like any layer input (Alg. 3
            // steps 1-2, strict compare of Eq. 2; each token its own mask); the slice's channels kept by either token
            // become one 64-channel list segment, ascending, the tokens' centred values side by side (0 where a token
            // pruned the channel), with the union's and the tokens' counts.
            constexpr int LPG = 8 / CPL;
            const bool gate_lane = (lane % LPG) < LPG / 2;
            float dz[BT][CPL];
            bool keep[BT][CPL], any[CPL];
            int chan[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int col = fcol + c;
                chan[c] = (col >> 3) * 4 + (col & 3);
                const bool live = gate_lane && col < N && chan[c] < F;
                any[c] = false;
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float up = __shfl_down(p[b][c], LPG / 2, kWave);
                    const float z = p[b][c] / (1.f + expf(-p[b][c])) * up;
                    if (live && b < B && z_out) store_dev(&z_out[(int64_t)b * F + chan[c]], z);
                    const float d = z - m2;  // one fp32 subtraction
                    keep[b][c] = live && b < B && fabsf(d) > tau2;  // strict; NaN is pruned
                    dz[b][c] = keep[b][c] ? d : 0.f;
                    any[c] |= keep[b][c];
                }
            }
            const int seg = tile * WAVES + w;  // this slice's segment: channels seg * 64 ...
            const int nsegs = (F + kWave - 1) >> 6;
            if ((int64_t)seg * kWave < F) {  // wave-uniform
                int rank = 0, total_kept = 0;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const uint64_t bal = __ballot(any[c]);
                    rank += lanes_below(bal);
                    total_kept += __popcll(bal);
                }
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    if (any[c]) {
                        const int64_t e = (int64_t)seg * kWave + rank;
                        store_dev(&zl_idx[e], chan[c]);
                        store_dev(reinterpret_cast<unsigned long long*>(zl_d + e * BT),
                                  (unsigned long long)__float_as_uint(dz[0][c]) | ((unsigned long long)__float_as_uint(dz[1][c]) << 32));
                        ++rank;  // the lane's own earlier column comes first
                    }
                }
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    int kept_b = 0;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) kept_b += __popcll(__ballot(keep[b][c]));
                    if (lane == 0 && b < B) store_dev(&zl_cnt[(1 + b) * nsegs + seg], kept_b);
                }
                if (lane == 0) store_dev(&zl_cnt[seg], total_kept);
            }
        }
    };
    if (S == 1) {
        finish(sum);
        return;
    }

    // ------------------------------------------------------------------ 4a. split-K hand-over in fixed point
    // As in the one-token kernel (scap_gemv1.hpp, 4a), one 64-bit word per (token, column): every arrival adds its
    // partial, rounded to 2^-frac and biased, and a 1 in the arrival count with ONE atomic; whoever completes a
    // column's count holds its sum, converts it once, applies scale and bias and stores y.  A partial that is not
    // finite or not below 2^20 travels as fp32 through its partial-sum slot and the column's escape mask.
    if constexpr (FUSE != kFuseSwiglu) {
        if (fx_acc != nullptr) {
            const int limit_bits = fx_limit_bits(S);
            const int frac = limit_bits - kFxRangeBits;
            const double to_fixed = __hiloint2double((1023 + frac) << 20, 0);    // 2^frac
            const double from_fixed = __hiloint2double((1023 - frac) << 20, 0);  // 2^-frac
            const unsigned long long fbias = 1ull << limit_bits;
            unsigned long long* escw = fx_acc + kFxCols;
            const uint32_t pstride = (uint32_t)T * B * TILE * 4u;
            const uint32_t pmine = (uint32_t)((tile * B * TILE + w * SLICE + lane * CPL) * 4);
            const uint32_t ptok = (uint32_t)TILE * 4u;
            bool esc[BT][CPL];
            bool any_esc = false;
#pragma unroll
            for (int b = 0; b < BT; ++b)
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    esc[b][c] = b < B && fcol + c * CSTR < N && !(fabsf(sum[b].v[c]) < 1048576.f);  // also NaN and Inf
                    any_esc |= esc[b][c];
                }
            if (__ballot(any_esc) != 0ull) {  // rare
                const __amdgpu_buffer_rsrc_t pbuf = make_raw_buffer(partial, (uint32_t)S * T * B * TILE * 4u);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    if (b < B) sum[b].store_coherent(pbuf, split * pstride + pmine + b * ptok);
#pragma unroll
                    for (int c = 0; c < CPL; ++c)
                        if (esc[b][c])
                            __hip_atomic_fetch_or(&escw[(size_t)b * N + fcol + c * CSTR], 1ull << split, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                wait_memory_ops();  // values and mask bits are in place before the arrivals are counted
            }
            unsigned long long now_c[BT][CPL];  // all of the lane's atomics first, then what they returned
#pragma unroll
            for (int b = 0; b < BT; ++b)
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    now_c[b][c] = 0ull;
                    if (!(b < B && fcol + c * CSTR < N)) continue;
                    const long long vfix = esc[b][c] ? 0ll : __double2ll_rn((double)sum[b].v[c] * to_fixed);
                    const unsigned long long inc = (1ull << 57) | (esc[b][c] ? 1ull << 50 : 0ull) | (unsigned long long)(vfix + (long long)fbias);
                    now_c[b][c] = __hip_atomic_fetch_add(&fx_acc[(size_t)b * N + fcol + c * CSTR], inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + inc;
                }
#pragma unroll
            for (int b = 0; b < BT; ++b)
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const unsigned long long now = now_c[b][c];
                    if ((int)(now >> 57) != S) continue;  // not the column's last arrival (or no column: count 0, S > 1)
                    const long long total = (long long)(now & ((1ull << 50) - 1)) - (long long)S * (long long)fbias;
                    float yv = (float)((double)total * from_fixed);
                    const size_t word = (size_t)b * N + fcol + c * CSTR;
                    if ((now >> 50) & 127ull) {  // escaped partials: add them in split order
                        unsigned long long mask = load_dev(&escw[word]);
                        const float* pcol = partial + (size_t)(tile * B + b) * TILE + w * SLICE + lane * CPL + c;
                        while (mask) {
                            const int sp = __builtin_ctzll(mask);
                            mask &= mask - 1;
                            yv += load_dev(pcol + (size_t)sp * T * B * TILE);
                        }
                        store_dev(&escw[word], 0ull);
                    }
                    yv = (IS_I8 ? yv * cscale[c] : yv) + cbias[c];
                    store_dev(&y[word], yv);
                    store_dev(&fx_acc[word], 0ull);  // zero at rest
                }
            if (!want_lists || S == 1) return;
            // token w's list (tile 0, wavefront w < B) still needs the last of its writers to close the gaps: they
            // stored their pieces and counts before taking this ticket
            wait_memory_ops();
            unsigned long long* lt = reinterpret_cast<unsigned long long*>(counters + w * kG1TicketWords);
            unsigned long long got = 0;
            if (lane == 0) got = __hip_atomic_fetch_add(lt, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1ull;
            if (__builtin_amdgcn_readfirstlane((int)(uint32_t)got) != S) return;
            if (lane == 0) store_dev(lt, 0ull);
            const int run = close_list_rows(seg_cnt + (1 + w) * kMaxSplits, idx_out ? idx_out + (int64_t)w * K : nullptr, S, K, Kc, s_off, s_cnt);
            if (lane == 0 && nnz_out) nnz_out[w] = run;
            if (w == 0 && union_nnz_out) {
                int u = 0;
                for (int s0 = 0; s0 < S; s0 += kWave) u += s0 + lane < S ? load_dev(&seg_cnt[s0 + lane]) : 0;
                u = wave_sum(u);
                if (lane == 0) union_nnz_out[0] = u;
            }
            return;
        }
    }

    // ------------------------------------------------------------------ 4. split-K hand-over per (tile, slice)
    // partials [S][T][B][TILE]: as in the one-token kernel, B slices per arrival
    const __amdgpu_buffer_rsrc_t pbuf = make_raw_buffer(partial, (uint32_t)S * T * B * TILE * 4u);
    const uint32_t pstride = (uint32_t)T * B * TILE * 4u;  // bytes between consecutive splits
    const uint32_t pmine = (uint32_t)((tile * B * TILE + w * SLICE + lane * CPL) * 4);
    const uint32_t ptok = (uint32_t)TILE * 4u;  // bytes between consecutive tokens
#pragma unroll
    for (int b = 0; b < BT; ++b)
        if (b < B) sum[b].store_coherent(pbuf, split * pstride + pmine + b * ptok);
    wait_memory_ops();  // the wavefront's stores have been acknowledged
    unsigned long long* ticket = reinterpret_cast<unsigned long long*>(counters + tile * kCounterStride + w * kG1TicketWords);
    unsigned long long seen = 0;
    if (lane == 0)
        seen = __hip_atomic_fetch_add(ticket, ticket_increment(xcc_id()), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) +
               ticket_increment(xcc_id());
    const uint32_t seen_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)seen);
    const uint32_t seen_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(seen >> 32));
    seen = ((unsigned long long)seen_hi << 32) | seen_lo;
    if ((int)(seen & 0xFFFFull) != S) return;  // not the last arrival of this slice

    const bool near = ticket_all_one_xcd(seen) && !(flags & kG1FlagDeviceScope);
    if (near) asm volatile("buffer_inv sc0" ::: "memory");  // this compute unit's vector L1 holds nothing older
    constexpr int FLY = CPL == 1 ? 32 : 16;  // partial loads in flight per token, two tokens at a time
#pragma unroll
    for (int b0 = 0; b0 < BT; b0 += 2) {
        if (b0 >= B) break;
        slice_t total[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < CPL; ++c) total[t].v[c] = 0.f;
        for (int sp0 = 0; sp0 < S; sp0 += FLY) {
            slice_t v[2][FLY];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t tok = (uint32_t)min(b0 + t, B - 1) * ptok;  // a slot past the last token re-reads it
                if (near) {
#pragma unroll
                    for (int j = 0; j < FLY; ++j) v[t][j] = slice_t::load_plain(pbuf, min(sp0 + j, S - 1) * pstride + pmine + tok);
                } else {
#pragma unroll
                    for (int j = 0; j < FLY; ++j) v[t][j] = slice_t::load_coherent(pbuf, min(sp0 + j, S - 1) * pstride + pmine + tok);
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int j = 0; j < FLY; ++j) {
                    const bool in = sp0 + j < S;  // a slot past the last split re-read it: not added
#pragma unroll
                    for (int c = 0; c < CPL; ++c) total[t].v[c] += in ? v[t][j].v[c] : 0.f;
                }
            }
        }
        finish(total);
    }
    if (lane == 0) store_dev(ticket, 0ull);  // ready for the next call
    if (want_lists) {
        // token w's lists of all splits are complete: their writers stored them before taking this slice's ticket
        const int run = close_list_rows(seg_cnt + (1 + w) * kMaxSplits, idx_out ? idx_out + (int64_t)w * K : nullptr, S, K, Kc, s_off, s_cnt);
        if (lane == 0 && nnz_out) nnz_out[w] = run;
        if (w == 0 && union_nnz_out) {
            int u = 0;
            for (int s0 = 0; s0 < S; s0 += kWave) u += s0 + lane < S ? load_dev(&seg_cnt[s0 + lane]) : 0;
            u = wave_sum(u);
            if (lane == 0) union_nnz_out[0] = u;
        }
    }
}

// ---------------------------------------------------------------------------------------------- launch
struct Gemv1bArgs {
    Gemv1Args a;
    int B, bt;
};

template <int WDT, int NCH, int BT, int FUSE>
static int launch_gemv1b_one(const Gemv1bArgs& g, size_t lds, hipStream_t stream) {
    if (lds > 64 * 1024) {  // once per device and instantiation: allow the larger dynamic LDS
        constexpr int kMaxDevices = 64;
        static std::atomic<bool> asked[kMaxDevices];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SCAP_ERR_HIP;
        if (!asked[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv1b_kernel<WDT, NCH, BT, FUSE>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kG1bMaxLds) != hipSuccess)
                return SCAP_ERR_HIP;
            asked[dev].store(true, std::memory_order_release);
        }
    }
    const Gemv1Args& a = g.a;
    const dim3 grid((unsigned)(a.S * a.T)), block(kG1bWaves * kWave);
    hipLaunchKernelGGL((gemv1b_kernel<WDT, NCH, BT, FUSE>), grid, block, lds, stream, a.x, a.W, a.K, a.N, a.Kc, a.S, a.T, g.B,
                       a.mode, a.xdt, a.m, a.tau, a.flags, a.bias, a.y, a.partial, a.counters, a.col_scale, a.idx_out,
                       a.nnz_out, a.union_nnz_out, a.seg_cnt, a.m2, a.tau2, a.z_out, a.zl_idx, a.zl_d, a.zl_cnt, a.F,
                       FUSE == kFuseSwiglu ? nullptr : a.fx_acc);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

template <int WDT, int BT, int FUSE>
static int launch_gemv1b_nch(const Gemv1bArgs& g, hipStream_t stream) {
    constexpr int TILE = kWave * Vec<WDT>::kElems;
    const size_t lds = gemv1b_lds_bytes(TILE, g.a.Kc, BT);
    if (lds > (size_t)kG1bMaxLds) return SCAP_ERR_CONFIG;
    if (g.a.Kc <= kG1Chunk) return launch_gemv1b_one<WDT, 1, BT, FUSE>(g, lds, stream);
    if (g.a.Kc <= 2 * kG1Chunk) return launch_gemv1b_one<WDT, 2, BT, FUSE>(g, lds, stream);
    if (g.a.Kc <= 4 * kG1Chunk) return launch_gemv1b_one<WDT, 4, BT, FUSE>(g, lds, stream);
    return SCAP_ERR_CONFIG;
}

template <int WDT>
int launch_gemv1b_wdt(const Gemv1bArgs& g, hipStream_t stream) {
    if (g.bt == 2) return launch_gemv1b_nch<WDT, 2, kFusePlain>(g, stream);
    // four slots: 16-bit weights and int8 in 8-byte lanes (with 16-byte int8 lanes the wavefronts' sums of four tokens
    // do not fit LDS; those batches go to the matrix cores)
    if constexpr (WDT == kF16 || WDT == kBF16 || WDT == kI8Half) {
        if (g.bt == 4) return launch_gemv1b_nch<WDT, 4, kFusePlain>(g, stream);
    }
    return SCAP_ERR_CONFIG;
}

// the launches of the fused block of two tokens (fuse: kFuseSwiglu -- 16-byte int8 lanes only -- or kFuseList), and
// the down launch of a 16-bit block of 3-4 tokens (kFuseList, four slots)
template <int WDT>
int launch_gemv1b_block_wdt(const Gemv1bArgs& g, int fuse, hipStream_t stream) {
    if constexpr (WDT == kF16 || WDT == kBF16) {  // four slots: the down launch of a 16-bit block of 3-4 tokens
        if (g.bt == 4 && fuse == kFuseList) return launch_gemv1b_nch<WDT, 4, kFuseList>(g, stream);
    }
    if (g.bt != 2) return SCAP_ERR_CONFIG;
    if (fuse == kFuseList) return launch_gemv1b_nch<WDT, 2, kFuseList>(g, stream);
    if constexpr (WDT == kI8) {
        if (fuse == kFuseSwiglu) return launch_gemv1b_nch<WDT, 2, kFuseSwiglu>(g, stream);
    }
    return SCAP_ERR_CONFIG;
}

}  // namespace scap
