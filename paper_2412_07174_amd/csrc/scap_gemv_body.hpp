// Body of the column-gathered GEMV kernel (SCAP Alg. 3; Eq. 2, 3, 6), shared by the plain launch and the
// two launches of the fused SwiGLU block (Alg. 2).
#pragma once

#include "scap_gemv_parts.hpp"

namespace scap {

// 16 bytes of weight row `row` at this lane's columns.  `row` is wave-uniform, so the row base is
// formed on the scalar unit and the load takes a scalar base plus a 32-bit lane offset.
__device__ __forceinline__ uint4 load_row_vec(const char* __restrict__ wbase, uint32_t row, uint32_t row_bytes,
                                              uint32_t lane_off) {
    const uint64_t base = reinterpret_cast<uint64_t>(wbase) + (uint64_t)row * (uint64_t)row_bytes;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base >> 32));
    typedef __attribute__((address_space(1))) const char gchar_t;
    gchar_t* p = (gchar_t*)(((uint64_t)hi << 32) | lo);
    return load_weights16((global_u32x4_t*)(p + lane_off));
}

// LPR = lanes that share one weight row: 64 (a wavefront reads 1 KB of one row per load) or 32 (it reads
// 512 bytes of each of 2 rows).  Fewer lanes per row make the column tile narrower, so the same
// number of workgroups needs fewer K splits and the final reduction reads less.
// FUSE (kFusePlain / kFuseSwiglu / kFuseList) selects where the inputs come from and what the tile's last
// arrival does with the finished columns.
template <int WDT, int WAVES, int UNROLL, int BT, int LPR, int FUSE>
__device__ __forceinline__ void gemv_body(const GemvArgs& a) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr int TILE = LPR * ELEMS;
    constexpr int RPI = kWave / LPR;  // rows per load instruction
    constexpr int NT = WAVES * kWave;
    constexpr int GROUPS = TILE / 4;  // 4-column groups of a tile
    static_assert(GROUPS <= NT && NT % GROUPS == 0, "thread t finishes group t % GROUPS in every pass");

    extern __shared__ uint4 smem_raw[];
    Lds L = carve_lds<WAVES, BT>(reinterpret_cast<char*>(smem_raw), a.Kc);
    if constexpr (FUSE == kFuseSwiglu) {
        constexpr int RED = WAVES * RPI * TILE > NT * 4 ? WAVES * RPI * TILE : NT * 4;
        L.fin = L.red + RED;  // behind both uses of the reduction buffer
    }
    const int* s_idx = L.idx;
    const float* s_d = L.d;
    float* s_red = L.red;  // [WAVES*RPI][TILE]

    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;

    // constants of the column group this thread will finish (needed only at the very end: loaded now)
    const ColConst mine = load_col_const<WDT, TILE>(a, tile, tid % GROUPS);

    // ------------------------------------------------------------------ 1. centre, threshold, compact
    int cnt;
    if constexpr (FUSE == kFuseList)
        cnt = gather_lists<WAVES, BT>(a, split, L);
    else
        cnt = compact_inputs<WAVES, BT>(a, tile, split, L);

    // ------------------------------------------------------------------ 2. stream the kept rows
    float acc[BT][ELEMS];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int j = 0; j < ELEMS; ++j) acc[b][j] = 0.f;

    const int sub_row = lane / LPR;  // which of the RPI rows of a load this lane reads
    const int col0 = tile * TILE + (lane % LPR) * ELEMS;
    const bool col_ok = col0 < a.N;
    const uint32_t lane_off = col_ok ? (uint32_t)col0 * Vec<WDT>::kBytes : 0u;
    const uint32_t row_bytes = (uint32_t)a.N * Vec<WDT>::kBytes;
    const char* wbase = reinterpret_cast<const char*>(a.W);

    if constexpr (LPR == kWave) {
        const int n_w = (cnt > w) ? (cnt - w + WAVES - 1) / WAVES : 0;  // entries w, w+WAVES, ...
        for (int i0 = 0; i0 < n_w; i0 += kWave) {
            const int e = w + WAVES * (i0 + lane);
            const bool in = e < cnt;
            const int vidx = in ? s_idx[e] : 0;
            float vd[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) vd[b] = in ? s_d[b * a.Kc + e] : 0.f;
            const int nb = min(kWave, n_w - i0);
            for (int u = 0; u < nb; u += UNROLL) {
                const int rem = nb - u;  // wave-uniform
                // Issue UNROLL row loads together.  In a ragged last group the spare slots re-read the
                // group's last row (same cache lines, no extra HBM traffic) and are not accumulated.
                uint4 r[UNROLL];
#pragma unroll
                for (int q = 0; q < UNROLL; ++q) {
                    const uint32_t row = (uint32_t)__builtin_amdgcn_readlane(vidx, min(u + q, nb - 1));
                    r[q] = load_row_vec(wbase, row, row_bytes, lane_off);
                }
                if (rem >= UNROLL) {
#pragma unroll
                    for (int q = 0; q < UNROLL; ++q) {
#pragma unroll
                        for (int b = 0; b < BT; ++b) fma_vec<WDT>(acc[b], r[q], read_lane_f(vd[b], u + q));
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < UNROLL - 1; ++q) {
                        if (q < rem) {
#pragma unroll
                            for (int b = 0; b < BT; ++b) fma_vec<WDT>(acc[b], r[q], read_lane_f(vd[b], u + q));
                        }
                    }
                }
            }
        }
    } else {
        // The list is consumed in blocks of RPI consecutive entries, blocks round-robin over the
        // wavefronts; lane group `sub_row` of a wavefront takes entry sub_row of the block.  Lanes past
        // the end of the list are masked off for the load and the accumulation alike.
        const int n_blocks = (cnt + RPI - 1) / RPI;
        const int n_w = (n_blocks > w) ? (n_blocks - w + WAVES - 1) / WAVES : 0;
        // Whole groups of UNROLL complete blocks first, without a predicate anywhere (a conditional load keeps
        // the compiler from issuing a group's loads together); the ragged rest goes through the masked form.
        const int n_complete = cnt / RPI;  // blocks whose RPI entries all exist
        const int n_cw = (n_complete > w) ? (n_complete - w + WAVES - 1) / WAVES : 0;
        const int n_main = n_cw - n_cw % UNROLL;
        for (int i0 = 0; i0 < n_main; i0 += UNROLL) {
            uint4 r[UNROLL];
            float dv[UNROLL][BT];
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                const int e = (w + WAVES * (i0 + q)) * RPI + sub_row;
                const uint32_t row = (uint32_t)s_idx[e];
                r[q] = load_weights16(wbase + (uint64_t)row * row_bytes + lane_off);
#pragma unroll
                for (int b = 0; b < BT; ++b) dv[q][b] = s_d[b * a.Kc + e];
            }
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
#pragma unroll
                for (int b = 0; b < BT; ++b) fma_vec<WDT>(acc[b], r[q], dv[q][b]);
            }
        }
        for (int i0 = n_main; i0 < n_w; i0 += UNROLL) {
            uint4 r[UNROLL];
            float dv[UNROLL][BT];
            bool ok[UNROLL];
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                const int e = (w + WAVES * (i0 + q)) * RPI + sub_row;
                ok[q] = (i0 + q < n_w) && (e < cnt);
                r[q] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                for (int b = 0; b < BT; ++b) dv[q][b] = 0.f;
                if (ok[q]) {
                    const uint32_t row = (uint32_t)s_idx[e];
                    r[q] = load_weights16(wbase + (uint64_t)row * row_bytes + lane_off);
#pragma unroll
                    for (int b = 0; b < BT; ++b) dv[q][b] = s_d[b * a.Kc + e];
                }
            }
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                if (ok[q]) {
#pragma unroll
                    for (int b = 0; b < BT; ++b) fma_vec<WDT>(acc[b], r[q], dv[q][b]);
                }
            }
        }
    }

    // ------------------------------------------------------------------ 3. add the wavefronts' sums
    const __amdgpu_buffer_rsrc_t pbuf = partial_buffer<TILE>(a);
    __syncthreads();  // the list is no longer needed; its LDS becomes the reduction buffer
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        if (b < a.B) {
            // lane group sub_row of wavefront w holds the sums of row slot (w*RPI + sub_row)
            float4* dst = reinterpret_cast<float4*>(s_red + (w * RPI + sub_row) * TILE + (lane % LPR) * ELEMS);
#pragma unroll
            for (int j = 0; j < ELEMS / 4; ++j)
                dst[j] = make_float4(acc[b][4 * j], acc[b][4 * j + 1], acc[b][4 * j + 2], acc[b][4 * j + 3]);
            __syncthreads();
            for (int g = tid; g < GROUPS; g += NT) {
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int i = 0; i < WAVES * RPI; ++i) {
                    const float4 v = *reinterpret_cast<const float4*>(s_red + i * TILE + 4 * g);
                    s.x += v.x;
                    s.y += v.y;
                    s.z += v.z;
                    s.w += v.w;
                }
                emit_group<WDT, TILE, FUSE>(a, pbuf, tile, split, b, g, s, L.fin, mine);  // g == tid here
            }
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ 4. last arrival finishes the tile
    finish_tile<WDT, WAVES, TILE, BT, FUSE>(a, pbuf, tile, L, mine);
}

}  // namespace scap
