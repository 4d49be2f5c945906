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
#include "scap_device.hpp"
#include "scap_internal.hpp"

namespace scap {

constexpr int kHdrBytes = 2048;  // LDS header: per-wave counts + flags

// Data handed from one workgroup to another inside a launch (split-K partials, per-split index lists,
// arrival counters) bypasses the non-coherent cache levels: device-scope relaxed atomics for single
// words, buffer loads/stores with the device-coherent cache policy for the 16-byte partial sums.
// Such stores write through to the device's coherence point and such loads read from it, so no
// workgroup has to write back or invalidate its whole L2 -- on an 8-XCD part one device-scope fence
// per workgroup costs several times the GEMV itself.  A compute unit pulls coherent data at only a few
// tens of GB/s, so these accesses are kept few and wide.
// Ordering: every thread waits until its own stores are acknowledged (s_waitcnt vmcnt(0)), the workgroup
// barriers, then one thread takes the arrival ticket; the last arrival barriers again before anyone
// reads.

constexpr int kAuxDeviceCoherent = 1 << 4;  // "sc1" bit of the buffer cache policy

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_raw_buffer(void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ void store_coherent16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, float4 v) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t t = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    __builtin_amdgcn_raw_buffer_store_b128(t, r, (int)byte_off, 0, kAuxDeviceCoherent);
}
__device__ __forceinline__ float4 load_coherent16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
    const auto t = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kAuxDeviceCoherent);
    return make_float4(__uint_as_float(t[0]), __uint_as_float(t[1]), __uint_as_float(t[2]), __uint_as_float(t[3]));
}
// all of this thread's earlier memory operations have completed
__device__ __forceinline__ void wait_memory_ops() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <typename T>
__device__ __forceinline__ void store_dev(T* p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T load_dev(const T* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16 bytes of weight row `row` at this lane's columns.  `row` is wave-uniform, so the row base is
// formed on the scalar unit and the load takes a scalar base plus a 32-bit lane offset.
__device__ __forceinline__ uint4 load_row_vec(const char* __restrict__ wbase, uint32_t row, uint32_t row_bytes,
                                              uint32_t lane_off) {
    const uint64_t base = reinterpret_cast<uint64_t>(wbase) + (uint64_t)row * (uint64_t)row_bytes;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base >> 32));
    typedef __attribute__((address_space(1))) const char gchar_t;
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(1))) const u32x4_t gvec_t;
    gchar_t* p = (gchar_t*)(((uint64_t)hi << 32) | lo);
    const u32x4_t v = *(gvec_t*)(p + lane_off);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// LPR = lanes that share one weight row: 64 (a wavefront reads 1 KB of one row per load) or 32 (it reads
// 512 bytes of each of 2 rows).  Fewer lanes per row make the column tile narrower, so the same
// number of workgroups needs fewer K splits and the final reduction reads less.
template <int WDT, int WAVES, int UNROLL, int BT, int LPR>
__global__ __launch_bounds__(WAVES * kWave) void gemv_kernel(const GemvArgs a) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr int TILE = LPR * ELEMS;
    constexpr int RPI = kWave / LPR;  // rows per load instruction
    constexpr int NT = WAVES * kWave;

    extern __shared__ uint4 smem_raw[];
    char* smem = reinterpret_cast<char*>(smem_raw);
    int* s_hdr = reinterpret_cast<int*>(smem);              // [(1+BT)][WAVES] wave counts, then flags
    int* s_flag = s_hdr + (1 + BT) * WAVES;                 // [0] last-arrival flag
    int* s_idx = reinterpret_cast<int*>(smem + kHdrBytes);  // [Kc]
    float* s_d = reinterpret_cast<float*>(s_idx + a.Kc);    // [BT][Kc]
    float* s_red = reinterpret_cast<float*>(smem + kHdrBytes);  // [WAVES*RPI][TILE], reuses the list space

    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;
    const int k0 = split * a.Kc;
    const int kend = min(k0 + a.Kc, a.K);
    const bool per_token = BT > 1 && tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr);
    const bool want_idx = tile == 0 && a.idx_out != nullptr;

    // ------------------------------------------------------------------ 1. centre, threshold, compact
    const int nchunk = (kend - k0 + kWave - 1) / kWave;
    const int cpw = (nchunk + WAVES - 1) / WAVES;
    const int c_begin = min(w * cpw, nchunk);
    const int c_end = min(c_begin + cpw, nchunk);

    auto eval = [&](int b, int k, bool valid, float& d) -> bool {
        d = 0.f;
        if (b >= a.B || !valid) return false;
        if (a.mode == kModeFold) {
            d = a.m;
            return true;
        }
        const float xf = act_to_f32(a.x, (int64_t)b * a.K + k, a.xdt);
        if (a.mode == kModeDense) {
            d = xf;
            return true;
        }
        d = xf - a.m;               // one fp32 subtraction
        return fabsf(d) > a.tau;    // strict; NaN compares false
    };

    {
        int ucount = 0;
        int tcount[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) tcount[b] = 0;
        for (int c = c_begin; c < c_end; ++c) {
            const int k = k0 + c * kWave + lane;
            const bool valid = k < kend;
            bool any = false;
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float d;
                const bool keep = eval(b, k, valid, d);
                any |= keep;
                if (per_token) tcount[b] += __popcll(__ballot(keep));
            }
            ucount += __popcll(__ballot(any));
        }
        if (lane == 0) {
            s_hdr[w] = ucount;
            if (per_token) {
#pragma unroll
                for (int b = 0; b < BT; ++b) s_hdr[(1 + b) * WAVES + w] = tcount[b];
            }
        }
    }
    __syncthreads();
    int ubase = 0, cnt = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        const int v = s_hdr[i];
        if (i < w) ubase += v;
        cnt += v;
    }
    cnt = uniform(cnt);
    ubase = uniform(ubase);
    {
        int tbase[BT];
        int ttotal[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            tbase[b] = 0;
            ttotal[b] = 0;
            if (per_token) {
                for (int i = 0; i < WAVES; ++i) {
                    const int v = s_hdr[(1 + b) * WAVES + i];
                    if (i < w) tbase[b] += v;
                    ttotal[b] += v;
                }
            }
        }
        for (int c = c_begin; c < c_end; ++c) {
            const int k = k0 + c * kWave + lane;
            const bool valid = k < kend;
            bool any = false;
            float d[BT];
            bool keep[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                keep[b] = eval(b, k, valid, d[b]);
                any |= keep[b];
            }
            const uint64_t ub = __ballot(any);
            if (any) {
                const int pos = ubase + lanes_below(ub);
                s_idx[pos] = k;
#pragma unroll
                for (int b = 0; b < BT; ++b) s_d[b * a.Kc + pos] = keep[b] ? d[b] : 0.f;
                if (BT == 1 && want_idx) store_dev(&a.idx_out[k0 + pos], k);
            }
            ubase += __popcll(ub);
            if (BT > 1 && per_token) {
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const uint64_t tb = __ballot(keep[b]);
                    if (want_idx && keep[b]) store_dev(&a.idx_out[(int64_t)b * a.K + k0 + tbase[b] + lanes_below(tb)], k);
                    tbase[b] += __popcll(tb);
                }
            }
        }
        if (tile == 0 && tid == 0) {
            store_dev(&a.seg_cnt[a.B * a.S + split], cnt);  // union
            if (BT == 1) {
                store_dev(&a.seg_cnt[split], cnt);
            } else if (per_token) {
#pragma unroll
                for (int b = 0; b < BT; ++b)
                    if (b < a.B) store_dev(&a.seg_cnt[b * a.S + split], ttotal[b]);
            }
        }
    }
    __syncthreads();

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
        for (int i0 = 0; i0 < n_w; i0 += UNROLL) {
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
                    r[q] = *reinterpret_cast<const uint4*>(wbase + (uint64_t)row * row_bytes + lane_off);
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
    constexpr int GROUPS = TILE / 4;  // 4-column groups of a tile
    auto finish_columns = [&](int b, int g, float4 s) {  // scale, add the fused bias, store y
        const int col = tile * TILE + 4 * g;
        if (col >= a.N) return;  // N is a multiple of 8: a group is inside or outside as a whole
        if (WDT == kI8) {
            s.x *= f16_bits_to_f32(a.col_scale[col]);
            s.y *= f16_bits_to_f32(a.col_scale[col + 1]);
            s.z *= f16_bits_to_f32(a.col_scale[col + 2]);
            s.w *= f16_bits_to_f32(a.col_scale[col + 3]);
        }
        if (a.bias) {
            const float4 bv = *reinterpret_cast<const float4*>(a.bias + col);
            s.x += bv.x;
            s.y += bv.y;
            s.z += bv.z;
            s.w += bv.w;
        }
        *reinterpret_cast<float4*>(a.y + (int64_t)b * a.N + col) = s;
    };

    // split-K partials of this call: [B][S][T][TILE] floats, addressed by byte offset
    const __amdgpu_buffer_rsrc_t pbuf = make_raw_buffer(a.partial, (uint32_t)a.B * a.S * a.T * TILE * 4u);
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
                if (a.S == 1)
                    finish_columns(b, g, s);
                else
                    store_coherent16(pbuf, (uint32_t)((((b * a.S + split) * a.T + tile) * TILE + 4 * g) * 4), s);
            }
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ 4. last arrival finishes the tile
    const bool wants_lists = tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr || a.union_nnz_out != nullptr);
    if (a.S > 1) {
        wait_memory_ops();  // my coherent stores have been acknowledged
        __syncthreads();
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(&a.counters[tile * kCounterStride], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_flag[0] = (old == a.S - 1);
        }
        __syncthreads();
        if (s_flag[0] == 0) return;
        // The S partials of a 4-column group are shared out over Q threads (splits q, q+Q, ...), each adds
        // its share in ascending split order, then the Q shares are added in ascending q: a fixed
        // association, so y does not depend on which workgroup arrived last or when.
        constexpr int Q = (NT / GROUPS) > 0 ? (NT / GROUPS) : 1;
        constexpr int PASSES = (GROUPS + NT - 1) / NT;  // > 1 only when a workgroup has fewer threads than groups
        const uint32_t pstride = (uint32_t)a.T * TILE * 4u;  // bytes between consecutive splits
        for (int b = 0; b < a.B; ++b) {
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                const int g = (tid % GROUPS) + pass * NT;
                const int q = (PASSES > 1) ? 0 : tid / GROUPS;
                if (g < GROUPS && q < Q) {
                    const uint32_t pc = (uint32_t)(((b * a.S * a.T + tile) * TILE + 4 * g) * 4);
                    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                    for (int sp0 = q; sp0 < a.S; sp0 += 8 * Q) {  // 8 loads in flight
                        float4 v[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int sp = sp0 + j * Q;
                            v[j] = sp < a.S ? load_coherent16(pbuf, pc + sp * pstride) : make_float4(0.f, 0.f, 0.f, 0.f);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            s.x += v[j].x;
                            s.y += v[j].y;
                            s.z += v[j].z;
                            s.w += v[j].w;
                        }
                    }
                    *reinterpret_cast<float4*>(s_red + q * TILE + 4 * g) = s;
                }
            }
            __syncthreads();
            for (int g = tid; g < GROUPS; g += NT) {
                float4 s = *reinterpret_cast<const float4*>(s_red + 4 * g);
#pragma unroll
                for (int q = 1; q < Q; ++q) {
                    const float4 v = *reinterpret_cast<const float4*>(s_red + q * TILE + 4 * g);
                    s.x += v.x;
                    s.y += v.y;
                    s.z += v.z;
                    s.w += v.w;
                }
                finish_columns(b, g, s);
            }
            __syncthreads();
        }
        if (tid == 0) store_dev(&a.counters[tile * kCounterStride], 0);  // ready for the next call
    }

    // ------------------------------------------------------------------ index lists (tile 0 only)
    if (!wants_lists) return;
    // Each split left its ascending list in place at idx_out[b*K + split*Kc ...]; close the gaps.
    // Every entry moves left or stays, so reading a block of source positions, synchronising, then
    // writing it, block after block from the left, never overwrites an entry that is still to be read.
    __syncthreads();
    int* s_off = s_idx;               // [S] exclusive offsets
    int* s_cnt = s_idx + kMaxSplits;  // [S] counts
    const int nlist = a.B + 1;
    for (int l = 0; l < nlist; ++l) {
        const bool is_union = l == a.B;
        if (is_union && a.union_nnz_out == nullptr) continue;
        if (!is_union && a.nnz_out == nullptr) continue;
        const int src_l = (BT == 1) ? 0 : l;  // with one token the union list is the token's list
        __syncthreads();
        if (w == 0) {
            int run = 0;
            for (int s0 = 0; s0 < a.S; s0 += kWave) {
                const int sp = s0 + lane;
                const int v = sp < a.S ? load_dev(&a.seg_cnt[(is_union ? a.B : src_l) * a.S + sp]) : 0;
                const int inc = wave_inclusive_scan(v);
                if (sp < a.S) {
                    s_off[sp] = run + inc - v;
                    s_cnt[sp] = v;
                }
                run += __shfl(inc, kWave - 1, kWave);
            }
            if (lane == 0) {
                if (is_union)
                    a.union_nnz_out[0] = run;
                else
                    a.nnz_out[l] = run;
            }
        }
        __syncthreads();
        if (!is_union && a.idx_out != nullptr && a.S > 1) {
            int32_t* base = a.idx_out + (int64_t)l * a.K;
            constexpr int PER = 16;
            for (int c0 = 0; c0 < a.K; c0 += NT * PER) {
                int vals[PER], dsts[PER];
#pragma unroll
                for (int j = 0; j < PER; ++j) {
                    const int p = c0 + j * NT + tid;
                    dsts[j] = -1;
                    vals[j] = 0;
                    if (p < a.K) {
                        const int seg = p / a.Kc;
                        const int r = p - seg * a.Kc;
                        if (r < s_cnt[seg]) {
                            vals[j] = load_dev(&base[p]);
                            dsts[j] = s_off[seg] + r;
                        }
                    }
                }
                __syncthreads();
#pragma unroll
                for (int j = 0; j < PER; ++j)
                    if (dsts[j] >= 0) base[dsts[j]] = vals[j];
                __syncthreads();
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- launch
template <int WDT, int WAVES, int UNROLL, int BT, int LPR>
static int launch_one(const GemvArgs& a, hipStream_t stream) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    const size_t list_bytes = (size_t)a.Kc * 4 * (1 + BT);
    const size_t red_bytes = (size_t)WAVES * kWave * ELEMS * 4;
    const size_t off_bytes = (size_t)kMaxSplits * 8;
    size_t body = list_bytes > red_bytes ? list_bytes : red_bytes;
    if (body < off_bytes) body = off_bytes;
    const size_t lds = kHdrBytes + body;
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
        return SCAP_ERR_CONFIG;
    } else {
        if (waves == 8 && unroll == 4 && lpr == 64) return launch_one<WDT, 8, 4, BT, 64>(a, stream);
        return SCAP_ERR_CONFIG;
    }
}

template <int WDT>
static int launch_wdt(const GemvArgs& a, int bt, int waves, int unroll, int lpr, hipStream_t stream) {
    switch (bt) {
        case 1: return launch_bt<WDT, 1>(a, waves, unroll, lpr, stream);
        case 2: return launch_bt<WDT, 2>(a, waves, unroll, lpr, stream);
        case 4: return launch_bt<WDT, 4>(a, waves, unroll, lpr, stream);
        case 8: return launch_bt<WDT, 8>(a, waves, unroll, lpr, stream);
        case 16: return launch_bt<WDT, 16>(a, waves, unroll, lpr, stream);
    }
    return SCAP_ERR_SHAPE;
}

int launch_gemv(const GemvArgs& a_in, int wdt, const scap_launch_cfg* cfg, hipStream_t stream) {
    GemvArgs a = a_in;
    int bt = 1;
    while (bt < a.B) bt <<= 1;
    if (bt > SCAP_MAX_TOKENS) return SCAP_ERR_SHAPE;

    int waves = 8, unroll = (bt <= 4) ? 8 : 4, kc = 0, lpr = 64;
    if (cfg) {
        if (cfg->waves_per_group) waves = cfg->waves_per_group;
        if (cfg->unroll) unroll = cfg->unroll;
        if (cfg->rows_per_group) kc = cfg->rows_per_group;
        if (cfg->lanes_per_row) lpr = cfg->lanes_per_row;
        if (kc < 0 || (kc % kWave) != 0) return SCAP_ERR_CONFIG;
        if (lpr != 64 && lpr != 32) return SCAP_ERR_CONFIG;
    }
    const int elems = (wdt == kI8) ? 16 : 8;
    const int tile = lpr * elems;
    a.T = (int)((a.N + tile - 1) / tile);
    if (a.T > kMaxTiles) return (cfg && cfg->lanes_per_row) ? SCAP_ERR_CONFIG : SCAP_ERR_SHAPE;

    if (kc == 0) {
        // about one workgroup per compute unit (256): more splits only lengthen the final reduction,
        // fewer leave compute units -- each limited to ~100 GB/s of misses -- without work
        const int want_groups = 256;
        int s = (want_groups + a.T - 1) / a.T;
        if (s < 1) s = 1;
        kc = (int)align_up((size_t)((a.K + s - 1) / s), kWave);
        if (kc < 128) kc = 128;
    }
    // bounds from the workspace: at most kMaxSplits splits and partial_capacity floats per token
    const size_t tile_cols = (size_t)a.T * tile;
    size_t s_cap = partial_capacity(a.N) / tile_cols;
    if (s_cap > (size_t)kMaxSplits) s_cap = kMaxSplits;
    if (s_cap < 1) s_cap = 1;
    int s = (a.K + kc - 1) / kc;
    if ((size_t)s > s_cap) {
        kc = (int)align_up((size_t)((a.K + s_cap - 1) / s_cap), kWave);
        s = (a.K + kc - 1) / kc;
    }
    // LDS budget: the list of one workgroup must fit
    const int kc_lds = (int)((64 * 1024 - kHdrBytes) / (4 * (1 + bt)) / kWave * kWave);
    if (kc > kc_lds) {
        if (cfg && cfg->rows_per_group) return SCAP_ERR_CONFIG;
        kc = kc_lds;
        s = (a.K + kc - 1) / kc;
        if ((size_t)s > s_cap) return SCAP_ERR_SHAPE;
    }
    a.Kc = kc;
    a.S = s;

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

// Streaming read of `nvec` 16-byte vectors; a per-workgroup checksum keeps the loads alive.
constexpr int kProbeGroups = 2048;
__global__ __launch_bounds__(512) void read_probe_kernel(const uint4* __restrict__ src, size_t nvec, uint32_t* out) {
    __shared__ uint32_t sh[8];
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        const uint4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        acc += v0.x ^ v0.y ^ v0.z ^ v0.w;
        acc += v1.x ^ v1.y ^ v1.z ^ v1.w;
        acc += v2.x ^ v2.y ^ v2.z ^ v2.w;
        acc += v3.x ^ v3.y ^ v3.z ^ v3.w;
    }
    for (; i < nvec; i += stride) {
        const uint4 v = src[i];
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
