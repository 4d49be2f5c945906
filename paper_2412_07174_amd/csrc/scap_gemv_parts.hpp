// Pieces shared by the GEMV (vector ALU) and batched (MFMA) kernels of libscap: LDS carving, the
// centre/threshold/compact prologue (SCAP Alg. 3 steps 1-2, Eq. 2), and the split-K epilogue.
#pragma once

#include "scap_device.hpp"
#include "scap_internal.hpp"

namespace scap {

constexpr int kHdrBytes = 2048;  // LDS header: per-wave counts + flags

// What surrounds the gathered GEMV of a launch:
constexpr int kFusePlain = 0;   // inputs from x, outputs to y
constexpr int kFuseSwiglu = 1;  // columns are gate|up interleaved in groups of 4; the tile's last arrival forms
                                // z = silu(gate) * up, centres and thresholds it and leaves compacted lists
constexpr int kFuseList = 2;    // inputs are those lists instead of x

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


// ---------------------------------------------------------------------------------------------- LDS
struct Lds {
    int* hdr;    // [(1+BT)][WAVES] per-wave kept counts (union first, then per token)
    int* flag;   // [0] last-arrival flag
    int* idx;    // [Kc] kept channel indices, ascending (LDS, or global for the batched path)
    float* d;    // centred values, token-major [BT][Kc] (0 where the token pruned the channel)
    float* red;  // reduction buffer; reuses the list space once the rows have been streamed
    float* fin;  // kFuseSwiglu: the tile's finished columns (after scale and bias), [BT][TILE]
};

template <int WAVES, int BT>
__device__ __forceinline__ Lds carve_lds(char* smem, int Kc) {
    Lds L;
    L.hdr = reinterpret_cast<int*>(smem);
    L.flag = L.hdr + (1 + BT) * WAVES;
    L.idx = reinterpret_cast<int*>(smem + kHdrBytes);
    L.d = reinterpret_cast<float*>(L.idx + Kc);
    L.red = reinterpret_cast<float*>(smem + kHdrBytes);
    L.fin = nullptr;
    return L;
}

// ---------------------------------------------------------------------------------------------- prologue
// Centre and threshold the workgroup's Kc inputs of every token, and compact the channels kept by any
// token into an ascending list in LDS (wave64 ballot + prefix counts; cross-wave offsets through LDS).
// Workgroups of column tile 0 also leave the per-token lists in idx_out and the counts in seg_cnt when
// the caller asked for them.  Returns the list length (wave-uniform); ends with a barrier.
template <int WAVES, int BT>
__device__ __forceinline__ int compact_inputs(const GemvArgs& a, int tile, int split, const Lds& L) {
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int k0 = split * a.Kc;
    const int kend = min(k0 + a.Kc, a.K);
    const bool per_token = BT > 1 && tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr);
    const bool want_idx = tile == 0 && a.idx_out != nullptr;

    const int nchunk = (kend - k0 + kWave - 1) / kWave;
    const int cpw = (nchunk + WAVES - 1) / WAVES;
    const int c_begin = min(w * cpw, nchunk);
    const int c_end = min(c_begin + cpw, nchunk);

    // Centred value and keep test of every token at channel k.  The loads of all tokens are issued
    // together (no control flow between them) so that one memory latency covers the whole batch.
    auto eval_all = [&](int k, bool valid, float (&d)[BT], bool (&keep)[BT]) {
        // branch-free loads: a lane past the end or a token slot past the batch re-reads the last valid
        // element (it is masked below); only the bias-folding mode, which has no input, skips them
        uint32_t xb[BT];
        const int kc_ = min(k, a.K - 1);
#pragma unroll
        for (int b = 0; b < BT; ++b) xb[b] = 0u;
        if (a.mode != kModeFold) {
#pragma unroll
            for (int b = 0; b < BT; ++b) xb[b] = (uint32_t)a.x[(int64_t)min(b, a.B - 1) * a.K + kc_];
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const float xf = a.xdt == kBF16 ? bf16_bits_to_f32(xb[b]) : f16_bits_to_f32(xb[b]);
            const bool live = valid && b < a.B;
            float dv = xf - a.m;  // one fp32 subtraction
            bool kp = fabsf(dv) > a.tau;  // strict; NaN compares false
            if (a.mode == kModeDense) {
                dv = xf;
                kp = true;
            } else if (a.mode == kModeFold) {
                dv = a.m;
                kp = true;
            }
            keep[b] = live && kp;
            d[b] = keep[b] ? dv : 0.f;
        }
    };

    // One token and few chunks per wavefront (the usual launch shapes): the centred values and keep
    // ballots of the counting pass stay in registers, so the inputs are loaded once.
    constexpr int kRegChunks = 4;
    if (BT == 1 && cpw <= kRegChunks) {
        float dreg[kRegChunks];
        uint64_t breg[kRegChunks];
        int ucount = 0;
#pragma unroll
        for (int j = 0; j < kRegChunks; ++j) {
            const int c = c_begin + j;
            dreg[j] = 0.f;
            breg[j] = 0;
            if (c < c_end) {
                const int k = k0 + c * kWave + lane;
                float d[BT];
                bool keep[BT];
                eval_all(k, k < kend, d, keep);
                dreg[j] = d[0];
                breg[j] = __ballot(keep[0]);
                ucount += __popcll(breg[j]);
            }
        }
        if (lane == 0) L.hdr[w] = ucount;
        __syncthreads();
        int ubase = 0, cnt = 0;
#pragma unroll
        for (int i = 0; i < WAVES; ++i) {
            const int v = L.hdr[i];
            if (i < w) ubase += v;
            cnt += v;
        }
        cnt = uniform(cnt);
        ubase = uniform(ubase);
#pragma unroll
        for (int j = 0; j < kRegChunks; ++j) {
            const int c = c_begin + j;
            if (c < c_end) {
                if ((breg[j] >> lane) & 1) {
                    const int k = k0 + c * kWave + lane;
                    const int pos = ubase + lanes_below(breg[j]);
                    L.idx[pos] = k;
                    L.d[pos] = dreg[j];
                    if (want_idx) store_dev(&a.idx_out[k0 + pos], k);
                }
                ubase += __popcll(breg[j]);
            }
        }
        if (tile == 0 && tid == 0) {
            store_dev(&a.seg_cnt[a.B * a.Sl + split], cnt);  // union
            store_dev(&a.seg_cnt[split], cnt);
        }
        __syncthreads();
        return cnt;
    }

    {
        int ucount = 0;
        int tcount[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) tcount[b] = 0;
        for (int c = c_begin; c < c_end; ++c) {
            const int k = k0 + c * kWave + lane;
            const bool valid = k < kend;
            bool any = false;
            float d[BT];
            bool keep[BT];
            eval_all(k, valid, d, keep);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                any |= keep[b];
                if (per_token) tcount[b] += __popcll(__ballot(keep[b]));
            }
            ucount += __popcll(__ballot(any));
        }
        if (lane == 0) {
            L.hdr[w] = ucount;
            if (per_token) {
#pragma unroll
                for (int b = 0; b < BT; ++b) L.hdr[(1 + b) * WAVES + w] = tcount[b];
            }
        }
    }
    __syncthreads();
    int ubase = 0, cnt = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        const int v = L.hdr[i];
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
                    const int v = L.hdr[(1 + b) * WAVES + i];
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
            eval_all(k, valid, d, keep);
#pragma unroll
            for (int b = 0; b < BT; ++b) any |= keep[b];
            const uint64_t ub = __ballot(any);
            if (any) {
                const int pos = ubase + lanes_below(ub);
                L.idx[pos] = k;
#pragma unroll
                for (int b = 0; b < BT; ++b) L.d[b * a.Kc + pos] = d[b];
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
            store_dev(&a.seg_cnt[a.B * a.Sl + split], cnt);  // union
            if (BT == 1) {
                store_dev(&a.seg_cnt[split], cnt);
            } else if (per_token) {
#pragma unroll
                for (int b = 0; b < BT; ++b)
                    if (b < a.B) store_dev(&a.seg_cnt[b * a.Sl + split], ttotal[b]);
            }
        }
    }
    __syncthreads();
    return cnt;
}

// The same prologue for the matrix-core kernel, whose workgroups own long channel ranges: a wavefront handles
// up to MAXC chunks of 64 channels and issues the loads of ALL its chunks and tokens before it looks at any of
// them (one memory round trip instead of one per chunk and pass; the chunk loop of compact_inputs has a
// loop-carried wait).  Centred values, per-token keep bits and the union ballots stay in registers between
// the counting and the placing pass.  Requires Kc <= WAVES * 64 * MAXC.
template <int WAVES, int BT, int MAXC>
__device__ __forceinline__ int compact_inputs_wide(const GemvArgs& a, int tile, int split, const Lds& L) {
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int k0 = split * a.Kc;
    const int kend = min(k0 + a.Kc, a.K);
    const bool per_token = tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr);
    const bool want_idx = tile == 0 && a.idx_out != nullptr;
    const int nchunk = (kend - k0 + kWave - 1) / kWave;
    const int cpw = (nchunk + WAVES - 1) / WAVES;
    const int c_begin = min(w * cpw, nchunk);
    const int c_end = min(c_begin + cpw, nchunk);

    // ---- all loads, branch-free: chunk slots past c_end and token slots past B re-read a valid element
    uint32_t xb[MAXC][BT];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int k = min(k0 + (c_begin + j) * kWave + lane, a.K - 1);
#pragma unroll
        for (int b = 0; b < BT; ++b) xb[j][b] = (uint32_t)a.x[(int64_t)min(b, a.B - 1) * a.K + k];
    }
    // ---- centre, threshold, count
    float d[MAXC][BT];
    uint32_t keepmask[MAXC];
    uint64_t ub[MAXC];
    int ucount = 0;
    int tcount[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) tcount[b] = 0;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int k = k0 + (c_begin + j) * kWave + lane;
        const bool valid = (c_begin + j) < c_end && k < kend;
        keepmask[j] = 0;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const float xf = a.xdt == kBF16 ? bf16_bits_to_f32(xb[j][b]) : f16_bits_to_f32(xb[j][b]);
            const float dv = (a.mode == kModeDense) ? xf : xf - a.m;  // one fp32 subtraction
            const bool keep = valid && b < a.B && (a.mode == kModeDense || fabsf(dv) > a.tau);  // strict; NaN is pruned
            keepmask[j] |= keep ? (1u << b) : 0u;
            d[j][b] = keep ? dv : 0.f;
        }
        ub[j] = __ballot(keepmask[j] != 0);
        ucount += __popcll(ub[j]);
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b) tcount[b] += __popcll(__ballot((keepmask[j] >> b) & 1u));
        }
    }
    if (lane == 0) {
        L.hdr[w] = ucount;
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b) L.hdr[(1 + b) * WAVES + w] = tcount[b];
        }
    }
    __syncthreads();
    int ubase = 0, cnt = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        const int v = L.hdr[i];
        if (i < w) ubase += v;
        cnt += v;
    }
    cnt = uniform(cnt);
    ubase = uniform(ubase);
    int tbase[BT], ttotal[BT];
#pragma unroll
    for (int b = 0; b < BT; ++b) {
        tbase[b] = 0;
        ttotal[b] = 0;
        if (per_token) {
            for (int i = 0; i < WAVES; ++i) {
                const int v = L.hdr[(1 + b) * WAVES + i];
                if (i < w) tbase[b] += v;
                ttotal[b] += v;
            }
        }
    }
    // ---- place
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int k = k0 + (c_begin + j) * kWave + lane;
        if (keepmask[j] != 0) {
            const int pos = ubase + lanes_below(ub[j]);
            L.idx[pos] = k;
#pragma unroll
            for (int b = 0; b < BT; ++b) L.d[b * a.Kc + pos] = d[j][b];
        }
        ubase += __popcll(ub[j]);
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const bool kb = (keepmask[j] >> b) & 1u;
                const uint64_t tb = __ballot(kb);
                if (want_idx && kb) store_dev(&a.idx_out[(int64_t)b * a.K + k0 + tbase[b] + lanes_below(tb)], k);
                tbase[b] += __popcll(tb);
            }
        }
    }
    if (tile == 0 && tid == 0) {
        store_dev(&a.seg_cnt[a.B * a.Sl + split], cnt);  // union
        if (per_token) {
#pragma unroll
            for (int b = 0; b < BT; ++b)
                if (b < a.B) store_dev(&a.seg_cnt[b * a.Sl + split], ttotal[b]);
        }
    }
    __syncthreads();
    return cnt;
}

// ---------------------------------------------------------------------------------------------- list input
// Lists of the gated product (fused SwiGLU block), one segment per 64 channels, BT = tokens rounded up to
// a power of two:
//   zl_idx[seg*64 + r]            r-th channel of the segment kept by at least one token, ascending
//   zl_d[(seg*64 + r)*BT + b]     token b's centred value there, 0 where token b pruned the channel
//   zl_cnt[seg]                   entries of the segment;  zl_cnt[(1+b)*nsegs + seg]  those kept by token b
//
// kFuseList prologue: the workgroup's Kc channels are Kc/64 segments.  The segment counts and every entry
// slot are loaded together (one memory latency); entry r of a segment goes to position (entries of the
// earlier segments) + r.  Requires Kc/64 <= 64.  Ends with a barrier.
template <int WAVES, int BT>
__device__ __forceinline__ int gather_lists(const GemvArgs& a, int split, const Lds& L) {
    constexpr int PER_WAVE = kWave / WAVES;  // segments a wavefront may have to move
    typedef float dvec_t __attribute__((ext_vector_type(BT)));
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int spw = a.Kc >> 6;
    const int seg0 = split * spw;
    const int nseg = min(spw, a.Sl - seg0);
    int cv = lane < nseg ? a.zl_cnt[seg0 + lane] : 0;
    cv = min(max(cv, 0), kWave);  // a segment never holds more; keeps LDS writes in range whatever the memory holds
    int vi[PER_WAVE];
    float vd[PER_WAVE][BT];
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int sl = w + j * WAVES;
        vi[j] = 0;
#pragma unroll
        for (int b = 0; b < BT; ++b) vd[j][b] = 0.f;
        if (sl < nseg) {
            const int64_t p = (int64_t)(seg0 + sl) * kWave + lane;
            vi[j] = a.zl_idx[p];
            if constexpr (BT == 1) {
                vd[j][0] = a.zl_d[p];
            } else {
                const dvec_t v = *reinterpret_cast<const dvec_t*>(a.zl_d + p * BT);
#pragma unroll
                for (int b = 0; b < BT; ++b) vd[j][b] = v[b];
            }
        }
    }
    const int inc = wave_inclusive_scan(cv);
    const int total = __shfl(inc, kWave - 1, kWave);
    const int excl = inc - cv;
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int sl = w + j * WAVES;
        if (sl < nseg) {
            const int c = __shfl(cv, sl, kWave);
            const int off = __shfl(excl, sl, kWave);
            if (lane < c) {
                L.idx[off + lane] = vi[j];
#pragma unroll
                for (int b = 0; b < BT; ++b) L.d[b * a.Kc + off + lane] = vd[j][b];
            }
        }
    }
    __syncthreads();
    return uniform(total);
}

// kFuseSwiglu: the finished columns of a tile (s_fin[b*TILE + column]) hold, per 8 columns, 4 gate then the 4
// matching up pre-activations.  Form z = silu(gate) * up (Alg. 2), centre and threshold it like any other
// layer input (Alg. 3 steps 1-2, strict compare of Eq. 2; each token its own mask) and leave each 64-channel
// segment's kept channels, compacted, for the down launch.  Called by every thread of the tile's last arrival.
template <int WAVES, int TILE, int BT>
__device__ __forceinline__ void gate_and_compact(const GemvArgs& a, int tile, float* s_fin) {
    constexpr int HALF = TILE / 2;  // gated outputs per tile; a multiple of 64
    constexpr int NT = WAVES * kWave;
    constexpr bool SPREAD = BT >= 4;  // several tokens: the activation is evaluated by all threads first
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int nsegs = (a.F + kWave - 1) / kWave;
    // centred, thresholded gated product of (token b, channel t of the tile); 0 where pruned or absent
    auto gated = [&](int b, int t) {
        const int c = tile * HALF + t;
        if (!(b < a.B && t < HALF && c < a.F)) return 0.f;
        const int p = b * TILE + (t >> 2) * 8 + (t & 3);
        const float g = s_fin[p], u = s_fin[p + 4];
        const float z = g / (1.f + expf(-g)) * u;
        if (a.z_out) a.z_out[(int64_t)b * a.F + c] = z;
        const float d = z - a.m2;
        return fabsf(d) > a.tau2 ? d : 0.f;
    };
    if constexpr (SPREAD) {
        // One thread per (token, channel) instead of one per channel with the tokens in sequence (the exponential
        // and the division are ~50 instructions each, and only HALF of the NT threads have a channel).  The
        // results replace the gate values in s_fin; kept means |d| > tau >= 0, so a kept value is never 0.
        constexpr int PER = (BT * HALF + NT - 1) / NT;
        float dreg[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int item = i * NT + tid;
            dreg[i] = item < BT * HALF ? gated(item / HALF, item % HALF) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int item = i * NT + tid;
            const int b = item / HALF, t = item % HALF;
            if (item < BT * HALF) s_fin[b * TILE + (t >> 2) * 8 + (t & 3)] = dreg[i];
        }
        __syncthreads();
    }
    for (int t0 = 0; t0 < HALF; t0 += NT) {
        const int t = t0 + tid;
        const int c = tile * HALF + t;
        float dv[BT];
        bool keep[BT];
        bool any = false;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            if constexpr (SPREAD)
                dv[b] = (b < a.B && t < HALF && c < a.F) ? s_fin[b * TILE + (t >> 2) * 8 + (t & 3)] : 0.f;
            else
                dv[b] = gated(b, t);
            keep[b] = dv[b] != 0.f;
            any |= keep[b];
        }
        const uint64_t bal = __ballot(any);
        const int seg = uniform((tile * HALF + t0 + (tid & ~63)) >> 6);
        const bool seg_ok = t0 + (tid & ~63) < HALF && seg < nsegs;  // wave-uniform
        if (seg_ok) {
            if (any) {
                const int64_t p = (int64_t)seg * kWave + lanes_below(bal);
                a.zl_idx[p] = c;
#pragma unroll
                for (int b = 0; b < BT; ++b) a.zl_d[p * BT + b] = dv[b];
            }
            if (lane == 0) a.zl_cnt[seg] = __popcll(bal);
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const uint64_t tb = __ballot(keep[b]);
            if (seg_ok && lane == 0 && b < a.B) a.zl_cnt[(1 + b) * nsegs + seg] = __popcll(tb);
        }
    }
}

// kFuseList, last arrival of tile 0: kept-channel count and gap-free ascending list of every token, from the
// segment lists (an entry belongs to token b where its centred value is non-zero: kept means |d| > tau >= 0).
// Other workgroups may still be reading the segment lists, so those stay as they are.
template <int WAVES, int BT>
__device__ __forceinline__ void close_block_lists(const GemvArgs& a, const Lds& L) {
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    int* s_off = L.idx;  // [Sl] exclusive offsets of the token's entries
    for (int b = 0; b < a.B; ++b) {
        __syncthreads();
        if (w == 0) {
            int run = 0;
            for (int s0 = 0; s0 < a.Sl; s0 += kWave) {
                const int sp = s0 + lane;
                const int v = sp < a.Sl ? a.zl_cnt[(1 + b) * a.Sl + sp] : 0;
                const int inc = wave_inclusive_scan(v);
                if (sp < a.Sl) s_off[sp] = run + inc - v;
                run += __shfl(inc, kWave - 1, kWave);
            }
            if (lane == 0 && a.nnz_out) a.nnz_out[b] = run;
        }
        __syncthreads();
        if (a.idx_out == nullptr) continue;
        for (int seg = w; seg < a.Sl; seg += WAVES) {
            const int n = min(max(a.zl_cnt[seg], 0), kWave);
            const int64_t p = (int64_t)seg * kWave + lane;
            const bool mine = lane < n && a.zl_d[p * BT + b] != 0.f;
            const uint64_t bal = __ballot(mine);
            if (mine) a.idx_out[(int64_t)b * a.K + s_off[seg] + lanes_below(bal)] = a.zl_idx[p];
        }
    }
}

// ---------------------------------------------------------------------------------------------- epilogue
// Per-column constants of a 4-column group: fused bias and (int8) column scales.  A thread that will finish
// group g loads them when the kernel starts, so that the tile's last arrival does not add another memory
// round trip after it has read the partial sums.
struct ColConst {
    float4 bias, scale;
};
template <int WDT, int TILE>
__device__ __forceinline__ ColConst load_col_const(const GemvArgs& a, int tile, int g) {
    ColConst c;
    c.bias = make_float4(0.f, 0.f, 0.f, 0.f);
    c.scale = make_float4(1.f, 1.f, 1.f, 1.f);
    const int col = tile * TILE + 4 * g;
    if (col < a.N) {  // N is a multiple of 8: a group is inside or outside as a whole
        if (a.bias) c.bias = *reinterpret_cast<const float4*>(a.bias + col);
        if (WDT == kI8) {
            const uint2 h = *reinterpret_cast<const uint2*>(a.col_scale + col);
            c.scale = make_float4(f16_bits_to_f32(h.x & 0xFFFFu), f16_bits_to_f32(h.x >> 16), f16_bits_to_f32(h.y & 0xFFFFu),
                                  f16_bits_to_f32(h.y >> 16));
        }
    }
    return c;
}

// scale (int8), add the fused bias, store 4 columns of y
template <int WDT, int TILE, int FUSE = kFusePlain>
__device__ __forceinline__ void finish_columns(const GemvArgs& a, int tile, int b, int g, float4 s, float* s_fin,
                                               const ColConst& c) {
    const int col = tile * TILE + 4 * g;
    if (col >= a.N) return;
    if (WDT == kI8) {
        s.x *= c.scale.x;
        s.y *= c.scale.y;
        s.z *= c.scale.z;
        s.w *= c.scale.w;
    }
    s.x += c.bias.x;
    s.y += c.bias.y;
    s.z += c.bias.z;
    s.w += c.bias.w;
    if constexpr (FUSE == kFuseSwiglu)
        *reinterpret_cast<float4*>(s_fin + b * TILE + 4 * g) = s;
    else
        // written through to memory: lines left modified in L2 are paid for when the kernel ends
        store_coherent16(make_raw_buffer(a.y, (uint32_t)((size_t)a.B * a.N * 4)), (uint32_t)(((int64_t)b * a.N + col) * 4), s);
}

// split-K partials of one call: [B][S][T][TILE] floats, addressed by byte offset
template <int TILE>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t partial_buffer(const GemvArgs& a) {
    return make_raw_buffer(a.partial, (uint32_t)a.B * a.S * a.T * TILE * 4u);
}

// the workgroup's sum of 4 columns for token b: final output if there is one split, else a partial
// (`c` = constants of group g, loaded beforehand or here)
template <int WDT, int TILE, int FUSE = kFusePlain>
__device__ __forceinline__ void emit_group(const GemvArgs& a, __amdgpu_buffer_rsrc_t pbuf, int tile, int split, int b,
                                           int g, float4 s, float* s_fin, const ColConst& c) {
    if (a.S == 1)
        finish_columns<WDT, TILE, FUSE>(a, tile, b, g, s, s_fin, c);
    else
        store_coherent16(pbuf, (uint32_t)((((b * a.S + split) * a.T + tile) * TILE + 4 * g) * 4), s);
}

// Arrival ticket; the last arrival of a tile adds the S partials (fixed association), writes y and clears
// the counter; the last arrival of tile 0 also closes the gaps between the per-split index lists.
// Every thread of the workgroup must call this after its last emit_group().
// `mine` = constants of group (tid % GROUPS), the group this thread finishes in every pass.
template <int WDT, int WAVES, int TILE, int BT, int FUSE = kFusePlain>
__device__ __forceinline__ void finish_tile(const GemvArgs& a, __amdgpu_buffer_rsrc_t pbuf, int tile, const Lds& L,
                                            const ColConst& mine) {
    constexpr int NT = WAVES * kWave;
    constexpr int GROUPS = TILE / 4;
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    float* s_red = L.red;
    const bool wants_lists = tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr || a.union_nnz_out != nullptr);
    if (a.S > 1) {
        wait_memory_ops();  // my coherent stores have been acknowledged
        __syncthreads();
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(&a.counters[tile * kCounterStride], 1, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
            L.flag[0] = (old == a.S - 1);
        }
        __syncthreads();
        if (L.flag[0] == 0) return;
        // Work items are (token, 4-column group) pairs.  The S partials of an item are shared out over
        // Q threads (splits q, q+Q, ...), each adds its share in ascending split order, then the Q shares
        // are added in ascending q: a fixed association, so y does not depend on which workgroup arrived
        // last or when.  All items of a pass have their loads in flight together.
        const int nitems = a.B * GROUPS;
        const int per_pass = nitems < NT ? nitems : NT;
        const int Q = NT / per_pass;
        const uint32_t pstride = (uint32_t)a.T * TILE * 4u;  // bytes between consecutive splits
        const int li = tid % per_pass, q = tid / per_pass;
        for (int i0 = 0; i0 < nitems; i0 += per_pass) {
            const int item = i0 + li;
            const int b = item / GROUPS, g = item - b * GROUPS;
            if (q < Q && item < nitems) {
                const uint32_t pc = (uint32_t)(((b * a.S * a.T + tile) * TILE + 4 * g) * 4);
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                // int8 weights with 16 token slots: 256-column tiles, so 16 splits and 16 partials per thread.
                // There 16 loads are in flight, no branch between them (one round trip of these device-scope
                // loads costs about 1 us; 14336 x 4096 int8, 16 tokens: 24.8 -> 24.4 us).  Everywhere else the
                // larger epilogue costs more than it gains.
                if constexpr (WDT == kI8 && BT == 16) {
                    for (int sp0 = q; sp0 < a.S; sp0 += 16 * Q) {
                        float4 v[16];
#pragma unroll
                        for (int j = 0; j < 16; ++j) v[j] = load_coherent16(pbuf, pc + min(sp0 + j * Q, a.S - 1) * pstride);
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const bool in = sp0 + j * Q < a.S;  // a slot past the last split re-read it: not added
                            s.x += in ? v[j].x : 0.f;
                            s.y += in ? v[j].y : 0.f;
                            s.z += in ? v[j].z : 0.f;
                            s.w += in ? v[j].w : 0.f;
                        }
                    }
                } else
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
                *reinterpret_cast<float4*>(s_red + (q * per_pass + li) * 4) = s;
            }
            __syncthreads();
            if (q == 0 && item < nitems) {
                float4 s = *reinterpret_cast<const float4*>(s_red + li * 4);
                for (int qq = 1; qq < Q; ++qq) {
                    const float4 v = *reinterpret_cast<const float4*>(s_red + (qq * per_pass + li) * 4);
                    s.x += v.x;
                    s.y += v.y;
                    s.z += v.z;
                    s.w += v.w;
                }
                finish_columns<WDT, TILE, FUSE>(a, tile, b, g, s, L.fin, mine);  // g == tid % GROUPS
            }
            __syncthreads();
        }
        if (tid == 0) store_dev(&a.counters[tile * kCounterStride], 0);  // ready for the next call
    }
    if constexpr (FUSE == kFuseSwiglu) {
        __syncthreads();  // the tile's columns are complete in L.fin
        gate_and_compact<WAVES, TILE, BT>(a, tile, L.fin);
    }
    if constexpr (FUSE == kFuseList) {
        if (tile == 0 && (a.nnz_out != nullptr || a.idx_out != nullptr)) close_block_lists<WAVES, BT>(a, L);
        return;
    }

    if (!wants_lists) return;
    // Each split left its ascending list in place at idx_out[b*K + segment*Kl ...]; close the gaps.
    // Every entry moves left or stays, so reading a block of source positions, synchronising, then
    // writing it, block after block from the left, never overwrites an entry that is still to be read.
    __syncthreads();
    int* s_off = L.idx;          // [Sl] exclusive offsets
    int* s_cnt = L.idx + a.Sl;   // [Sl] counts
    const int nlist = a.B + 1;
    for (int l = 0; l < nlist; ++l) {
        const bool is_union = l == a.B;
        if (is_union && a.union_nnz_out == nullptr) continue;
        if (!is_union && a.nnz_out == nullptr) continue;
        const int src_l = (BT == 1) ? 0 : l;  // with one token the union list is the token's list
        __syncthreads();
        if (w == 0) {
            int run = 0;
            for (int s0 = 0; s0 < a.Sl; s0 += kWave) {
                const int sp = s0 + lane;
                const int v = sp < a.Sl ? load_dev(&a.seg_cnt[(is_union ? a.B : src_l) * a.Sl + sp]) : 0;
                const int inc = wave_inclusive_scan(v);
                if (sp < a.Sl) {
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
        if (!is_union && a.idx_out != nullptr && a.Sl > 1) {
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
                        const int seg = p / a.Kl;
                        const int r = p - seg * a.Kl;
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

// LDS bytes one workgroup needs: header + max(list, reduction buffers, offset tables)
inline size_t lds_bytes(int Kc, int floats_per_entry, size_t red_bytes) {
    const size_t list_bytes = (size_t)Kc * 4 * (1 + floats_per_entry);
    const size_t off_bytes = (size_t)kMaxSplits * 8;
    size_t body = list_bytes > red_bytes ? list_bytes : red_bytes;
    if (body < off_bytes) body = off_bytes;
    return kHdrBytes + body;
}

// Choose the K split of a launch: fills a.T, a.Kc, a.S.  `tile` = columns per workgroup, `kc` = requested
// rows per workgroup (0 = about one workgroup per compute unit).  Returns a scap_status.
// `lds_budget` = LDS bytes one workgroup may use for its list.
int plan_splits(GemvArgs& a, int tile, int floats_per_entry, int kc, bool kc_forced, size_t lds_budget = 64 * 1024,
                int granule = kWave);

}  // namespace scap
