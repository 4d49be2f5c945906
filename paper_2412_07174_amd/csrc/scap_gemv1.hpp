// One-token column-gathered GEMV (SCAP Alg. 3; Eq. 2, 3, 6) for gfx950: the decode-time hot path in one launch,
// built around what a launch costs when no weight is streaming.
//
// The K input channels are cut into S ranges of Kc channels and the N columns into T tiles of one 16-byte vector
// per lane (512 columns of 16-bit weights, 1024 of int8).  Workgroup (split, tile), WAVES = 8 (or 4) wavefronts:
//   1. EVERY wavefront tests all Kc inputs of the workgroup itself: one 16-byte load per lane covers 512
//      channels, eight subtract-compare-ballot steps give the keep masks (Alg. 3 steps 1-2, strict compare of
//      Eq. 2).  A kept channel's position in the workgroup's list follows from the ballots; wavefront w takes
//      the positions p with p % WAVES == w.  No count is exchanged, so there is no barrier before the first weight
//      load, and the kept rows are spread evenly over the wavefronts whatever the mask looks like.
//   2. a wavefront streams its rows with UNROLL 16-byte loads per lane in flight, re-issuing a load as soon as
//      its predecessor in the ring has been consumed (Eq. 3: only kept rows are ever addressed).
//   3. one barrier; wavefront w then adds the wavefronts' sums of ITS slice of the tile (1/WAVES of the
//      columns), stores the slice's split-K partial and takes the slice's arrival ticket.  The last arrival of a
//      (tile, slice) adds the S partials in split order -- a fixed order, so y is bit-reproducible -- applies
//      the int8 scale and the fused bias (Eq. 6) and writes y.  WAVES tickets per tile instead of one: the
//      final sums of a tile are collected by up to WAVES compute units in parallel, each pulling S x 256 bytes,
//      and no wavefront waits for another after the barrier.
//
// Hand-over of the partials between workgroups.  The stores are device-coherent write-through stores and the
// ticket is a device-scope atomic, so a reader anywhere on the device may fetch them with device-coherent
// loads once it holds the last ticket.  Those loads go to the device's coherence point, past the L2 of the
// reader's accelerator die (XCD).  When every contributor of a (tile, slice) ran on the reader's own XCD -- the
// usual placement, workgroups being dealt round-robin to the 8 XCDs and a tile's workgroups being 8 apart --
// their stores all went through the L2 the reader uses, which therefore holds the current data or nothing;
// the reader then invalidates its compute unit's vector L1 and uses ordinary loads.  Whether that holds is
// decided at run time from the hardware's XCC id: each arrival adds (1, id, id^2) to the ticket word, and the
// last arrival takes the short way only if count * sum(id^2) == sum(id)^2, i.e. all ids are equal.  Where the
// dispatcher puts a workgroup thus decides speed only, never correctness.
#pragma once

#include "scap_gemv_body.hpp"

namespace scap {

constexpr int kG1MaxWaves = 8;       // wavefronts per workgroup: 4 or 8
constexpr int kG1Chunk = 8 * kWave;  // channels a wavefront tests per 16-byte load per lane
constexpr int kG1MaxChunks = 4;      // Kc <= 2048
constexpr int kG1HdrBytes = 2048;    // offsets and counts of up to 256 splits (closing the caller's lists)
constexpr int kG1TicketWords = 32;   // int32 words between the tickets of a tile's slices (128 bytes)

constexpr int kG1FlagDeviceScope = 1;  // always fetch the partials with device-coherent loads
constexpr int kG1FlagAccumulate = 4;   // y += result: every workgroup adds its share to y with fp32 atomics
constexpr int kG1FlagPartials = 8;     // hand split-K partial sums over as fp32 values (not as fixed-point atomics)
constexpr int kG1FlagParkSlices = 16;  // gating epilogue: always take the way through memory (for tests)

// Fixed-point hand-over: one 64-bit word per output column, updated by ONE atomic add per arrival:
//   bits 63-57 arrivals so far, bits 56-50 how many of them escaped, bits 49-0 the sum of (partial * 2^frac + BIAS).
constexpr int kFxMaxSplits = 64;
constexpr int kFxRangeBits = 20;  // partial sums below 2^20 in magnitude travel as fixed point; others escape
__host__ __device__ inline int fx_limit_bits(int S) {  // bits of one arrival's magnitude: S biased values fit 50 bits
    int hs = 0;
    while ((1 << hs) < S) ++hs;
    return 49 - hs;
}

// int8 weights read 8 bytes per lane instead of 16 (internal to this kernel): the column tile is 512 columns
// instead of 1024, so a layer with few columns gets twice the tiles and half the K splits.  With 4096 columns
// that is 8 tiles of 32 splits instead of 4 of 64: half as many partial sums per finished slice.
constexpr int kI8Half = 3;
template <> struct Vec<kI8Half> { static constexpr int kElems = 8; static constexpr int kBytes = 1; };

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(1))) const u32x2_t global_u32x2_t;

// this lane's vector of weight row `row` (wave-uniform): scalar row base plus the lane's byte offset
template <int WDT>
__device__ __forceinline__ uint4 load_row(const char* __restrict__ wbase, uint32_t row, uint32_t row_bytes, uint32_t lane_off) {
    if constexpr (WDT == kI8Half) {
        const uint64_t base = reinterpret_cast<uint64_t>(wbase) + (uint64_t)row * (uint64_t)row_bytes;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base >> 32));
        typedef __attribute__((address_space(1))) const char gchar_t;
        gchar_t* p = (gchar_t*)(((uint64_t)hi << 32) | lo);
        const u32x2_t v = __builtin_nontemporal_load((global_u32x2_t*)(p + lane_off));
        return make_uint4(v.x, v.y, 0u, 0u);
    } else {
        return load_row_vec(wbase, row, row_bytes, lane_off);
    }
}

template <int WDT>
__device__ __forceinline__ void fma_row(float* __restrict__ acc, const uint4& r, float d) {
    if constexpr (WDT == kI8Half) {
        const uint32_t w[2] = {r.x, r.y};
#pragma unroll
        for (int q = 0; q < 2; ++q) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int v = ((int)(w[q] << (24 - 8 * j))) >> 24;
                acc[4 * q + j] = fmaf((float)v, d, acc[4 * q + j]);
            }
        }
    } else {
        fma_vec<WDT>(acc, r, d);
    }
}

struct Gemv1Args {
    const void* W;
    const uint16_t* x;
    const uint16_t* col_scale;
    const float* bias;
    float* y;
    float* partial;      // [S][T][TILE] fp32
    int32_t* counters;   // ticket of (tile, slice) at word tile*kCounterStride + slice*kG1TicketWords (64-bit)
    int32_t* idx_out;
    int32_t* nnz_out;
    int32_t* union_nnz_out;
    int32_t* seg_cnt;    // [S] kept channels per split (only when the caller wants lists)
    int K, N, Kc, S, T, mode, xdt, flags;
    float m, tau;
    // Fused SwiGLU block (Alg. 2), one token.  The gate|up launch (FUSE = kFuseSwiglu) leaves the gated product z,
    // centred and thresholded, as one compacted list per `segz` channels -- the channels a wavefront slice
    // finishes --; the down launch (kFuseList) takes those lists as its input.
    float m2, tau2;    // mode estimate and threshold of the gated product
    float* z_out;      // optional fp32 [F]: the gated product itself
    int32_t* zl_idx;   // [nseg][segz] kept channels of each segment, ascending
    float* zl_d;       // [nseg][segz] their centred values
    int32_t* zl_cnt;   // [nseg] entries per segment
    int F, segz;       // channels of the gated product; channels per list segment (32 or 64)
    unsigned long long* fx_acc;  // fixed-point hand-over words and escape masks, or NULL: partial sums
};

// id of the accelerator die (XCD) this wavefront runs on: hardware register XCC_ID (20), bits 3:0
__device__ __forceinline__ uint32_t xcc_id() { return __builtin_amdgcn_s_getreg(((4 - 1) << 11) | (0 << 6) | 20) & 0xFu; }

// what an arrival adds to the 64-bit ticket: count in bits 0-15, sum of ids in 16-31, sum of squares in 32-63
__device__ __forceinline__ unsigned long long ticket_increment(uint32_t id) {
    return 1ull | ((unsigned long long)id << 16) | ((unsigned long long)(id * id) << 32);
}
__device__ __forceinline__ bool ticket_all_one_xcd(unsigned long long t) {
    const unsigned long long n = t & 0xFFFFull, sum = (t >> 16) & 0xFFFFull, sq = t >> 32;
    return n * sq == sum * sum;  // zero variance of the ids
}

template <int CPL> struct SliceVec;
template <> struct SliceVec<1> {
    float v[1];
    __device__ __forceinline__ static SliceVec load_coherent(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        SliceVec s;
        s.v[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, kAuxDeviceCoherent));
        return s;
    }
    __device__ __forceinline__ static SliceVec load_plain(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        SliceVec s;
        s.v[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
        return s;
    }
    __device__ __forceinline__ void store_coherent(__amdgpu_buffer_rsrc_t r, uint32_t off) const {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[0]), r, (int)off, 0, kAuxDeviceCoherent);
    }
};
template <> struct SliceVec<2> {
    float v[2];
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    __device__ __forceinline__ static SliceVec load_coherent(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, kAuxDeviceCoherent);
        SliceVec s;
        s.v[0] = __uint_as_float(t[0]);
        s.v[1] = __uint_as_float(t[1]);
        return s;
    }
    __device__ __forceinline__ static SliceVec load_plain(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
        SliceVec s;
        s.v[0] = __uint_as_float(t[0]);
        s.v[1] = __uint_as_float(t[1]);
        return s;
    }
    __device__ __forceinline__ void store_coherent(__amdgpu_buffer_rsrc_t r, uint32_t off) const {
        const u32x2_t t = {__float_as_uint(v[0]), __float_as_uint(v[1])};
        __builtin_amdgcn_raw_buffer_store_b64(t, r, (int)off, 0, kAuxDeviceCoherent);
    }
};

template <> struct SliceVec<4> {
    float v[4];
    __device__ __forceinline__ static SliceVec from(const float4& t) {
        SliceVec s;
        s.v[0] = t.x;
        s.v[1] = t.y;
        s.v[2] = t.z;
        s.v[3] = t.w;
        return s;
    }
    __device__ __forceinline__ static SliceVec load_coherent(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        return from(load_coherent16(r, off));
    }
    __device__ __forceinline__ static SliceVec load_plain(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        const auto t = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
        return from(make_float4(__uint_as_float(t[0]), __uint_as_float(t[1]), __uint_as_float(t[2]), __uint_as_float(t[3])));
    }
    __device__ __forceinline__ void store_coherent(__amdgpu_buffer_rsrc_t r, uint32_t off) const {
        store_coherent16(r, off, make_float4(v[0], v[1], v[2], v[3]));
    }
};

// exclusive prefix sum across the 64 lanes of a wave
__device__ __forceinline__ int wave_exclusive_scan(int v) { return wave_inclusive_scan(v) - v; }

// Close the gaps of one token's list: every split's ascending list sits at idx[split*Kc ...] with its count in
// seg_cnt[split].  Returns the total (in every lane).  One wavefront; entries only move left, and a block of source
// positions is read completely before any of it is written, so nothing is overwritten before it has been read.
__device__ __forceinline__ int close_list_rows(const int32_t* seg_cnt, int32_t* idx, int S, int K, int Kc, int* s_off,
                                               int* s_cnt) {
    const int lane = lane_id();
    int run = 0;
    for (int s0 = 0; s0 < S; s0 += kWave) {
        const int sp = s0 + lane;
        const int v = sp < S ? load_dev(&seg_cnt[sp]) : 0;
        const int inc = wave_inclusive_scan(v);
        if (sp < S) {
            s_off[sp] = run + inc - v;
            s_cnt[sp] = v;
        }
        run += __shfl(inc, kWave - 1, kWave);
    }
    if (idx == nullptr || S == 1) return run;
    __builtin_amdgcn_wave_barrier();
    constexpr int PER = 16;
    for (int c0 = 0; c0 < K; c0 += kWave * PER) {
        int vals[PER], dsts[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int p = c0 + j * kWave + lane;
            dsts[j] = -1;
            vals[j] = 0;
            if (p < K) {
                const int seg = p / Kc;
                const int r = p - seg * Kc;
                if (r < s_cnt[seg]) {
                    vals[j] = load_dev(&idx[p]);
                    dsts[j] = s_off[seg] + r;
                }
            }
        }
        wait_memory_ops();
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (dsts[j] >= 0) store_dev(&idx[dsts[j]], vals[j]);
        wait_memory_ops();
    }
    return run;
}

// Last arrival of (tile 0, slice 0) of the one-token kernel: write the total and close the gaps.
__device__ __forceinline__ void close_lists_wave(const Gemv1Args& a, int* s_off, int* s_cnt) {
    const int run = close_list_rows(a.seg_cnt, a.idx_out, a.S, a.K, a.Kc, s_off, s_cnt);
    if (lane_id() == 0) {
        if (a.nnz_out) a.nnz_out[0] = run;
        if (a.union_nnz_out) a.union_nnz_out[0] = run;
    }
}

// The arguments are passed one by one, the ones the prologue needs first: the leading 16 dwords of a kernel's
// scalar arguments can be placed in registers by the dispatcher (kernel-argument preload), which takes the
// argument fetch -- one memory round trip -- off the path to the first input load.
template <int WDT, int WAVES, int UNROLL, int NCH, int FUSE>
__global__ __launch_bounds__(WAVES * kWave) void gemv1_kernel(const uint16_t* x, const void* W, int K, int N, int Kc, int S,
                                                           int T, int mode, int xdt, int flags, float m, float tau,
                                                           const float* bias, float* y, float* partial,
                                                           int32_t* counters, const uint16_t* col_scale, int32_t* idx_out,
                                                           int32_t* nnz_out, int32_t* union_nnz_out, int32_t* seg_cnt,
                                                           float m2, float tau2, float* z_out, int32_t* zl_idx, float* zl_d,
                                                           int32_t* zl_cnt, int F, int segz, unsigned long long* fx_acc) {
    Gemv1Args a;
    a.W = W; a.x = x; a.col_scale = col_scale; a.bias = bias; a.y = y; a.partial = partial; a.counters = counters;
    a.idx_out = idx_out; a.nnz_out = nnz_out; a.union_nnz_out = union_nnz_out; a.seg_cnt = seg_cnt;
    a.K = K; a.N = N; a.Kc = Kc; a.S = S; a.T = T; a.mode = mode; a.xdt = xdt; a.flags = flags; a.m = m; a.tau = tau;
    a.m2 = m2; a.tau2 = tau2; a.z_out = z_out; a.zl_idx = zl_idx; a.zl_d = zl_d; a.zl_cnt = zl_cnt; a.F = F; a.segz = segz;
    a.fx_acc = fx_acc;
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr bool IS_I8 = WDT == kI8 || WDT == kI8Half;
    constexpr int TILE = kWave * ELEMS;
    constexpr int CPL = ELEMS / WAVES;  // columns per lane of a wavefront's slice
    constexpr int SLICE = kWave * CPL;  // columns per slice: 1/WAVES of the tile
    static_assert(CPL == 1 || CPL == 2 || CPL == 4, "a slice is 4, 8 or 16 bytes per lane");
    typedef SliceVec<CPL> slice_t;

    extern __shared__ uint4 smem_raw[];
    char* smem = reinterpret_cast<char*>(smem_raw);
    int* s_off = reinterpret_cast<int*>(smem);
    int* s_cnt = s_off + kMaxSplits;
    float* s_red = reinterpret_cast<float*>(smem + kG1HdrBytes);                           // [8][TILE]
    int2* s_list = reinterpret_cast<int2*>(smem + kG1HdrBytes + WAVES * TILE * 4);  // [WAVES][slots]
    const int slots = a.Kc / WAVES + 1;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = uniform(tid >> 6);
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;
    const int k0 = split * a.Kc;
    const int kend = min(k0 + a.Kc, a.K);

    // ------------------------------------------------------------------ 1. inputs: every wavefront, all Kc
    uint4 xv[NCH];
    if constexpr (FUSE != kFuseList) {
    #pragma unroll
        for (int c = 0; c < NCH; ++c) {
            xv[c] = make_uint4(0u, 0u, 0u, 0u);
            const int kb = k0 + c * kG1Chunk + 8 * lane;
            if (a.mode != kModeFold && kb < kend) {
                if (kb + 8 <= a.K) {
                    xv[c] = *reinterpret_cast<const uint4*>(a.x + kb);
                } else {  // the last octet of an input whose length is not a multiple of 8: element by element
                    uint32_t h[8];
    #pragma unroll
                    for (int j = 0; j < 8; ++j) h[j] = kb + j < a.K ? (uint32_t)a.x[kb + j] : 0u;
                    xv[c] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
                }
            }
        }
    }
    // constants of the columns this lane finishes, needed only at the very end: loaded now, behind the inputs
    // Column c of this lane is fcol + c * CSTR: lanes side by side, so that every store and atomic of the hand-over
    // covers 64 consecutive words (with the lane's columns adjacent one instruction spread over twice or four times
    // the cache lines, and the atomics of a 2-column slice took 2 us instead of 0.7).
    constexpr int CSTR = kWave;
    constexpr int LSTR = 1;
    const int fcol = tile * TILE + w * SLICE + lane * LSTR;
    float cbias[CPL], cscale[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        cbias[c] = 0.f;
        cscale[c] = 1.f;
        if (fcol + c * CSTR < a.N) {
            if (a.bias) cbias[c] = a.bias[fcol + c * CSTR];
            if (IS_I8) cscale[c] = f16_bits_to_f32(a.col_scale[fcol + c * CSTR]);
        }
    }

    const bool want_lists = FUSE != kFuseSwiglu && tile == 0 && w == 0 && (a.nnz_out != nullptr || a.union_nnz_out != nullptr);
    int2* mylist = s_list + w * slots;
    int cnt = 0;    // kept channels so far, in (chunk, element, lane) order -- wave-uniform
    int lcnt = 0;   // the same in ascending channel order (caller's list)
    if constexpr (FUSE == kFuseList) {
        // The workgroup's channels are Kc / segz list segments of the gated product.  Lane l takes the count of
        // segment l (at most 64 segments), a prefix sum gives every entry its position; the entries are fetched 64
        // at a time (whole segments side by side).
        const int seg0 = k0 / a.segz;
        const int nsegw = (kend - k0 + a.segz - 1) / a.segz;
        const int per_it = kWave / a.segz;       // segments per fetch of 64 entries: 2 or 1
        const int sub = lane / a.segz, r = lane - sub * a.segz;
        constexpr int ITS = 8 * NCH;             // Kc / 64 fetches at most
        // every entry slot of the workgroup's segments, whatever the counts will say: one memory round trip for
        // counts and entries together (slots past a segment's count hold stale entries and are dropped below)
        int2 ent[ITS];
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int sg = it * per_it + sub;
            ent[it] = make_int2(0, 0);
            if (sg < nsegw) {
                const int64_t e = (int64_t)(seg0 + sg) * a.segz + r;
                ent[it] = make_int2(a.zl_idx[e], __float_as_int(a.zl_d[e]));
            }
        }
        int c_l = lane < nsegw ? a.zl_cnt[seg0 + lane] : 0;
        c_l = min(max(c_l, 0), a.segz);  // keeps LDS writes in range whatever the memory holds
        const int inc = wave_inclusive_scan(c_l);
        const int off_l = inc - c_l;
        cnt = __shfl(inc, kWave - 1, kWave);
        int pos[ITS];
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int sg = it * per_it + sub;
            const int c_s = __shfl(c_l, sg & 63, kWave), o_s = __shfl(off_l, sg & 63, kWave);
            pos[it] = (sg < nsegw && r < c_s) ? o_s + r : -1;
        }
#pragma unroll
        for (int it = 0; it < ITS; ++it)
            if (pos[it] >= 0 && (pos[it] & (WAVES - 1)) == w) mylist[pos[it] / WAVES] = ent[it];
        if (want_lists) {
            // kept channels of z before this workgroup's: the counts of all earlier segments (ascending lists
            // need no gap closing here: every workgroup can work out its own offset)
            int before = 0;
            for (int s0 = 0; s0 < seg0; s0 += kWave) {
                const int sg = s0 + lane;
                before += sg < seg0 ? min(max(a.zl_cnt[sg], 0), a.segz) : 0;
            }
            before = wave_sum(before);
            if (a.idx_out) {
#pragma unroll
                for (int it = 0; it < ITS; ++it)
                    if (pos[it] >= 0) a.idx_out[before + pos[it]] = ent[it].x;
            }
            if (split == a.S - 1 && lane == 0) {
                if (a.nnz_out) a.nnz_out[0] = before + cnt;
                if (a.union_nnz_out) a.union_nnz_out[0] = before + cnt;
            }
        }
    } else {
    #pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if (k0 + c * kG1Chunk < kend) {  // wave-uniform
                const int kb = k0 + c * kG1Chunk + 8 * lane;
                const int nvalid = kend - kb;  // elements j < nvalid of this lane exist
                const uint32_t wd[4] = {xv[c].x, xv[c].y, xv[c].z, xv[c].w};
                float xf[8];
                if (a.xdt == kBF16) {
    #pragma unroll
                    for (int j = 0; j < 8; ++j) xf[j] = __uint_as_float((j & 1) ? (wd[j >> 1] & 0xFFFF0000u) : (wd[j >> 1] << 16));
                } else {
    #pragma unroll
                    for (int j = 0; j < 8; ++j) xf[j] = f16_bits_to_f32((j & 1) ? (wd[j >> 1] >> 16) : (wd[j >> 1] & 0xFFFFu));
                }
                uint64_t bal[8];
                // position of a kept channel in the workgroup's list, and the entries this wavefront owns
                auto place = [&](int j, float dv) {
                    const int pos = cnt + lanes_below(bal[j]);
                    if (((bal[j] >> lane) & 1) && (pos & (WAVES - 1)) == w) mylist[pos / WAVES] = make_int2(kb + j, __float_as_int(dv));
                    cnt += __popcll(bal[j]);
                };
                if (a.mode == kModeSparse) {
    #pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float dv = xf[j] - a.m;                          // one fp32 subtraction
                        bal[j] = __ballot(fabsf(dv) > a.tau && j < nvalid);    // strict; NaN is pruned
                        place(j, dv);
                    }
                } else {
    #pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        bal[j] = __ballot(j < nvalid);  // dense (Eq. 1) and bias folding (Eq. 6): every channel
                        place(j, a.mode == kModeFold ? a.m : xf[j]);
                    }
                }
                if (want_lists) {
                    uint32_t kbits = 0;
    #pragma unroll
                    for (int j = 0; j < 8; ++j) kbits |= (uint32_t)((bal[j] >> lane) & 1) << j;
                    const int mine = __popc(kbits);
                    const int inc = wave_inclusive_scan(mine);
                    if (a.idx_out) {
                        int p = k0 + lcnt + inc - mine;
    #pragma unroll
                        for (int j = 0; j < 8; ++j)
                            if ((kbits >> j) & 1u) store_dev(&a.idx_out[p++], kb + j);
                    }
                    lcnt += __shfl(inc, kWave - 1, kWave);
                }
            }
        }
    }
    cnt = uniform(cnt);
    if (FUSE != kFuseList && want_lists && lane == 0) {
        if (a.S == 1) {
            if (a.nnz_out) a.nnz_out[0] = cnt;
            if (a.union_nnz_out) a.union_nnz_out[0] = cnt;
        } else {
            store_dev(&a.seg_cnt[split], cnt);
        }
    }
    __builtin_amdgcn_wave_barrier();  // the list is this wavefront's own: written above, read below, in order

    // ------------------------------------------------------------------ 2. stream the kept rows
    float acc[ELEMS];
#pragma unroll
    for (int j = 0; j < ELEMS; ++j) acc[j] = 0.f;
    const int col0 = tile * TILE + lane * ELEMS;
    const uint32_t lane_off = col0 < a.N ? (uint32_t)col0 * Vec<WDT>::kBytes : 0u;  // lanes past N re-read column 0
    const uint32_t row_bytes = (uint32_t)a.N * Vec<WDT>::kBytes;
    const char* wbase = reinterpret_cast<const char*>(a.W);
    const int n_w = cnt > w ? (cnt - w + WAVES - 1) / WAVES : 0;  // positions w, w + WAVES, ...

    for (int i0 = 0; i0 < n_w; i0 += kWave) {
        const int e = i0 + lane;
        const int2 ent = e < n_w ? mylist[e] : make_int2(0, 0);
        const int vidx = ent.x;
        const float vd = __int_as_float(ent.y);
        const int nb = min((int)kWave, n_w - i0);
        auto row_load = [&](int i) {
            return load_row<WDT>(wbase, (uint32_t)__builtin_amdgcn_readlane(vidx, i), row_bytes, lane_off);
        };
        uint4 r[UNROLL];
        if (nb < UNROLL) {
#pragma unroll
            for (int q = 0; q < UNROLL - 1; ++q)
                if (q < nb) r[q] = row_load(q);
#pragma unroll
            for (int q = 0; q < UNROLL - 1; ++q)
                if (q < nb) fma_row<WDT>(acc, r[q], read_lane_f(vd, q));
        } else {
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) r[q] = row_load(q);
            int u = 0;
            for (; u + 2 * UNROLL <= nb; u += UNROLL) {
#pragma unroll
                for (int q = 0; q < UNROLL; ++q) {
                    fma_row<WDT>(acc, r[q], read_lane_f(vd, u + q));
                    r[q] = row_load(u + UNROLL + q);
                    __builtin_amdgcn_sched_barrier(0);  // keep each load where it is: right behind the row it replaces
                }
            }
            // rows u .. u+UNROLL-1 are in flight; fewer than UNROLL further rows are left to issue
            const int rest = nb - u - UNROLL;
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                fma_row<WDT>(acc, r[q], read_lane_f(vd, u + q));
                if (q < rest) r[q] = row_load(u + UNROLL + q);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int q = 0; q < UNROLL - 1; ++q)
                if (q < rest) fma_row<WDT>(acc, r[q], read_lane_f(vd, u + UNROLL + q));
        }
    }

    // ------------------------------------------------------------------ 3. add the wavefronts' sums, slice by slice
    {
        float4* dst = reinterpret_cast<float4*>(s_red + w * TILE + lane * ELEMS);
#pragma unroll
        for (int j = 0; j < ELEMS / 4; ++j) dst[j] = make_float4(acc[4 * j], acc[4 * j + 1], acc[4 * j + 2], acc[4 * j + 3]);
    }
    __syncthreads();
    slice_t sum;
#pragma unroll
    for (int c = 0; c < CPL; ++c) sum.v[c] = 0.f;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
#pragma unroll
        for (int c = 0; c < CPL; ++c) sum.v[c] += s_red[i * TILE + w * SLICE + lane * LSTR + c * CSTR];
    }

    // what happens to a slice whose columns are finished (p: scaled for int8, fused bias added) in this wavefront
    auto emit = [&](const float* pt) {
        if constexpr (FUSE != kFuseSwiglu) {
            const float* p = pt;
#pragma unroll
            for (int c = 0; c < CPL; ++c)  // written through: lines left modified in L2 are paid for when the kernel ends
                if (fcol + c * CSTR < a.N) store_dev(&a.y[fcol + c * CSTR], p[c]);
        } else {
            // Columns come in groups of 8: 4 gate pre-activations, then the 4 matching up pre-activations.  The
            // lanes that hold gate columns fetch their up partners from 4 columns further on, form
            // z = silu(gate) * up (Alg. 2), centre and threshold it like any layer input (Alg. 3 steps 1-2, strict
            // compare of Eq. 2) and leave the slice's kept channels, compacted and ascending, as one list segment.
            // Here a lane needs CPL ADJACENT columns (a group's gate and up columns sit in neighbouring lanes): column
            // acol + c = slice column lane * CPL + c, which lane (that number mod 64) holds as its (number / 64)-th.
            float p[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int j = lane * CPL + c;
                p[c] = 0.f;
#pragma unroll
                for (int cc = 0; cc < CPL; ++cc) {
                    const float t = __shfl(pt[cc], j & 63, kWave);
                    if ((j >> 6) == cc) p[c] = t;
                }
            }
            const int acol = tile * TILE + w * SLICE + lane * CPL;
            constexpr int LPG = 8 / CPL;  // lanes per group of 8 columns
            const bool gate_lane = (lane % LPG) < LPG / 2;
            float dz[CPL];
            bool keep[CPL];
            int chan[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const float up = __shfl_down(p[c], LPG / 2, kWave);
                const int col = acol + c;
                chan[c] = (col >> 3) * 4 + (col & 3);
                const bool live = gate_lane && col < a.N && chan[c] < a.F;
                const float z = p[c] / (1.f + expf(-p[c])) * up;
                if (live && a.z_out) store_dev(&a.z_out[chan[c]], z);
                dz[c] = z - a.m2;  // one fp32 subtraction
                keep[c] = live && fabsf(dz[c]) > a.tau2;  // strict; NaN is pruned
            }
            const int seg = tile * WAVES + w;  // this slice's segment: SLICE / 2 channels from seg * (SLICE / 2) on
            if ((int64_t)seg * (SLICE / 2) < a.F) {
                int rank = 0, total_kept = 0;
                uint64_t bal[CPL];
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    bal[c] = __ballot(keep[c]);
                    rank += lanes_below(bal[c]);
                    total_kept += __popcll(bal[c]);
                }
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    if (keep[c]) {
                        const int64_t e = (int64_t)seg * (SLICE / 2) + rank;
                        store_dev(&a.zl_idx[e], chan[c]);
                        store_dev(&a.zl_d[e], dz[c]);
                        ++rank;  // the lane's own earlier column comes first
                    }
                }
                if (lane == 0) store_dev(&a.zl_cnt[seg], total_kept);
            }
        }
    };
    auto finish = [&](const slice_t& s) {
        float p[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) p[c] = (IS_I8 ? s.v[c] * cscale[c] : s.v[c]) + cbias[c];
        emit(p);
    };
    if constexpr (FUSE != kFuseSwiglu) {
        if (a.flags & kG1FlagAccumulate) {
            // y already holds what the result is to be added to (a residual stream, say).  Every workgroup adds its
            // share of the slice with device-scope fp32 atomic adds and is done: no partial sums, no ticket, no
            // last arrival -- and no fixed order of the additions, so the last bits of y differ from run to run.
            // The workgroups of split 0 bring the fused bias (Eq. 6).
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const float p = (IS_I8 ? sum.v[c] * cscale[c] : sum.v[c]) + (split == 0 ? cbias[c] : 0.f);
                if (fcol + c * CSTR < a.N) __hip_atomic_fetch_add(&a.y[fcol + c * CSTR], p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (FUSE != kFusePlain || !want_lists || a.S == 1) return;
            // the caller's lists still need the last arrival of (tile 0, slice 0) to close their gaps
            wait_memory_ops();
            unsigned long long* lt = reinterpret_cast<unsigned long long*>(a.counters);
            unsigned long long got = 0;
            if (lane == 0) got = __hip_atomic_fetch_add(lt, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1ull;
            if (__builtin_amdgcn_readfirstlane((int)(uint32_t)got) != a.S) return;
            if (lane == 0) store_dev(lt, 0ull);
            close_lists_wave(a, s_off, s_cnt);
            return;
        }
    }
    if (a.S == 1) {
        finish(sum);
        return;
    }

    // ------------------------------------------------------------------ 4a. split-K hand-over in fixed point
    // The S partial sums of a column are added as INTEGERS: each arrival rounds its partial to a multiple of
    // 2^-frac (frac chosen so that S of them fit 50 bits with 2^20 of range; 2^-24 for 32 splits) and adds it,
    // biased to be non-negative, to the column's 64-bit word together with a 1 in the arrival count -- ONE
    // atomic with return per column.  Integer addition is associative, so the sum does not depend on the order of
    // the arrivals (y is bit-reproducible) and nobody has to collect anything: whoever sees the count reach S holds
    // the complete sum in the value its own atomic returned, converts it once (fp64, one rounding to fp32), applies
    // scale and bias, stores y and clears the word.  One memory round trip after the last row instead of three.
    // A partial that is not finite or not below 2^20 in magnitude ESCAPES: it is handed over the old way -- stored
    // as fp32 into its partial-sum slot, its split marked in the column's escape mask, both acknowledged before the
    // atomic, which then carries a zero and a 1 in the escape count -- and the finisher adds the escaped values, in
    // split order, to the converted sum.  So every input gives the IEEE result the partial-sum hand-over gives, up
    // to the rounding of the non-escaped partials to 2^-frac.
    {
        if (a.fx_acc != nullptr) {
            const int limit_bits = fx_limit_bits(a.S);
            const int frac = limit_bits - kFxRangeBits;
            const double to_fixed = __hiloint2double((1023 + frac) << 20, 0);     // 2^frac
            const double from_fixed = __hiloint2double((1023 - frac) << 20, 0);   // 2^-frac
            const unsigned long long bias = 1ull << limit_bits;
            unsigned long long* escw = a.fx_acc + kFxCols;
            bool esc[CPL];
            bool any_esc = false;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                esc[c] = fcol + c * CSTR < a.N && !(fabsf(sum.v[c]) < 1048576.f);  // also NaN and Inf
                any_esc |= esc[c];
            }
            if (__ballot(any_esc) != 0ull) {  // rare: some partial of this slice escapes
                const __amdgpu_buffer_rsrc_t pbuf = make_raw_buffer(a.partial, (uint32_t)a.S * a.T * TILE * 4u);
                const uint32_t pstride = (uint32_t)a.T * TILE * 4u;
                const uint32_t pmine = (uint32_t)((tile * TILE + w * SLICE + lane * CPL) * 4);
                sum.store_coherent(pbuf, split * pstride + pmine);
#pragma unroll
                for (int c = 0; c < CPL; ++c)
                    if (esc[c]) __hip_atomic_fetch_or(&escw[fcol + c * CSTR], 1ull << split, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                wait_memory_ops();  // value and mask bit are in place before the arrival is counted
            }
            float fin_p[CPL];  // the gating epilogue: finished columns stay in registers
            bool fin_done[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                fin_p[c] = 0.f;
                fin_done[c] = false;
            }
            // all of the lane's atomics first (one round trip for the lot), then what they returned
            unsigned long long now_c[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                now_c[c] = 0ull;
                if (fcol + c * CSTR >= a.N) continue;
                const long long vfix = esc[c] ? 0ll : __double2ll_rn((double)sum.v[c] * to_fixed);
                const unsigned long long inc = (1ull << 57) | (esc[c] ? 1ull << 50 : 0ull) | (unsigned long long)(vfix + (long long)bias);
                now_c[c] = __hip_atomic_fetch_add(&a.fx_acc[fcol + c * CSTR], inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + inc;
            }
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const unsigned long long now = now_c[c];
                if ((int)(now >> 57) != a.S) continue;  // not the column's last arrival (or no column: count 0, S > 1)
                const long long total = (long long)(now & ((1ull << 50) - 1)) - (long long)a.S * (long long)bias;
                float yv = (float)((double)total * from_fixed);
                if ((now >> 50) & 127ull) {  // escaped partials: add them in split order
                    unsigned long long mask = load_dev(&escw[fcol + c * CSTR]);
                    const float* pcol = a.partial + (size_t)tile * TILE + (w * SLICE + lane * CPL + c);
                    while (mask) {
                        const int sp = __builtin_ctzll(mask);
                        mask &= mask - 1;
                        yv += load_dev(pcol + (size_t)sp * a.T * TILE);
                    }
                    store_dev(&escw[fcol + c * CSTR], 0ull);
                }
                yv = (IS_I8 ? yv * cscale[c] : yv) + cbias[c];
                if constexpr (FUSE != kFuseSwiglu) store_dev(&a.y[fcol + c * CSTR], yv);
                fin_p[c] = yv;
                fin_done[c] = true;
                store_dev(&a.fx_acc[fcol + c * CSTR], 0ull);  // zero at rest
            }
            if constexpr (FUSE == kFuseSwiglu) {
                // The gating epilogue works on a whole slice (gate and up columns side by side, one compacted list
                // segment).  Nearly always the wavefront that finishes one column of a slice finishes all of them:
                // then the slice is gated from registers.  Otherwise the finished columns are parked in memory and
                // counted on the slice's ticket; whoever completes the count fetches the slice and gates it.
                const int first = tile * TILE + w * SLICE;
                const int live_cols = min(max(a.N - first, 0), SLICE);  // columns of this slice that exist
                if (live_cols == 0) return;
                bool all_done = true, any_done = false;
                int n_done = 0;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    if (fcol + c * CSTR < a.N) all_done &= fin_done[c];
                    any_done |= fin_done[c];
                    n_done += fin_done[c] ? 1 : 0;
                }
                if (__ballot(!all_done) == 0ull && !(a.flags & kG1FlagParkSlices)) {
                    emit(fin_p);
                    return;
                }
                if (__ballot(any_done) == 0ull) return;
                float* park = a.partial + (size_t)a.S * a.T * TILE;  // behind the partial-sum slots (room checked on the host)
#pragma unroll
                for (int c = 0; c < CPL; ++c)
                    if (fin_done[c]) store_dev(&park[fcol + c * CSTR], fin_p[c]);
                wait_memory_ops();
                n_done = wave_sum(n_done);
                unsigned long long* st = reinterpret_cast<unsigned long long*>(a.counters + tile * kCounterStride + w * kG1TicketWords);
                unsigned long long got = 0;
                if (lane == 0) got = __hip_atomic_fetch_add(st, (unsigned long long)n_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + (unsigned long long)n_done;
                if (__builtin_amdgcn_readfirstlane((int)(uint32_t)got) != live_cols) return;
                if (lane == 0) store_dev(st, 0ull);
#pragma unroll
                for (int c = 0; c < CPL; ++c) fin_p[c] = fcol + c * CSTR < a.N ? load_dev(&park[fcol + c * CSTR]) : 0.f;
                emit(fin_p);
                return;
            }
            if (FUSE != kFusePlain || !want_lists) return;
            // the caller's lists still need the last arrival of (tile 0, slice 0) to close their gaps
            wait_memory_ops();
            unsigned long long* lt = reinterpret_cast<unsigned long long*>(a.counters);
            unsigned long long got = 0;
            if (lane == 0) got = __hip_atomic_fetch_add(lt, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1ull;
            if (__builtin_amdgcn_readfirstlane((int)(uint32_t)got) != a.S) return;
            if (lane == 0) store_dev(lt, 0ull);
            close_lists_wave(a, s_off, s_cnt);
            return;
        }
    }

    // ------------------------------------------------------------------ 4. split-K hand-over per (tile, slice)
    const __amdgpu_buffer_rsrc_t pbuf = make_raw_buffer(a.partial, (uint32_t)a.S * a.T * TILE * 4u);
    const uint32_t pstride = (uint32_t)a.T * TILE * 4u;  // bytes between consecutive splits
    const uint32_t pmine = (uint32_t)((tile * TILE + w * SLICE + lane * CPL) * 4);
    sum.store_coherent(pbuf, split * pstride + pmine);
    wait_memory_ops();  // the wavefront's stores have been acknowledged
    unsigned long long* ticket =
        reinterpret_cast<unsigned long long*>(a.counters + tile * kCounterStride + w * kG1TicketWords);
    unsigned long long seen = 0;
    if (lane == 0)
        seen = __hip_atomic_fetch_add(ticket, ticket_increment(xcc_id()), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) +
               ticket_increment(xcc_id());
    const uint32_t seen_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)seen);
    const uint32_t seen_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(seen >> 32));
    seen = ((unsigned long long)seen_hi << 32) | seen_lo;
    if ((int)(seen & 0xFFFFull) != a.S) return;  // not the last arrival of this slice

    const bool near = ticket_all_one_xcd(seen) && !(a.flags & kG1FlagDeviceScope);
    if (near) asm volatile("buffer_inv sc0" ::: "memory");  // this compute unit's vector L1 holds nothing older
    slice_t total;
#pragma unroll
    for (int c = 0; c < CPL; ++c) total.v[c] = 0.f;
    constexpr int FLY = CPL == 4 ? 16 : 32;  // partial loads in flight
    for (int sp0 = 0; sp0 < a.S; sp0 += FLY) {
        slice_t v[FLY];
        if (near) {
#pragma unroll
            for (int j = 0; j < FLY; ++j) v[j] = slice_t::load_plain(pbuf, min(sp0 + j, a.S - 1) * pstride + pmine);
        } else {
#pragma unroll
            for (int j = 0; j < FLY; ++j) v[j] = slice_t::load_coherent(pbuf, min(sp0 + j, a.S - 1) * pstride + pmine);
        }
#pragma unroll
        for (int j = 0; j < FLY; ++j) {
            const bool in = sp0 + j < a.S;  // a slot past the last split re-read it: not added
#pragma unroll
            for (int c = 0; c < CPL; ++c) total.v[c] += in ? v[j].v[c] : 0.f;
        }
    }
    finish(total);
    if (lane == 0) store_dev(ticket, 0ull);  // ready for the next call
    if (FUSE == kFusePlain && want_lists) close_lists_wave(a, s_off, s_cnt);
}

// ---------------------------------------------------------------------------------------------- launch
inline size_t gemv1_lds_bytes(int tile_cols, int Kc, int waves) {
    return (size_t)kG1HdrBytes + (size_t)waves * tile_cols * 4 + (size_t)waves * (Kc / waves + 1) * 8;
}

#define G1_ARGS                                                                                                    \
    a.x, a.W, a.K, a.N, a.Kc, a.S, a.T, a.mode, a.xdt, a.flags, a.m, a.tau, a.bias, a.y, a.partial, a.counters, \
        a.col_scale, a.idx_out, a.nnz_out, a.union_nnz_out, a.seg_cnt, a.m2, a.tau2, a.z_out, a.zl_idx, a.zl_d,  \
        a.zl_cnt, a.F, a.segz, a.fx_acc
template <int WDT, int WAVES, int UNROLL, int FUSE = kFusePlain>
static int launch_gemv1_nch(const Gemv1Args& a, hipStream_t stream) {
    constexpr int TILE = kWave * Vec<WDT>::kElems;
    const size_t lds = gemv1_lds_bytes(TILE, a.Kc, WAVES);
    if (lds > 64 * 1024) return SCAP_ERR_CONFIG;
    const dim3 grid((unsigned)(a.S * a.T)), block(WAVES * kWave);
    if (a.Kc <= kG1Chunk)
        hipLaunchKernelGGL((gemv1_kernel<WDT, WAVES, UNROLL, 1, FUSE>), grid, block, lds, stream, G1_ARGS);
    else if (a.Kc <= 2 * kG1Chunk)
        hipLaunchKernelGGL((gemv1_kernel<WDT, WAVES, UNROLL, 2, FUSE>), grid, block, lds, stream, G1_ARGS);
    else if (a.Kc <= 4 * kG1Chunk)
        hipLaunchKernelGGL((gemv1_kernel<WDT, WAVES, UNROLL, 4, FUSE>), grid, block, lds, stream, G1_ARGS);
    else
        return SCAP_ERR_CONFIG;
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}
template <int WDT, int WAVES>
static int launch_gemv1_unroll(const Gemv1Args& a, int unroll, hipStream_t stream) {
    switch (unroll) {
        case 4: return launch_gemv1_nch<WDT, WAVES, 4>(a, stream);
        case 8: return launch_gemv1_nch<WDT, WAVES, 8>(a, stream);
        case 16: return launch_gemv1_nch<WDT, WAVES, 16>(a, stream);
    }
    return SCAP_ERR_CONFIG;
}

template <int WDT>
int launch_gemv1_wdt(const Gemv1Args& a, int waves, int unroll, hipStream_t stream) {
    if (waves == 8) return launch_gemv1_unroll<WDT, 8>(a, unroll, stream);
    if (waves == 4) return launch_gemv1_unroll<WDT, 4>(a, unroll, stream);
    return SCAP_ERR_CONFIG;
}

// the two launches of the fused block: default shape only (8 wavefronts, 4 x 1 KB or 8 x 512 bytes in flight)
template <int WDT, int FUSE>
int launch_gemv1_block(const Gemv1Args& a, hipStream_t stream) {
    return launch_gemv1_nch<WDT, 8, WDT == kI8Half ? 8 : 4, FUSE>(a, stream);
}

#undef G1_ARGS

}  // namespace scap
