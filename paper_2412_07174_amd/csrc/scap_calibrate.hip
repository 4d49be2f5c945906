// Offline calibration (SCAP Eq. 2: tau = Quantile(|X_calib|, s); Section 3: mode estimate first, threshold
// on the centred sample).
//
// The calibration activations are 16-bit codes, so a pooled sample of any size has at most 65 536 distinct
// values.  ONE streaming pass over the sample counts how often each code occurs; every statistic the
// estimators need is then a function of those 65 536 counts and is evaluated on the host with the same
// IEEE operations the pruner uses on the device (widening is exact, d = fp32(x) - m is one fp32
// subtraction): order statistics by walking the counts in value order -- exact, no float error -- the mean
// as an fp64 sum of count x value, the histogram mode from fp64 bin arithmetic.
#include <math.h>
#include <cmath>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <utility>
#include <vector>

#include "scap_device.hpp"
#include "scap_internal.hpp"

namespace scap {

constexpr int kCodes = 65536;
constexpr int kHalf = 32768;        // codes counted by one workgroup: 128 KB of LDS counters (gfx950: 160 KB per workgroup)
constexpr int kHistThreads = 1024;
constexpr int kHistChunks = 128;    // workgroups per half of the code space

// Workgroup (chunk, half) reads its share of the sample 16 bytes per lane and counts the codes whose top bit
// equals `half` (the sign) in LDS, then adds its non-zero counters to the global histogram.  The kernel is bound
// by instruction issue (shift, compare, masked LDS add per code), so every code is looked at by as few
// workgroups as LDS allows: two.
__global__ __launch_bounds__(kHistThreads) void code_hist_kernel(const uint16_t* __restrict__ X, int64_t M,
                                                                unsigned long long* __restrict__ hist) {
    extern __shared__ uint32_t sh[];  // [kHalf]
    const int tid = threadIdx.x;
    // The two workgroups that read the same share sit on one XCD (blockIdx % 8) and start together, so the share
    // comes from HBM once and from that XCD's L2 the second time.
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const uint32_t half = (uint32_t)j & 1u;
    const int chunk = xcd + 8 * (j >> 1);
    const int nchunk = gridDim.x >> 1;
    for (int i = tid; i < kHalf; i += kHistThreads) sh[i] = 0;
    __syncthreads();
    auto count = [&](uint32_t code) {
        if ((code >> 15) == half) atomicAdd(&sh[code & (kHalf - 1)], 1u);
    };
    const int64_t nvec = M / 8;
    const uint4* __restrict__ X8 = reinterpret_cast<const uint4*>(X);
    auto count8 = [&](const uint4& v) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            count(w[q] & 0xFFFFu);
            count(w[q] >> 16);
        }
    };
    // four loads in flight per lane: with 16 wavefronts per compute unit (the counters fill LDS) one load per lane
    // leaves the memory latency exposed
    constexpr int FLY = 4;
    const int64_t stride = (int64_t)nchunk * kHistThreads;
    int64_t i = (int64_t)chunk * kHistThreads + tid;
    for (; i + (FLY - 1) * stride < nvec; i += FLY * stride) {
        uint4 v[FLY];
#pragma unroll
        for (int u = 0; u < FLY; ++u) v[u] = X8[i + u * stride];
#pragma unroll
        for (int u = 0; u < FLY; ++u) count8(v[u]);
    }
    for (; i < nvec; i += stride) count8(X8[i]);
    if (chunk == 0) {
        const int64_t j = nvec * 8 + tid;  // the last M % 8 codes
        if (j < M) count(X[j]);
    }
    __syncthreads();
    for (int i = tid; i < kHalf; i += kHistThreads) {
        const uint32_t v = sh[i];
        if (v) atomicAdd(&hist[half * kHalf + i], (unsigned long long)v);
    }
}

namespace {

bool ok(hipError_t e) { return e == hipSuccess; }

// exact widening of a 16-bit code on the host
float code_to_float(uint32_t c, int xdt) {
    uint32_t u;
    if (xdt == kBF16) {
        u = c << 16;
    } else {
        const uint32_t sign = (c & 0x8000u) << 16, e = (c >> 10) & 0x1Fu, f = c & 0x3FFu;
        if (e == 0x1Fu) {
            u = sign | 0x7F800000u | (f << 13);
        } else if (e != 0) {
            u = sign | ((e + 112u) << 23) | (f << 13);
        } else if (f == 0) {
            u = sign;
        } else {  // subnormal half: normalise
            int sh = 0;
            uint32_t m = f;
            while (!(m & 0x400u)) {
                m <<= 1;
                ++sh;
            }
            u = sign | ((113u - sh) << 23) | ((m & 0x3FFu) << 13);
        }
    }
    float v;
    memcpy(&v, &u, 4);
    return v;
}

// The sample as (value, count) pairs in ascending value order; NaNs counted apart (they rank last).
struct Table {
    std::vector<float> val;
    std::vector<unsigned long long> cnt;
    unsigned long long nans = 0;
};

Table make_table(const std::vector<unsigned long long>& hist, int xdt) {
    Table t;
    auto push = [&](uint32_t c) {
        if (!hist[c]) return;
        const float v = code_to_float(c, xdt);
        if (v != v) {
            t.nans += hist[c];
        } else {
            t.val.push_back(v);
            t.cnt.push_back(hist[c]);
        }
    };
    // both formats order like sign-magnitude integers: negatives from the largest magnitude down, then
    // positives up (-0 sorts before +0; they are equal as numbers, which no statistic below can tell apart)
    for (int c = 0xFFFF; c >= 0x8000; --c) push((uint32_t)c);
    for (int c = 0x0000; c <= 0x7FFF; ++c) push((uint32_t)c);
    return t;
}

float quiet_nan() {
    const uint32_t u = 0x7FFFFFFFu;
    float v;
    memcpy(&v, &u, 4);
    return v;
}

// k-th smallest of the raw values, 1 <= k <= M
float select_raw(const Table& t, unsigned long long k) {
    unsigned long long run = 0;
    for (size_t i = 0; i < t.val.size(); ++i) {
        run += t.cnt[i];
        if (k <= run) return t.val[i];
    }
    return quiet_nan();
}

// k-th smallest of |value - m| (one fp32 subtraction, as the pruner forms it).  Below m the importance
// falls as the value rises, above m it rises (fp32 rounding is monotone), so the sorted order is a merge
// of the two runs that start at the value nearest m.
float select_centred(const Table& t, float m, unsigned long long k) {
    if (m != m) return quiet_nan();
    const size_t n = t.val.size();
    std::vector<float> imp(n);
    size_t p = n;  // first entry with value - m >= 0
    bool any_nan = false;
    for (size_t i = 0; i < n; ++i) {
        volatile float d = t.val[i] - m;
        imp[i] = fabsf(d);
        any_nan |= imp[i] != imp[i];
        if (p == n && !(d < 0.f)) p = i;
    }
    if (any_nan) {
        // infinite m meeting an infinite sample: no monotone runs; sort outright, NaN importances last
        std::vector<std::pair<float, unsigned long long>> e;
        unsigned long long run = 0;
        for (size_t i = 0; i < n; ++i)
            if (imp[i] == imp[i]) e.emplace_back(imp[i], t.cnt[i]);
        std::sort(e.begin(), e.end());
        for (const auto& x : e) {
            run += x.second;
            if (k <= run) return x.first;
        }
        return quiet_nan();
    }
    size_t up = p;          // next candidate of the rising run
    size_t down = p;        // one past the next candidate of the falling run
    unsigned long long run = 0;
    while (up < n || down > 0) {
        size_t pick;
        if (up >= n)
            pick = --down;
        else if (down == 0)
            pick = up++;
        else if (imp[down - 1] <= imp[up])
            pick = --down;
        else
            pick = up++;
        run += t.cnt[pick];
        if (k <= run) return imp[pick];
    }
    return quiet_nan();
}

// 1-based rank of the q-quantile among M pooled values: the smallest integer >= q*M (product formed in fp64),
// kept inside [0, M]
int64_t quantile_rank(double q, int64_t M) {
    return std::min<int64_t>(M, std::max<int64_t>(0, (int64_t)std::ceil(q * (double)M)));
}

// Histogram estimate of the mode from the (value, count) table: kHistBins equal bins between the 0.001 and
// 0.999 order statistics (a value equal to the upper one belongs to the last bin), each bin scored by the
// number of samples in the five bins centred on it (fewer at the edges), the centre of the first bin with the
// top score.  The bins are filled as a running total, so a score is the difference of two totals.
float histogram_mode(const Table& t, int64_t M) {
#pragma clang fp contract(off)  // (b + 1/2) * w and lo + ... each round once, in fp64
    const float lo = select_raw(t, (unsigned long long)std::max<int64_t>(1, quantile_rank(0.001, M)));
    const float hi = select_raw(t, (unsigned long long)std::max<int64_t>(1, quantile_rank(0.999, M)));
    if (!(hi > lo)) return lo;
    const double width = ((double)hi - (double)lo) / (double)kHistBins;
    // upto[b] = samples in bins 0 .. b-1; the table is ascending, so bins are met in order
    std::vector<unsigned long long> upto(kHistBins + 1, 0);
    for (size_t i = 0; i < t.val.size(); ++i) {
        const float v = t.val[i];
        if (v < lo || v > hi) continue;
        const double pos = std::floor(((double)v - (double)lo) / width);
        const int bin = pos >= (double)kHistBins ? kHistBins - 1 : (int)pos;
        upto[bin + 1] += t.cnt[i];
    }
    for (int b = 0; b < kHistBins; ++b) upto[b + 1] += upto[b];
    int top_bin = 0;
    unsigned long long top = 0;
    for (int b = 0; b < kHistBins; ++b) {
        const unsigned long long score = upto[std::min(b + 3, kHistBins)] - upto[std::max(b - 2, 0)];
        if (b == 0 || score > top) {
            top = score;
            top_bin = b;
        }
    }
    const double offset = ((double)top_bin + 0.5) * width;
    const double centre = (double)lo + offset;
    return (float)centre;
}

}  // namespace

int run_calibrate(const uint16_t* X, int64_t M, int xdt, float s, int est, float* m_out, float* tau_out, void* workspace,
                  hipStream_t stream) {
    if (est < SCAP_MODE_ZERO || est > SCAP_MODE_HIST) return SCAP_ERR_DTYPE;
    unsigned long long* d_hist = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + kOffCodeHist);
    int rc = launch_zero_words(reinterpret_cast<int32_t*>(d_hist), 2 * (size_t)kCodes, stream);
    if (rc != SCAP_OK) return rc;
    {
        // 128 KB of dynamic LDS: above the default limit, asked for once per device
        constexpr int kMaxDevices = 64;
        static std::atomic<bool> asked[kMaxDevices];
        int dev = 0;
        if (!ok(hipGetDevice(&dev)) || dev < 0 || dev >= kMaxDevices) return SCAP_ERR_HIP;
        if (!asked[dev].load(std::memory_order_acquire)) {
            if (!ok(hipFuncSetAttribute(reinterpret_cast<const void*>(&code_hist_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kHalf * 4)))
                return SCAP_ERR_HIP;
            asked[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL(code_hist_kernel, dim3(2 * kHistChunks), dim3(kHistThreads), kHalf * 4, stream, X, M, d_hist);
    if (!ok(hipGetLastError())) return SCAP_ERR_HIP;
    std::vector<unsigned long long> hist(kCodes);
    if (!ok(hipMemcpyAsync(hist.data(), d_hist, sizeof(unsigned long long) * kCodes, hipMemcpyDeviceToHost, stream)))
        return SCAP_ERR_HIP;
    if (!ok(hipStreamSynchronize(stream))) return SCAP_ERR_HIP;
    const Table t = make_table(hist, xdt);

    float m = 0.f;
    if (est == SCAP_MODE_MEAN) {
        double sum = t.nans ? (double)quiet_nan() : 0.0;
        for (size_t i = 0; i < t.val.size(); ++i) sum += (double)t.cnt[i] * (double)t.val[i];
        m = (float)(sum / (double)M);
    } else if (est == SCAP_MODE_MEDIAN) {
        if (M % 2 == 1) {
            m = select_raw(t, (unsigned long long)(M / 2 + 1));
        } else {
            const float a = select_raw(t, (unsigned long long)(M / 2));
            const float b = select_raw(t, (unsigned long long)(M / 2 + 1));
            m = (float)(((double)a + (double)b) / 2.0);
        }
    } else if (est == SCAP_MODE_HIST) {
        m = histogram_mode(t, M);
    }

    float tau = 0.f;
    const int64_t k = quantile_rank((double)s, M);
    if (k > 0) tau = select_centred(t, m, (unsigned long long)k);
    *m_out = m;
    *tau_out = tau;
    return SCAP_OK;
}

}  // namespace scap
