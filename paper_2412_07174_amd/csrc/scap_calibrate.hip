// Offline calibration on the GPU (SCAP Eq. 2: tau = Quantile(|X_calib|, s); Section 3: mode estimate
// first, threshold on the centred sample).  Order statistics are exact: an 8-bit-digit radix select over
// the fp32 bit patterns (four histogram passes per rank), so tau and the median carry no float error.
#include <math.h>

#include <vector>

#include "scap_device.hpp"
#include "scap_internal.hpp"

namespace scap {

// ascending numeric order == ascending unsigned key; every NaN ranks last
__device__ __forceinline__ uint32_t order_key(float v) {
    if (v != v) return 0xFFFFFFFFu;
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

static float key_to_float(uint32_t key) {
    const uint32_t u = (key & 0x80000000u) ? (key ^ 0x80000000u) : ~key;
    union { uint32_t u; float f; } cv;
    cv.u = u;
    return cv.f;
}

// value whose order statistics are wanted: the raw activation, or its importance |fp32(x) - m|
__device__ __forceinline__ float calib_value(const uint16_t* __restrict__ X, int64_t j, int xdt, int centred, float m) {
    const float xf = act_to_f32(X, j, xdt);
    if (!centred) return xf;
    const float d = xf - m;  // formed exactly as the pruner forms it
    return fabsf(d);
}

__global__ __launch_bounds__(256) void radix_hist_kernel(const uint16_t* __restrict__ X, int64_t M, int xdt, int centred,
                                                         float m, uint32_t prefix, uint32_t prefix_mask, int shift,
                                                         unsigned long long* __restrict__ hist) {
    __shared__ uint32_t sh[256];
    sh[threadIdx.x] = 0;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < M; j += stride) {
        const uint32_t key = order_key(calib_value(X, j, xdt, centred, m));
        if ((key & prefix_mask) == prefix) atomicAdd(&sh[(key >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    const uint32_t v = sh[threadIdx.x];
    if (v) atomicAdd(&hist[threadIdx.x], (unsigned long long)v);
}

__global__ __launch_bounds__(256) void block_sum_kernel(const uint16_t* __restrict__ X, int64_t M, int xdt,
                                                        double* __restrict__ sums) {
    __shared__ double sh[256];
    double acc = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < M; j += stride)
        acc += (double)act_to_f32(X, j, xdt);
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) sums[blockIdx.x] = sh[0];
}

// equal-width histogram between lo and hi (inclusive), bin = floor((v - lo) / w) in fp64
__global__ __launch_bounds__(256) void mode_hist_kernel(const uint16_t* __restrict__ X, int64_t M, int xdt, float lo,
                                                        float hi, double w, unsigned long long* __restrict__ hist) {
    __shared__ uint32_t sh[kHistBins];
    for (int i = threadIdx.x; i < kHistBins; i += blockDim.x) sh[i] = 0;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < M; j += stride) {
        const float v = act_to_f32(X, j, xdt);
        if (!(v >= lo && v <= hi)) continue;
        long long b = (long long)floor(((double)v - (double)lo) / w);
        if (b > kHistBins - 1) b = kHistBins - 1;
        if (b < 0) b = 0;
        atomicAdd(&sh[b], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHistBins; i += blockDim.x) {
        const uint32_t v = sh[i];
        if (v) atomicAdd(&hist[i], (unsigned long long)v);
    }
}

namespace {

struct Ctx {
    const uint16_t* X;
    int64_t M;
    int xdt;
    unsigned long long* d_hist;
    double* d_sums;
    hipStream_t stream;
    int blocks;
};

bool ok(hipError_t e) { return e == hipSuccess; }

int fetch(const Ctx& c, void* host, const void* dev, size_t bytes) {
    if (!ok(hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, c.stream))) return SCAP_ERR_HIP;
    if (!ok(hipStreamSynchronize(c.stream))) return SCAP_ERR_HIP;
    return SCAP_OK;
}

// k-th smallest (1-indexed, 1 <= k <= M) of the raw values (centred = 0) or of |x - m| (centred = 1)
int select_rank(const Ctx& c, int centred, float m, int64_t k, float* out) {
    uint32_t prefix = 0, mask = 0;
    unsigned long long h[256];
    unsigned long long want = (unsigned long long)k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        int rc = launch_zero_words(reinterpret_cast<int32_t*>(c.d_hist), 512, c.stream);
        if (rc != SCAP_OK) return rc;
        hipLaunchKernelGGL(radix_hist_kernel, dim3(c.blocks), dim3(256), 0, c.stream, c.X, c.M, c.xdt, centred, m, prefix,
                           mask, shift, c.d_hist);
        if (!ok(hipGetLastError())) return SCAP_ERR_HIP;
        rc = fetch(c, h, c.d_hist, sizeof(h));
        if (rc != SCAP_OK) return rc;
        int digit = 255;
        for (int d = 0; d < 256; ++d) {
            if (want <= h[d]) {
                digit = d;
                break;
            }
            want -= h[d];
        }
        prefix |= (uint32_t)digit << shift;
        mask |= 0xFFu << shift;
    }
    *out = key_to_float(prefix);
    return SCAP_OK;
}

int64_t rank_of(double q, int64_t M) {
    int64_t k = (int64_t)ceil(q * (double)M);
    if (k < 0) k = 0;
    if (k > M) k = M;
    return k;
}

}  // namespace

int run_calibrate(const uint16_t* X, int64_t M, int xdt, float s, int est, float* m_out, float* tau_out, void* workspace,
                  hipStream_t stream) {
    Ctx c;
    c.X = X;
    c.M = M;
    c.xdt = xdt;
    c.d_hist = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + kOffHist);
    c.d_sums = reinterpret_cast<double*>(static_cast<char*>(workspace) + kOffSums);
    c.stream = stream;
    int64_t blocks = (M + 256 * 16 - 1) / (256 * 16);
    if (blocks < 1) blocks = 1;
    if (blocks > kSumSlots) blocks = kSumSlots;
    c.blocks = (int)blocks;

    float m = 0.f;
    int rc;
    if (est == SCAP_MODE_MEAN) {
        hipLaunchKernelGGL(block_sum_kernel, dim3(c.blocks), dim3(256), 0, stream, X, M, xdt, c.d_sums);
        if (!ok(hipGetLastError())) return SCAP_ERR_HIP;
        std::vector<double> part((size_t)c.blocks);
        rc = fetch(c, part.data(), c.d_sums, sizeof(double) * (size_t)c.blocks);
        if (rc != SCAP_OK) return rc;
        double sum = 0.0;
        for (double p : part) sum += p;
        m = (float)(sum / (double)M);
    } else if (est == SCAP_MODE_MEDIAN) {
        float a, b;
        if (M % 2 == 1) {
            rc = select_rank(c, 0, 0.f, M / 2 + 1, &a);
            if (rc != SCAP_OK) return rc;
            m = a;
        } else {
            rc = select_rank(c, 0, 0.f, M / 2, &a);
            if (rc != SCAP_OK) return rc;
            rc = select_rank(c, 0, 0.f, M / 2 + 1, &b);
            if (rc != SCAP_OK) return rc;
            m = (float)(((double)a + (double)b) / 2.0);
        }
    } else if (est == SCAP_MODE_HIST) {
        float lo, hi;
        int64_t klo = rank_of(0.001, M), khi = rank_of(0.999, M);
        if (klo < 1) klo = 1;
        if (khi < 1) khi = 1;
        rc = select_rank(c, 0, 0.f, klo, &lo);
        if (rc != SCAP_OK) return rc;
        rc = select_rank(c, 0, 0.f, khi, &hi);
        if (rc != SCAP_OK) return rc;
        if (!(hi > lo)) {
            m = lo;
        } else {
            const double w = ((double)hi - (double)lo) / (double)kHistBins;
            rc = launch_zero_words(reinterpret_cast<int32_t*>(c.d_hist), 2 * kHistBins, stream);
            if (rc != SCAP_OK) return rc;
            hipLaunchKernelGGL(mode_hist_kernel, dim3(c.blocks), dim3(256), 0, stream, X, M, xdt, lo, hi, w, c.d_hist);
            if (!ok(hipGetLastError())) return SCAP_ERR_HIP;
            std::vector<unsigned long long> cnt(kHistBins);
            rc = fetch(c, cnt.data(), c.d_hist, sizeof(unsigned long long) * kHistBins);
            if (rc != SCAP_OK) return rc;
            long long best = -1;
            int bestb = 0;
            for (int b = 0; b < kHistBins; ++b) {
                long long sum = 0;
                for (int t = b - 2; t <= b + 2; ++t)
                    if (t >= 0 && t < kHistBins) sum += (long long)cnt[t];
                if (sum > best) {
                    best = sum;
                    bestb = b;
                }
            }
            volatile double centre = ((double)bestb + 0.5) * w;
            volatile double mode = (double)lo + centre;
            m = (float)mode;
        }
    } else if (est != SCAP_MODE_ZERO) {
        return SCAP_ERR_DTYPE;
    }

    float tau = 0.f;
    const int64_t k = rank_of((double)s, M);
    if (k > 0) {
        rc = select_rank(c, 1, m, k, &tau);
        if (rc != SCAP_OK) return rc;
    }
    *m_out = m;
    *tau_out = tau;
    return SCAP_OK;
}

}  // namespace scap
