// Device-side helpers shared by the HIP kernels of libscap (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scap_internal.hpp"

namespace scap {

constexpr int kWave = 64;


__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ float f16_bits_to_f32(uint32_t b) {
    union { uint16_t u; _Float16 h; } cv;
    cv.u = (uint16_t)b;
    return (float)cv.h;
}

__device__ __forceinline__ float act_to_f32(const uint16_t* __restrict__ x, int64_t pos, int xdt) {
    const uint32_t b = x[pos];
    return xdt == kBF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
}

// 16 bytes of weights through a global pointer, marked non-temporal: every weight byte is used exactly once
// per call, and streaming loads that do not claim cache lines read HBM about 15 % faster than plain ones
// (6.1 against 5.3 TB/s in a pure read sweep on this part).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const u32x4_t global_u32x4_t;
__device__ __forceinline__ uint4 load_weights16(global_u32x4_t* p) {
    const u32x4_t v = __builtin_nontemporal_load(p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load_weights16(const void* p) {
    return load_weights16((global_u32x4_t*)(uint64_t)p);
}

// number of weight elements in one 16-byte load
template <int WDT> struct Vec { static constexpr int kElems = (WDT == kI8) ? 16 : 8; static constexpr int kBytes = (WDT == kI8) ? 1 : 2; };

// acc[j] += d * w[j] for the elements packed in one 16-byte vector
template <int WDT>
__device__ __forceinline__ void fma_vec(float* __restrict__ acc, const uint4& r, float d) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
    if constexpr (WDT == kBF16) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            acc[2 * q + 0] = fmaf(__uint_as_float(w[q] << 16), d, acc[2 * q + 0]);
            acc[2 * q + 1] = fmaf(__uint_as_float(w[q] & 0xFFFF0000u), d, acc[2 * q + 1]);
        }
    } else if constexpr (WDT == kF16) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            union { uint32_t u; _Float16 h[2]; } cv;
            cv.u = w[q];
            acc[2 * q + 0] = fmaf((float)cv.h[0], d, acc[2 * q + 0]);
            acc[2 * q + 1] = fmaf((float)cv.h[1], d, acc[2 * q + 1]);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int v = ((int)(w[q] << (24 - 8 * j))) >> 24;
                acc[4 * q + j] = fmaf((float)v, d, acc[4 * q + j]);
            }
        }
    }
}

// lanes below mine that have their bit set in a 64-bit ballot
__device__ __forceinline__ int lanes_below(uint64_t ballot) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ float read_lane_f(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// inclusive prefix sum across the 64 lanes of a wave
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(v, off, kWave);
        if (lane >= off) v += t;
    }
    return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

}  // namespace scap
