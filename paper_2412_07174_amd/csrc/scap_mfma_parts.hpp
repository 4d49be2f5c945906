// Pieces shared by the kernels that run the gathered product on the matrix cores (gfx950 MFMA):
//
//     Y[16 tokens, 16 columns] += D[16 tokens, 16 rows] * W[16 rows, 16 columns]     v_mfma_f32_16x16x16_bf16
//     Y[16 tokens, 16 columns] += D[16 tokens, 32 rows] * W[32 rows, 16 columns]     v_mfma_f32_16x16x32_bf16
//
// (the second, gfx950's own shape, in the staged-tile kernel: mfma_block32 below -- same lane layout with 8
// instead of 4 k-slots per lane, A[m = l%16][k = 8*(l/16) + j], B[k = 8*(l/16) + j][n = l%16], j = 0..7, fed from
// two 16-row blocks of the list at a time; half the matrix instructions for the same rows)
//
// Operand layout without any transposition.  For this instruction lane l holds
//     A[m = l%16][k = 4*(l/16) + j],   B[k = 4*(l/16) + j][n = l%16],   C[m = 4*(l/16) + i][n = l%16],  i,j = 0..3.
// The weights are K-major, so a lane cannot fetch four rows of one column in one access; but it can fetch
// 16 bytes = ELEMS columns of one row.  Lane l loads columns ELEMS*(l%16) .. of the four list rows 4*(l/16) + j
// of a 16-row block, and element e of those four vectors is exactly this lane's B operand of the MFMA that
// produces columns {ELEMS*n + e}.  The C registers of lane l then hold tokens 4*(l/16)+i and ELEMS
// consecutive columns.  The A operand (centred values of token l%16 at rows 4*(l/16)+j) is split into a
// bf16 head and a bf16 tail (d = hi + lo) and fed through two MFMAs, so the bf16 rounding of d costs about
// 2^-17 relative instead of 2^-9.  int8 weights are widened exactly to bf16 in registers.  fp16 weights use
// v_mfma_f32_16x16x16_f16 (same lane layout) with the A operand split into an fp16 head and tail.
#pragma once

#include "scap_gemv_parts.hpp"

namespace scap {

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaTile = 128;    // columns per workgroup with bf16 weights (16 lanes x 8); int8: 256
constexpr int kMfmaTokens = 16;   // M of the MFMA; tokens beyond B are zero rows
constexpr int kMfmaBlock = 16;    // list rows per MFMA (K of the MFMA)
constexpr int kCompactWaves = 8;

__device__ __forceinline__ uint32_t bf16_rne_bits(float v) {
    const uint32_t u = __float_as_uint(v);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;  // finite or infinite input (NaN never reaches the list)
}

// 4 centred values -> bf16 head and tail operands
__device__ __forceinline__ void split_bf16x4(const float4& d, s16x4_t& hi, s16x4_t& lo) {
    const float v[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t h = bf16_rne_bits(v[j]);
        const float hf = __uint_as_float(h << 16);
        const float rest = ((h & 0x7FFFu) != 0x7F80u) ? v[j] - hf : 0.f;  // an infinite head has no tail
        hi[j] = (short)h;
        lo[j] = (short)bf16_rne_bits(rest);
    }
}

// 4 centred values -> fp16 head and tail operands (as raw 16-bit patterns).  The head is clamped to the largest
// finite fp16 so that a finite value never turns into an infinite head; the tail then carries the rest (the
// activations are fp16 or bf16 values minus a small mode, so the rest is small).  Values below fp16's
// subnormal step (6e-8) lose their tail, an absolute error far inside the output tolerance.
__device__ __forceinline__ void split_f16x4(const float4& d, s16x4_t& hi, s16x4_t& lo) {
    const float v[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool inf = fabsf(v[j]) == __builtin_huge_valf();
        const float c = inf ? v[j] : fminf(fmaxf(v[j], -65504.f), 65504.f);
        const _Float16 h = (_Float16)c;
        const _Float16 l = (_Float16)(inf ? 0.f : v[j] - (float)h);
        union { _Float16 f; short s; } a, b;
        a.f = h;
        b.f = l;
        hi[j] = a.s;
        lo[j] = b.s;
    }
}

// head / tail split of the A operand in the format the weights' MFMA takes
template <int WDT>
__device__ __forceinline__ void split_operand(const float4& d, s16x4_t& hi, s16x4_t& lo) {
    if constexpr (WDT == kF16)
        split_f16x4(d, hi, lo);
    else
        split_bf16x4(d, hi, lo);
}

// One 16-row block: r[j] = this lane's 16 bytes of list row 4*(l/16)+j (zeros for a slot past the list),
// a_hi / a_lo = its A operand.  acc[e] += A * B_e for the ELEMS column elements.
template <int WDT>
__device__ __forceinline__ void mfma_block(f32x4_t* __restrict__ acc, s16x4_t a_hi, s16x4_t a_lo, const uint4 (&r)[4]) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    const uint32_t q0[4] = {r[0].x, r[0].y, r[0].z, r[0].w};
    const uint32_t q1[4] = {r[1].x, r[1].y, r[1].z, r[1].w};
    const uint32_t q2[4] = {r[2].x, r[2].y, r[2].z, r[2].w};
    const uint32_t q3[4] = {r[3].x, r[3].y, r[3].z, r[3].w};
#pragma unroll
    for (int e = 0; e < ELEMS; ++e) {
        uint32_t lo01, lo23;  // rows (0,1) and (2,3) of column element e, packed as two bf16
        if constexpr (WDT == kBF16 || WDT == kF16) {
            const int q = e >> 1;
            if ((e & 1) == 0) {
                lo01 = (q0[q] & 0xFFFFu) | (q1[q] << 16);
                lo23 = (q2[q] & 0xFFFFu) | (q3[q] << 16);
            } else {
                lo01 = (q0[q] >> 16) | (q1[q] & 0xFFFF0000u);
                lo23 = (q2[q] >> 16) | (q3[q] & 0xFFFF0000u);
            }
        } else {
            // byte e of each row, sign-extended, as a float: its low 16 bits are zero (|v| <= 128)
            const int q = e >> 2, sh = 24 - 8 * (e & 3);
            const uint32_t f0 = __float_as_uint((float)(((int)(q0[q] << sh)) >> 24));
            const uint32_t f1 = __float_as_uint((float)(((int)(q1[q] << sh)) >> 24));
            const uint32_t f2 = __float_as_uint((float)(((int)(q2[q] << sh)) >> 24));
            const uint32_t f3 = __float_as_uint((float)(((int)(q3[q] << sh)) >> 24));
            lo01 = (f0 >> 16) | f1;
            lo23 = (f2 >> 16) | f3;
        }
        union { uint32_t u32[2]; s16x4_t v; } bop;
        bop.u32[0] = lo01;
        bop.u32[1] = lo23;
        if constexpr (WDT == kF16) {
            union { s16x4_t s; f16x4_t h; } ah, al, bh;
            ah.s = a_hi;
            al.s = a_lo;
            bh.s = bop.v;
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(ah.h, bh.h, acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(al.h, bh.h, acc[e], 0, 0, 0);
        } else {
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, bop.v, acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, bop.v, acc[e], 0, 0, 0);
        }
    }
}

typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

// Two 16-row blocks at once on the 32-deep instruction: r[0..3] = this lane's 16 bytes of rows 4*(l/16)+j of the
// first block, r[4..7] of the second (zeros for slots past the list); a_hi / a_lo = heads and tails of the eight
// matching centred values.  Which list row sits in which of the lane's 8 k-slots is free as long as A and B
// agree.  acc[e] += A * B_e for the ELEMS column elements.
template <int WDT>
__device__ __forceinline__ void mfma_block32(f32x4_t* __restrict__ acc, const s16x4_t (&a_hi)[2], const s16x4_t (&a_lo)[2],
                                             const uint4 (&r)[8]) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    union { s16x4_t h[2]; bf16x8_t b; f16x8_t f; } ah, al;
    ah.h[0] = a_hi[0];
    ah.h[1] = a_hi[1];
    al.h[0] = a_lo[0];
    al.h[1] = a_lo[1];
    uint32_t q[8][4];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        q[j][0] = r[j].x;
        q[j][1] = r[j].y;
        q[j][2] = r[j].z;
        q[j][3] = r[j].w;
    }
#pragma unroll
    for (int e = 0; e < ELEMS; ++e) {
        union { uint32_t u32[4]; bf16x8_t b; f16x8_t f; } bop;  // rows (0,1), (2,3), (4,5), (6,7) of column element e
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const uint32_t* x0 = q[2 * pr];
            const uint32_t* x1 = q[2 * pr + 1];
            if constexpr (WDT == kBF16 || WDT == kF16) {
                const int c = e >> 1;
                bop.u32[pr] = (e & 1) == 0 ? ((x0[c] & 0xFFFFu) | (x1[c] << 16)) : ((x0[c] >> 16) | (x1[c] & 0xFFFF0000u));
            } else {
                // byte e of each row, sign-extended, as a float: its low 16 bits are zero (|v| <= 128)
                const int c = e >> 2, sh = 24 - 8 * (e & 3);
                const uint32_t f0 = __float_as_uint((float)(((int)(x0[c] << sh)) >> 24));
                const uint32_t f1 = __float_as_uint((float)(((int)(x1[c] << sh)) >> 24));
                bop.u32[pr] = (f0 >> 16) | f1;
            }
        }
        if constexpr (WDT == kF16) {
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah.f, bop.f, acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al.f, bop.f, acc[e], 0, 0, 0);
        } else {
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah.b, bop.b, acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al.b, bop.b, acc[e], 0, 0, 0);
        }
    }
}

// Every wavefront holds a full [16 tokens x TILE columns] tile of sums in the same lane layout
// (acc[e][i] = token 4*(l/16) + i, column ELEMS*(l%16) + e of the tile).  They are added through LDS (32 KB at
// s_tree) in a fixed order and emitted by one thread per (token, 4-column group).  Ends with a barrier.
// (FUSE / s_fin: see finish_columns -- with one split the sums are final and may go to the gating step)
// ONE_LEVEL (8 wavefronts): the form described inside; otherwise a binary tree over the wavefronts.  The
// two-launch kernel keeps the tree: the one-level form costs it registers it needs for two workgroups per CU.
template <int WDT, int WAVES, int FUSE = kFusePlain, bool ONE_LEVEL = false>
__device__ __forceinline__ void reduce_waves_and_emit(const GemvArgs& a, __amdgpu_buffer_rsrc_t pbuf, int tile, int split,
                                                      f32x4_t* __restrict__ acc, float* s_red, float* s_fin = nullptr) {
    constexpr int ELEMS = Vec<WDT>::kElems;
    constexpr int TILE = 16 * ELEMS;
    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int cg = lane & 15, kg = lane >> 4;
    f32x4_t* s_tree = reinterpret_cast<f32x4_t*>(s_red);
    static_assert(!ONE_LEVEL || WAVES == 8, "the one-level form is written for 8 wavefronts");
    if constexpr (ONE_LEVEL) {
        // One level, eight columns per lane at a time, the wavefronts in two halves: four wavefronts write their
        // [16 tokens x 32 groups of 4 columns] (4 x 512 items x 16 bytes = 32 KB), every thread adds the four
        // values of its (token, group) in wavefront order, then the other four -- a fixed association -- and
        // emits the sum: consecutive threads hold consecutive groups, so a wavefront's stores are one contiguous
        // KB (write-through stores of half-filled 32-byte sectors cost visibly more).  Four barriers per 8
        // columns instead of seven with a tree plus a hand-over to the storing threads (1.3 -> 0.6 us at 16 tokens).
        constexpr int ITEMS = kMfmaTokens * 32;
        constexpr int H = WAVES / 2;
        static_assert(H * ITEMS * 16 <= 32 * 1024 && ITEMS == WAVES * kWave, "reduction buffer, one item per thread");
        static_assert(ELEMS % 8 == 0, "accumulators are handed over eight columns at a time");
#pragma unroll
        for (int c0 = 0; c0 < ELEMS; c0 += 8) {
            f32x4_t t = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int hw = 0; hw < 2; ++hw) {
                __syncthreads();  // the buffer is free (the list, or the previous values, have been read)
                if (w / H == hw) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
#pragma unroll
                        for (int v = 0; v < 2; ++v)
                            s_tree[(w % H) * ITEMS + (4 * kg + i) * 32 + 2 * cg + v] =
                                f32x4_t{acc[c0 + 4 * v][i], acc[c0 + 4 * v + 1][i], acc[c0 + 4 * v + 2][i], acc[c0 + 4 * v + 3][i]};
                    }
                }
                __syncthreads();
#pragma unroll
                for (int ww = 0; ww < H; ++ww) t += s_tree[ww * ITEMS + tid];
            }
            const int b = tid >> 5, gi = tid & 31;
            if (b < a.B) {
                const int g = ((gi >> 1) * ELEMS + c0) / 4 + (gi & 1);
                // one split: this is the finished value, and the group's constants are loaded here
                emit_group<WDT, TILE, FUSE>(a, pbuf, tile, split, b, g, make_float4(t[0], t[1], t[2], t[3]), s_fin,
                                            a.S == 1 ? load_col_const<WDT, TILE>(a, tile, g) : ColConst{});
            }
        }
        __syncthreads();
        return;
    }
    constexpr int CH = (WAVES <= 8) ? 8 : 4;  // binary tree: (WAVES/2) * CH * 64 lanes * 16 bytes = 32 KB of LDS
    static_assert(ELEMS % CH == 0, "accumulators are handed over in whole chunks");
#pragma unroll
    for (int c0 = 0; c0 < ELEMS; c0 += CH) {
#pragma unroll
        for (int half = WAVES / 2; half >= 1; half >>= 1) {
            __syncthreads();  // the buffer is free (previous level or chunk has been read)
            if (w >= half && w < 2 * half) {
#pragma unroll
                for (int e = 0; e < CH; ++e) s_tree[((w - half) * CH + e) * kWave + lane] = acc[c0 + e];
            }
            __syncthreads();
            if (w < half) {
#pragma unroll
                for (int e = 0; e < CH; ++e) acc[c0 + e] += s_tree[(w * CH + e) * kWave + lane];
            }
        }
        // Wavefront 0 holds the chunk's sums (lane = column group x row group).  They pass through LDS once more
        // so that every thread emits one 4-column group of one token (straight from wavefront 0's registers they
        // were strided stores of one wavefront, ~2 us of the kernel).
        constexpr int GPC = 16 * (CH / 4);  // 4-column groups of the chunk per token
        if (w == 0) {  // the only reader of the last tree level: no barrier needed before it writes
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int v = 0; v < CH / 4; ++v)
                    s_tree[(4 * kg + i) * GPC + cg * (CH / 4) + v] =
                        f32x4_t{acc[c0 + 4 * v][i], acc[c0 + 4 * v + 1][i], acc[c0 + 4 * v + 2][i], acc[c0 + 4 * v + 3][i]};
            }
        }
        __syncthreads();
        for (int item = tid; item < kMfmaTokens * GPC; item += WAVES * kWave) {
            const int b = item / GPC, gi = item - b * GPC;
            if (b < a.B) {
                const f32x4_t t = s_tree[item];
                const int g = ((gi / (CH / 4)) * ELEMS + c0) / 4 + gi % (CH / 4);
                emit_group<WDT, TILE, FUSE>(a, pbuf, tile, split, b, g, make_float4(t[0], t[1], t[2], t[3]), s_fin,
                                            a.S == 1 ? load_col_const<WDT, TILE>(a, tile, g) : ColConst{});
            }
        }
    }
    __syncthreads();
}

}  // namespace scap
