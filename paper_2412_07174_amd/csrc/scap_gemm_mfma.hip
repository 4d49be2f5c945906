// Batched sparse FC on the matrix cores (gfx950 MFMA), bf16 weights, 4..16 tokens.
//
// With several tokens each token keeps its own mask (SCAP Eq. 2 is elementwise); the rows that have to be
// read are the union of the masks (Appendix C), and what multiplies them is a [tokens x kept-rows] matrix of
// centred values with zeros where a token pruned the channel -- a dense contraction, so it goes to MFMA:
//
//     Y[16 tokens, 16 columns] += D[16 tokens, 16 rows] * W[16 rows, 16 columns]     v_mfma_f32_16x16x16_bf16
//
// Two launches.  `batch_compact_kernel` (one workgroup per K split) centres and thresholds the inputs of all
// tokens once and leaves, in the workspace, the ascending union list of its split and the centred values
// packed the way the matrix-core kernel reads them.  Doing this inside every (split, column tile) workgroup,
// as the one-token kernel does, repeats 16 tokens' worth of work per tile and took longer than the GEMM.
// `gemm_mfma_kernel` (split, tile of 128 columns) then only streams rows.
//
// Operand layout without any transposition.  For this instruction lane l holds
//     A[m = l%16][k = 4*(l/16) + j],   B[k = 4*(l/16) + j][n = l%16],   C[m = 4*(l/16) + i][n = l%16],  i,j = 0..3.
// The weights are K-major, so a lane cannot fetch four rows of one column in one access; but it can fetch
// 16 bytes = 8 columns of one row.  Lane l therefore loads columns 8*(l%16) .. +7 of the four list rows
// 4*(l/16) + j of a 16-row block (a load instruction covers four 256-byte row segments), and element e of
// those four vectors is exactly this lane's B operand of the MFMA that produces columns {8*n + e}.  Eight
// MFMAs (e = 0..7) per block cover the wavefront's 128 columns; the C registers of lane l then hold tokens
// 4*(l/16)+i and 8 consecutive columns.  The A operand (centred values of token l%16 at rows 4*(l/16)+j)
// is one 16-byte vector of the packed list; it is split into a bf16 head and a bf16 tail (d = hi + lo) and
// fed through two MFMAs, so the bf16 rounding of d costs about 2^-17 relative instead of 2^-9.
#include "scap_gemv_parts.hpp"

namespace scap {

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaTile = 128;    // columns per workgroup
constexpr int kMfmaTokens = 16;   // M of the MFMA; tokens beyond B are zero rows
constexpr int kMfmaBlock = 16;    // list rows per MFMA (K of the MFMA)
constexpr int kCompactWaves = 16;

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

// ---------------------------------------------------------------------------------------------- launch 1
// Workgroup `split`: union list of channels [split*Kc, (split+1)*Kc) -> u_idx[split*Kc ...] (ascending),
// centred values -> u_d (16 floats per entry, packed by d_at<kDPacked16>), list length -> seg_cnt[B*S+split];
// per-token lists and counts for idx_out / nnz_out as in the one-token kernel.
__global__ __launch_bounds__(kCompactWaves * kWave) void batch_compact_kernel(const GemvArgs a) {
    __shared__ int s_hdr[kHdrBytes / 4];
    const int split = blockIdx.x;
    Lds L;
    L.hdr = s_hdr;
    L.flag = s_hdr + (1 + kMfmaTokens) * kCompactWaves;
    L.idx = a.u_idx + (int64_t)split * a.Kc;
    L.d = a.u_d + (int64_t)split * a.Kc * kMfmaTokens;
    L.red = nullptr;
    compact_inputs<kCompactWaves, kMfmaTokens, kDPacked16>(a, 0, split, L);
}

// ---------------------------------------------------------------------------------------------- launch 2
template <int WAVES, int UB>
__global__ __launch_bounds__(WAVES * kWave) void gemm_mfma_kernel(const GemvArgs a) {
    constexpr int BT = kMfmaTokens;
    constexpr int TILE = kMfmaTile;
    constexpr int NT = WAVES * kWave;
    constexpr int GROUPS = TILE / 4;

    extern __shared__ uint4 smem_raw[];
    const Lds L = carve_lds<WAVES, BT>(reinterpret_cast<char*>(smem_raw), 0);
    float* s_red = L.red;  // [WAVES][4 token groups][TILE]

    const int tid = threadIdx.x;
    const int w = uniform(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x % a.T;
    const int split = blockIdx.x / a.T;

    const int cnt = uniform(a.seg_cnt[a.B * a.S + split]);  // written by the previous launch
    const int4* __restrict__ lidx = reinterpret_cast<const int4*>(a.u_idx + (int64_t)split * a.Kc);
    const float4* __restrict__ ld4 = reinterpret_cast<const float4*>(a.u_d + (int64_t)split * a.Kc * BT);

    const int cg = lane & 15;   // column group: columns 8*cg .. 8*cg+7 of the tile (B/C index n)
    const int kg = lane >> 4;   // row group: list rows 4*kg .. 4*kg+3 of a block (k of A and B); token group of C
    const int tok = lane & 15;  // token whose centred values this lane supplies (A index m)
    const int col0 = tile * TILE + cg * 8;
    const uint32_t lane_off = (col0 < a.N) ? (uint32_t)col0 * 2u : 0u;
    const uint32_t row_bytes = (uint32_t)a.N * 2u;
    const char* wbase = reinterpret_cast<const char*>(a.W);

    f32x4_t acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Entry group (blk, kg) = list entries blk*16 + 4*kg .. +3: one int4 of indices, and for token `tok` one
    // float4 of centred values at float4 index (blk*4 + kg)*16 + tok.  Groups at or past the end of the list
    // are not loaded; inside the last group, entries >= cnt are masked.
    auto load_idx = [&](int blk) -> int4 {
        const int g4 = blk * 4 + kg;
        return (g4 * 4 < cnt) ? lidx[g4] : make_int4(0, 0, 0, 0);
    };

    const int n_blocks = (cnt + kMfmaBlock - 1) / kMfmaBlock;
    int4 ix[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) ix[u] = load_idx(w + u * WAVES);

    for (int blk0 = w; blk0 < n_blocks; blk0 += WAVES * UB) {
        uint4 r[UB][4];
        float4 dv[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int blk = blk0 + u * WAVES;
            const int e0 = blk * kMfmaBlock + 4 * kg;
            const int rows[4] = {ix[u].x, ix[u].y, ix[u].z, ix[u].w};
            dv[u] = (e0 < cnt) ? ld4[(blk * 4 + kg) * 16 + tok] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                r[u][j] = make_uint4(0u, 0u, 0u, 0u);
                if (e0 + j < cnt)
                    r[u][j] = *reinterpret_cast<const uint4*>(wbase + (uint64_t)(uint32_t)rows[j] * row_bytes + lane_off);
            }
            if (e0 + 1 >= cnt) dv[u].y = 0.f;
            if (e0 + 2 >= cnt) dv[u].z = 0.f;
            if (e0 + 3 >= cnt) dv[u].w = 0.f;
        }
        int4 ixn[UB];  // indices of the next iteration, fetched while this one computes
#pragma unroll
        for (int u = 0; u < UB; ++u) ixn[u] = load_idx(blk0 + (UB + u) * WAVES);
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            s16x4_t a_hi, a_lo;
            split_bf16x4(dv[u], a_hi, a_lo);
            const uint32_t q0[4] = {r[u][0].x, r[u][0].y, r[u][0].z, r[u][0].w};
            const uint32_t q1[4] = {r[u][1].x, r[u][1].y, r[u][1].z, r[u][1].w};
            const uint32_t q2[4] = {r[u][2].x, r[u][2].y, r[u][2].z, r[u][2].w};
            const uint32_t q3[4] = {r[u][3].x, r[u][3].y, r[u][3].z, r[u][3].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int q = e >> 1;
                uint32_t lo01, lo23;  // rows (0,1) and (2,3) of column element e, packed as two bf16
                if ((e & 1) == 0) {
                    lo01 = (q0[q] & 0xFFFFu) | (q1[q] << 16);
                    lo23 = (q2[q] & 0xFFFFu) | (q3[q] << 16);
                } else {
                    lo01 = (q0[q] >> 16) | (q1[q] & 0xFFFF0000u);
                    lo23 = (q2[q] >> 16) | (q3[q] & 0xFFFF0000u);
                }
                union { uint32_t u32[2]; s16x4_t v; } bop;
                bop.u32[0] = lo01;
                bop.u32[1] = lo23;
                acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, bop.v, acc[e], 0, 0, 0);
                acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, bop.v, acc[e], 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) ix[u] = ixn[u];
    }

    // ------------------------------------------------------------------ add the wavefronts' sums
    // acc[e][i] = token 4*kg + i, column col0 + e.  One pass per i: 4 tokens x 128 columns per wavefront.
    const __amdgpu_buffer_rsrc_t pbuf = partial_buffer<TILE>(a);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float4* dst = reinterpret_cast<float4*>(s_red + (w * 4 + kg) * TILE + cg * 8);
        dst[0] = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
        dst[1] = make_float4(acc[4][i], acc[5][i], acc[6][i], acc[7][i]);
        __syncthreads();
        for (int t = tid; t < 4 * GROUPS; t += NT) {
            const int mg = t / GROUPS, g = t % GROUPS;
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) {
                const float4 v = *reinterpret_cast<const float4*>(s_red + (ww * 4 + mg) * TILE + 4 * g);
                s.x += v.x;
                s.y += v.y;
                s.z += v.z;
                s.w += v.w;
            }
            const int b = 4 * mg + i;
            if (b < a.B) emit_group<kBF16, TILE>(a, pbuf, tile, split, b, g, s);
        }
        __syncthreads();
    }

    finish_tile<kBF16, WAVES, TILE, BT>(a, pbuf, tile, L);
}

int launch_gemm_mfma(const GemvArgs& a_in, const scap_launch_cfg* cfg, hipStream_t stream) {
    GemvArgs a = a_in;
    constexpr int WAVES = 16;
    if (!a.u_idx || !a.u_d) return SCAP_ERR_WORKSPACE;
    int kc = 0;
    if (cfg && cfg->rows_per_group) {
        kc = cfg->rows_per_group;
        if (kc < 0 || (kc % kWave) != 0) return SCAP_ERR_CONFIG;
    }
    // no list in LDS: the split is bounded only by the workspace
    const int rc = plan_splits(a, kMfmaTile, 0, kc, kc != 0);
    if (rc != SCAP_OK) return rc;
    if ((size_t)a.S * a.Kc > union_list_entries(a.K)) return SCAP_ERR_CONFIG;

    hipLaunchKernelGGL(batch_compact_kernel, dim3((unsigned)a.S), dim3(kCompactWaves * kWave), 0, stream, a);
    if (hipGetLastError() != hipSuccess) return SCAP_ERR_HIP;

    // reduction buffers: WAVES x 4 token groups x 128 columns (the final reduction needs less)
    const size_t red = (size_t)WAVES * 4 * kMfmaTile * 4;
    const size_t lds = lds_bytes(0, 0, red);
    const dim3 grid((unsigned)(a.S * a.T));
    const dim3 block(WAVES * kWave);
    hipLaunchKernelGGL((gemm_mfma_kernel<WAVES, 2>), grid, block, lds, stream, a);
    return hipGetLastError() == hipSuccess ? SCAP_OK : SCAP_ERR_HIP;
}

}  // namespace scap
