// Host-side internals of libscap: workspace layout, kernel argument blocks, launcher prototypes.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/scap.h"

namespace scap {

// dtype codes, numerically equal to scap_dtype
constexpr int kF16 = SCAP_F16;
constexpr int kBF16 = SCAP_BF16;
constexpr int kI8 = SCAP_I8_COLSCALE;

// GEMV input modes
constexpr int kModeSparse = 0;  // d = x - m, keep = |d| > tau        (Alg. 3)
constexpr int kModeDense = 1;   // d = x, every channel kept          (Eq. 1)
constexpr int kModeFold = 2;    // d = m for every channel            (Eq. 6, eta * column sums)

// ---------------------------------------------------------------------------------------------
// Workspace layout (byte offsets into the caller's buffer)
//   [65536, +32768)      int32 seg_cnt[17][256]  kept-channel counts per (token | union, K split)
//   [131072, +1 MiB)     int32 counter per column tile, one every 1 KiB so that the arrival tickets of
//                        different tiles go to different memory channels; zero at rest
//   [1179648, +2 MiB)    one-token kernel, fixed-point hand-over: uint64 acc[131072] (per output column: arrival
//                        count, escape count and the biased fixed-point sum of the arrivals' partial sums), then
//                        uint64 esc[131072] (which splits handed their partial over as fp32 instead); zero at rest
//   [3276800, +4*B*cap)  float partial[B][S][T][tile]   split-K partial sums; during calibration the first
//                        512 KiB hold the uint64 count of every 16-bit code
//   [.., +68*(K+16384))  batched path (B >= 2): union list of every list segment (64 bytes of A operands and
//                        the channel index per entry)
// ---------------------------------------------------------------------------------------------
constexpr size_t kOffSegCnt = 65536;
constexpr size_t kOffCounters = 131072;
constexpr int kCounterStride = 256;  // int32 words between the counters of neighbouring tiles
constexpr size_t kOffFx = kOffCounters + 1024 * (size_t)kCounterStride * 4;
constexpr int kFxCols = 131072;  // output columns the fixed-point hand-over covers (wider layers use partial sums)
constexpr size_t kOffPartial = kOffFx + (size_t)kFxCols * 16;
constexpr size_t kOffCodeHist = kOffPartial;
constexpr size_t kCalibBytes = kOffCodeHist + 65536 * 8;  // workspace bytes calibration needs
constexpr int kMaxTiles = 1024;
constexpr int kMaxSplits = 256;
constexpr int kHistBins = 2048;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// columns rounded up to whole 1024-column blocks (covers the 512- and 1024-column tiles)
// entries of union-list storage for a K-channel layer: every split may round up to a multiple of 64
inline size_t union_list_entries(int64_t K) { return (size_t)K + 64 * 256; }

inline size_t padded_cols(int64_t N) { return align_up((size_t)N, 1024); }

// floats of split-K partial storage per token
inline size_t partial_capacity(int64_t N) {
    const size_t np = padded_cols(N);
    const size_t cap = np * 16;
    return cap > ((size_t)1 << 20) ? cap : ((size_t)1 << 20);
}

struct GemvArgs {
    const void* W;
    const uint16_t* col_scale;
    const uint16_t* x;
    const float* bias;
    float* y;
    int32_t* idx_out;
    int32_t* nnz_out;
    int32_t* union_nnz_out;
    int32_t* counters;
    int32_t* seg_cnt;
    unsigned long long* fx_acc;  // fixed-point hand-over words [kFxCols], then the escape masks [kFxCols]; or NULL
    float* partial;
    int32_t* u_idx;  // batched path: union list of each segment, [Sl][Kl] channel indices
    float* u_d;      // batched path: the union list's centred values as MFMA A operands: per 16 entries 64 lanes x
                     // (4 bf16 heads, 4 bf16 tails) = 1 KB, i.e. 64 bytes per entry
    int K, N, B, Kc, S, T, mode, xdt;
    int Kl, Sl;  // segmentation of the kept-channel lists: Sl segments of Kl channels (= S, Kc unless batched)
    float m, tau;
    // Fused SwiGLU block (Alg. 2).  The gate|up launch leaves the gated product z, centred and thresholded,
    // as one compacted list per 64 channels; the down launch takes those lists as its input.
    float m2, tau2;   // mode estimate and threshold of the gated product
    float* z_out;     // optional fp32 [B][F]: the gated product itself
    int32_t* zl_idx;  // [ceil(F/64)][64] channels of each 64-channel segment kept by any token, ascending
    float* zl_d;      // [ceil(F/64)][64][BT] their centred values per token (BT = B rounded up to 1, 2 or 4)
    int32_t* zl_cnt;  // [1 + BT][ceil(F/64)] entries per segment: union first, then per token
    int F;            // channels of the gated product (half the columns of the gate|up launch)
};

// Enqueue one GEMV (sparse / dense / fold mode).  Returns a scap_status.
int launch_gemv(const GemvArgs& a, int wdt, const scap_launch_cfg* cfg, hipStream_t stream);

// One token (B == 1) through the one-token kernel.  Returns a scap_status, or kG1NotApplicable (positive) when a
// workgroup would own more channels than that kernel tests per wavefront: the caller takes launch_gemv's kernel.
constexpr int kG1NotApplicable = 1;
int launch_gemv1(const GemvArgs& a, int wdt, const scap_launch_cfg* cfg, hipStream_t stream);
// Two to four tokens through that kernel's two- / four-slot form; kG1NotApplicable likewise (also for another token count, bias
// folding and an input length that is not a multiple of 8).
int launch_gemv1b(const GemvArgs& a, int wdt, int flags, hipStream_t stream);
// The fused block of one token on the same kernel (two launches); kG1NotApplicable likewise.
// Two-token block: whether launch `part` (0: gate|up with the gating epilogue, 1: down reading the lists) can run on the
// two- / four-slot kernel, and that launch.  Both use the batched block kernels' list format, so the parts mix with theirs.
bool swiglu_block2_part_applies(const GemvArgs& up, const GemvArgs& down, int wdt, int part);
int launch_swiglu_block2_part(const GemvArgs& up, const GemvArgs& down, int wdt, int part, hipStream_t stream);
int launch_swiglu_block1(const GemvArgs& up, const GemvArgs& down, int wdt, int up_flags, int down_flags,
                         hipStream_t stream);

// Fused SwiGLU block: two launches (gate|up with the gating epilogue, then down reading the lists).
// `up` and `down` carry the two layers' arguments; the list pointers and m2/tau2 are set in both.
constexpr int kBlockVectorTokens = 4;  // tokens per fused-block call on the vector kernel (any weight dtype)
constexpr int kBlockMaxTokens = 16;    // ... on the matrix cores (bf16 and int8 weights)
// token slots of the block's lists for B tokens
inline int block_token_slots(int64_t B) { return B <= 1 ? 1 : (B == 2 ? 2 : (B <= 4 ? 4 : 16)); }
int launch_swiglu_block(const GemvArgs& up, const GemvArgs& down, int wdt, hipStream_t stream, int flags1 = 0);

// Interleave two [rows, F] arrays of `elem_bytes`-byte elements in groups of 4 columns: out[rows, 2F].
int launch_pack_gate_up(const void* gate, const void* up, int64_t rows, int64_t F, int elem_bytes, void* out,
                        hipStream_t stream);

// Batched tokens over bf16 or int8 weights on the matrix cores: possible from kMfmaMinTokens tokens on (the
// workspace then carries the union lists of the two-launch form), chosen by default from kMfmaAutoTokens
// (bf16) / kMfmaAutoTokensI8 (int8) tokens on.  Below that the vector kernel is as fast or faster (bf16, 4
// tokens on 14336 x 4096: 28.9 us against 28.3 us; 2 tokens: 25.1 against 27.5); with int8 weights the vector
// kernel is bound by its per-element converts from 3 tokens on (34.6 us against 20.7 us).
constexpr int kMfmaMinTokens = 2;
constexpr int kMfmaAutoTokens = 5;
constexpr int kMfmaAutoTokensI8 = 3;
int launch_gemm_mfma(const GemvArgs& a, int wdt, const scap_launch_cfg* cfg, hipStream_t stream);
// The same in one launch: each workgroup compacts its own inputs into LDS (up to 160 KB on gfx950).
// SCAP_ERR_SHAPE when the input is too long to split into LDS-sized pieces.
int launch_gemm_inline(const GemvArgs& a, int wdt, const scap_launch_cfg* cfg, hipStream_t stream, bool slots16 = false);
// The fused block's two launches on the same kernel (bf16 / int8, up to 16 tokens).
int launch_swiglu_block_inline(const GemvArgs& up, const GemvArgs& down, int wdt, hipStream_t stream);

// Fill `n` int32 words with zero using a kernel (safe to record into a HIP graph).
int launch_zero_words(int32_t* p, size_t n, hipStream_t stream);

// Zero the fixed header of a workspace (arrival counters, calibration scratch, segment counts).
int launch_workspace_init(void* workspace, size_t bytes, hipStream_t stream);

int launch_read_probe(const void* src, size_t bytes, uint32_t* out, hipStream_t stream);

// Calibration (synchronous; returns a scap_status).
int run_calibrate(const uint16_t* X, int64_t M, int xdt, float s, int est, float* m_out, float* tau_out,
                  void* workspace, hipStream_t stream);

}  // namespace scap
