/*
 * scap.h -- C ABI of the MI355X (gfx950) library for the decode-time sparse fully-connected
 * layer of SCAP, "Statistical Calibrated Activation Pruning" (arXiv 2412.07174).
 *
 * The layer, in the paper's notation (Section 2 Eq. 1-3, Section 3 Eq. 4-6, Appendix B Alg. 3):
 *
 *     d    = x - eta                      eta: per-layer scalar mode estimate ("m" below)
 *     keep = |d| > tau                    tau: per-layer scalar threshold (strict compare, Eq. 2)
 *     y    = (d * keep) W + b_fused       b_fused = b + eta * (column sums of W)      (Eq. 6)
 *
 * W is the paper's IC x OC matrix stored K-major: element (i, o) of a K x N matrix is at
 * W[i*N + o], so a pruned input channel is one contiguous row that is never fetched.
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are HIP device pointers owned by the caller; pointers marked HOST are
 *     ordinary host pointers.  The library allocates and frees no device memory and keeps no state
 *     between calls other than what lives in the caller's workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls marked ASYNC only
 *     enqueue work on it and return; calls marked SYNC wait for the stream before returning.
 *   - Every call returns a scap_status.  Arguments are validated on the host before anything is
 *     enqueued; on an error nothing is launched and no output is written.  No call throws, aborts
 *     or prints.
 *   - Device pointers of W, x, y, bias, col_scale and the workspace must be 16-byte aligned.  N must
 *     be a multiple of 8 (16-bit weights) or 16 (int8 weights).  A layer has at most 2^20 input channels
 *     and 2^19 output columns (SCAP_ERR_SHAPE beyond; scap_calibrate pools up to 2^34 values of rows up to
 *     2^24 wide).  An explicit launch shape that cannot hold such a layer is SCAP_ERR_CONFIG.
 *   - A workspace is a caller-allocated device buffer of at least scap_workspace_bytes(...) bytes
 *     that has been passed once to scap_workspace_init().  Kernels leave it ready for the next
 *     call.  Two calls that share one workspace must not overlap in time (use one workspace per
 *     stream).
 */
#ifndef SCAP_H
#define SCAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SCAP_OK = 0,
    SCAP_ERR_NULL = -1,      /* a required pointer is NULL */
    SCAP_ERR_SHAPE = -2,     /* K, N, B or n out of range, or N not a multiple of the vector width */
    SCAP_ERR_DTYPE = -3,     /* unknown dtype / estimator code, or a combination not supported */
    SCAP_ERR_ALIGN = -4,     /* a device pointer is not 16-byte aligned */
    SCAP_ERR_VALUE = -5,     /* tau negative or NaN, m not finite, target sparsity outside [0, 1) */
    SCAP_ERR_WORKSPACE = -6, /* workspace NULL or smaller than scap_workspace_bytes() */
    SCAP_ERR_HIP = -7,       /* a HIP runtime call or launch reported an error */
    SCAP_ERR_UNIMPL = -8,    /* valid request that this build does not implement */
    SCAP_ERR_CONFIG = -9     /* invalid scap_launch_cfg */
} scap_status;

/* storage types of weights and activations */
typedef enum {
    SCAP_F16 = 0,         /* IEEE binary16 */
    SCAP_BF16 = 1,        /* bfloat16 */
    SCAP_I8_COLSCALE = 2  /* weights only: symmetric int8, w[i,o] = col_scale[o] * q[i,o], fp16 scales */
} scap_dtype;

/* mode estimators (Section 3, "Determination of mode value") */
typedef enum {
    SCAP_MODE_ZERO = 0,   /* m = 0: inputs already centred (GLU blocks, Section 4 "Implementation") */
    SCAP_MODE_MEAN = 1,   /* mean of the pooled sample */
    SCAP_MODE_MEDIAN = 2, /* median of the pooled sample (mean of the two middle values if even) */
    SCAP_MODE_HIST = 3    /* histogram stand-in for a density-estimate mode: 2048 bins between the
                             0.001 and 0.999 order statistics, 5-bin box smoothing, fullest bin */
} scap_mode_est;

/* Optional launch shape of the kernels (for tuning sweeps and tests).  Zero fields mean "choose".
 * lanes_per_row selects the kernel: 64 or 32 = the vector kernel (column tile = lanes_per_row x 8 columns,
 * x 16 for int8; more than 4 tokens: 64 only; one token with 8 wavefronts and 64 lanes per row, the default, runs
 * the one-token kernel unless flags says otherwise or a workgroup would own more than 2048 channels); 16 = the single-launch matrix-core kernel and 1 = the two-launch
 * matrix-core form with its lists in the workspace (both: 2..16 tokens over bf16 or int8 weights; the
 * single-launch kernel also 5..16 tokens over fp16 weights; there waves_per_group must be 0 or 8 -- the
 * two-launch form also takes 16 with bf16 -- and rows_per_group is a multiple of 64, rounded up to whole
 * 512-channel list segments by the two-launch form, whose unroll (1, 2, 4; int8: 1, 2) counts 16-row blocks
 * in flight per wavefront).  By default batches of 5 or more tokens (3 or more over int8 weights) run on
 * the matrix cores. */
typedef struct {
    int32_t waves_per_group; /* 4, 8 or 16 wavefronts per workgroup */
    int32_t rows_per_group;  /* input channels owned by one workgroup; multiple of 64 */
    int32_t unroll;          /* weight rows in flight per wavefront: 4, 8 or 16 */
    int32_t lanes_per_row;   /* 64, 32, 16 or 1: see above */
    int32_t flags;           /* bit 0 (SCAP_CFG_DEVICE_SCOPE_LOADS): the one-token kernel fetches split-K partial sums
                                with device-coherent loads even when all their writers ran on the reader's own
                                accelerator die (results are identical; for tests and measurements);
                                bit 1 (SCAP_CFG_GENERAL_KERNEL): one to four tokens through the general kernels
                                instead of the one-token kernel and its two- and four-slot forms;
                                bit 2 (SCAP_CFG_ACCUMULATE): NOT a tuning knob -- y += result instead of y = result.
                                y must hold the addend (a residual stream, say) when the call is enqueued; every
                                workgroup adds its share with fp32 atomic adds, which removes the split-K hand-over
                                (about 1.5 us of a one-token launch) and with it the fixed order of the additions:
                                the last bits of y may differ from run to run.  One token through the one-token
                                kernel only (sparse or dense mode); SCAP_ERR_CONFIG where that kernel does not
                                apply.  idx_out / nnz_out are exact as always;
                                bit 3 (SCAP_CFG_PARTIAL_SUMS): the one-token kernel hands its split-K partial sums
                                over as fp32 values that the last arrival collects and adds in split order, instead
                                of adding them as fixed-point integers with one atomic per column (both are
                                bit-reproducible; they differ in the last bits of y).  Bit 0 implies it;
                                bit 4 (SCAP_CFG_PARK_SLICES, scap_swiglu_block_ex only, for tests): the first launch
                                of a one-token block gates every slice by the way a slice takes when its columns were
                                finished by more than one wavefront (through memory) */
} scap_launch_cfg;
#define SCAP_CFG_DEVICE_SCOPE_LOADS 1
#define SCAP_CFG_GENERAL_KERNEL 2
#define SCAP_CFG_ACCUMULATE 4
#define SCAP_CFG_PARTIAL_SUMS 8
#define SCAP_CFG_PARK_SLICES 16

/* Static, NUL-terminated description of a status code.  Never freed. */
const char* scap_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int scap_version(void);

/*
 * Bytes of workspace that scap_sparse_fc / scap_dense_fc / scap_fold_bias need for a K x N layer and
 * B tokens, and that scap_calibrate needs for an n x K sample (pass N = 0, B = n).  Returns 0 for
 * arguments out of range.
 */
size_t scap_workspace_bytes(int64_t K, int64_t N, int64_t B);

/*
 * ASYNC.  Prepares a freshly allocated workspace: clears its arrival counters with a fill kernel.
 * Must be called once before the workspace is first used, and again after any call that failed
 * with SCAP_ERR_HIP.
 *   workspace  DEVICE, 16-byte aligned, workspace_bytes >= 4096.
 */
int scap_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * SYNC, offline.  Calibration of one layer (Eq. 2: tau = Quantile(|X_calib|, s); Section 3: the mode
 * is estimated first and the threshold is taken on the centred sample).
 *   X_calib          DEVICE  [n, K] row-major activations captured at the layer input, dtype xdt
 *                            (SCAP_F16 or SCAP_BF16); all n*K values are pooled.
 *   target_sparsity  s in [0, 1).
 *   est              scap_mode_est.
 *   m_out, tau_out   HOST    receive the mode estimate and the threshold (fp32).
 *                            tau is the k-th smallest of |fp32(x) - m| over the pool, k = ceil(s*n*K),
 *                            no interpolation (k = 0 gives tau = 0); |.| is formed exactly as
 *                            scap_sparse_fc forms it, so the sample's own sparsity is >= s.
 *   workspace        DEVICE  scap_workspace_bytes(K, 0, n) bytes, initialised (a layer's workspace is large
 *                            enough as well).
 * The sample is read in one pass that counts the occurrences of each 16-bit code; the statistics are then
 * exact functions of those counts.  NaN samples rank above every number.
 */
int scap_calibrate(const void* X_calib, int64_t n, int64_t K, int xdt, float target_sparsity, int est,
                   float* m_out, float* tau_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ASYNC, offline.  Fused bias of Eq. 6: b_fused[o] = bias[o] + m * sum_i W[i,o].
 *   W            DEVICE  [K, N] K-major, dtype wdt.
 *   col_scale    DEVICE  fp16 [N] when wdt == SCAP_I8_COLSCALE, else NULL.
 *   bias         DEVICE  fp32 [N] or NULL (= zeros; Alg. 2 is bias-free).
 *   b_fused_out  DEVICE  fp32 [N].
 */
int scap_fold_bias(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const float* bias,
                   float m, float* b_fused_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ASYNC, the decode-time hot path (Alg. 3 with the strict compare of Eq. 2; Eq. 3 / Eq. 6).
 * One launch: centre, threshold, compact the kept channels, read only their weight rows, reduce (two
 * launches -- union of the masks, then the gathered product -- only for a batch whose input is too long for a
 * workgroup's share of it to fit LDS: more than about 600 000 channels).
 *   W, col_scale   as in scap_fold_bias.
 *   x              DEVICE  [B, K] row-major, dtype xdt (SCAP_F16 or SCAP_BF16).
 *   m, tau         layer constants from scap_calibrate (tau >= 0, both finite).
 *   b_fused        DEVICE  fp32 [N] from scap_fold_bias, or NULL (= zeros).
 *   y              DEVICE  fp32 [B, N]; fully overwritten.
 *   idx_out        DEVICE  int32 [B, K] or NULL: token b's kept channels, ascending, in
 *                          idx_out[b*K .. b*K + nnz_out[b]); entries past nnz are unspecified.
 *   nnz_out        DEVICE  int32 [B] or NULL (required when idx_out is given).
 *   union_nnz_out  DEVICE  int32 [1] or NULL: number of distinct weight rows read (union of the B
 *                          masks, Appendix C; equals nnz_out[0] for B = 1).
 * Each token has its own mask (Eq. 2 is elementwise); a row in the union contributes zero to tokens
 * that pruned it.  d = fp32(x) - m is one fp32 subtraction; products accumulate in fp32.
 * NaN inputs are pruned (the compare is false); infinities are kept and propagate.
 * B is limited to SCAP_MAX_TOKENS.
 */
#define SCAP_MAX_TOKENS 16
int scap_sparse_fc(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                   int64_t B, float m, float tau, const float* b_fused, float* y, int32_t* idx_out,
                   int32_t* nnz_out, int32_t* union_nnz_out, void* workspace, size_t workspace_bytes,
                   void* stream);

/*
 * ASYNC.  scap_sparse_fc for callers that cannot allocate device memory or pass a workspace: code recorded into a
 * HIP graph, tight serving loops, harnesses that forbid allocation.  Arguments and results as scap_sparse_fc
 * (same kernels, bit-identical outputs); the scratch is an array of SCAP_STATIC_SCRATCH_BYTES bytes inside the
 * library's code object, one copy per GPU, held until the process ends.  The call allocates and frees nothing.
 *   - Refused with SCAP_ERR_WORKSPACE when scap_workspace_bytes(K, N, B) exceeds SCAP_STATIC_SCRATCH_BYTES
 *     (one token: any layer up to about 300 000 output columns; four tokens: up to 65536 columns and about
 *     50 000 input channels; 16 tokens never fit).  Nothing is launched then.
 *   - The device that is current when the call is made must be the stream's device.  The first call on a
 *     device (and the first after a call that failed with SCAP_ERR_HIP) looks up the array's address and clears
 *     its header with a fill kernel on `stream`.
 *   - All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in time on one GPU
 *     race and give wrong results.  Serialise them (one stream, or events), or use scap_sparse_fc with one
 *     workspace per stream.
 */
#define SCAP_STATIC_SCRATCH_BYTES (24 * 1024 * 1024)
int scap_sparse_fc_static(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x,
                          int xdt, int64_t B, float m, float tau, const float* b_fused, float* y,
                          int32_t* idx_out, int32_t* nnz_out, int32_t* union_nnz_out, void* stream);

/* Same as scap_sparse_fc with an explicit launch shape (cfg may be NULL). */
int scap_sparse_fc_ex(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x,
                      int xdt, int64_t B, float m, float tau, const float* b_fused, float* y, int32_t* idx_out,
                      int32_t* nnz_out, int32_t* union_nnz_out, void* workspace, size_t workspace_bytes,
                      void* stream, const scap_launch_cfg* cfg);

/*
 * ASYNC.  Dense baseline on the same kernels (Eq. 1): y[b,o] = bias[o] + sum_i x[b,i] W[i,o] over every
 * channel, nothing centred or pruned.  Arguments as in scap_sparse_fc; cfg may be NULL.
 */
int scap_dense_fc(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                  int64_t B, const float* bias, float* y, void* workspace, size_t workspace_bytes, void* stream,
                  const scap_launch_cfg* cfg);

/*
 * ASYNC, offline.  Column layout of the fused block's first matrix: interleaves two row-major [rows, F]
 * arrays in groups of 4 columns, out[r, 8j + 0..3] = gate[r, 4j + 0..3], out[r, 8j + 4..7] = up[r, 4j + 0..3].
 * Serves the weights (rows = K; elem_bytes 2, or 1 for int8), their column scales (rows = 1, elem_bytes 2)
 * and biases (rows = 1, elem_bytes 4).  Gate and up share one input mask (Section 4, "Implementation"), so
 * the pair is one layer with 2F columns; this order puts matching gate and up columns in one 16-byte load.
 *   gate, up, out  DEVICE, 16-byte aligned; F a multiple of 4; out must not overlap the inputs.
 */
int scap_pack_gate_up(const void* gate, const void* up, int64_t rows, int64_t F, int elem_bytes, void* out,
                      void* stream);

/* Bytes of workspace scap_swiglu_block needs (hidden size K, intermediate size F, output size N, B tokens);
 * such a workspace also serves every other call on layers no larger than the block's two.  0 = out of range. */
size_t scap_swiglu_workspace_bytes(int64_t K, int64_t F, int64_t N, int64_t B);

/*
 * ASYNC.  SwiGLU feed-forward block of 1 to 16 tokens (Appendix B, Alg. 2; each scap_fc in the centred form of
 * Alg. 3):   z = scap_fc(x; W_up) * silu(scap_fc(x; W_gate)),   y = scap_fc(z; W_down)
 * in two launches.  The first reads the kept rows of the interleaved gate|up matrix; the workgroup that
 * completes a column tile forms z in fp32 (silu(t) = t / (1 + exp(-t))), subtracts m_z, applies the strict
 * threshold tau_z and leaves the kept channels compacted in the workspace.  The second takes those lists as
 * its input.  z is never rounded to 16 bits.
 *   W_gu, gu_scale   DEVICE  [K, 2F] from scap_pack_gate_up (and its packed fp16 scales for int8, else NULL).
 *   W_down, down_scale DEVICE [F, N] K-major (scales for int8, else NULL); same dtype wdt as W_gu.
 *   x                DEVICE  [B, K], dtype xdt.   B <= 16 (matrix cores from 5 tokens, int8 from 3); each token
 *                            has its own masks, a weight row is read when any token keeps its channel
 *                            (Appendix C).
 *   m_x, tau_x       constants of the block input;  b_gu_fused  DEVICE fp32 [2F] packed fused bias or NULL
 *                    (scap_fold_bias on W_gu with the packed bias gives it).
 *   m_z, tau_z       constants of the gated product;  b_down_fused  DEVICE fp32 [N] or NULL.
 *   y                DEVICE  fp32 [B, N], fully overwritten.
 *   z_out            DEVICE  fp32 [B, F] or NULL: the gated product before centring.
 *   idx_z_out        DEVICE  int32 [B, F] or NULL: token b's kept channels of z, ascending, in
 *                            idx_z_out[b*F .. b*F + nnz_z_out[b]).
 *   nnz_z_out        DEVICE  int32 [B] or NULL (required with idx_z_out).
 *   workspace        scap_swiglu_workspace_bytes(K, F, N, B) bytes, initialised.
 * F must be a multiple of 4 (8 for int8) and at most 262144.
 */
int scap_swiglu_block(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale, int64_t K,
                      int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x, float tau_x,
                      const float* b_gu_fused, float m_z, float tau_z, const float* b_down_fused, float* y,
                      float* z_out, int32_t* idx_z_out, int32_t* nnz_z_out, void* workspace, size_t workspace_bytes,
                      void* stream);

/* Same as scap_swiglu_block with launch flags for its one-token form (cfg may be NULL): of cfg only the flags
 * SCAP_CFG_PARTIAL_SUMS and SCAP_CFG_PARK_SLICES (B == 1) and SCAP_CFG_GENERAL_KERNEL (B <= 4: both launches on the
 * general kernels instead of the one-token kernel and its two- and four-slot forms) are read.  For tests and measurements. */
int scap_swiglu_block_ex(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale, int64_t K,
                         int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x, float tau_x,
                         const float* b_gu_fused, float m_z, float tau_z, const float* b_down_fused, float* y,
                         float* z_out, int32_t* idx_z_out, int32_t* nnz_z_out, void* workspace, size_t workspace_bytes,
                         void* stream, const scap_launch_cfg* cfg);

/*
 * ASYNC.  The same block of ONE token with its output ADDED to y: y[o] += block(x)[o], y holding the residual
 * stream when the call is enqueued (the feed-forward block of a decoder layer ends in that addition).  The down
 * launch then adds every workgroup's share to y with fp32 atomic adds instead of collecting split-K partial sums:
 * one dependent memory round trip instead of three at the end of the block, and no fixed order of the additions
 * (the last bits of y may differ from run to run).  Arguments as in scap_swiglu_block; B must be 1 and both layers
 * must fit the one-token kernel (SCAP_ERR_CONFIG otherwise).  z_out, idx_z_out and nnz_z_out are exact as always.
 */
int scap_swiglu_block_residual(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale,
                               int64_t K, int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x,
                               float tau_x, const float* b_gu_fused, float m_z, float tau_z,
                               const float* b_down_fused, float* y, float* z_out, int32_t* idx_z_out,
                               int32_t* nnz_z_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ASYNC.  Streaming-read probe used to measure the HBM read ceiling of the box: reads `bytes` bytes at
 * `src` (DEVICE, 16-byte aligned, bytes a multiple of 16) with 2048 workgroups and stores one uint32
 * checksum per workgroup to out (DEVICE, uint32 [SCAP_PROBE_SLOTS]).
 */
#define SCAP_PROBE_SLOTS 2048
int scap_read_probe(const void* src, size_t bytes, uint32_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SCAP_H */
