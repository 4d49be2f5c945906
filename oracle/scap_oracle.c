/*
 * CPU oracle for the sparse fully-connected layer of SCAP (arXiv 2412.07174).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  Nothing in the product path may call, link or import
 * it; only the tests, the smoke check and the benchmark's "cpu_baseline" leg do.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * What it evaluates, in the paper's notation (X input, W of shape IC x OC, eta the
 * mode estimate, tau the threshold, s the target sparsity):
 *
 *   dense FC            Y = X W + b                                   (Eq. 1)
 *   pruner              keep X_ij iff |X_ij| > tau, else 0            (Eq. 2)
 *   threshold           tau = Quantile(|X_calib|, s)                  (Eq. 2, text after it)
 *   sparse FC           Y' = X' W' + b                                (Eq. 3)
 *   mode centring       Y = (X - eta) W + eta W + b                   (Eq. 4-5)
 *   fused bias          Y = (X - eta) W + b_fused, b_fused = b + eta W (Eq. 6)
 *   centred sparse FC   x_eta = x - eta; Mask = |x_eta| vs tau;
 *                       y = (x_eta * Mask) W + b_fused                (Appendix B, Alg. 3)
 *   mode estimate       mean or median of the calibration sample      (Section 3, "Determination
 *                                                                      of mode value")
 *   SwiGLU block        z = scap_fc(x; W_up) * silu(scap_fc(x; W_gate));
 *                       y = scap_fc(z; W_down)                        (Appendix B, Alg. 2)
 *   FFN sparsity        2/3 s_x + 1/3 s_gated                         (Appendix B)
 *
 * Readings of points the paper leaves open (also listed in the design notes):
 *   - the threshold comparison is the strict one of Eq. 2 (an entry equal to tau is pruned);
 *   - Alg. 3's last step multiplies the masked, centred input by W;
 *   - eta and tau are one fp32 scalar each per layer;
 *   - storage is 16-bit (fp16 / bf16); x - eta is ONE fp32 subtraction, |.| > tau an fp32
 *     compare; sums run in fp64 over ascending input channel; y is rounded to fp32 once;
 *   - the quantile is an order statistic without interpolation: with M pooled values sorted
 *     ascending and k = ceil(s*M), tau is the k-th smallest (k = 0 gives tau = 0);
 *   - the median of an even count is the mean of the two middle values (in fp64, then fp32);
 *   - NaN inputs compare false and are pruned; for sorting, NaN ranks above every number;
 *   - with several tokens each token has its own mask (Eq. 2 is elementwise); the union of
 *     the masks is reported because it is the set of weight rows a kernel has to read
 *     (Appendix C);
 *   - inside a SwiGLU block the gated product is an fp32 vector (it is never stored in 16 bits) and
 *     the last call of Alg. 2 takes it, not x, as its input;
 *   - int8 weights are symmetric with one fp16 scale per output channel: w = scale[o]*q[i,o].
 *
 * Parity unpinned: none.  The histogram mode estimator (ORACLE_MODE_HIST) is pinned, by samples
 * built by hand on a grid whose bin contents and winning bin are worked out on paper, against
 * the definition written at hist_mode() below.  That definition is itself a stand-in: the paper
 * (Section 3, "Determination of mode value") names kernel density estimation but fixes neither
 * bandwidth nor grid, so there is no printed value of the paper's own estimator to compare with;
 * the stand-in is also checked to land within one bin of the closed-form mode of synthetic laws.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_F16 0
#define ORACLE_BF16 1
#define ORACLE_I8 2
#define ORACLE_F32 3 /* activations only: plain fp32 values (the gated product inside a SwiGLU block) */

#define ORACLE_MODE_ZERO 0
#define ORACLE_MODE_MEAN 1
#define ORACLE_MODE_MEDIAN 2
#define ORACLE_MODE_HIST 3

/* ---------------------------------------------------------------- storage -> fp32 */
static float half_bits_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t out;
    if (exp == 0) {
        if (man == 0) {
            out = sign;
        } else { /* subnormal half: value = man * 2^-24, exact in fp32 */
            float f = (float)man * (1.0f / 16777216.0f);
            memcpy(&out, &f, 4);
            out |= sign;
        }
    } else if (exp == 31) {
        out = sign | 0x7F800000u | (man << 13);
    } else {
        out = sign | ((exp + 112u) << 23) | (man << 13);
    }
    float r;
    memcpy(&r, &out, 4);
    return r;
}

static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float r;
    memcpy(&r, &u, 4);
    return r;
}

float oracle_to_f32(uint16_t bits, int dt)
{
    return dt == ORACLE_BF16 ? bf16_bits_to_float(bits) : half_bits_to_float(bits);
}

static double weight_at(const void *W, int wdt, int64_t pos)
{
    if (wdt == ORACLE_I8)
        return (double)((const int8_t *)W)[pos];
    return (double)oracle_to_f32(((const uint16_t *)W)[pos], wdt);
}

/* ---------------------------------------------------------------- Alg. 3, steps 1-2 */
/* activation i of a vector stored as 16-bit codes, or as fp32 when xdt == ORACLE_F32 */
static float act_at(const void *x, int xdt, int64_t i)
{
    if (xdt == ORACLE_F32)
        return ((const float *)x)[i];
    return oracle_to_f32(((const uint16_t *)x)[i], xdt);
}

static size_t act_bytes(int xdt) { return xdt == ORACLE_F32 ? 4 : 2; }

/* d[i] = x[i] - eta (fp32), keep[i] = |d[i]| > tau (strict, Eq. 2).  Returns the count kept. */
int64_t oracle_centre_threshold(const void *x, int xdt, int64_t K, float eta, float tau,
                                float *d, uint8_t *keep)
{
    int64_t cnt = 0;
    for (int64_t i = 0; i < K; ++i) {
        volatile float xf = act_at(x, xdt, i);
        volatile float di = xf - eta; /* one IEEE fp32 subtraction */
        int k = fabsf(di) > tau;      /* NaN compares false */
        d[i] = di;
        keep[i] = (uint8_t)k;
        cnt += k;
    }
    return cnt;
}

/* ---------------------------------------------------------------- Eq. 3 / Eq. 6 / Alg. 3 step 3 */
/* Output columns [o0, o1) of one token: y[o] = b_fused[o] + scale[o] * sum_{i kept} d_i W[i,o]. */
static void fc_columns(const void *W, const uint16_t *col_scale, int64_t N, int wdt,
                       const int32_t *idx, int64_t nnz, const float *d, const float *b_fused,
                       float *y, int64_t o0, int64_t o1)
{
    int64_t n = o1 - o0;
    if (n <= 0)
        return;
    double *acc = (double *)calloc((size_t)n, sizeof(double));
    for (int64_t j = 0; j < nnz; ++j) {
        int64_t i = idx[j];
        double di = (double)d[i];
        for (int64_t o = o0; o < o1; ++o)
            acc[o - o0] += di * weight_at(W, wdt, i * N + o);
    }
    for (int64_t o = o0; o < o1; ++o) {
        double a = acc[o - o0];
        if (wdt == ORACLE_I8)
            a *= (double)half_bits_to_float(col_scale[o]);
        if (b_fused)
            a += (double)b_fused[o];
        y[o] = (float)a;
    }
    free(acc);
}

/*
 * Centred, thresholded FC for B tokens (Alg. 3 per token; Eq. 2 is elementwise over X_ij).
 *   W [K,N] K-major; x [B,K] (16-bit codes, or fp32 values for ORACLE_F32); y [B,N] fp32; idx [B,K] (ascending kept channels, first nnz[b]
 *   valid per token) or NULL; nnz [B] or NULL; union_idx [K] / union_nnz [1] or NULL.
 * nthreads > 1 splits the output columns over that many threads; the loop nest is unchanged.
 */
int oracle_sparse_fc(const void *W, const uint16_t *col_scale, int64_t K, int64_t N, int wdt,
                     const void *x, int xdt, int64_t B, float eta, float tau,
                     const float *b_fused, float *y, int32_t *idx, int32_t *nnz,
                     int32_t *union_idx, int32_t *union_nnz, int nthreads)
{
    if (!W || !x || !y || K < 1 || N < 1 || B < 1)
        return -1;
    if (wdt == ORACLE_I8 && !col_scale)
        return -1;
    float *d = (float *)malloc((size_t)K * sizeof(float));
    uint8_t *keep = (uint8_t *)malloc((size_t)K);
    uint8_t *any = (uint8_t *)calloc((size_t)K, 1);
    int32_t *list = (int32_t *)malloc((size_t)K * sizeof(int32_t));
    for (int64_t b = 0; b < B; ++b) {
        oracle_centre_threshold((const char *)x + (size_t)(b * K) * act_bytes(xdt), xdt, K, eta, tau, d, keep);
        int64_t cnt = 0;
        for (int64_t i = 0; i < K; ++i)
            if (keep[i]) {
                list[cnt++] = (int32_t)i;
                any[i] = 1;
            }
        if (idx)
            memcpy(idx + b * K, list, (size_t)cnt * sizeof(int32_t));
        if (nnz)
            nnz[b] = (int32_t)cnt;
        float *yb = y + b * N;
        if (nthreads <= 1) {
            fc_columns(W, col_scale, N, wdt, list, cnt, d, b_fused, yb, 0, N);
        } else {
#pragma omp parallel for num_threads(nthreads) schedule(static)
            for (int t = 0; t < nthreads; ++t) {
                int64_t o0 = N * t / nthreads, o1 = N * (t + 1) / nthreads;
                fc_columns(W, col_scale, N, wdt, list, cnt, d, b_fused, yb, o0, o1);
            }
        }
    }
    int64_t ucnt = 0;
    for (int64_t i = 0; i < K; ++i)
        if (any[i]) {
            if (union_idx)
                union_idx[ucnt] = (int32_t)i;
            ++ucnt;
        }
    if (union_nnz)
        *union_nnz = (int32_t)ucnt;
    free(d);
    free(keep);
    free(any);
    free(list);
    return 0;
}

/* Dense FC, Eq. 1: y[b,o] = bias[o] + sum_i x[b,i] W[i,o] over every channel, fp64 sums. */
int oracle_dense_fc(const void *W, const uint16_t *col_scale, int64_t K, int64_t N, int wdt,
                    const uint16_t *x, int xdt, int64_t B, const float *bias, float *y)
{
    if (!W || !x || !y || K < 1 || N < 1 || B < 1)
        return -1;
    if (wdt == ORACLE_I8 && !col_scale)
        return -1;
    float *xf = (float *)malloc((size_t)K * sizeof(float));
    int32_t *all = (int32_t *)malloc((size_t)K * sizeof(int32_t));
    for (int64_t i = 0; i < K; ++i)
        all[i] = (int32_t)i;
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t i = 0; i < K; ++i)
            xf[i] = oracle_to_f32(x[b * K + i], xdt);
        fc_columns(W, col_scale, N, wdt, all, K, xf, bias, y + b * N, 0, N);
    }
    free(xf);
    free(all);
    return 0;
}

/* Eq. 5-6: b_fused[o] = b[o] + eta * sum_i W[i,o]   (bias == NULL means b = 0). */
int oracle_fold_bias(const void *W, const uint16_t *col_scale, int64_t K, int64_t N, int wdt,
                     const float *bias, float eta, float *b_fused)
{
    if (!W || !b_fused || K < 1 || N < 1)
        return -1;
    if (wdt == ORACLE_I8 && !col_scale)
        return -1;
    for (int64_t o = 0; o < N; ++o) {
        double colsum = 0.0;
        for (int64_t i = 0; i < K; ++i)
            colsum += weight_at(W, wdt, i * N + o);
        if (wdt == ORACLE_I8)
            colsum *= (double)half_bits_to_float(col_scale[o]);
        double b0 = bias ? (double)bias[o] : 0.0;
        b_fused[o] = (float)(b0 + (double)eta * colsum);
    }
    return 0;
}

/* ---------------------------------------------------------------- calibration */
static int cmp_float_nan_last(const void *pa, const void *pb)
{
    float a = *(const float *)pa, b = *(const float *)pb;
    int an = isnan(a), bn = isnan(b);
    if (an || bn)
        return an - bn;
    return (a > b) - (a < b);
}

/* k-th smallest (1-indexed) of a sorted array; k is clamped to [1, M]. */
static float order_stat(const float *sorted, int64_t M, int64_t k)
{
    if (k < 1)
        k = 1;
    if (k > M)
        k = M;
    return sorted[k - 1];
}

static int64_t rank_of(double q, int64_t M)
{
    int64_t k = (int64_t)ceil(q * (double)M);
    if (k < 0)
        k = 0;
    if (k > M)
        k = M;
    return k;
}

#define HIST_BINS 2048

/* Histogram stand-in for a density-estimate mode: HIST_BINS equal bins between the 0.001 and
 * 0.999 order statistics, counts smoothed with a 5-bin box, centre of the fullest bin (lowest
 * bin on ties). */
static float hist_mode(const float *sorted, int64_t M)
{
    int64_t klo = rank_of(0.001, M), khi = rank_of(0.999, M);
    float lo = order_stat(sorted, M, klo), hi = order_stat(sorted, M, khi);
    if (!(hi > lo))
        return lo;
    double w = ((double)hi - (double)lo) / (double)HIST_BINS;
    int64_t *cnt = (int64_t *)calloc(HIST_BINS, sizeof(int64_t));
    for (int64_t j = 0; j < M; ++j) {
        float v = sorted[j];
        if (!(v >= lo && v <= hi))
            continue;
        int64_t b = (int64_t)floor(((double)v - (double)lo) / w);
        if (b > HIST_BINS - 1)
            b = HIST_BINS - 1;
        if (b < 0)
            b = 0;
        cnt[b]++;
    }
    int64_t best = -1, bestb = 0;
    for (int64_t b = 0; b < HIST_BINS; ++b) {
        int64_t s = 0;
        for (int64_t t = b - 2; t <= b + 2; ++t)
            if (t >= 0 && t < HIST_BINS)
                s += cnt[t];
        if (s > best) {
            best = s;
            bestb = b;
        }
    }
    free(cnt);
    volatile double centre = ((double)bestb + 0.5) * w;
    volatile double mode = (double)lo + centre;
    return (float)mode;
}

/*
 * eta = mode estimate of the pooled sample; tau = Quantile(|X - eta|, s)  (Eq. 2 and Section 3).
 * X [n,K] row-major 16-bit.  The pool is all n*K values of the layer input.
 */
int oracle_calibrate(const uint16_t *X, int64_t n, int64_t K, int xdt, float s, int est,
                     float *eta_out, float *tau_out)
{
    if (!X || !eta_out || !tau_out || n < 1 || K < 1)
        return -1;
    if (!(s >= 0.0f && s < 1.0f))
        return -2;
    int64_t M = n * K;
    float *v = (float *)malloc((size_t)M * sizeof(float));
    for (int64_t j = 0; j < M; ++j)
        v[j] = oracle_to_f32(X[j], xdt);

    float eta = 0.0f;
    if (est == ORACLE_MODE_MEAN) {
        double sum = 0.0;
        for (int64_t j = 0; j < M; ++j)
            sum += (double)v[j];
        eta = (float)(sum / (double)M);
    } else if (est == ORACLE_MODE_MEDIAN || est == ORACLE_MODE_HIST) {
        float *sorted = (float *)malloc((size_t)M * sizeof(float));
        memcpy(sorted, v, (size_t)M * sizeof(float));
        qsort(sorted, (size_t)M, sizeof(float), cmp_float_nan_last);
        if (est == ORACLE_MODE_MEDIAN) {
            if (M % 2 == 1) {
                eta = sorted[M / 2];
            } else {
                double a = (double)sorted[M / 2 - 1], b = (double)sorted[M / 2];
                eta = (float)((a + b) / 2.0);
            }
        } else {
            eta = hist_mode(sorted, M);
        }
        free(sorted);
    } else if (est != ORACLE_MODE_ZERO) {
        free(v);
        return -3;
    }

    /* importance |x - eta|, formed exactly as the pruner forms it */
    for (int64_t j = 0; j < M; ++j) {
        volatile float dj = v[j] - eta;
        v[j] = fabsf(dj);
    }
    qsort(v, (size_t)M, sizeof(float), cmp_float_nan_last);
    int64_t k = rank_of((double)s, M);
    *tau_out = (k == 0) ? 0.0f : v[k - 1];
    *eta_out = eta;
    free(v);
    return 0;
}

/*
 * SwiGLU feed-forward block of one token, Appendix B Alg. 2, each of its three scap_fc calls being the
 * centred form of Alg. 3 (the paper notes the two can be merged; eta = 0 and a NULL bias give Alg. 2 as
 * printed):
 *     g = scap_fc(tau_x, x, W_gate)     u = scap_fc(tau_x, x, W_up)        one mask for both
 *     z = u * silu(g)                   silu(t) = t / (1 + exp(-t))
 *     y = scap_fc(tau_z, z, W_down)     (the printed listing passes x here; the gated product is meant)
 * g and u are the fp32 outputs of the first two calls; the product is formed in fp64 and rounded once
 * to fp32; z stays fp32 (it is never stored in 16 bits), so the second pruner compares
 * |fp32(z) - eta_z| with tau_z in fp32 exactly as the first compares the input.
 * Outputs: g, u, z [F], y [N]; idx_x/nnz_x and idx_z/nnz_z as in oracle_sparse_fc (may be NULL).
 */
int oracle_swiglu_block(const void *W_gate, const uint16_t *gate_scale, const void *W_up,
                        const uint16_t *up_scale, const void *W_down, const uint16_t *down_scale,
                        int64_t K, int64_t F, int64_t N, int wdt, const void *x, int xdt,
                        float eta_x, float tau_x, const float *b_gate, const float *b_up,
                        float eta_z, float tau_z, const float *b_down,
                        float *g, float *u, float *z, float *y,
                        int32_t *idx_x, int32_t *nnz_x, int32_t *idx_z, int32_t *nnz_z, int nthreads)
{
    if (!g || !u || !z || !y)
        return -1;
    int rc = oracle_sparse_fc(W_gate, gate_scale, K, F, wdt, x, xdt, 1, eta_x, tau_x, b_gate, g,
                              idx_x, nnz_x, NULL, NULL, nthreads);
    if (rc)
        return rc;
    rc = oracle_sparse_fc(W_up, up_scale, K, F, wdt, x, xdt, 1, eta_x, tau_x, b_up, u,
                          NULL, NULL, NULL, NULL, nthreads);
    if (rc)
        return rc;
    for (int64_t i = 0; i < F; ++i) {
        double t = (double)g[i];
        double silu = t / (1.0 + exp(-t));
        z[i] = (float)((double)u[i] * silu);
    }
    return oracle_sparse_fc(W_down, down_scale, F, N, wdt, z, ORACLE_F32, 1, eta_z, tau_z, b_down, y,
                            idx_z, nnz_z, NULL, NULL, nthreads);
}

/* Appendix B: three equal-sized FCs, Up and Gate share the input sparsity s_x. */
double oracle_ffn_sparsity(double s_x, double s_gated)
{
    return (2.0 * s_x + s_gated) / 3.0;
}
