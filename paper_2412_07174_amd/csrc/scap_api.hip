// extern "C" entry points of libscap: argument validation and dispatch.  See include/scap.h.
#include <math.h>

#include <mutex>

#include "scap_internal.hpp"

using namespace scap;

namespace {

constexpr int64_t kMaxK = (int64_t)1 << 20;  // input channels of a layer
constexpr int64_t kMaxN = (int64_t)1 << 19;  // output columns of a layer

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool weight_dtype_ok(int wdt) { return wdt == SCAP_F16 || wdt == SCAP_BF16 || wdt == SCAP_I8_COLSCALE; }
bool act_dtype_ok(int xdt) { return xdt == SCAP_F16 || xdt == SCAP_BF16; }

int check_layer(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt) {
    if (!W) return SCAP_ERR_NULL;
    if (!weight_dtype_ok(wdt)) return SCAP_ERR_DTYPE;
    if (wdt == SCAP_I8_COLSCALE && !col_scale) return SCAP_ERR_NULL;
    if (K < 1 || N < 1 || K > kMaxK || N > kMaxN) return SCAP_ERR_SHAPE;
    const int64_t vec = (wdt == SCAP_I8_COLSCALE) ? 16 : 8;
    if (N % vec != 0) return SCAP_ERR_SHAPE;
    if (!aligned16(W) || (col_scale && !aligned16(col_scale))) return SCAP_ERR_ALIGN;
    return SCAP_OK;
}

int check_workspace(void* ws, size_t bytes, int64_t K, int64_t N, int64_t B) {
    if (!ws) return SCAP_ERR_WORKSPACE;
    if (!aligned16(ws)) return SCAP_ERR_ALIGN;
    const size_t need = scap_workspace_bytes(K, N, B);
    if (need == 0 || bytes < need) return SCAP_ERR_WORKSPACE;
    return SCAP_OK;
}

size_t union_list_offset(int64_t N, int64_t B) { return kOffPartial + 4 * (size_t)B * partial_capacity(N); }

void fill_workspace_ptrs(GemvArgs& a, void* ws, int64_t K, int64_t N, int64_t B) {
    char* base = static_cast<char*>(ws);
    a.counters = reinterpret_cast<int32_t*>(base + kOffCounters);
    a.seg_cnt = reinterpret_cast<int32_t*>(base + kOffSegCnt);
    a.fx_acc = reinterpret_cast<unsigned long long*>(base + kOffFx);
    a.partial = reinterpret_cast<float*>(base + kOffPartial);
    a.u_idx = nullptr;
    a.u_d = nullptr;
    if (B >= kMfmaMinTokens) {
        char* lists = base + union_list_offset(N, B);
        a.u_d = reinterpret_cast<float*>(lists);
        a.u_idx = reinterpret_cast<int32_t*>(lists + union_list_entries(K) * 64);
    }
}

// argument checks of an FC call, workspace apart
int check_fc_args(int mode, const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                  int64_t B, float m, float tau, const float* bias, const float* y, const int32_t* idx_out,
                  const int32_t* nnz_out) {
    const int rc = check_layer(W, col_scale, K, N, wdt);
    if (rc != SCAP_OK) return rc;
    if (!y) return SCAP_ERR_NULL;
    if (mode != kModeFold) {
        if (!x) return SCAP_ERR_NULL;
        if (!act_dtype_ok(xdt)) return SCAP_ERR_DTYPE;
        if (!aligned16(x)) return SCAP_ERR_ALIGN;
    }
    if (B < 1 || B > SCAP_MAX_TOKENS) return SCAP_ERR_SHAPE;
    if (!aligned16(y) || (bias && !aligned16(bias))) return SCAP_ERR_ALIGN;
    if (idx_out && !nnz_out) return SCAP_ERR_NULL;
    if (mode == kModeSparse) {
        if (!(tau >= 0.f) || !isfinite(tau) || !isfinite(m)) return SCAP_ERR_VALUE;
    } else if (mode == kModeFold) {
        if (!isfinite(m)) return SCAP_ERR_VALUE;
    }
    return SCAP_OK;
}

int fc_common(int mode, const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
              int64_t B, float m, float tau, const float* bias, float* y, int32_t* idx_out, int32_t* nnz_out,
              int32_t* union_nnz_out, void* workspace, size_t workspace_bytes, void* stream, const scap_launch_cfg* cfg) {
    int rc = check_fc_args(mode, W, col_scale, K, N, wdt, x, xdt, B, m, tau, bias, y, idx_out, nnz_out);
    if (rc != SCAP_OK) return rc;
    rc = check_workspace(workspace, workspace_bytes, K, N, B);
    if (rc != SCAP_OK) return rc;

    GemvArgs a{};
    a.W = W;
    a.col_scale = static_cast<const uint16_t*>(col_scale);
    a.x = static_cast<const uint16_t*>(x);
    a.bias = bias;
    a.y = y;
    a.idx_out = idx_out;
    a.nnz_out = nnz_out;
    a.union_nnz_out = union_nnz_out;
    a.K = (int)K;
    a.N = (int)N;
    a.B = (int)B;
    a.mode = mode;
    a.xdt = xdt;
    a.m = m;
    a.tau = tau;
    fill_workspace_ptrs(a, workspace, K, N, B);
    return launch_gemv(a, wdt, cfg, static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------------------------------------
// Scratch of scap_sparse_fc_static: the workspace of a call, held in the code object instead of a caller's
// allocation.  Each GPU that loads the library has its own copy at its own address; host code never uses the
// array's name as an address, only what hipGetSymbolAddress returned for the current device.
static __device__ __align__(256) unsigned char scratch[SCAP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct StaticScratch {
    void* ptr = nullptr;   // device address of `scratch` on this GPU
    bool clean = false;    // header (arrival counters, segment counts) known to be zero
};
StaticScratch g_static[kMaxDevices];
std::mutex g_static_mutex;

// Address of the current device's scratch, its header cleared if it may be dirty.  SCAP_ERR_HIP on failure.
int static_scratch(hipStream_t stream, void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SCAP_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticScratch& st = g_static[dev];
    if (st.ptr == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SCAP_ERR_HIP;
        st.ptr = p;
    }
    if (!st.clean) {
        // a fill kernel, not hipMemsetAsync: the call may be recorded into a HIP graph
        const int rc = launch_workspace_init(st.ptr, SCAP_STATIC_SCRATCH_BYTES, stream);
        if (rc != SCAP_OK) return rc;
        st.clean = true;
    }
    *out = st.ptr;
    return SCAP_OK;
}

void static_scratch_failed() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    g_static[dev].clean = false;
}

constexpr int64_t kMaxGated = 262144;  // channels of the gated product: 4096 segments of 64

size_t block_list_offset(int64_t F, int64_t N, int64_t B) {
    const size_t c1 = partial_capacity(2 * F), c2 = partial_capacity(N);
    return kOffPartial + 4 * (size_t)B * (c1 > c2 ? c1 : c2);
}

}  // namespace

extern "C" {

const char* scap_status_string(int status) {
    switch (status) {
        case SCAP_OK: return "ok";
        case SCAP_ERR_NULL: return "a required pointer is NULL";
        case SCAP_ERR_SHAPE: return "shape out of range or N not a multiple of the vector width";
        case SCAP_ERR_DTYPE: return "unknown or unsupported dtype / estimator code";
        case SCAP_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case SCAP_ERR_VALUE: return "tau negative or NaN, m not finite, or sparsity outside [0,1)";
        case SCAP_ERR_WORKSPACE: return "workspace missing or too small";
        case SCAP_ERR_HIP: return "HIP runtime error";
        case SCAP_ERR_UNIMPL: return "not implemented in this build";
        case SCAP_ERR_CONFIG: return "invalid launch configuration";
    }
    return "unknown status";
}

int scap_version(void) { return 100; }

size_t scap_workspace_bytes(int64_t K, int64_t N, int64_t B) {
    if (K < 1 || N < 0 || B < 1) return 0;
    if (N == 0) return kCalibBytes;  // calibration only: fixed header + the code histogram
    if (K > kMaxK || N > kMaxN || B > SCAP_MAX_TOKENS) return 0;
    return union_list_offset(N, B) + (B >= kMfmaMinTokens ? union_list_entries(K) * 68 : 0);
}

int scap_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace) return SCAP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SCAP_ERR_ALIGN;
    if (workspace_bytes < 4096) return SCAP_ERR_WORKSPACE;
    return launch_workspace_init(workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int scap_calibrate(const void* X_calib, int64_t n, int64_t K, int xdt, float target_sparsity, int est, float* m_out,
                   float* tau_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!X_calib || !m_out || !tau_out) return SCAP_ERR_NULL;
    if (!act_dtype_ok(xdt)) return SCAP_ERR_DTYPE;
    if (est < SCAP_MODE_ZERO || est > SCAP_MODE_HIST) return SCAP_ERR_DTYPE;
    if (n < 1 || K < 1 || K > ((int64_t)1 << 24) || n > ((int64_t)1 << 34) / K) return SCAP_ERR_SHAPE;
    if (!(target_sparsity >= 0.f && target_sparsity < 1.f)) return SCAP_ERR_VALUE;
    if (!aligned16(X_calib)) return SCAP_ERR_ALIGN;
    if (!workspace || workspace_bytes < kCalibBytes) return SCAP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SCAP_ERR_ALIGN;
    return run_calibrate(static_cast<const uint16_t*>(X_calib), n * K, xdt, target_sparsity, est, m_out, tau_out,
                         workspace, static_cast<hipStream_t>(stream));
}

int scap_fold_bias(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const float* bias, float m,
                   float* b_fused_out, void* workspace, size_t workspace_bytes, void* stream) {
    return fc_common(kModeFold, W, col_scale, K, N, wdt, nullptr, SCAP_BF16, 1, m, 0.f, bias, b_fused_out, nullptr,
                     nullptr, nullptr, workspace, workspace_bytes, stream, nullptr);
}

int scap_sparse_fc_ex(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                      int64_t B, float m, float tau, const float* b_fused, float* y, int32_t* idx_out,
                      int32_t* nnz_out, int32_t* union_nnz_out, void* workspace, size_t workspace_bytes, void* stream,
                      const scap_launch_cfg* cfg) {
    return fc_common(kModeSparse, W, col_scale, K, N, wdt, x, xdt, B, m, tau, b_fused, y, idx_out, nnz_out,
                     union_nnz_out, workspace, workspace_bytes, stream, cfg);
}

int scap_sparse_fc(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                   int64_t B, float m, float tau, const float* b_fused, float* y, int32_t* idx_out, int32_t* nnz_out,
                   int32_t* union_nnz_out, void* workspace, size_t workspace_bytes, void* stream) {
    return fc_common(kModeSparse, W, col_scale, K, N, wdt, x, xdt, B, m, tau, b_fused, y, idx_out, nnz_out,
                     union_nnz_out, workspace, workspace_bytes, stream, nullptr);
}

int scap_sparse_fc_static(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                          int64_t B, float m, float tau, const float* b_fused, float* y, int32_t* idx_out,
                          int32_t* nnz_out, int32_t* union_nnz_out, void* stream) {
    int rc = check_fc_args(kModeSparse, W, col_scale, K, N, wdt, x, xdt, B, m, tau, b_fused, y, idx_out, nnz_out);
    if (rc != SCAP_OK) return rc;
    // a layer and batch whose workspace would not fit the static scratch is refused before anything is touched
    const size_t need = scap_workspace_bytes(K, N, B);
    if (need == 0) return SCAP_ERR_SHAPE;
    if (need > (size_t)SCAP_STATIC_SCRATCH_BYTES) return SCAP_ERR_WORKSPACE;
    void* ws = nullptr;
    rc = static_scratch(static_cast<hipStream_t>(stream), &ws);
    if (rc != SCAP_OK) return rc;
    rc = fc_common(kModeSparse, W, col_scale, K, N, wdt, x, xdt, B, m, tau, b_fused, y, idx_out, nnz_out,
                   union_nnz_out, ws, SCAP_STATIC_SCRATCH_BYTES, stream, nullptr);
    if (rc == SCAP_ERR_HIP) static_scratch_failed();
    return rc;
}

int scap_dense_fc(const void* W, const void* col_scale, int64_t K, int64_t N, int wdt, const void* x, int xdt,
                  int64_t B, const float* bias, float* y, void* workspace, size_t workspace_bytes, void* stream,
                  const scap_launch_cfg* cfg) {
    return fc_common(kModeDense, W, col_scale, K, N, wdt, x, xdt, B, 0.f, 0.f, bias, y, nullptr, nullptr, nullptr,
                     workspace, workspace_bytes, stream, cfg);
}

int scap_pack_gate_up(const void* gate, const void* up, int64_t rows, int64_t F, int elem_bytes, void* out,
                      void* stream) {
    if (!gate || !up || !out) return SCAP_ERR_NULL;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4) return SCAP_ERR_DTYPE;
    if (rows < 1 || F < 4 || F % 4 != 0 || F > ((int64_t)1 << 24) || rows > ((int64_t)1 << 24)) return SCAP_ERR_SHAPE;
    if (!aligned16(gate) || !aligned16(up) || !aligned16(out)) return SCAP_ERR_ALIGN;
    return launch_pack_gate_up(gate, up, rows, F, elem_bytes, out, static_cast<hipStream_t>(stream));
}

size_t scap_swiglu_workspace_bytes(int64_t K, int64_t F, int64_t N, int64_t B) {
    if (K < 1 || F < 1 || N < 1 || B < 1 || B > SCAP_MAX_TOKENS) return 0;
    if (K > kMaxK || F > kMaxGated || N > kMaxN) return 0;
    const size_t segs = (size_t)((F + 63) / 64);
    const size_t bt = (size_t)block_token_slots(B);
    size_t bytes = block_list_offset(F, N, B) + segs * 64 * 4 * (1 + bt) + align_up(segs * 4 * (1 + bt), 256);
    const size_t a = scap_workspace_bytes(K, 2 * F, B), b = scap_workspace_bytes(F, N, B);
    if (bytes < a) bytes = a;
    if (bytes < b) bytes = b;
    return bytes;
}

}  // extern "C"

namespace {
// both block entry points; residual: y += block output (one token, the one-token kernel's atomic-add epilogue)
int block_common(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale, int64_t K,
                 int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x, float tau_x,
                 const float* b_gu_fused, float m_z, float tau_z, const float* b_down_fused, float* y, float* z_out,
                 int32_t* idx_z_out, int32_t* nnz_z_out, void* workspace, size_t workspace_bytes, void* stream,
                 bool residual, int flags1) {
    if (F < 1 || F > kMaxGated) return SCAP_ERR_SHAPE;
    int rc = check_layer(W_gu, gu_scale, K, 2 * F, wdt);
    if (rc != SCAP_OK) return rc;
    rc = check_layer(W_down, down_scale, F, N, wdt);
    if (rc != SCAP_OK) return rc;
    if (F % 4 != 0) return SCAP_ERR_SHAPE;
    if (!x || !y) return SCAP_ERR_NULL;
    if (!act_dtype_ok(xdt)) return SCAP_ERR_DTYPE;
    if (B < 1 || B > SCAP_MAX_TOKENS) return SCAP_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y) || (b_gu_fused && !aligned16(b_gu_fused)) ||
        (b_down_fused && !aligned16(b_down_fused)) || (z_out && !aligned16(z_out)))
        return SCAP_ERR_ALIGN;
    if (idx_z_out && !nnz_z_out) return SCAP_ERR_NULL;
    if (!(tau_x >= 0.f) || !isfinite(tau_x) || !isfinite(m_x)) return SCAP_ERR_VALUE;
    if (!(tau_z >= 0.f) || !isfinite(tau_z) || !isfinite(m_z)) return SCAP_ERR_VALUE;
    if (!workspace) return SCAP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SCAP_ERR_ALIGN;
    const size_t need = scap_swiglu_workspace_bytes(K, F, N, B);
    if (need == 0 || workspace_bytes < need) return SCAP_ERR_WORKSPACE;

    char* base = static_cast<char*>(workspace);
    const size_t segs = (size_t)((F + 63) / 64);
    char* lists = base + block_list_offset(F, N, B);

    GemvArgs up{};
    up.W = W_gu;
    up.col_scale = static_cast<const uint16_t*>(gu_scale);
    up.x = static_cast<const uint16_t*>(x);
    up.bias = b_gu_fused;
    up.K = (int)K;
    up.N = (int)(2 * F);
    up.B = (int)B;
    up.mode = kModeSparse;
    up.xdt = xdt;
    up.m = m_x;
    up.tau = tau_x;
    up.counters = reinterpret_cast<int32_t*>(base + kOffCounters);
    up.seg_cnt = reinterpret_cast<int32_t*>(base + kOffSegCnt);
    up.fx_acc = reinterpret_cast<unsigned long long*>(base + kOffFx);
    up.partial = reinterpret_cast<float*>(base + kOffPartial);
    up.m2 = m_z;
    up.tau2 = tau_z;
    up.z_out = z_out;
    const size_t bt = (size_t)block_token_slots(B);
    up.zl_d = reinterpret_cast<float*>(lists);
    up.zl_idx = reinterpret_cast<int32_t*>(lists + segs * 256 * bt);
    up.zl_cnt = reinterpret_cast<int32_t*>(lists + segs * 256 * (bt + 1));
    up.F = (int)F;

    GemvArgs dn = up;
    dn.W = W_down;
    dn.col_scale = static_cast<const uint16_t*>(down_scale);
    dn.x = nullptr;
    dn.bias = b_down_fused;
    dn.y = y;
    dn.K = (int)F;
    dn.N = (int)N;
    dn.m = m_z;
    dn.tau = tau_z;
    dn.idx_out = idx_z_out;
    dn.nnz_out = nnz_z_out;
    dn.seg_cnt = up.zl_cnt;  // the counts the list-closing step reads
    dn.z_out = nullptr;
    if (residual) {
        if (B != 1) return SCAP_ERR_CONFIG;
        const int rc = launch_swiglu_block1(up, dn, wdt, flags1, SCAP_CFG_ACCUMULATE, static_cast<hipStream_t>(stream));
        return rc == kG1NotApplicable ? SCAP_ERR_CONFIG : rc;
    }
    return launch_swiglu_block(up, dn, wdt, static_cast<hipStream_t>(stream), flags1);
}
}  // namespace

extern "C" {

int scap_swiglu_block(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale, int64_t K,
                      int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x, float tau_x,
                      const float* b_gu_fused, float m_z, float tau_z, const float* b_down_fused, float* y,
                      float* z_out, int32_t* idx_z_out, int32_t* nnz_z_out, void* workspace, size_t workspace_bytes,
                      void* stream) {
    return block_common(W_gu, gu_scale, W_down, down_scale, K, F, N, wdt, x, xdt, B, m_x, tau_x, b_gu_fused, m_z, tau_z,
                        b_down_fused, y, z_out, idx_z_out, nnz_z_out, workspace, workspace_bytes, stream, false, 0);
}

int scap_swiglu_block_ex(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale, int64_t K,
                         int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x, float tau_x,
                         const float* b_gu_fused, float m_z, float tau_z, const float* b_down_fused, float* y,
                         float* z_out, int32_t* idx_z_out, int32_t* nnz_z_out, void* workspace, size_t workspace_bytes,
                         void* stream, const scap_launch_cfg* cfg) {
    const int flags1 = cfg ? cfg->flags & (SCAP_CFG_PARTIAL_SUMS | SCAP_CFG_PARK_SLICES | SCAP_CFG_GENERAL_KERNEL) : 0;
    return block_common(W_gu, gu_scale, W_down, down_scale, K, F, N, wdt, x, xdt, B, m_x, tau_x, b_gu_fused, m_z, tau_z,
                        b_down_fused, y, z_out, idx_z_out, nnz_z_out, workspace, workspace_bytes, stream, false, flags1);
}

int scap_swiglu_block_residual(const void* W_gu, const void* gu_scale, const void* W_down, const void* down_scale,
                               int64_t K, int64_t F, int64_t N, int wdt, const void* x, int xdt, int64_t B, float m_x,
                               float tau_x, const float* b_gu_fused, float m_z, float tau_z,
                               const float* b_down_fused, float* y, float* z_out, int32_t* idx_z_out,
                               int32_t* nnz_z_out, void* workspace, size_t workspace_bytes, void* stream) {
    return block_common(W_gu, gu_scale, W_down, down_scale, K, F, N, wdt, x, xdt, B, m_x, tau_x, b_gu_fused, m_z, tau_z,
                        b_down_fused, y, z_out, idx_z_out, nnz_z_out, workspace, workspace_bytes, stream, true, 0);
}

int scap_read_probe(const void* src, size_t bytes, uint32_t* out, void* stream) {
    if (!src || !out) return SCAP_ERR_NULL;
    if (!aligned16(src)) return SCAP_ERR_ALIGN;
    if (bytes == 0 || bytes % 16 != 0) return SCAP_ERR_SHAPE;
    return launch_read_probe(src, bytes, out, static_cast<hipStream_t>(stream));
}

}  // extern "C"
