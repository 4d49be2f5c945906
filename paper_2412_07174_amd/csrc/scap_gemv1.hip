// Launch of the one-token GEMV kernel (scap_gemv1.hpp): K split, argument block, dispatch by weight type.
#include "scap_gemv1b.hpp"

namespace scap {

extern template int launch_gemv1_wdt<kF16>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1_wdt<kBF16>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1_wdt<kI8>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1_wdt<kI8Half>(const Gemv1Args&, int, int, hipStream_t);
extern template int launch_gemv1b_wdt<kF16>(const Gemv1bArgs&, hipStream_t);
extern template int launch_gemv1b_wdt<kBF16>(const Gemv1bArgs&, hipStream_t);
extern template int launch_gemv1b_wdt<kI8>(const Gemv1bArgs&, hipStream_t);
extern template int launch_gemv1b_wdt<kI8Half>(const Gemv1bArgs&, hipStream_t);
extern template int launch_gemv1b_block_wdt<kF16>(const Gemv1bArgs&, int, hipStream_t);
extern template int launch_gemv1b_block_wdt<kBF16>(const Gemv1bArgs&, int, hipStream_t);
extern template int launch_gemv1b_block_wdt<kI8>(const Gemv1bArgs&, int, hipStream_t);
extern template int launch_gemv1b_block_wdt<kI8Half>(const Gemv1bArgs&, int, hipStream_t);
#define SCAP_G1_BLOCK_EXTERN(WD)                                                             \
    extern template int launch_gemv1_block<WD, kFuseSwiglu>(const Gemv1Args&, hipStream_t); \
    extern template int launch_gemv1_block<WD, kFuseList>(const Gemv1Args&, hipStream_t);
SCAP_G1_BLOCK_EXTERN(kF16)
SCAP_G1_BLOCK_EXTERN(kBF16)
SCAP_G1_BLOCK_EXTERN(kI8)
SCAP_G1_BLOCK_EXTERN(kI8Half)
#undef SCAP_G1_BLOCK_EXTERN

// One token through a K x N layer (sparse, dense or bias-folding mode).  Returns a scap_status, or
// kG1NotApplicable when the shape needs more than 2048 channels per workgroup (the caller then takes the
// general kernel).  cfg: rows_per_group and unroll are honoured, flags bit 0 forces device-scope loads.
namespace {

struct Plan1 {
    bool i8_half;
    int elems, tile, Kc, S, T;
};

// K split and lane width of one launch.  SCAP_OK, kG1NotApplicable or a scap_status.
// bt = token slots: 1 (one-token kernel), 2 or 4 (its multi-token forms, 8 wavefronts).
int plan_gemv1(const GemvArgs& g, int wdt, int kc, bool kc_forced, int waves, int granule_min, int bt, Plan1* out) {
    // int8 weights: 16 bytes per lane (1024-column tiles) unless that leaves at most 4 tiles -- then 8 bytes per
    // lane, twice the tiles and half the K splits (14336 x 4096 int8: 15.9 -> 14.2 us dense)
    out->i8_half = wdt == kI8 && g.N <= 4 * 1024;
    out->elems = wdt == kI8 && !out->i8_half ? 16 : 8;
    out->tile = kWave * out->elems;
    GemvArgs p = g;
    // LDS: header, the wavefronts' sums, then 8 bytes per listed channel (16 with 2 token slots)
    const int entry = bt == 1 ? 8 : (bt == 2 ? 16 : 32);
    const int64_t fixed_lds = bt == 1 ? (int64_t)waves * out->tile * 4 + 64 + kG1HdrBytes
                                      : (int64_t)bt * kG1HdrBytes + (int64_t)kG1bWaves * bt * out->tile * 4 + (int64_t)kG1bWaves * 4 * entry;
    const int64_t lds_max = bt == 1 ? 64 * 1024 : kG1bMaxLds;
    // (four slots of 1024-column tiles: the wavefronts' sums alone would fill LDS)
    if (fixed_lds + (int64_t)kWave * (4 + entry) > lds_max) return kG1NotApplicable;
    const size_t lds_budget = (size_t)(lds_max - fixed_lds) + kHdrBytes;
    // Rows per workgroup in multiples of 64, unless the input is so short that 64-row pieces would leave compute
    // units without a workgroup (1024 x 4096: 16 splits x 8 tiles; with 32-row pieces 8.5 -> 6.5 us dense)
    p.T = (p.N + out->tile - 1) / out->tile;
    int granule = ((int64_t)((p.K + kWave - 1) / kWave) * p.T < 256) ? 8 : kWave;
    if (granule < granule_min) granule = granule_min;
    const int rc = plan_splits(p, out->tile, entry / 4 - 1, kc, kc_forced, lds_budget, granule);
    if (rc != SCAP_OK) return rc == SCAP_ERR_SHAPE ? kG1NotApplicable : rc;
    if (p.Kc > kG1MaxChunks * kG1Chunk) return kG1NotApplicable;
    out->Kc = p.Kc;
    out->S = p.S;
    out->T = p.T;
    return SCAP_OK;
}

Gemv1Args args_of(const GemvArgs& g, const Plan1& pl, int flags) {
    Gemv1Args a{};
    a.W = g.W;
    a.x = g.x;
    a.col_scale = g.col_scale;
    a.bias = g.bias;
    a.y = g.y;
    a.partial = g.partial;
    a.counters = g.counters;
    a.idx_out = g.idx_out;
    a.nnz_out = g.nnz_out;
    a.union_nnz_out = g.union_nnz_out;
    a.seg_cnt = g.seg_cnt;
    a.K = g.K;
    a.N = g.N;
    a.Kc = pl.Kc;
    a.S = pl.S;
    a.T = pl.T;
    a.mode = g.mode;
    a.xdt = g.xdt;
    a.flags = flags;
    a.m = g.m;
    a.tau = g.tau;
    // fixed-point hand-over unless the caller asks for partial sums (either flag), the layer is wider than the
    // words provided or a column has more arrivals than a word counts
    const bool fx = !(flags & (kG1FlagPartials | kG1FlagDeviceScope)) && g.N <= kFxCols && pl.S <= kFxMaxSplits;
    a.fx_acc = fx ? g.fx_acc : nullptr;
    return a;
}

}  // namespace

// One token (B == 1) through a K x N layer (sparse, dense or bias-folding mode).  Returns a scap_status, or
// kG1NotApplicable when the shape needs more than 2048 channels per workgroup (the caller then takes the
// general kernel).  cfg: wavefronts (4, 8), rows_per_group and unroll are honoured, flags bit 0 forces device-scope loads.
int launch_gemv1(const GemvArgs& g, int wdt, const scap_launch_cfg* cfg, hipStream_t stream) {
    if (g.B != 1) return kG1NotApplicable;
    int kc = 0, unroll = 0, flags = 0, waves = 8;
    if (cfg) {
        if (cfg->rows_per_group) kc = cfg->rows_per_group;
        if (cfg->unroll) unroll = cfg->unroll;
        if (cfg->waves_per_group) waves = cfg->waves_per_group;
        flags = cfg->flags;
        if (kc < 0 || (kc % 8) != 0) return SCAP_ERR_CONFIG;  // whole octets of channels per workgroup
        if (kc > kG1MaxChunks * kG1Chunk) return kG1NotApplicable;
    }
    Plan1 pl;
    const int rc = plan_gemv1(g, wdt, kc, cfg && cfg->rows_per_group, waves, 8, 1, &pl);
    if (rc != SCAP_OK) return rc;
    // rows in flight per wavefront: 4 x 1 KB (16-byte lanes), 8 x 512 bytes (8-byte lanes)
    if (unroll == 0) unroll = pl.i8_half ? 8 : 4;
    const Gemv1Args a = args_of(g, pl, flags);
    switch (wdt) {
        case kF16: return launch_gemv1_wdt<kF16>(a, waves, unroll, stream);
        case kBF16: return launch_gemv1_wdt<kBF16>(a, waves, unroll, stream);
        case kI8: return pl.i8_half ? launch_gemv1_wdt<kI8Half>(a, waves, unroll, stream) : launch_gemv1_wdt<kI8>(a, waves, unroll, stream);
    }
    return SCAP_ERR_DTYPE;
}

// Two tokens, or three to four (16-bit weights; int8 where N <= 4096, i.e. 8-byte lanes), through the two- /
// four-slot form of the one-token kernel (sparse or dense mode).  Returns a scap_status, or kG1NotApplicable: another token count, bias folding, an input length
// that is not a multiple of 8 (the later tokens' rows would not be 16-byte aligned), more than 2048 channels per
// workgroup, or four slots without the fixed-point hand-over.  flags as for launch_gemv1.
int launch_gemv1b(const GemvArgs& g, int wdt, int flags, hipStream_t stream) {
    if (g.B < 2 || g.B > 4 || g.mode == kModeFold || (g.K % 8) != 0) return kG1NotApplicable;

    Gemv1bArgs b;
    b.B = g.B;
    b.bt = g.B == 2 ? 2 : 4;
    Plan1 pl;
    const int rc = plan_gemv1(g, wdt, 0, false, kG1bWaves, 8, b.bt, &pl);
    if (rc != SCAP_OK) return rc;
    b.a = args_of(g, pl, flags);
    if ((size_t)g.B * (size_t)g.N > (size_t)kFxCols) b.a.fx_acc = nullptr;  // one fixed-point word per (token, column)
    // with four slots the partial-sum hand-over loses to the other kernels (its last arrivals fetch 4 S slices)
    if (b.bt == 4 && b.a.fx_acc == nullptr) return kG1NotApplicable;
    switch (wdt) {
        case kF16: return launch_gemv1b_wdt<kF16>(b, stream);
        case kBF16: return launch_gemv1b_wdt<kBF16>(b, stream);
        case kI8: return pl.i8_half ? launch_gemv1b_wdt<kI8Half>(b, stream) : launch_gemv1b_wdt<kI8>(b, stream);
    }
    return SCAP_ERR_DTYPE;
}

template <int FUSE>
static int launch_block_half(const Gemv1Args& a, int wdt, bool i8_half, hipStream_t stream) {
    switch (wdt) {
        case kF16: return launch_gemv1_block<kF16, FUSE>(a, stream);
        case kBF16: return launch_gemv1_block<kBF16, FUSE>(a, stream);
        case kI8: return i8_half ? launch_gemv1_block<kI8Half, FUSE>(a, stream) : launch_gemv1_block<kI8, FUSE>(a, stream);
    }
    return SCAP_ERR_DTYPE;
}

// Fused SwiGLU block of one token on the one-token kernel: the gate|up launch with the gating epilogue, then the
// down launch reading the lists.  `up` and `down` as for launch_swiglu_block; up_flags, down_flags: the launches'
// flags (kG1FlagPartials; up: kG1FlagParkSlices; down: kG1FlagAccumulate, y += block output).  kG1NotApplicable when either layer needs more than 2048 channels per
// workgroup.
int launch_swiglu_block1(const GemvArgs& up, const GemvArgs& dn, int wdt, int up_flags, int down_flags, hipStream_t stream) {
    if (up.B != 1) return kG1NotApplicable;
    Plan1 pu, pd;
    int rc = plan_gemv1(up, wdt, 0, false, 8, kWave, 1, &pu);
    if (rc != SCAP_OK) return rc;
    rc = plan_gemv1(dn, wdt, 0, false, 8, kWave, 1, &pd);  // whole 64-channel pieces: whole list segments
    if (rc != SCAP_OK) return rc;
    const int segz = pu.tile / 8 / 2;  // gated channels a wavefront slice of the gate|up launch finishes: 32 or 64
    if (pd.Kc % segz != 0 || pd.Kc / segz > kWave) return kG1NotApplicable;
    Gemv1Args a = args_of(up, pu, up_flags);
    Gemv1Args b = args_of(dn, pd, down_flags);
    for (Gemv1Args* q : {&a, &b}) {
        q->m2 = up.m2;
        q->tau2 = up.tau2;
        q->zl_idx = up.zl_idx;
        q->zl_d = up.zl_d;
        q->zl_cnt = up.zl_cnt;
        q->F = up.F;
        q->segz = segz;
    }
    a.z_out = up.z_out;
    // the gating epilogue parks finished columns behind the partial-sum slots when a slice is finished piecemeal
    if ((size_t)(pu.S + 1) * pu.T * pu.tile > partial_capacity(up.N)) a.fx_acc = nullptr;
    a.idx_out = a.nnz_out = a.union_nnz_out = nullptr;
    b.x = nullptr;
    rc = launch_block_half<kFuseSwiglu>(a, wdt, pu.i8_half, stream);
    if (rc != SCAP_OK) return rc;
    return launch_block_half<kFuseList>(b, wdt, pd.i8_half, stream);
}

// Fused SwiGLU block of two tokens (down launch: up to four): each of its launches can run on the multi-slot kernel, in the list format of the
// batched block kernels (64-channel segments, 2 token slots), so either can be paired with the general kernel's.
//   part 0, the gate|up launch with the gating epilogue: int8 weights in 16-byte lanes (2F > 4096; a wavefront's
//           slice is then 128 columns = one segment), input length a multiple of 8;
//   part 1, the down launch reading the lists: any weights, unless 16-bit and too wide for the fixed-point hand-over
//           (with partial sums handed over the general kernel's down launch measured 0.5 us faster).
// Measured on 4096 -> 14336 -> 4096, two tokens, both launches general / these (us): int8 45.8 / 41.9 with nothing
// pruned, 38.0 / 34.5 at 50 %, 21.8 / 19.6 at 90 %; bf16 (down launch only) 65.3 / 64.3, 55.9 / 54.7, 25.9 / 24.8.
// Returns SCAP_OK and fills *g, or kG1NotApplicable.
static int plan_block2_part(const GemvArgs& up, const GemvArgs& dn, int wdt, int part, Gemv1bArgs* g, bool* i8_half) {
    // 3-4 tokens: the down launch only, 16-bit weights, on the four-slot form (the lists then carry 4 token slots)
    const bool four = (up.B == 3 || up.B == 4) && part == 1 && wdt != kI8;
    if (up.B != 2 && !four) return kG1NotApplicable;
    const GemvArgs& src = part == 0 ? up : dn;
    if (part == 0 && (wdt != kI8 || (src.K % 8) != 0)) return kG1NotApplicable;
    if (part == 1 && wdt != kI8 && (int64_t)up.B * (int64_t)src.N > (int64_t)kFxCols) return kG1NotApplicable;
    Plan1 pl;
    const int rc = plan_gemv1(src, wdt, 0, false, kG1bWaves, kWave, four ? 4 : 2, &pl);  // whole 64-channel pieces: whole segments
    if (rc != SCAP_OK) return kG1NotApplicable;
    if (four && pl.Kc > 2 * kG1Chunk) return kG1NotApplicable;  // (its prologue holds every entry slot in registers)
    if (part == 0 && pl.i8_half) return kG1NotApplicable;
    if (part == 1 && (pl.Kc % kWave) != 0) return kG1NotApplicable;
    g->B = (int)up.B;
    g->bt = four ? 4 : 2;
    g->a = args_of(src, pl, 0);
    if (part == 0 || (size_t)up.B * (size_t)src.N > (size_t)kFxCols) g->a.fx_acc = nullptr;
    if (four && g->a.fx_acc == nullptr) return kG1NotApplicable;  // four slots: fixed-point hand-over only
    g->a.m2 = up.m2;
    g->a.tau2 = up.tau2;
    g->a.zl_idx = up.zl_idx;
    g->a.zl_d = up.zl_d;
    g->a.zl_cnt = up.zl_cnt;
    g->a.F = up.F;
    if (part == 0) {
        g->a.z_out = up.z_out;
        g->a.idx_out = g->a.nnz_out = g->a.union_nnz_out = nullptr;
    } else {
        g->a.x = nullptr;
        g->a.z_out = nullptr;
    }
    *i8_half = pl.i8_half;
    return SCAP_OK;
}

bool swiglu_block2_part_applies(const GemvArgs& up, const GemvArgs& dn, int wdt, int part) {
    Gemv1bArgs g;
    bool half = false;
    return plan_block2_part(up, dn, wdt, part, &g, &half) == SCAP_OK;
}

int launch_swiglu_block2_part(const GemvArgs& up, const GemvArgs& dn, int wdt, int part, hipStream_t stream) {
    Gemv1bArgs g;
    bool half = false;
    const int rc = plan_block2_part(up, dn, wdt, part, &g, &half);
    if (rc != SCAP_OK) return rc;
    const int fuse = part == 0 ? kFuseSwiglu : kFuseList;
    switch (wdt) {
        case kF16: return launch_gemv1b_block_wdt<kF16>(g, fuse, stream);
        case kBF16: return launch_gemv1b_block_wdt<kBF16>(g, fuse, stream);
        case kI8: return half ? launch_gemv1b_block_wdt<kI8Half>(g, fuse, stream) : launch_gemv1b_block_wdt<kI8>(g, fuse, stream);
    }
    return SCAP_ERR_DTYPE;
}

}  // namespace scap
