// Host layer of the DynamicRad library: argument validation, the fp64 per-t table of the
// radial window and split rule (paper Eqs. 1-6), scratch management and kernel launches.
#include "../../include/dynamicrad.h"
#include "../../include/dynamicrad_probe.h"
#include "dr_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

using namespace dr;

// Scratch of dr_sparse_attn_fwd_static: one copy per GPU the library runs on, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress (dr_create resolves it, per device); kernels get the address.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct dr_ctx {
    int device = 0;
    unsigned char* static_scratch = nullptr;   // device address of `scratch` on this context's device
    std::string err;
    // stage (a) scratch
    float* pooled = nullptr;
    size_t pooled_bytes = 0;
    // stage (b) scratch
    uint32_t* keepbits = nullptr;
    int32_t* counts = nullptr;
    size_t keep_bytes = 0, count_bytes = 0;
    // stage (c) scratch (block sizes 32 / 64): merged key-block lists per 128-row group
    int32_t* gcol = nullptr;
    int32_t* gcount = nullptr;
    size_t gcol_bytes = 0, gcount_bytes = 0;
    // stage (c) scratch (bf16 MFMA paths): per-wave range flags of the fast pass, read by the fp32-scaled second pass
    int32_t* attn_flags = nullptr;
    size_t attn_flags_bytes = 0;
    bool attn_pairs = true;      // block size 128: the kernel that walks pairs of query blocks (DR_ATTN_PAIRS=0 turns it off)
    // cached selection of the uniform rule (it depends on geometry, ratios and seed only): one mask of Sb rows
    uint32_t* uni_keep = nullptr;
    int32_t* uni_counts = nullptr;
    size_t uni_keep_bytes = 0, uni_count_bytes = 0;
    bool uni_valid = false;
    struct UniKey { double ratio, ratio_far; uint32_t seed; int32_t pad; } uni_key{};
    // proxy objective: per (b, h) and slice partial sums
    double* proxy_partial = nullptr;
    size_t proxy_bytes = 0;
    // token-level order: link bytes [B, masks, N, N] when the caller does not ask for them
    uint8_t* links = nullptr;
    size_t links_bytes = 0;
    // cached candidate geometry
    uint8_t* class_map = nullptr;
    uint64_t* class_bits = nullptr;      // the classes as lane masks (block rows of at most kWaveSelectMaxBlocks)
    size_t class_bits_bytes = 0;
    int32_t* row_sel = nullptr;
    unsigned long long* totals = nullptr;     // device [2]
    size_t class_bytes = 0, rowsel_bytes = 0;
    bool geom_valid = false;
    struct Key { int32_t N, Nf, Nt, Bs; double gamma, lambda, theta_c, theta_m; } key{};
    int64_t cand_total = 0;
    int32_t max_sel = 0;
};

namespace {

dr_status fail(dr_ctx* ctx, dr_status st, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return st;
}

#define DR_HIP(ctx, call)                                                                          \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(ctx, DR_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        if (prev != dev) ok = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

const dr_mask_params kDefaults = {1.0, 0.15, 0.60, -1.0, 2, 0, 0.0, 0u, {0, 0, 0}};

dr_status grow(dr_ctx* ctx, void** p, size_t* have, size_t need) {
    if (*have >= need) return DR_OK;
    if (*p) {
        DR_HIP(ctx, hipFree(*p));
        *p = nullptr;
        *have = 0;
    }
    hipError_t e = hipMalloc(p, need);
    if (e != hipSuccess) {
        *p = nullptr;
        return fail(ctx, DR_ERR_NOMEM, "hipMalloc(%zu): %s", need, hipGetErrorString(e));
    }
    *have = need;
    return DR_OK;
}

dr_status check_geometry(dr_ctx* ctx, const dr_shape* s) {
    if (!s) return fail(ctx, DR_ERR_INVALID_ARG, "shape is NULL");
    if (s->Nf <= 0 || s->Hg <= 0 || s->Wg <= 0 || s->N <= 0) return fail(ctx, DR_ERR_INVALID_ARG, "non-positive dimension");
    if ((int64_t)s->Nf * s->Hg * s->Wg != (int64_t)s->N)
        return fail(ctx, DR_ERR_INVALID_ARG, "N=%d != Nf*Hg*Wg=%lld", s->N, (long long)s->Nf * s->Hg * s->Wg);
    if (s->Bs != 32 && s->Bs != 64 && s->Bs != 128) return fail(ctx, DR_ERR_UNSUPPORTED, "Bs=%d not in {32,64,128}", s->Bs);
    if (s->Nf > kMaxFrames) return fail(ctx, DR_ERR_UNSUPPORTED, "Nf=%d exceeds %d", s->Nf, kMaxFrames);
    if (s->reserved0 != 0) return fail(ctx, DR_ERR_INVALID_ARG, "reserved0 must be 0");
    return DR_OK;
}

dr_status check_tensor_shape(dr_ctx* ctx, const dr_shape* s) {
    dr_status st = check_geometry(ctx, s);
    if (st != DR_OK) return st;
    if (s->B <= 0 || s->H <= 0) return fail(ctx, DR_ERR_INVALID_ARG, "non-positive B or H");
    if (s->B > 32767 || s->H > 65535) return fail(ctx, DR_ERR_UNSUPPORTED, "B or H too large for the launch grid");
    if (s->d != 64 && s->d != 128) return fail(ctx, DR_ERR_UNSUPPORTED, "d=%d not in {64,128}", s->d);
    if (s->dtype != DR_F32 && s->dtype != DR_BF16) return fail(ctx, DR_ERR_INVALID_ARG, "unknown dtype %d", s->dtype);
    const int64_t es = s->dtype == DR_BF16 ? 2 : 4;
    if (s->stride_n < s->d || s->stride_h <= 0 || s->stride_b <= 0) return fail(ctx, DR_ERR_INVALID_ARG, "bad strides");
    if ((s->stride_n * es) % 16 || (s->stride_h * es) % 16 || (s->stride_b * es) % 16)
        return fail(ctx, DR_ERR_INVALID_ARG, "strides must keep rows 16-byte aligned");
    return DR_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

dr_status check_params(dr_ctx* ctx, const dr_mask_params* p, double lambda) {
    if (!(lambda > 0.0) || !std::isfinite(lambda)) return fail(ctx, DR_ERR_INVALID_ARG, "lambda must be > 0");
    if (!(p->gamma > 0.0) || !std::isfinite(p->gamma)) return fail(ctx, DR_ERR_INVALID_ARG, "gamma must be > 0");
    if (!(p->theta_c >= 0.0 && p->theta_c < 1.0)) return fail(ctx, DR_ERR_INVALID_ARG, "theta_c must be in [0,1)");
    if (!(p->theta_m >= 0.0 && p->theta_m < 1.0)) return fail(ctx, DR_ERR_INVALID_ARG, "theta_m must be in [0,1)");
    if (p->ratio_far > 1.0 || p->ratio_far == 0.0 || std::isnan(p->ratio_far))
        return fail(ctx, DR_ERR_INVALID_ARG, "ratio_far must be < 0 (unused) or in (0,1]");
    if (p->head_fuse < 0) return fail(ctx, DR_ERR_INVALID_ARG, "head_fuse must be >= 0");
    if (p->has_tau_far != 0 && p->has_tau_far != 1) return fail(ctx, DR_ERR_INVALID_ARG, "has_tau_far must be 0 or 1");
    if (p->has_tau_far && std::isnan(p->tau_far)) return fail(ctx, DR_ERR_INVALID_ARG, "tau_far is NaN");
    for (int i = 0; i < 3; ++i)
        if (p->reserved[i] != 0) return fail(ctx, DR_ERR_INVALID_ARG, "reserved fields must be 0");
    return DR_OK;
}

// Smallest integer count c in 0..n with c / n > theta (IEEE double division); n + 1 if there is none.
int32_t min_count_exceeding(int n, double theta) {
    for (int c = 0; c <= n; ++c)
        if ((double)c / (double)n > theta) return c;
    return n + 1;
}

// Paper Eqs. 1-6, one entry per temporal distance t.
void fill_frame_table(int Nf, int Nt, int Bs, double gamma, double lambda, FrameTab* tab) {
    std::memset(tab, 0, sizeof *tab);
    long long L0 = 1;
    while (L0 < Nt) L0 <<= 1;                                      // 2^ceil(log2 Nt)
    for (int t = 0; t < Nf; ++t) {
        if (t <= 1) {                                              // Eq. 3 first case; never pruned
            tab->w[t] = Nt;
            tab->flags[t] = (uint8_t)(1 | (DR_CLASS_FORCED << 1));
            continue;
        }
        int group = 0;                                             // floor(log2 t) + 1 == bit length of t
        for (int x = t; x > 0; x >>= 1) ++group;
        const double base = (double)L0 / (double)(1ll << group);
        const double decay = base * gamma;                         // Eq. 2
        const double lsplit = base * lambda;                       // Eq. 4
        const long long rounded = (long long)std::floor(decay + 0.5);
        const long long w = rounded > Bs ? rounded : Bs;           // Eq. 3
        long long sf = (long long)std::floor((double)Bs / (lsplit + 1e-6));   // Eq. 5
        if (sf < 1) sf = 1;
        const bool retained = (t % sf) == 0;                       // Eq. 6
        const int cls = decay >= (double)Bs ? DR_CLASS_NEAR : DR_CLASS_FAR;   // Eq. 8 cases
        tab->w[t] = (int32_t)(w > 0x3fffffff ? 0x3fffffff : w);
        tab->flags[t] = (uint8_t)((retained ? 1 : 0) | (cls << 1));
    }
}

Geometry make_geometry(const dr_shape* s, const dr_mask_params* p) {
    Geometry g{};
    const int Sb = (s->N + s->Bs - 1) / s->Bs;
    g.N = s->N; g.Nt = s->Hg * s->Wg; g.Nf = s->Nf; g.Bs = s->Bs; g.Sb = Sb;
    const int tail = s->N - (Sb - 1) * s->Bs;
    g.row_min_full = min_count_exceeding(s->Bs, p->theta_c);
    g.row_min_tail = min_count_exceeding(tail, p->theta_c);
    g.col_min_full = min_count_exceeding(s->Bs, p->theta_m);
    g.col_min_tail = min_count_exceeding(tail, p->theta_m);
    return g;
}

dr_status ensure_geometry(dr_ctx* ctx, const dr_shape* s, double lambda, const dr_mask_params* p, hipStream_t stream) {
    const int Nt = s->Hg * s->Wg;
    dr_ctx::Key k{s->N, s->Nf, Nt, s->Bs, p->gamma, lambda, p->theta_c, p->theta_m};
    if (ctx->geom_valid && std::memcmp(&k, &ctx->key, sizeof k) == 0) return DR_OK;
    ctx->geom_valid = false;
    ctx->uni_valid = false;
    const int Sb = (s->N + s->Bs - 1) / s->Bs;
    dr_status st;
    if ((st = grow(ctx, (void**)&ctx->class_map, &ctx->class_bytes, (size_t)Sb * Sb)) != DR_OK) return st;
    if ((st = grow(ctx, (void**)&ctx->row_sel, &ctx->rowsel_bytes, (size_t)Sb * 4)) != DR_OK) return st;
    const bool lane_masks = Sb <= kWaveSelectMaxBlocks;
    if (lane_masks && (st = grow(ctx, (void**)&ctx->class_bits, &ctx->class_bits_bytes,
                                 (size_t)Sb * wave_select_slots(Sb) * 3 * sizeof(uint64_t))) != DR_OK) return st;
    if (!ctx->totals) DR_HIP(ctx, hipMalloc((void**)&ctx->totals, 2 * sizeof(unsigned long long)));
    const Geometry g = make_geometry(s, p);
    FrameTab tab;
    fill_frame_table(s->Nf, Nt, s->Bs, p->gamma, lambda, &tab);
    DR_HIP(ctx, hipMemsetAsync(ctx->totals, 0, 2 * sizeof(unsigned long long), stream));
    DR_HIP(ctx, launch_class_map(g, tab, ctx->class_map, lane_masks ? ctx->class_bits : nullptr, ctx->row_sel, ctx->totals, stream));
    unsigned long long host_tot[2] = {0, 0};
    DR_HIP(ctx, hipMemcpyAsync(host_tot, ctx->totals, sizeof host_tot, hipMemcpyDeviceToHost, stream));
    DR_HIP(ctx, hipStreamSynchronize(stream));
    ctx->cand_total = (int64_t)host_tot[0];
    ctx->max_sel = (int32_t)host_tot[1];
    std::memcpy(&ctx->key, &k, sizeof k);     // memcmp-compared later: copy padding-free fields bytewise
    ctx->geom_valid = true;
    return DR_OK;
}

}  // namespace

extern "C" {

const char* dr_version(void) { return "dynamicrad-gfx950 0.3"; }

dr_status dr_create(dr_ctx** out, int device) {
    if (!out) return DR_ERR_INVALID_ARG;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return DR_ERR_INVALID_ARG;
    dr_ctx* c = new (std::nothrow) dr_ctx();
    if (!c) return DR_ERR_NOMEM;
    c->device = device;
    std::memset(&c->key, 0, sizeof c->key);
    if (const char* e = std::getenv("DR_ATTN_PAIRS")) c->attn_pairs = !(e[0] == '0' && e[1] == 0);
    {
        DeviceGuard g(device);
        void* p = nullptr;
        if (!g.ok || hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            delete c;
            return DR_ERR_HIP;
        }
        c->static_scratch = static_cast<unsigned char*>(p);
    }
    *out = c;
    return DR_OK;
}

void dr_destroy(dr_ctx* ctx) {
    if (!ctx) return;
    {
        DeviceGuard g(ctx->device);
        void* ptrs[] = {ctx->pooled, ctx->keepbits, ctx->counts, ctx->class_map, ctx->class_bits, ctx->row_sel, ctx->totals, ctx->gcol,
                        ctx->gcount, ctx->attn_flags, ctx->uni_keep, ctx->uni_counts, ctx->links, ctx->proxy_partial};
        for (void* p : ptrs)
            if (p) (void)hipFree(p);
    }
    delete ctx;
}

const char* dr_last_error(const dr_ctx* ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

dr_status dr_class_map(dr_ctx* ctx, const dr_shape* shape, double lambda, const dr_mask_params* params,
                       uint8_t* class_map, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    const dr_mask_params* p = params ? params : &kDefaults;
    dr_status st;
    if ((st = check_geometry(ctx, shape)) != DR_OK) return st;
    if ((st = check_params(ctx, p, lambda)) != DR_OK) return st;
    if (!class_map) return fail(ctx, DR_ERR_INVALID_ARG, "class_map is NULL");
    DeviceGuard g(ctx->device);
    hipStream_t s = (hipStream_t)stream;
    if ((st = ensure_geometry(ctx, shape, lambda, p, s)) != DR_OK) return st;
    const int Sb = (shape->N + shape->Bs - 1) / shape->Bs;
    DR_HIP(ctx, hipMemcpyAsync(class_map, ctx->class_map, (size_t)Sb * Sb, hipMemcpyDeviceToDevice, s));
    return DR_OK;
}

dr_status dr_mask_capacity(dr_ctx* ctx, const dr_shape* shape, double lambda, const dr_mask_params* params,
                           int64_t* candidate_blocks, int32_t* max_selectable_per_row) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    const dr_mask_params* p = params ? params : &kDefaults;
    dr_status st;
    if ((st = check_geometry(ctx, shape)) != DR_OK) return st;
    if ((st = check_params(ctx, p, lambda)) != DR_OK) return st;
    if (!candidate_blocks) return fail(ctx, DR_ERR_INVALID_ARG, "candidate_blocks is NULL");
    DeviceGuard g(ctx->device);
    if ((st = ensure_geometry(ctx, shape, lambda, p, nullptr)) != DR_OK) return st;
    *candidate_blocks = ctx->cand_total;
    if (max_selectable_per_row) *max_selectable_per_row = ctx->max_sel;
    return DR_OK;
}

dr_status dr_static_ratio_for_sparsity(dr_ctx* ctx, const dr_shape* shape, double lambda, const dr_mask_params* params,
                                       double target, double* ratio, double* achieved) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    const dr_mask_params* p = params ? params : &kDefaults;
    dr_status st;
    if ((st = check_geometry(ctx, shape)) != DR_OK) return st;
    if ((st = check_params(ctx, p, lambda)) != DR_OK) return st;
    if (!ratio) return fail(ctx, DR_ERR_INVALID_ARG, "ratio is NULL");
    if (!(target > 0.0 && target < 1.0)) return fail(ctx, DR_ERR_INVALID_ARG, "target must be in (0,1)");
    DeviceGuard g(ctx->device);
    if ((st = ensure_geometry(ctx, shape, lambda, p, nullptr)) != DR_OK) return st;
    const int Sb = (shape->N + shape->Bs - 1) / shape->Bs;
    std::vector<int32_t> n_row((size_t)Sb);
    DR_HIP(ctx, hipMemcpy(n_row.data(), ctx->row_sel, (size_t)Sb * 4, hipMemcpyDeviceToHost));
    int64_t selectable = 0;
    for (int32_t n : n_row) selectable += n;
    const int64_t forced = ctx->cand_total - selectable;
    const double pairs = (double)Sb * (double)Sb;
    bool found = false;
    for (int i = 1; i <= 1000; ++i) {
        const double rho = (double)i * 1e-3;
        int64_t kept = forced;
        for (int32_t n : n_row) {
            if (n <= 0) continue;
            const int64_t k = (int64_t)std::floor((double)n * rho);      // Eq. 8's keep rule
            kept += k < 1 ? 1 : k;
        }
        const double sparsity = 1.0 - (double)kept / pairs;
        if (sparsity >= target) {
            *ratio = rho;
            if (achieved) *achieved = sparsity;
            found = true;
        }
    }
    if (!found) return fail(ctx, DR_ERR_UNSUPPORTED, "no ratio reaches sparsity %.4f: the never-pruned zone alone keeps %lld of %.0f block pairs",
                            target, (long long)forced, pairs);
    return DR_OK;
}

dr_status dr_block_scores(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, int32_t head_fuse,
                          float* scores, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    dr_status st;
    if ((st = check_tensor_shape(ctx, shape)) != DR_OK) return st;
    if (!Q || !K || !scores) return fail(ctx, DR_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(Q) || misaligned(K)) return fail(ctx, DR_ERR_INVALID_ARG, "Q/K must be 16-byte aligned");
    if (head_fuse < 0 || head_fuse > shape->H) return fail(ctx, DR_ERR_INVALID_ARG, "head_fuse=%d outside 0..H", head_fuse);
    DeviceGuard g(ctx->device);
    const int Sb = (shape->N + shape->Bs - 1) / shape->Bs;
    const int Hs = head_fuse > 0 ? head_fuse : shape->H;
    const int masks = head_fuse > 0 ? 1 : shape->H;
    const int hpm = head_fuse > 0 ? head_fuse : 1;
    const size_t need = (size_t)2 * shape->B * Hs * Sb * shape->d * sizeof(float);
    if ((st = grow(ctx, (void**)&ctx->pooled, &ctx->pooled_bytes, need)) != DR_OK) return st;
    TensorDesc td{shape->stride_b, shape->stride_h, shape->stride_n, shape->B, shape->H, shape->N, shape->d};
    hipStream_t s = (hipStream_t)stream;
    DR_HIP(ctx, launch_pool(Q, K, shape->dtype == DR_BF16, td, Hs, shape->Bs, Sb, ctx->pooled, s));
    DR_HIP(ctx, launch_scores(ctx->pooled, shape->B, Hs, masks, hpm, Sb, shape->d, scores, s));
    return DR_OK;
}

dr_status dr_build_mask(dr_ctx* ctx, const dr_shape* shape, int32_t mode, double ratio_or_tau, double lambda,
                        const dr_mask_params* params, const float* scores, int32_t* rowptr, int32_t* colidx,
                        int64_t colidx_capacity, int64_t* nnz, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    const dr_mask_params* p = params ? params : &kDefaults;
    dr_status st;
    if ((st = check_geometry(ctx, shape)) != DR_OK) return st;
    if ((st = check_params(ctx, p, lambda)) != DR_OK) return st;
    if (shape->B <= 0 || shape->H <= 0) return fail(ctx, DR_ERR_INVALID_ARG, "non-positive B or H");
    if (shape->B > 65535 || shape->H > 65535) return fail(ctx, DR_ERR_UNSUPPORTED, "B or H too large for the launch grid");
    if (mode < DR_MODE_STATIC_RATIO || mode > DR_MODE_UNIFORM_RATIO)
        return fail(ctx, DR_ERR_INVALID_ARG, "unknown mode %d", mode);
    if (mode == DR_MODE_ZSCORE_THRESHOLD) {
        if (std::isnan(ratio_or_tau)) return fail(ctx, DR_ERR_INVALID_ARG, "tau_1 is NaN");
    } else if (!(ratio_or_tau > 0.0 && ratio_or_tau <= 1.0)) {
        return fail(ctx, DR_ERR_INVALID_ARG, "%s must be in (0,1]", mode == DR_MODE_DYNAMIC_THRESHOLD ? "tau" : "ratio");
    }
    if (p->head_fuse > shape->H) return fail(ctx, DR_ERR_INVALID_ARG, "head_fuse=%d > H", p->head_fuse);
    if ((!scores && mode != DR_MODE_UNIFORM_RATIO) || !rowptr || !colidx || !nnz)
        return fail(ctx, DR_ERR_INVALID_ARG, "NULL output or scores pointer");
    if (colidx_capacity <= 0) return fail(ctx, DR_ERR_CAPACITY, "colidx_capacity must be > 0");
    const int Sb = (shape->N + shape->Bs - 1) / shape->Bs;
    if (mode == DR_MODE_ZSCORE_THRESHOLD &&
        select_zscore_lds_bytes(Sb, shape->Hg * shape->Wg, shape->Nf, shape->Bs) > kSelectZscoreMaxLds)
        return fail(ctx, DR_ERR_UNSUPPORTED, "z-score mode: a row tile of %d frames x %d key blocks per frame exceeds the LDS",
                    shape->Nf, (shape->Hg * shape->Wg + shape->Bs - 1) / shape->Bs + 1);
    DeviceGuard g(ctx->device);
    hipStream_t s = (hipStream_t)stream;
    if ((st = ensure_geometry(ctx, shape, lambda, p, s)) != DR_OK) return st;
    const int masks = p->head_fuse > 0 ? 1 : shape->H;
    if (ctx->max_sel > kMaxSelectablePerRow)
        return fail(ctx, DR_ERR_UNSUPPORTED, "%d selectable blocks in a row exceed %d", ctx->max_sel, kMaxSelectablePerRow);
    const size_t rows = (size_t)shape->B * masks * Sb;
    const size_t words = (Sb + 31) / 32;
    const bool uniform = mode == DR_MODE_UNIFORM_RATIO;
    if (uniform) {
        // The sample is the same for every batch element and head and for every call with this geometry, these
        // ratios and this seed (paper: the static mask is computed once, "Selector Efficiency" appendix): select once
        // for one mask, keep it in the context, and only write it out per call.
        if ((st = grow(ctx, (void**)&ctx->uni_keep, &ctx->uni_keep_bytes, (size_t)Sb * words * 4)) != DR_OK) return st;
        if ((st = grow(ctx, (void**)&ctx->uni_counts, &ctx->uni_count_bytes, (size_t)Sb * 4)) != DR_OK) return st;
    } else {
        if ((st = grow(ctx, (void**)&ctx->keepbits, &ctx->keep_bytes, rows * words * 4)) != DR_OK) return st;
        if ((st = grow(ctx, (void**)&ctx->counts, &ctx->count_bytes, rows * 4)) != DR_OK) return st;
    }
    SelectArgs a{};
    a.mode = mode;
    a.two_ratio = ((mode == DR_MODE_STATIC_RATIO || mode == DR_MODE_UNIFORM_RATIO) && p->ratio_far > 0.0) ? 1 : 0;
    a.ratio = ratio_or_tau;
    a.ratio_far = p->ratio_far;
    a.tau = ratio_or_tau;
    int cap = 1;
    while (cap < ctx->max_sel) cap <<= 1;
    a.sort_cap = cap;
    a.tau_near = ratio_or_tau;
    a.tau_far = p->has_tau_far ? p->tau_far : ratio_or_tau;
    a.seed = p->seed;
    a.N = shape->N; a.Nt = shape->Hg * shape->Wg; a.Nf = shape->Nf; a.Bs = shape->Bs;
    if (uniform) {
        dr_ctx::UniKey uk{};
        uk.ratio = ratio_or_tau; uk.ratio_far = p->ratio_far; uk.seed = p->seed;
        if (!ctx->uni_valid || std::memcmp(&uk, &ctx->uni_key, sizeof uk) != 0) {
            ctx->uni_valid = false;
            DR_HIP(ctx, launch_select(ctx->class_map, Sb <= kWaveSelectMaxBlocks ? ctx->class_bits : nullptr, nullptr, 1, 1, Sb, a, ctx->uni_keep, ctx->uni_counts, s));
            std::memcpy(&ctx->uni_key, &uk, sizeof uk);
            ctx->uni_valid = true;
        }
        DR_HIP(ctx, launch_emit(ctx->uni_keep, ctx->uni_counts, shape->B, masks, Sb, true, rowptr, colidx, colidx_capacity, nnz, s));
        return DR_OK;
    }
    if (mode == DR_MODE_ZSCORE_THRESHOLD) {
        FrameTab tab;
        fill_frame_table(shape->Nf, a.Nt, shape->Bs, p->gamma, lambda, &tab);
        for (int t = 0; t < shape->Nf; ++t)
            if (((tab.flags[t] >> 1) & 3) == DR_CLASS_NEAR) a.near_mask[t >> 6] |= 1ull << (t & 63);
    }
    if (mode == DR_MODE_ZSCORE_THRESHOLD)
        DR_HIP(ctx, launch_select_zscore(ctx->class_map, scores, shape->B, masks, Sb, a, ctx->keepbits, ctx->counts, s));
    else
        DR_HIP(ctx, launch_select(ctx->class_map, Sb <= kWaveSelectMaxBlocks ? ctx->class_bits : nullptr, scores, shape->B, masks, Sb, a, ctx->keepbits, ctx->counts, s));
    DR_HIP(ctx, launch_emit(ctx->keepbits, ctx->counts, shape->B, masks, Sb, false, rowptr, colidx, colidx_capacity, nnz, s));
    return DR_OK;
}

dr_status dr_token_scores(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, int32_t head_fuse,
                          float* scores, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    dr_status st;
    if ((st = check_tensor_shape(ctx, shape)) != DR_OK) return st;
    if (!Q || !K || !scores) return fail(ctx, DR_ERR_INVALID_ARG, "NULL tensor pointer");
    if (head_fuse < 0 || head_fuse > shape->H) return fail(ctx, DR_ERR_INVALID_ARG, "head_fuse=%d outside 0..H", head_fuse);
    if (shape->N > kMaxTokensTokenLevel)
        return fail(ctx, DR_ERR_UNSUPPORTED, "N=%d exceeds %d for the token-level order", shape->N, kMaxTokensTokenLevel);
    const int masks = head_fuse > 0 ? 1 : shape->H;
    if ((int64_t)shape->B * masks > 65535) return fail(ctx, DR_ERR_UNSUPPORTED, "B * masks too large for the launch grid");
    DeviceGuard g(ctx->device);
    TensorDesc td{shape->stride_b, shape->stride_h, shape->stride_n, shape->B, shape->H, shape->N, shape->d};
    DR_HIP(ctx, launch_token_scores(Q, K, shape->dtype == DR_BF16, td, masks, head_fuse > 0 ? head_fuse : 1, scores,
                                    (hipStream_t)stream));
    return DR_OK;
}

dr_status dr_build_mask_tokens(dr_ctx* ctx, const dr_shape* shape, double tau_near, double lambda,
                               const dr_mask_params* params, const float* token_scores, int32_t* rowptr,
                               int32_t* colidx, int64_t colidx_capacity, int64_t* nnz, uint8_t* links, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    const dr_mask_params* p = params ? params : &kDefaults;
    dr_status st;
    if ((st = check_geometry(ctx, shape)) != DR_OK) return st;
    if ((st = check_params(ctx, p, lambda)) != DR_OK) return st;
    if (shape->B <= 0 || shape->H <= 0) return fail(ctx, DR_ERR_INVALID_ARG, "non-positive B or H");
    if (shape->B > 65535 || shape->H > 65535) return fail(ctx, DR_ERR_UNSUPPORTED, "B or H too large for the launch grid");
    if (std::isnan(tau_near)) return fail(ctx, DR_ERR_INVALID_ARG, "tau_1 is NaN");
    if (p->head_fuse > shape->H) return fail(ctx, DR_ERR_INVALID_ARG, "head_fuse=%d > H", p->head_fuse);
    if (!token_scores || !rowptr || !colidx || !nnz) return fail(ctx, DR_ERR_INVALID_ARG, "NULL output or scores pointer");
    if (colidx_capacity <= 0) return fail(ctx, DR_ERR_CAPACITY, "colidx_capacity must be > 0");
    const int Nt = shape->Hg * shape->Wg;
    if (shape->N > kMaxTokensTokenLevel || Nt > kMaxFrameTokensTokenLevel)
        return fail(ctx, DR_ERR_UNSUPPORTED, "N=%d / Nt=%d exceed %d / %d for the token-level order", shape->N, Nt,
                    kMaxTokensTokenLevel, kMaxFrameTokensTokenLevel);
    DeviceGuard g(ctx->device);
    hipStream_t s = (hipStream_t)stream;
    if ((st = ensure_geometry(ctx, shape, lambda, p, s)) != DR_OK) return st;
    const int Sb = (shape->N + shape->Bs - 1) / shape->Bs;
    const int masks = p->head_fuse > 0 ? 1 : shape->H;
    const size_t rows = (size_t)shape->B * masks * Sb;
    const size_t words = (Sb + 31) / 32;
    if ((st = grow(ctx, (void**)&ctx->keepbits, &ctx->keep_bytes, rows * words * 4)) != DR_OK) return st;
    if ((st = grow(ctx, (void**)&ctx->counts, &ctx->count_bytes, rows * 4)) != DR_OK) return st;
    if (!links) {
        const size_t need = (size_t)shape->B * masks * (size_t)shape->N * (size_t)shape->N;
        if ((st = grow(ctx, (void**)&ctx->links, &ctx->links_bytes, need)) != DR_OK) return st;
        links = ctx->links;
    }
    FrameTab tab;
    fill_frame_table(shape->Nf, Nt, shape->Bs, p->gamma, lambda, &tab);
    const Geometry geo = make_geometry(shape, p);
    DR_HIP(ctx, launch_pair_links(token_scores, tab, shape->B, masks, shape->N, Nt, shape->Nf, tau_near,
                                  p->has_tau_far ? p->tau_far : tau_near, links, s));
    DR_HIP(ctx, launch_aggregate_links(links, ctx->class_map, geo, shape->B, masks, ctx->keepbits, ctx->counts, s));
    DR_HIP(ctx, launch_emit(ctx->keepbits, ctx->counts, shape->B, masks, Sb, false, rowptr, colidx, colidx_capacity, nnz, s));
    return DR_OK;
}

namespace {

// Scratch that the attention kernels need beyond their inputs and outputs, in bytes: the per-wave range flags of the
// bf16 MFMA paths, and for the paths that walk merged key-block lists (block sizes 32 / 64, and the pair kernel of
// block size 128) the lists and their lengths.  Zero for the fp32 arithmetic path.
struct AttnScratchNeed { size_t flags, gcount, gcol; };

AttnScratchNeed attn_scratch_need(const AttnArgs& a, bool pairs) {
    AttnScratchNeed n{0, 0, 0};
    if (!attn_mfma_supported(a) && !attn_mfma_small_supported(a)) return n;
    const size_t groups128 = ((size_t)a.td.N + 127) / 128;
    n.flags = (size_t)a.td.B * a.td.H * groups128 * 4 * sizeof(int32_t);
    const bool lists = attn_mfma_small_supported(a) || pairs;
    if (lists) {
        const size_t groups = attn_mfma_small_supported(a) ? groups128 : ((size_t)a.Sb + 1) / 2;
        n.gcount = (size_t)a.td.B * a.mask_heads * groups * sizeof(int32_t);
        n.gcol = ((size_t)a.td.B * a.mask_heads * (size_t)a.colidx_stride + 1) * sizeof(int32_t);
    }
    return n;
}

dr_status attn_prepare(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, const void* V, const int32_t* rowptr,
                       const int32_t* colidx, int32_t mask_heads, int64_t colidx_stride, void* O, float* lse, AttnArgs* out) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    dr_status st;
    if ((st = check_tensor_shape(ctx, shape)) != DR_OK) return st;
    if (!Q || !K || !V || !O || !rowptr || !colidx) return fail(ctx, DR_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, DR_ERR_INVALID_ARG, "Q/K/V/O must be 16-byte aligned");
    if (mask_heads != 1 && mask_heads != shape->H) return fail(ctx, DR_ERR_INVALID_ARG, "mask_heads must be 1 or H");
    if (colidx_stride < 0) return fail(ctx, DR_ERR_INVALID_ARG, "negative colidx_stride");
    AttnArgs a{};
    a.Q = Q; a.K = K; a.V = V; a.O = O; a.lse = lse;
    a.rowptr = rowptr; a.colidx = colidx; a.colidx_stride = colidx_stride; a.mask_heads = mask_heads;
    a.td = TensorDesc{shape->stride_b, shape->stride_h, shape->stride_n, shape->B, shape->H, shape->N, shape->d};
    a.Bs = shape->Bs;
    a.Sb = (shape->N + shape->Bs - 1) / shape->Bs;
    a.bf16 = shape->dtype == DR_BF16;
    if (attn_mfma_small_supported(a) && a.Sb >= (1 << 28))
        return fail(ctx, DR_ERR_UNSUPPORTED, "too many blocks for the packed group lists");
    // the pre-pass that merges the rows of a workgroup's query blocks keeps one presence bitmap of Sb bits per row in LDS
    if (a.bf16 && a.td.d == 128 && (size_t)(256 / a.Bs) * (((size_t)a.Sb + 31) / 32) * 4 > 160 * 1024)
        return fail(ctx, DR_ERR_UNSUPPORTED, "%d key blocks per row: the list-merging pre-pass holds %d bitmaps of that many bits in "
                    "160 KB of LDS", a.Sb, 256 / a.Bs);
    *out = a;
    return DR_OK;
}

// The 256 queries of two (block size 128), four (64) or eight (32) adjacent query blocks walk the union of their rows,
// one wavefront per SIMD; rows that kernel flags are taken again by the second pass of the kernels with one 128-row group
// per workgroup.
bool attn_wants_pairs(const dr_ctx* ctx, const AttnArgs& a) {
    return ctx->attn_pairs && a.bf16 && a.td.d == 128 && (a.Bs == 128 || a.Bs == 64 || a.Bs == 32) && a.td.N >= 64 &&
           a.Sb < (a.Bs == 32 ? (1 << 24) : (1 << 28));
}

dr_status attn_launch(dr_ctx* ctx, const AttnArgs& a, bool pairs, hipStream_t s) {
    if (pairs && attn_mfma_pair_supported(a)) {
        DR_HIP(ctx, launch_attn_mfma_pair(a, s));
        if (a.Bs == 128) DR_HIP(ctx, launch_attn_mfma_second_pass(a, s));
        else DR_HIP(ctx, launch_attn_mfma_small_second_pass(a, s));
    } else if (attn_mfma_supported(a)) {
        DR_HIP(ctx, launch_attn_mfma(a, s));
    } else if (attn_mfma_small_supported(a)) {
        DR_HIP(ctx, launch_attn_mfma_small(a, s));
    } else {
        DR_HIP(ctx, launch_attn_generic(a, s));
    }
    return DR_OK;
}

}  // namespace

dr_status dr_sparse_attn_fwd(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, const void* V,
                             const int32_t* rowptr, const int32_t* colidx, int32_t mask_heads, int64_t colidx_stride,
                             void* O, float* lse, void* stream) {
    AttnArgs a{};
    dr_status st;
    if ((st = attn_prepare(ctx, shape, Q, K, V, rowptr, colidx, mask_heads, colidx_stride, O, lse, &a)) != DR_OK) return st;
    DeviceGuard g(ctx->device);
    const bool pairs = attn_wants_pairs(ctx, a);
    const AttnScratchNeed need = attn_scratch_need(a, pairs);
    if (need.flags && (st = grow(ctx, (void**)&ctx->attn_flags, &ctx->attn_flags_bytes, need.flags)) != DR_OK) return st;
    if (need.gcol && (st = grow(ctx, (void**)&ctx->gcol, &ctx->gcol_bytes, need.gcol)) != DR_OK) return st;
    if (need.gcount && (st = grow(ctx, (void**)&ctx->gcount, &ctx->gcount_bytes, need.gcount)) != DR_OK) return st;
    a.flags = need.flags ? ctx->attn_flags : nullptr;
    a.gcol = need.gcol ? ctx->gcol : nullptr;
    a.gcount = need.gcount ? ctx->gcount : nullptr;
    return attn_launch(ctx, a, pairs, (hipStream_t)stream);
}

dr_status dr_sparse_attn_fwd_static(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, const void* V,
                                    const int32_t* rowptr, const int32_t* colidx, int32_t mask_heads, int64_t colidx_stride,
                                    void* O, float* lse, void* stream) {
    AttnArgs a{};
    dr_status st;
    if ((st = attn_prepare(ctx, shape, Q, K, V, rowptr, colidx, mask_heads, colidx_stride, O, lse, &a)) != DR_OK) return st;
    if (!ctx->static_scratch) return fail(ctx, DR_ERR_HIP, "the static scratch area of this device was not resolved at dr_create");
    DeviceGuard g(ctx->device);
    const bool pairs = attn_wants_pairs(ctx, a);
    const AttnScratchNeed need = attn_scratch_need(a, pairs);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t total = up(need.flags) + up(need.gcount) + up(need.gcol);
    if (total > kStaticScratchBytes)
        return fail(ctx, DR_ERR_UNSUPPORTED, "this call needs %zu bytes of scratch (flags %zu, list lengths %zu, merged lists %zu); "
                    "the static area holds %zu: use dr_sparse_attn_fwd", total, need.flags, need.gcount, need.gcol, kStaticScratchBytes);
    unsigned char* base = ctx->static_scratch;
    a.flags = need.flags ? reinterpret_cast<int32_t*>(base) : nullptr;
    a.gcount = need.gcount ? reinterpret_cast<int32_t*>(base + up(need.flags)) : nullptr;
    a.gcol = need.gcol ? reinterpret_cast<int32_t*>(base + up(need.flags) + up(need.gcount)) : nullptr;
    return attn_launch(ctx, a, pairs, (hipStream_t)stream);
}

dr_status dr_proxy_loss(dr_ctx* ctx, const float* A_dense, const float* A_sparse, int32_t B, int32_t H, int32_t N,
                        const int64_t* nnz, int32_t masks, int32_t Sb, double target, double alpha, double* out,
                        void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    if (!A_dense || !A_sparse || !nnz || !out) return fail(ctx, DR_ERR_INVALID_ARG, "NULL pointer");
    if (B <= 0 || H <= 0 || N <= 0 || masks <= 0 || Sb <= 0) return fail(ctx, DR_ERR_INVALID_ARG, "non-positive size");
    if ((int64_t)B * H > 65535) return fail(ctx, DR_ERR_UNSUPPORTED, "B * H too large for the launch grid");
    if (std::isnan(target) || std::isnan(alpha)) return fail(ctx, DR_ERR_INVALID_ARG, "target or alpha is NaN");
    DeviceGuard g(ctx->device);
    dr_status st;
    const size_t need = (size_t)B * H * kProxySlices * 2 * sizeof(double);
    if ((st = grow(ctx, (void**)&ctx->proxy_partial, &ctx->proxy_bytes, need)) != DR_OK) return st;
    DR_HIP(ctx, launch_proxy_loss(A_dense, A_sparse, B * H, N, nnz, B * masks, Sb, target, alpha, ctx->proxy_partial, out,
                                  (hipStream_t)stream));
    return DR_OK;
}

dr_status dr_clock_probe(dr_ctx* ctx, uint64_t window_us, uint64_t* out, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    if (!out) return fail(ctx, DR_ERR_INVALID_ARG, "NULL output pointer");
    if (window_us == 0 || window_us > 2000000) return fail(ctx, DR_ERR_INVALID_ARG, "window must be 1 us .. 2 s");
    DeviceGuard g(ctx->device);
    DR_HIP(ctx, launch_clock_probe(window_us * 100ull, reinterpret_cast<unsigned long long*>(out), (hipStream_t)stream));
    return DR_OK;
}

dr_status dr_mfma_probe(dr_ctx* ctx, int32_t shape, int32_t workgroups, int32_t iters, int32_t random_operands,
                        float* sink, double* flop, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    if (!sink) return fail(ctx, DR_ERR_INVALID_ARG, "NULL sink pointer");
    if (shape != 32 && shape != 16) return fail(ctx, DR_ERR_INVALID_ARG, "shape must be 32 (32x32x16) or 16 (16x16x32)");
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || iters > (1 << 24) || (iters & 7))
        return fail(ctx, DR_ERR_INVALID_ARG, "workgroups must be 1 .. 2^20 and iters a multiple of 8 in 8 .. 2^24");
    // the kernel cannot be pre-empted: keep a launch to tens of milliseconds of matrix work on a full device
    if ((int64_t)workgroups * iters > (1ll << 26))
        return fail(ctx, DR_ERR_INVALID_ARG, "workgroups * iters = %lld exceeds 2^26", (long long)workgroups * iters);
    DeviceGuard g(ctx->device);
    DR_HIP(ctx, launch_mfma_probe(shape, workgroups, iters, random_operands ? 1 : 0, sink, (hipStream_t)stream));
    if (flop) *flop = (double)workgroups * 4.0 * (double)iters * 8.0 * (shape == 32 ? 32768.0 : 16384.0);
    return DR_OK;
}

dr_status dr_mfma_mix_probe(dr_ctx* ctx, int32_t workgroups, int32_t iters, float* sink, double* flop, void* stream) {
    if (!ctx) return DR_ERR_INVALID_ARG;
    if (!sink) return fail(ctx, DR_ERR_INVALID_ARG, "NULL sink pointer");
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || iters > (1 << 24))
        return fail(ctx, DR_ERR_INVALID_ARG, "workgroups must be 1 .. 2^20 and iters 1 .. 2^24");
    // the kernel cannot be pre-empted: keep a launch to tens of milliseconds on a full device
    if ((int64_t)workgroups * iters > (1ll << 26))
        return fail(ctx, DR_ERR_INVALID_ARG, "workgroups * iters = %lld exceeds 2^26", (long long)workgroups * iters);
    DeviceGuard g(ctx->device);
    DR_HIP(ctx, launch_mfma_mix_probe(workgroups, iters, sink, (hipStream_t)stream));
    if (flop) *flop = (double)workgroups * 4.0 * (double)iters * 8.0 * 32768.0;
    return DR_OK;
}

}  // extern "C"
