// C ABI of libdip: argument validation on the host, then kernel launches on the caller's
// stream.  Nothing here allocates device memory, synchronises, or reads device data.

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "dip_internal.h"

namespace dip {

static thread_local char t_err[512] = "";

int32_t fail(int32_t status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_err, sizeof(t_err), fmt, ap);
    va_end(ap);
    return status;
}

int32_t check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return DIP_OK;
    return fail(DIP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// ---- per-launch timing pool ---------------------------------------------------------------
namespace {
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> start, stop;
    std::vector<int> kind;
    size_t used = 0;
} g_prof;
}  // namespace

bool prof_next(int kind, hipEvent_t* start, hipEvent_t* stop) {
    if (!g_prof.on || g_prof.used >= g_prof.start.size()) return false;
    *start = g_prof.start[g_prof.used];
    *stop = g_prof.stop[g_prof.used];
    g_prof.kind[g_prof.used] = kind;
    ++g_prof.used;
    return true;
}

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int elem_bits(int dtype) { return dtype == DIP_F32 ? 32 : (dtype == DIP_BF16 ? 16 : 4); }

int32_t validate_weight(const dip_weight* w, const char* name) {
    if (!w) return fail(DIP_ERR_INVALID_ARG, "%s: null descriptor", name);
    if (!w->data) return fail(DIP_ERR_INVALID_ARG, "%s: null data pointer", name);
    if (w->n_in < 1 || w->n_out < 1) return fail(DIP_ERR_INVALID_ARG, "%s: n_in and n_out must be >= 1", name);
    if (w->reserved != 0) return fail(DIP_ERR_INVALID_ARG, "%s: reserved must be 0", name);
    if (w->dtype != DIP_F32 && w->dtype != DIP_BF16 && w->dtype != DIP_INT4_G128)
        return fail(DIP_ERR_UNSUPPORTED, "%s: unknown dtype %d", name, w->dtype);
    const int bits = elem_bits(w->dtype);
    const int per_load = 128 / bits;
    if (w->dtype == DIP_INT4_G128) {
        if (!w->scales) return fail(DIP_ERR_INVALID_ARG, "%s: int4 weights need a scales pointer", name);
        if (w->n_out % 128) return fail(DIP_ERR_UNSUPPORTED, "%s: int4 rows must be whole groups of 128", name);
        if (!aligned(w->scales, 2)) return fail(DIP_ERR_UNSUPPORTED, "%s: scales must be 2-byte aligned", name);
    }
    if (w->n_out % per_load) return fail(DIP_ERR_UNSUPPORTED, "%s: n_out must be a multiple of %d", name, per_load);
    if (w->row_stride_bytes < (int64_t)w->n_out * bits / 8)
        return fail(DIP_ERR_INVALID_ARG, "%s: row_stride_bytes smaller than a row", name);
    if (w->row_stride_bytes % 16 || !aligned(w->data, 16))
        return fail(DIP_ERR_UNSUPPORTED, "%s: rows must start on 16-byte boundaries", name);
    return DIP_OK;
}

int32_t validate_cache(const dip_cache* c, int n, const char* name) {
    if (!c->bits || !c->stamp || !c->meta) return fail(DIP_ERR_INVALID_ARG, "%s: null state pointer", name);
    if (c->n < 1 || c->n > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "%s: n must be in [1, %d]", name, DIP_MAX_N);
    if (n >= 0 && c->n != n) return fail(DIP_ERR_INVALID_ARG, "%s: cache covers %d columns, layer has %d", name, c->n, n);
    if (c->capacity < 0 || c->capacity > c->n) return fail(DIP_ERR_INVALID_ARG, "%s: capacity outside [0, n]", name);
    if (c->policy != DIP_LRU && c->policy != DIP_LFU) return fail(DIP_ERR_INVALID_ARG, "%s: unknown policy", name);
    if (c->reserved != 0) return fail(DIP_ERR_INVALID_ARG, "%s: reserved must be 0", name);
    return DIP_OK;
}

int32_t validate_gamma(float gamma) {
    if (!std::isfinite(gamma) || gamma < 0.f || gamma > 1.f)
        return fail(DIP_ERR_INVALID_ARG, "gamma must be finite and within [0, 1]");
    return DIP_OK;
}

// ---- workspace layout of the forward calls ---------------------------------------------------
// [ mask words of every layer: point 1, point 2 ]  kept until the cache updates at the end of the call
// [ scratch of one layer, shared by all layers   ]  index lists, h~, partial sums, ticket counters
constexpr size_t kMaskBytes = sizeof(uint32_t) * (DIP_MAX_N / 32);
constexpr int kMaxCounters = 2048;   // strips of the two products of a layer, at the narrowest strip width

struct ForwardPlan {
    int d, f;
    GemvShape ug, dn;          // selection and product launched apart
    GemvShape fug, fdn;        // product with the selection at its head
    bool fuse_ug, fuse_dn;
    int strips_ug, strips_dn;  // ticket counters (the larger of the two launch shapes)
    size_t off_idx1, off_val1, off_h, off_idx2, off_val2, off_part_ug, off_part_dn, off_cnt;
    size_t total;              // scratch of the layer, without the mask words
};

ForwardPlan plan_forward(const dip_mlp* mlp, int k_in, int k_mid) {
    ForwardPlan pl;
    pl.d = mlp->w_ug.n_in;
    pl.f = mlp->w_d.n_in;
    pl.ug = choose_gemv_shape(mlp->w_ug.dtype, pl.f, 2, k_in);
    pl.dn = choose_gemv_shape(mlp->w_d.dtype, pl.d, 1, k_mid);
    pl.fuse_ug = fused_shape(mlp->w_ug.dtype, pl.d, pl.f, 2, k_in, &pl.fug);
    pl.fuse_dn = fused_shape(mlp->w_d.dtype, pl.f, pl.d, 1, k_mid, &pl.fdn);
    pl.strips_ug = gemv_strips(pl.ug, mlp->w_ug.dtype, pl.f);
    pl.strips_dn = gemv_strips(pl.dn, mlp->w_d.dtype, pl.d);
    int ks_ug = pl.ug.ksplit, ks_dn = pl.dn.ksplit;
    if (pl.fuse_ug) {
        pl.strips_ug = std::max(pl.strips_ug, gemv_strips(pl.fug, mlp->w_ug.dtype, pl.f));
        ks_ug = std::max(ks_ug, pl.fug.ksplit);
    }
    if (pl.fuse_dn) {
        pl.strips_dn = std::max(pl.strips_dn, gemv_strips(pl.fdn, mlp->w_d.dtype, pl.d));
        ks_dn = std::max(ks_dn, pl.fdn.ksplit);
    }
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    // the ticket counters come first: they sit at the same place for every layer shape, are
    // cleared once per call and return to zero with every launch that uses them
    pl.off_cnt = take(sizeof(uint32_t) * kMaxCounters);
    pl.off_idx1 = take(sizeof(int32_t) * k_in);
    pl.off_val1 = take(sizeof(float) * k_in);
    pl.off_h = take(sizeof(float) * pl.f);
    pl.off_idx2 = take(sizeof(int32_t) * k_mid);
    pl.off_val2 = take(sizeof(float) * k_mid);
    pl.off_part_ug = take(ks_ug > 1 ? sizeof(float) * 2 * pl.f * ks_ug : 0);
    pl.off_part_dn = take(ks_dn > 1 ? sizeof(float) * pl.d * ks_dn : 0);
    pl.total = o;
    return pl;
}

int32_t validate_mlp(const dip_mlp* mlp, int k_in, int k_mid) {
    if (!mlp) return fail(DIP_ERR_INVALID_ARG, "mlp: null descriptor");
    int32_t st = validate_weight(&mlp->w_ug, "w_ug");
    if (st) return st;
    st = validate_weight(&mlp->w_d, "w_d");
    if (st) return st;
    const int d = mlp->w_ug.n_in, f = mlp->w_d.n_in;
    if (mlp->w_ug.n_out != 2 * f) return fail(DIP_ERR_INVALID_ARG, "w_ug.n_out must be 2 * w_d.n_in (bundled up/gate)");
    if (mlp->w_d.n_out != d) return fail(DIP_ERR_INVALID_ARG, "w_d.n_out must equal w_ug.n_in");
    if (d > DIP_MAX_N || f > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "d_model and d_ff must be <= %d", DIP_MAX_N);
    const int per_load = mlp->w_ug.dtype == DIP_INT4_G128 ? 128 : 128 / elem_bits(mlp->w_ug.dtype);
    if (f % per_load) return fail(DIP_ERR_UNSUPPORTED, "d_ff must be a multiple of %d", per_load);
    if (k_in < 1 || k_in > d) return fail(DIP_ERR_INVALID_ARG, "k_in must be in [1, d_model]");
    if (k_mid < 1 || k_mid > f) return fail(DIP_ERR_INVALID_ARG, "k_mid must be in [1, d_ff]");
    return DIP_OK;
}

// One token through one layer.  Launches, with a product that runs its own selection:
//   up/gate product   (scores + top-K of point 1 at its head)
//   down product      (scores + top-K of point 2 at its head)
// and otherwise selection and product apart (four launches).  Either way the masks go to the
// layer's two mask buffers and the cache updates are left to the caller, which runs them all
// in one launch at the end of the call: a cache is scored with its state from before this
// token (Alg. 1 takes c^(t-1)), and the update is in place before the next call scores it.
int32_t forward_one(const dip_mlp* mlp, const ForwardPlan& pl, const float* x, int k_in, int k_mid,
                    const dip_cache* cin, const dip_cache* cmid, float gamma, float* y,
                    const dip_debug* dbg, char* ws, uint32_t* mask1, uint32_t* mask2, hipStream_t stream,
                    std::vector<UpdatePiece>& updates, bool dense_in = false) {
    int32_t* idx1 = reinterpret_cast<int32_t*>(ws + pl.off_idx1);
    float* val1 = reinterpret_cast<float*>(ws + pl.off_val1);
    float* h = reinterpret_cast<float*>(ws + pl.off_h);
    int32_t* idx2 = reinterpret_cast<int32_t*>(ws + pl.off_idx2);
    float* val2 = reinterpret_cast<float*>(ws + pl.off_val2);
    float* part_ug = reinterpret_cast<float*>(ws + pl.off_part_ug);
    float* part_dn = reinterpret_cast<float*>(ws + pl.off_part_dn);
    uint32_t* cnt_ug = reinterpret_cast<uint32_t*>(ws + pl.off_cnt);
    uint32_t* cnt_dn = cnt_ug + pl.strips_ug;
    if (dbg && dbg->idx_in) idx1 = dbg->idx_in;
    if (dbg && dbg->idx_mid) idx2 = dbg->idx_mid;
    if (dbg && dbg->h) h = dbg->h;
    if (dbg && dbg->mask_in) mask1 = dbg->mask_in;
    if (dbg && dbg->mask_mid) mask2 = dbg->mask_mid;
    const bool want_mask1 = cin || (dbg && dbg->mask_in);
    const bool want_mask2 = cmid || (dbg && dbg->mask_mid);

    auto update_of = [](const dip_cache* c, const uint32_t* mask) {
        UpdatePiece u;
        u.mask = mask; u.bits = c->bits; u.stamp = c->stamp; u.meta = c->meta;
        u.n = c->n; u.capacity = c->capacity; u.policy = c->policy; u.pad = 0;
        return u;
    };

    int32_t st = DIP_OK;
    GemvParams g1;
    std::memset(&g1, 0, sizeof(g1));
    g1.w = mlp->w_ug.data; g1.row_stride = mlp->w_ug.row_stride_bytes;
    g1.scales = static_cast<const uint16_t*>(mlp->w_ug.scales); g1.scale_stride = mlp->w_ug.n_out / 128; g1.dtype = mlp->w_ug.dtype;
    g1.n_in = pl.d; g1.n_out = pl.f; g1.nseg = 2; g1.k = k_in; g1.out = h;
    g1.partial = part_ug; g1.counters = cnt_ug;
    if (dense_in) {
        // GLU pruning (Sec. 3.2): nothing is pruned at point 1, every stored row in order
        // (in the launch shape DIP would use with k_in = d_model, so that both give the same bits)
        g1.idx = nullptr; g1.val = x;
        st = check_hip(launch_gemv(g1, pl.fuse_ug ? pl.fug : pl.ug, stream, DIP_KERNEL_GEMV_UPGATE), "dense GEMV (up/gate)");
    } else if (pl.fuse_ug) {
        FusedParams fp;
        fp.g = g1;
        fp.s.v = x; fp.s.n = pl.d; fp.s.score_bits = cin ? cin->bits : nullptr; fp.s.gamma = gamma;
        fp.s.mask_out = want_mask1 ? mask1 : nullptr;
        fp.s.idx_out = dbg ? dbg->idx_in : nullptr;
        fp.s.s_out = dbg ? dbg->s_in : nullptr;
        st = check_hip(launch_fused(fp, pl.fug, stream, DIP_KERNEL_GEMV_UPGATE), "up/gate product with selection");
    } else {
        SelectParams s1;
        std::memset(&s1, 0, sizeof(s1));
        s1.v = x; s1.n = pl.d; s1.k = k_in; s1.gamma = gamma;
        s1.s_out = dbg ? dbg->s_in : nullptr;
        s1.mask_out = want_mask1 ? mask1 : nullptr;
        s1.idx_out = idx1; s1.val_out = val1;
        if (cin) s1.score_bits = cin->bits;
        st = check_hip(launch_select(s1, stream, DIP_KERNEL_SELECT_IN), "select (point 1)");
        if (st) return st;
        g1.idx = idx1; g1.val = val1;
        st = check_hip(launch_gemv(g1, pl.ug, stream, DIP_KERNEL_GEMV_UPGATE), "gathered GEMV (up/gate)");
    }
    if (st) return st;
    if (cin && !dense_in) updates.push_back(update_of(cin, mask1));

    GemvParams g2;
    std::memset(&g2, 0, sizeof(g2));
    g2.w = mlp->w_d.data; g2.row_stride = mlp->w_d.row_stride_bytes;
    g2.scales = static_cast<const uint16_t*>(mlp->w_d.scales); g2.scale_stride = mlp->w_d.n_out / 128; g2.dtype = mlp->w_d.dtype;
    g2.n_in = pl.f; g2.n_out = pl.d; g2.nseg = 1; g2.k = k_mid; g2.out = y;
    g2.partial = part_dn; g2.counters = cnt_dn;
    if (pl.fuse_dn) {
        FusedParams fp;
        fp.g = g2;
        fp.s.v = h; fp.s.n = pl.f; fp.s.score_bits = cmid ? cmid->bits : nullptr; fp.s.gamma = gamma;
        fp.s.mask_out = want_mask2 ? mask2 : nullptr;
        fp.s.idx_out = dbg ? dbg->idx_mid : nullptr;
        fp.s.s_out = dbg ? dbg->s_mid : nullptr;
        st = check_hip(launch_fused(fp, pl.fdn, stream, DIP_KERNEL_GEMV_DOWN), "down product with selection");
    } else {
        SelectParams s2;
        std::memset(&s2, 0, sizeof(s2));
        s2.v = h; s2.n = pl.f; s2.k = k_mid; s2.gamma = gamma;
        s2.s_out = dbg ? dbg->s_mid : nullptr;
        s2.mask_out = want_mask2 ? mask2 : nullptr;
        s2.idx_out = idx2; s2.val_out = val2;
        if (cmid) s2.score_bits = cmid->bits;
        st = check_hip(launch_select(s2, stream, DIP_KERNEL_SELECT_MID), "select (point 2)");
        if (st) return st;
        g2.idx = idx2; g2.val = val2;
        st = check_hip(launch_gemv(g2, pl.dn, stream, DIP_KERNEL_GEMV_DOWN), "gathered GEMV (down)");
    }
    if (st) return st;
    if (cmid) updates.push_back(update_of(cmid, mask2));
    return DIP_OK;
}

}  // namespace
}  // namespace dip

using namespace dip;

extern "C" {

int32_t dip_version(void) { return (DIP_VERSION_MAJOR << 16) | DIP_VERSION_MINOR; }

const char* dip_last_error(void) { return t_err; }

int32_t dip_ca_scores(const float* x, int32_t n, const uint32_t* cache_bits, float gamma,
                      float* s_out, void* stream) {
    if (!x || !s_out) return fail(DIP_ERR_INVALID_ARG, "dip_ca_scores: null pointer");
    if (n < 1) return fail(DIP_ERR_INVALID_ARG, "dip_ca_scores: n must be >= 1");
    if (n > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "dip_ca_scores: n must be <= %d", DIP_MAX_N);
    if (cache_bits) {
        int32_t st = validate_gamma(gamma);
        if (st) return st;
    }
    SelectParams p;
    std::memset(&p, 0, sizeof(p));
    p.v = x; p.n = n; p.k = 1; p.score_bits = cache_bits; p.gamma = gamma;
    p.scores_only = 1; p.s_out = s_out;
    return check_hip(launch_select(p, static_cast<hipStream_t>(stream), DIP_KERNEL_SELECT_IN), "dip_ca_scores");
}

int32_t dip_prune_topk(const float* s, int32_t n, int32_t k, uint32_t* mask_out, int32_t* idx_out,
                       void* stream) {
    if (!s) return fail(DIP_ERR_INVALID_ARG, "dip_prune_topk: null input");
    if (!mask_out && !idx_out) return fail(DIP_ERR_INVALID_ARG, "dip_prune_topk: no output requested");
    if (n < 1) return fail(DIP_ERR_INVALID_ARG, "dip_prune_topk: n must be >= 1");
    if (n > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "dip_prune_topk: n must be <= %d", DIP_MAX_N);
    if (k < 1 || k > n) return fail(DIP_ERR_INVALID_ARG, "dip_prune_topk: k must be in [1, n]");
    SelectParams p;
    std::memset(&p, 0, sizeof(p));
    p.v = s; p.n = n; p.k = k; p.mask_out = mask_out; p.idx_out = idx_out;
    return check_hip(launch_select(p, static_cast<hipStream_t>(stream), DIP_KERNEL_SELECT_IN), "dip_prune_topk");
}

int32_t dip_cache_init(const dip_cache* cache, const uint32_t* initial_bits, void* stream) {
    if (!cache) return fail(DIP_ERR_INVALID_ARG, "dip_cache_init: null descriptor");
    int32_t st = validate_cache(cache, -1, "dip_cache_init");
    if (st) return st;
    CacheInitParams p{cache->bits, cache->stamp, cache->meta, initial_bits, cache->n};
    return check_hip(launch_cache_init(p, static_cast<hipStream_t>(stream)), "dip_cache_init");
}

int32_t dip_cache_update(const dip_cache* cache, const uint32_t* mask_bits, void* stream) {
    if (!cache) return fail(DIP_ERR_INVALID_ARG, "dip_cache_update: null descriptor");
    if (!mask_bits) return fail(DIP_ERR_INVALID_ARG, "dip_cache_update: null mask");
    int32_t st = validate_cache(cache, -1, "dip_cache_update");
    if (st) return st;
    SelectParams p;
    std::memset(&p, 0, sizeof(p));
    p.n = cache->n; p.k = 1; p.mask_in = mask_bits;
    p.c_bits = cache->bits; p.c_stamp = cache->stamp; p.c_meta = cache->meta;
    p.capacity = cache->capacity; p.policy = cache->policy;
    return check_hip(launch_select(p, static_cast<hipStream_t>(stream), DIP_KERNEL_SELECT_IN), "dip_cache_update");
}

int32_t dip_cache_state_bytes(int32_t n, size_t* bits_bytes, size_t* stamp_bytes, size_t* meta_bytes) {
    if (n < 1 || n > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "dip_cache_state_bytes: n must be in [1, %d]", DIP_MAX_N);
    if (bits_bytes) *bits_bytes = sizeof(uint32_t) * (size_t)((n + 31) / 32);
    if (stamp_bytes) *stamp_bytes = sizeof(uint32_t) * (size_t)n;
    if (meta_bytes) *meta_bytes = sizeof(uint32_t) * DIP_CACHE_META_WORDS;
    return DIP_OK;
}

size_t dip_cache_blob_bytes(int32_t n) {
    if (n < 1 || n > DIP_MAX_N) return 0;
    return align_up(sizeof(uint32_t) * (size_t)((n + 31) / 32), 256) + align_up(sizeof(uint32_t) * (size_t)n, 256) +
           align_up(sizeof(uint32_t) * DIP_CACHE_META_WORDS, 256);
}

static int32_t cache_blob_copy(const dip_cache* cache, void* blob, size_t blob_bytes, void* stream,
                               bool to_blob, const char* name) {
    if (!cache || !blob) return fail(DIP_ERR_INVALID_ARG, "%s: null pointer", name);
    int32_t st = validate_cache(cache, -1, name);
    if (st) return st;
    if (blob_bytes < dip_cache_blob_bytes(cache->n))
        return fail(DIP_ERR_INVALID_ARG, "%s: blob smaller than dip_cache_blob_bytes(n)", name);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* b = static_cast<char*>(blob);
    const size_t nb = sizeof(uint32_t) * (size_t)((cache->n + 31) / 32), ns = sizeof(uint32_t) * (size_t)cache->n;
    const size_t nm = sizeof(uint32_t) * DIP_CACHE_META_WORDS;
    void* part[3] = {cache->bits, cache->stamp, cache->meta};
    const size_t bytes[3] = {nb, ns, nm};
    size_t off = 0;
    for (int i = 0; i < 3; ++i) {
        hipError_t e = to_blob ? hipMemcpyAsync(b + off, part[i], bytes[i], hipMemcpyDefault, hs)
                               : hipMemcpyAsync(part[i], b + off, bytes[i], hipMemcpyDefault, hs);
        if ((st = check_hip(e, name))) return st;
        off += align_up(bytes[i], 256);
    }
    return DIP_OK;
}

int32_t dip_cache_export(const dip_cache* cache, void* blob, size_t blob_bytes, void* stream) {
    return cache_blob_copy(cache, blob, blob_bytes, stream, true, "dip_cache_export");
}

int32_t dip_cache_import(const dip_cache* cache, const void* blob, size_t blob_bytes, void* stream) {
    return cache_blob_copy(cache, const_cast<void*>(blob), blob_bytes, stream, false, "dip_cache_import");
}

size_t dip_gathered_gemv_workspace_bytes(const dip_weight* w, int32_t k) {
    if (!w || w->n_out < 1 || k < 1) return 0;
    if (w->dtype != DIP_F32 && w->dtype != DIP_BF16 && w->dtype != DIP_INT4_G128) return 0;
    const GemvShape s = choose_gemv_shape(w->dtype, w->n_out, 1, k);
    const int strips = gemv_strips(s, w->dtype, w->n_out);
    size_t bytes = align_up(sizeof(uint32_t) * strips, 256);
    bytes += 2 * align_up(sizeof(float) * (size_t)k, 256);   // aligned copies of idx and x[idx]
    if (s.ksplit > 1) bytes += align_up(sizeof(float) * (size_t)w->n_out * s.ksplit, 256);
    return bytes;
}

int32_t dip_gathered_gemv(const dip_weight* w, const float* x, const int32_t* idx, int32_t k,
                          float* y_out, void* ws, size_t ws_bytes, void* stream) {
    int32_t st = validate_weight(w, "dip_gathered_gemv");
    if (st) return st;
    if (!x || !idx || !y_out) return fail(DIP_ERR_INVALID_ARG, "dip_gathered_gemv: null pointer");
    if (k < 1 || k > w->n_in) return fail(DIP_ERR_INVALID_ARG, "dip_gathered_gemv: k must be in [1, n_in]");
    const size_t need = dip_gathered_gemv_workspace_bytes(w, k);
    if (!ws || ws_bytes < need || !aligned(ws, 256))
        return fail(DIP_ERR_WORKSPACE, "dip_gathered_gemv: workspace must be 256-aligned and >= %zu bytes", need);
    const GemvShape s = choose_gemv_shape(w->dtype, w->n_out, 1, k);
    const int strips = gemv_strips(s, w->dtype, w->n_out);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    uint32_t* counters = reinterpret_cast<uint32_t*>(base);
    size_t o = align_up(sizeof(uint32_t) * strips, 256);
    int32_t* idx_copy = reinterpret_cast<int32_t*>(base + o);
    o += align_up(sizeof(float) * (size_t)k, 256);
    float* val = reinterpret_cast<float*>(base + o);
    o += align_up(sizeof(float) * (size_t)k, 256);
    float* partial = reinterpret_cast<float*>(base + o);
    if (s.ksplit > 1) {
        st = check_hip(launch_zero_u32(counters, strips, hs), "dip_gathered_gemv: counter reset");
        if (st) return st;
    }
    // the kernel reads (index, multiplier) pairs as aligned vectors
    st = check_hip(launch_gather(x, idx, k, w->n_in, val, idx_copy, hs), "dip_gathered_gemv: gather");
    if (st) return st;
    GemvParams p;
    std::memset(&p, 0, sizeof(p));
    p.w = w->data; p.row_stride = w->row_stride_bytes; p.dtype = w->dtype;
    p.scales = static_cast<const uint16_t*>(w->scales); p.scale_stride = w->n_out / 128; p.n_in = w->n_in; p.n_out = w->n_out;
    p.nseg = 1; p.idx = idx_copy; p.val = val; p.k = k; p.out = y_out;
    p.partial = partial; p.counters = counters;
    return check_hip(launch_gemv(p, s, hs, DIP_KERNEL_GEMV_DOWN), "dip_gathered_gemv");
}

size_t dip_swiglu_mlp_forward_workspace_bytes(const dip_mlp* mlp, int32_t k_in, int32_t k_mid) {
    if (validate_mlp(mlp, k_in, k_mid)) return 0;
    return 2 * kMaskBytes + plan_forward(mlp, k_in, k_mid).total;
}

size_t dip_swiglu_mlp_forward_stack_workspace_bytes(const dip_mlp* mlps, int32_t n_layers,
                                                    const int32_t* k_in, const int32_t* k_mid) {
    if (!mlps || !k_in || !k_mid || n_layers < 1) return 0;
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (validate_mlp(&mlps[l], k_in[l], k_mid[l])) return 0;
        need = std::max(need, plan_forward(&mlps[l], k_in[l], k_mid[l]).total);
    }
    return (size_t)n_layers * 2 * kMaskBytes + need;
}

// k_in / k_mid: one value per layer (k_stride = 1) or one for all (k_stride = 0)
static int32_t forward_checked(const dip_mlp* mlps, int32_t n_layers, const float* x, int64_t x_stride,
                               const int32_t* k_in, const int32_t* k_mid, int k_stride,
                               const dip_cache* caches_in, const dip_cache* caches_mid, float gamma,
                               float* y_out, int64_t y_stride, const dip_debug* dbg, void* ws,
                               size_t ws_bytes, void* stream, bool dense_in = false) {
    if (!mlps) return fail(DIP_ERR_INVALID_ARG, "forward: null mlp descriptor");
    if (n_layers < 1) return fail(DIP_ERR_INVALID_ARG, "forward: n_layers must be >= 1");
    if (!x || !y_out) return fail(DIP_ERR_INVALID_ARG, "forward: null x or y_out");
    if (!k_in || !k_mid) return fail(DIP_ERR_INVALID_ARG, "forward: null k_in or k_mid");
    if (caches_in || caches_mid) {
        int32_t st = validate_gamma(gamma);
        if (st) return st;
    }
    if (dbg && (!aligned(dbg->idx_in, 16) || !aligned(dbg->idx_mid, 16)))
        return fail(DIP_ERR_UNSUPPORTED, "forward: debug index lists must be 16-byte aligned");
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        int32_t st = validate_mlp(&mlps[l], k_in[l * k_stride], k_mid[l * k_stride]);
        if (st) return st;
        if (caches_in && (st = validate_cache(&caches_in[l], mlps[l].w_ug.n_in, "cache_in"))) return st;
        if (caches_mid && (st = validate_cache(&caches_mid[l], mlps[l].w_d.n_in, "cache_mid"))) return st;
        need = std::max(need, plan_forward(&mlps[l], k_in[l * k_stride], k_mid[l * k_stride]).total);
    }
    // Every cache is scored in its layer's launches and updated at the end of the call: two
    // layers (or the two points of one layer) that shared a cache would score the second use
    // against a state that lacks the first one's update.
    {
        std::vector<const uint32_t*> seen;
        for (int l = 0; l < n_layers; ++l) {
            if (caches_in) seen.push_back(caches_in[l].bits);
            if (caches_mid) seen.push_back(caches_mid[l].bits);
        }
        std::sort(seen.begin(), seen.end());
        if (std::adjacent_find(seen.begin(), seen.end()) != seen.end())
            return fail(DIP_ERR_INVALID_ARG, "forward: two pruning points share one cache state (every layer "
                                             "and point needs a dip_cache of its own)");
    }
    const size_t mask_bytes = (size_t)n_layers * 2 * kMaskBytes;
    need += mask_bytes;
    if (!ws || ws_bytes < need || !aligned(ws, 256))
        return fail(DIP_ERR_WORKSPACE, "forward: workspace must be 256-aligned and >= %zu bytes", need);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    char* scratch = base + mask_bytes;
    // the ticket counters of the products start at zero and return to zero with every launch
    int32_t st = check_hip(launch_zero_u32(reinterpret_cast<uint32_t*>(scratch), kMaxCounters, hs), "counter reset");
    if (st) return st;
    std::vector<UpdatePiece> updates;
    updates.reserve(2 * (size_t)n_layers);
    for (int l = 0; l < n_layers && !st; ++l) {
        const int ki = k_in[l * k_stride], km = k_mid[l * k_stride];
        const ForwardPlan pl = plan_forward(&mlps[l], ki, km);
        uint32_t* mask1 = reinterpret_cast<uint32_t*>(base + (size_t)(2 * l) * kMaskBytes);
        uint32_t* mask2 = reinterpret_cast<uint32_t*>(base + (size_t)(2 * l + 1) * kMaskBytes);
        st = forward_one(&mlps[l], pl, x + (int64_t)l * x_stride, ki, km,
                         caches_in ? &caches_in[l] : nullptr, caches_mid ? &caches_mid[l] : nullptr, gamma,
                         y_out + (int64_t)l * y_stride, dbg, scratch, mask1, mask2, hs, updates, dense_in);
    }
    // (after a failed launch: the updates of what was launched keep the caches consistent with it)
    if (!updates.empty()) {
        const int32_t st2 = check_hip(launch_update_batch(updates.data(), (int)updates.size(), hs, DIP_KERNEL_CACHE_UPDATE),
                                      "cache updates");
        if (!st) st = st2;
    }
    return st;
}

int32_t dip_swiglu_mlp_forward(const dip_mlp* mlp, const float* x, int32_t k_in, int32_t k_mid,
                               const dip_cache* cache_in, const dip_cache* cache_mid, float gamma,
                               float* y_out, const dip_debug* dbg, void* ws, size_t ws_bytes,
                               void* stream) {
    return forward_checked(mlp, 1, x, 0, &k_in, &k_mid, 0, cache_in, cache_mid, gamma, y_out, 0, dbg, ws,
                           ws_bytes, stream);
}

// ---- the forward for callers that cannot allocate ------------------------------------------
// The workspace of dip_swiglu_mlp_forward, held in the library's own device memory: one
// array per GPU, present from the moment the code object is loaded until the process ends.
// In host code `g_static_scratch` is only a handle for hipGetSymbolAddress; the address the
// kernels get is the one that call returns for the current device.
static __device__ __align__(256) unsigned char g_static_scratch[DIP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int32_t static_scratch(void** out) {
    int dev = -1;
    int32_t st = check_hip(hipGetDevice(&dev), "hipGetDevice");
    if (st) return st;
    if (dev < 0 || dev >= kMaxDevices) return fail(DIP_ERR_UNSUPPORTED, "device ordinal %d not supported", dev);
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // every thread that gets here asks for the same address of the same device
        st = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)), "hipGetSymbolAddress");
        if (st) return st;
        if (!p) return fail(DIP_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return DIP_OK;
}
}  // namespace

int32_t dip_swiglu_mlp_forward_noalloc(const dip_mlp* mlp, const float* x, int32_t k_in, int32_t k_mid,
                                       const dip_cache* cache_in, const dip_cache* cache_mid,
                                       float gamma, float* y_out, const dip_debug* dbg, void* stream) {
    int32_t st = validate_mlp(mlp, k_in, k_mid);
    if (st) return st;
    const size_t need = 2 * kMaskBytes + plan_forward(mlp, k_in, k_mid).total;
    if (need > (size_t)DIP_STATIC_SCRATCH_BYTES)
        return fail(DIP_ERR_WORKSPACE,
                    "dip_swiglu_mlp_forward_noalloc: this layer needs %zu bytes of scratch, the built-in "
                    "buffer holds %zu; use dip_swiglu_mlp_forward with a caller workspace",
                    need, (size_t)DIP_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if ((st = static_scratch(&ws))) return st;
    return forward_checked(mlp, 1, x, 0, &k_in, &k_mid, 0, cache_in, cache_mid, gamma, y_out, 0, dbg, ws,
                           (size_t)DIP_STATIC_SCRATCH_BYTES, stream);
}

int32_t dip_swiglu_mlp_forward_stack(const dip_mlp* mlps, int32_t n_layers, const float* x,
                                     int64_t x_stride, const int32_t* k_in, const int32_t* k_mid,
                                     const dip_cache* caches_in, const dip_cache* caches_mid,
                                     float gamma, float* y_out, int64_t y_stride, void* ws,
                                     size_t ws_bytes, void* stream) {
    return forward_checked(mlps, n_layers, x, x_stride, k_in, k_mid, 1, caches_in, caches_mid, gamma,
                           y_out, y_stride, nullptr, ws, ws_bytes, stream);
}

namespace {
struct BatchedPlan {
    int d, f, wd, wf, k1max, k2max, g1, g2;
    bool mc1, mc2;             // product on the matrix cores
    size_t off_rmax, off_m1, off_idx1, off_val1, off_m2, off_idx2, off_val2, off_cnt, off_h,
        off_part;
    size_t total;
};
BatchedPlan plan_batched(const dip_mlp* mlp, int B, int k_in, int k_mid) {
    BatchedPlan pl;
    pl.d = mlp->w_ug.n_in; pl.f = mlp->w_d.n_in;
    pl.wd = (pl.d + 31) / 32; pl.wf = (pl.f + 31) / 32;
    pl.k1max = std::min(pl.d, B * k_in);
    pl.k2max = std::min(pl.f, B * k_mid);
    pl.mc1 = batched_on_matrix_cores(mlp->w_ug.dtype, B, mlp->w_ug.n_in, mlp->w_ug.row_stride_bytes);
    pl.mc2 = batched_on_matrix_cores(mlp->w_d.dtype, B, mlp->w_d.n_in, mlp->w_d.row_stride_bytes);
    pl.g1 = batched_shares(mlp->w_ug.dtype, B, 2 * pl.f, pl.k1max, pl.mc1);
    pl.g2 = batched_shares(mlp->w_d.dtype, B, pl.d, pl.k2max, pl.mc2);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    pl.off_rmax = take(sizeof(uint32_t) * 16);     // per point: 8 row maxima
    pl.off_m1 = take(sizeof(uint32_t) * B * pl.wd);
    // index and multiplier lists carry 16 spare entries: the product reads whole vectors
    pl.off_idx1 = take(sizeof(int32_t) * (pl.k1max + 16));
    pl.off_val1 = take(sizeof(float) * (size_t)(pl.k1max + 16) * B);
    pl.off_m2 = take(sizeof(uint32_t) * B * pl.wf);
    pl.off_idx2 = take(sizeof(int32_t) * (pl.k2max + 16));
    pl.off_val2 = take(sizeof(float) * (size_t)(pl.k2max + 16) * B);
    pl.off_cnt = take(sizeof(uint32_t) * 2);
    pl.off_h = take(sizeof(float) * (size_t)B * pl.f);
    const size_t p1 = sizeof(float) * (size_t)pl.g1 * B * 2 * pl.f;
    const size_t p2 = sizeof(float) * (size_t)pl.g2 * B * pl.d;
    pl.off_part = take(std::max(p1, p2));
    pl.total = o;
    return pl;
}
}  // namespace

// Workspace of the batched calls: [ union mask words of every layer: point 1, point 2 ] kept
// until the cache updates at the end of the call, then the scratch of one layer.
size_t dip_swiglu_mlp_forward_batched_workspace_bytes(const dip_mlp* mlp, int32_t batch,
                                                      int32_t k_in, int32_t k_mid) {
    if (batch < 1 || batch > 8 || validate_mlp(mlp, k_in, k_mid)) return 0;
    return 2 * kMaskBytes + plan_batched(mlp, batch, k_in, k_mid).total;
}

size_t dip_swiglu_mlp_forward_batched_stack_workspace_bytes(const dip_mlp* mlps, int32_t n_layers, int32_t batch,
                                                            const int32_t* k_in, const int32_t* k_mid) {
    if (!mlps || !k_in || !k_mid || n_layers < 1 || batch < 1 || batch > 8) return 0;
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (validate_mlp(&mlps[l], k_in[l], k_mid[l])) return 0;
        need = std::max(need, plan_batched(&mlps[l], batch, k_in[l], k_mid[l]).total);
    }
    return (size_t)n_layers * 2 * kMaskBytes + need;
}

namespace {
// `batch` rows through one layer; the union masks go to uw1 / uw2 and the cache updates with
// them are left to the caller (one launch at the end of the call).
int32_t batched_one(const dip_mlp* mlp, const BatchedPlan& pl, const float* X, int batch, int k_in, int k_mid,
                    const dip_cache* cache_in, const dip_cache* cache_mid, float gamma, float* Y,
                    uint32_t* mask_in_out, float* h_out, uint32_t* mask_mid_out, char* base, uint32_t* uw1,
                    uint32_t* uw2, hipStream_t hs, std::vector<UpdatePiece>& updates) {
    int32_t st = DIP_OK;
    uint32_t* cnt = reinterpret_cast<uint32_t*>(base + pl.off_cnt);
    float* H = h_out ? h_out : reinterpret_cast<float*>(base + pl.off_h);
    float* part = reinterpret_cast<float*>(base + pl.off_part);

    struct Point {
        const float* v; int n, k, kmax, words; const dip_cache* cache; uint32_t* masks; uint32_t* uwords;
        int32_t* uidx; float* uval; uint32_t* count; int kind;
    };
    const Point pts[2] = {
        {X, pl.d, k_in, pl.k1max, pl.wd, cache_in,
         mask_in_out ? mask_in_out : reinterpret_cast<uint32_t*>(base + pl.off_m1), uw1,
         reinterpret_cast<int32_t*>(base + pl.off_idx1), reinterpret_cast<float*>(base + pl.off_val1), cnt,
         DIP_KERNEL_SELECT_IN},
        {H, pl.f, k_mid, pl.k2max, pl.wf, cache_mid,
         mask_mid_out ? mask_mid_out : reinterpret_cast<uint32_t*>(base + pl.off_m2), uw2,
         reinterpret_cast<int32_t*>(base + pl.off_idx2), reinterpret_cast<float*>(base + pl.off_val2), cnt + 1,
         DIP_KERNEL_SELECT_MID}};
    for (int pt = 0; pt < 2; ++pt) {
        const Point& q = pts[pt];
        // per-row scores and masks (state of the cache from before the step)
        SelectParams sp;
        std::memset(&sp, 0, sizeof(sp));
        sp.v = q.v; sp.n = q.n; sp.k = q.k; sp.gamma = gamma;
        sp.score_bits = q.cache ? q.cache->bits : nullptr;
        sp.mask_out = q.masks; sp.rows = batch; sp.v_row_stride = q.n; sp.words_row_stride = q.words;
        const bool mc = pt == 0 ? pl.mc1 : pl.mc2;
        uint32_t* rowmax = reinterpret_cast<uint32_t*>(base + pl.off_rmax) + 8 * pt;
        sp.rowmax_out = mc ? rowmax : nullptr;     // max |x| per row, for the matrix-core product's scaling
        if ((st = check_hip(launch_select_rows(sp, hs, q.kind), "forward_batched: select"))) return st;
        // union of the row masks, its index list and the row multipliers
        UnionParams up;
        std::memset(&up, 0, sizeof(up));
        up.masks = q.masks; up.words_stride = q.words; up.x = q.v; up.x_stride = q.n; up.n = q.n;
        up.batch = batch; up.union_words = q.uwords; up.uidx = q.uidx; up.uval = q.uval; up.count_out = q.count;
        if ((st = check_hip(launch_union(up, hs), "forward_batched: union"))) return st;
        // one cache update with the union mask (Alg. 1 step 3), run by the caller
        if (q.cache) {
            UpdatePiece u;
            u.mask = q.uwords; u.bits = q.cache->bits; u.stamp = q.cache->stamp; u.meta = q.cache->meta;
            u.n = q.n; u.capacity = q.cache->capacity; u.policy = q.cache->policy; u.pad = 0;
            updates.push_back(u);
        }
        // gathered product for all rows, then the reduction with its epilogue
        const dip_weight& w = pt == 0 ? mlp->w_ug : mlp->w_d;
        const int shares = pt == 0 ? pl.g1 : pl.g2;
        BatchedGemvParams gp;
        std::memset(&gp, 0, sizeof(gp));
        gp.w = w.data; gp.row_stride = w.row_stride_bytes;
        gp.scales = static_cast<const uint16_t*>(w.scales); gp.scale_stride = w.n_out / 128;
        gp.dtype = w.dtype; gp.n_in = w.n_in; gp.n_out = w.n_out;
        gp.uidx = q.uidx; gp.uval = q.uval; gp.k_dev = q.count; gp.k_max = q.kmax; gp.batch = batch;
        gp.partial = part; gp.rowmax = mc ? rowmax : nullptr;
        if ((st = check_hip(launch_batched_gemv(gp, shares, mc, hs, pt == 0 ? DIP_KERNEL_GEMV_UPGATE : DIP_KERNEL_GEMV_DOWN),
                            "forward_batched: gathered product")))
            return st;
        BatchedReduceParams rp;
        std::memset(&rp, 0, sizeof(rp));
        rp.partial = part; rp.shares = shares; rp.batch = batch; rp.n_out = w.n_out; rp.glu = pt == 0 ? 1 : 0;
        rp.out = pt == 0 ? H : Y; rp.out_stride = pt == 0 ? pl.f : pl.d;
        if ((st = check_hip(launch_batched_reduce(rp, hs), "forward_batched: reduction"))) return st;
    }
    return DIP_OK;
}

int32_t batched_checked(const dip_mlp* mlps, int n_layers, const float* X, int64_t x_stride, int batch,
                        const int32_t* k_in, const int32_t* k_mid, int k_stride, const dip_cache* caches_in,
                        const dip_cache* caches_mid, float gamma, float* Y, int64_t y_stride,
                        uint32_t* mask_in_out, float* h_out, uint32_t* mask_mid_out, void* ws, size_t ws_bytes,
                        void* stream) {
    if (batch < 1 || batch > 8) return fail(DIP_ERR_INVALID_ARG, "forward_batched: batch must be in [1, 8]");
    if (!mlps) return fail(DIP_ERR_INVALID_ARG, "forward_batched: null mlp descriptor");
    if (n_layers < 1) return fail(DIP_ERR_INVALID_ARG, "forward_batched: n_layers must be >= 1");
    if (!X || !Y) return fail(DIP_ERR_INVALID_ARG, "forward_batched: null X or Y");
    if (!k_in || !k_mid) return fail(DIP_ERR_INVALID_ARG, "forward_batched: null k_in or k_mid");
    int32_t st = DIP_OK;
    if (caches_in || caches_mid) {
        if ((st = validate_gamma(gamma))) return st;
    }
    size_t need = 0;
    std::vector<const uint32_t*> seen;
    for (int l = 0; l < n_layers; ++l) {
        if ((st = validate_mlp(&mlps[l], k_in[l * k_stride], k_mid[l * k_stride]))) return st;
        if (caches_in && (st = validate_cache(&caches_in[l], mlps[l].w_ug.n_in, "cache_in"))) return st;
        if (caches_mid && (st = validate_cache(&caches_mid[l], mlps[l].w_d.n_in, "cache_mid"))) return st;
        if (caches_in) seen.push_back(caches_in[l].bits);
        if (caches_mid) seen.push_back(caches_mid[l].bits);
        need = std::max(need, plan_batched(&mlps[l], batch, k_in[l * k_stride], k_mid[l * k_stride]).total);
    }
    std::sort(seen.begin(), seen.end());
    if (std::adjacent_find(seen.begin(), seen.end()) != seen.end())
        return fail(DIP_ERR_INVALID_ARG, "forward_batched: two pruning points share one cache state (every layer "
                                         "and point needs a dip_cache of its own)");
    const size_t mask_bytes = (size_t)n_layers * 2 * kMaskBytes;
    need += mask_bytes;
    if (!ws || ws_bytes < need || !aligned(ws, 256))
        return fail(DIP_ERR_WORKSPACE, "forward_batched: workspace must be 256-aligned and >= %zu bytes", need);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    std::vector<UpdatePiece> updates;
    updates.reserve(2 * (size_t)n_layers);
    for (int l = 0; l < n_layers && !st; ++l) {
        const int ki = k_in[l * k_stride], km = k_mid[l * k_stride];
        const BatchedPlan pl = plan_batched(&mlps[l], batch, ki, km);
        st = batched_one(&mlps[l], pl, X + (int64_t)l * x_stride, batch, ki, km,
                         caches_in ? &caches_in[l] : nullptr, caches_mid ? &caches_mid[l] : nullptr, gamma,
                         Y + (int64_t)l * y_stride, mask_in_out, h_out, mask_mid_out, base + mask_bytes,
                         reinterpret_cast<uint32_t*>(base + (size_t)(2 * l) * kMaskBytes),
                         reinterpret_cast<uint32_t*>(base + (size_t)(2 * l + 1) * kMaskBytes), hs, updates);
    }
    if (!updates.empty()) {
        const int32_t st2 = check_hip(launch_update_batch(updates.data(), (int)updates.size(), hs, DIP_KERNEL_CACHE_UPDATE),
                                      "forward_batched: cache updates");
        if (!st) st = st2;
    }
    return st;
}
}  // namespace

int32_t dip_swiglu_mlp_forward_batched(const dip_mlp* mlp, const float* X, int32_t batch,
                                       int32_t k_in, int32_t k_mid, const dip_cache* cache_in,
                                       const dip_cache* cache_mid, float gamma, float* Y,
                                       uint32_t* mask_in_out, float* h_out, uint32_t* mask_mid_out,
                                       void* ws, size_t ws_bytes, void* stream) {
    return batched_checked(mlp, 1, X, 0, batch, &k_in, &k_mid, 0, cache_in, cache_mid, gamma, Y, 0, mask_in_out,
                           h_out, mask_mid_out, ws, ws_bytes, stream);
}

int32_t dip_swiglu_mlp_forward_batched_stack(const dip_mlp* mlps, int32_t n_layers, const float* X,
                                             int64_t x_stride, int32_t batch, const int32_t* k_in,
                                             const int32_t* k_mid, const dip_cache* caches_in,
                                             const dip_cache* caches_mid, float gamma, float* Y,
                                             int64_t y_stride, void* ws, size_t ws_bytes, void* stream) {
    return batched_checked(mlps, n_layers, X, x_stride, batch, k_in, k_mid, 1, caches_in, caches_mid, gamma, Y,
                           y_stride, nullptr, nullptr, nullptr, ws, ws_bytes, stream);
}

int32_t dip_tune_gemv(int32_t lanes_per_row, int32_t waves, int32_t ksplit, int32_t unroll) {
    auto in = [](int v, std::initializer_list<int> ok) {
        for (int o : ok) if (v == o) return true;
        return false;
    };
    if (!in(lanes_per_row, {0, 8, 16, 32, 64})) return fail(DIP_ERR_INVALID_ARG, "dip_tune_gemv: lanes_per_row");
    if (!in(waves, {0, 2, 4, 8, 16})) return fail(DIP_ERR_INVALID_ARG, "dip_tune_gemv: waves");
    if (!in(unroll, {0, 1, 2, 4, 8})) return fail(DIP_ERR_INVALID_ARG, "dip_tune_gemv: unroll");
    if (ksplit < 0 || ksplit > 4096) return fail(DIP_ERR_INVALID_ARG, "dip_tune_gemv: ksplit");
    g_gemv_override = GemvShape{lanes_per_row, waves, ksplit, unroll};
    return DIP_OK;
}

// ---- Sec. 3.2 sibling schemes ------------------------------------------------------------------
int32_t dip_glu_pruning_forward(const dip_mlp* mlp, const float* x, int32_t k, float* y_out,
                                const dip_debug* dbg, void* ws, size_t ws_bytes, void* stream) {
    if (!mlp) return fail(DIP_ERR_INVALID_ARG, "dip_glu_pruning_forward: null mlp descriptor");
    if (dbg && (dbg->s_in || dbg->mask_in || dbg->idx_in))
        return fail(DIP_ERR_INVALID_ARG, "dip_glu_pruning_forward: there is no pruning point 1 to report");
    if (!aligned(x, 16)) return fail(DIP_ERR_UNSUPPORTED, "dip_glu_pruning_forward: x must be 16-byte aligned");
    const int32_t k_all = mlp->w_ug.n_in;
    return forward_checked(mlp, 1, x, 0, &k_all, &k, 0, nullptr, nullptr, 0.f, y_out, 0, dbg, ws,
                           ws_bytes, stream, true);
}

size_t dip_glu_pruning_forward_workspace_bytes(const dip_mlp* mlp, int32_t k) {
    if (!mlp) return 0;
    return dip_swiglu_mlp_forward_workspace_bytes(mlp, mlp->w_ug.n_in, k);
}

int32_t dip_gathered_rowdot(const dip_weight* w_rows, const float* x, const int32_t* idx, int32_t k,
                            float* out, void* stream) {
    int32_t st = validate_weight(w_rows, "dip_gathered_rowdot");
    if (st) return st;
    if (!x || !idx || !out) return fail(DIP_ERR_INVALID_ARG, "dip_gathered_rowdot: null pointer");
    if (k < 1 || k > w_rows->n_in) return fail(DIP_ERR_INVALID_ARG, "dip_gathered_rowdot: k must be in [1, stored rows]");
    if (!aligned(x, 16)) return fail(DIP_ERR_UNSUPPORTED, "dip_gathered_rowdot: x must be 16-byte aligned");
    if (w_rows->n_out > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "dip_gathered_rowdot: rows longer than %d", DIP_MAX_N);
    RowdotParams p;
    std::memset(&p, 0, sizeof(p));
    p.w = w_rows->data; p.row_stride = w_rows->row_stride_bytes;
    p.scales = static_cast<const uint16_t*>(w_rows->scales); p.scale_stride = w_rows->n_out / 128;
    p.dtype = w_rows->dtype; p.n_rows = w_rows->n_in; p.n_cols = w_rows->n_out;
    p.idx = idx; p.k = k; p.x = x; p.out = out;
    return check_hip(launch_rowdot(p, static_cast<hipStream_t>(stream), DIP_KERNEL_ROWDOT), "dip_gathered_rowdot");
}

namespace {
struct PartialPlan {
    int d, f;
    GemvShape dense, dn;
    int strips_dense, strips_dn;
    size_t off_a, off_idx, off_hsel, off_part_dense, off_part_dn, off_cnt, total;
};
PartialPlan plan_partial(const dip_mlp_split* mlp, int k) {
    PartialPlan pl;
    pl.d = mlp->w_dense.n_in;
    pl.f = mlp->w_dense.n_out;
    pl.dense = choose_gemv_shape(mlp->w_dense.dtype, pl.f, 1, pl.d);
    pl.dn = choose_gemv_shape(mlp->w_d.dtype, pl.d, 1, k);
    pl.strips_dense = gemv_strips(pl.dense, mlp->w_dense.dtype, pl.f);
    pl.strips_dn = gemv_strips(pl.dn, mlp->w_d.dtype, pl.d);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    pl.off_a = take(sizeof(float) * pl.f);
    pl.off_idx = take(sizeof(int32_t) * k);
    pl.off_hsel = take(sizeof(float) * k);
    pl.off_part_dense = take(pl.dense.ksplit > 1 ? sizeof(float) * pl.f * pl.dense.ksplit : 0);
    pl.off_part_dn = take(pl.dn.ksplit > 1 ? sizeof(float) * pl.d * pl.dn.ksplit : 0);
    pl.off_cnt = take(sizeof(uint32_t) * (pl.strips_dense + pl.strips_dn));
    pl.total = o;
    return pl;
}
int32_t validate_split(const dip_mlp_split* mlp, int k) {
    if (!mlp) return fail(DIP_ERR_INVALID_ARG, "mlp: null descriptor");
    int32_t st = validate_weight(&mlp->w_dense, "w_dense");
    if (st) return st;
    if ((st = validate_weight(&mlp->w_rows, "w_rows"))) return st;
    if ((st = validate_weight(&mlp->w_d, "w_d"))) return st;
    const int d = mlp->w_dense.n_in, f = mlp->w_dense.n_out;
    if (mlp->w_rows.n_in != f || mlp->w_rows.n_out != d)
        return fail(DIP_ERR_INVALID_ARG, "w_rows must hold d_ff stored rows of d_model elements");
    if (mlp->w_d.n_in != f || mlp->w_d.n_out != d)
        return fail(DIP_ERR_INVALID_ARG, "w_d must hold d_ff stored rows of d_model elements");
    if (d > DIP_MAX_N || f > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "d_model and d_ff must be <= %d", DIP_MAX_N);
    if (k < 1 || k > f) return fail(DIP_ERR_INVALID_ARG, "k must be in [1, d_ff]");
    return DIP_OK;
}
}  // namespace

size_t dip_partial_pruning_forward_workspace_bytes(const dip_mlp_split* mlp, int32_t k) {
    if (validate_split(mlp, k)) return 0;
    return plan_partial(mlp, k).total;
}

int32_t dip_partial_pruning_forward(const dip_mlp_split* mlp, int32_t scheme, const float* x, int32_t k,
                                    float* y_out, const dip_partial_debug* dbg, void* ws,
                                    size_t ws_bytes, void* stream) {
    int32_t st = validate_split(mlp, k);
    if (st) return st;
    if (scheme != DIP_GATE_PRUNING && scheme != DIP_UP_PRUNING)
        return fail(DIP_ERR_INVALID_ARG, "dip_partial_pruning_forward: scheme must be DIP_GATE_PRUNING or DIP_UP_PRUNING");
    if (!x || !y_out) return fail(DIP_ERR_INVALID_ARG, "dip_partial_pruning_forward: null x or y_out");
    if (!aligned(x, 16)) return fail(DIP_ERR_UNSUPPORTED, "dip_partial_pruning_forward: x must be 16-byte aligned");
    if (dbg && !aligned(dbg->idx, 16))
        return fail(DIP_ERR_UNSUPPORTED, "dip_partial_pruning_forward: debug index list must be 16-byte aligned");
    if (dbg && !aligned(dbg->h_sel, 16))
        return fail(DIP_ERR_UNSUPPORTED, "dip_partial_pruning_forward: debug h_sel must be 16-byte aligned");
    const PartialPlan pl = plan_partial(mlp, k);
    if (!ws || ws_bytes < pl.total || !aligned(ws, 256))
        return fail(DIP_ERR_WORKSPACE, "dip_partial_pruning_forward: workspace must be 256-aligned and >= %zu bytes", pl.total);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    float* a = dbg && dbg->a ? dbg->a : reinterpret_cast<float*>(base + pl.off_a);
    int32_t* idx = dbg && dbg->idx ? dbg->idx : reinterpret_cast<int32_t*>(base + pl.off_idx);
    float* hsel = dbg && dbg->h_sel ? dbg->h_sel : reinterpret_cast<float*>(base + pl.off_hsel);
    uint32_t* cnt_dense = reinterpret_cast<uint32_t*>(base + pl.off_cnt);
    uint32_t* cnt_dn = cnt_dense + pl.strips_dense;

    st = check_hip(launch_zero_u32(cnt_dense, pl.strips_dense + pl.strips_dn, hs), "counter reset");
    if (st) return st;

    // a = sigma(W^g x) (gate pruning) or W^u x (up pruning), all d_ff neurons
    GemvParams g1;
    std::memset(&g1, 0, sizeof(g1));
    g1.w = mlp->w_dense.data; g1.row_stride = mlp->w_dense.row_stride_bytes;
    g1.scales = static_cast<const uint16_t*>(mlp->w_dense.scales); g1.scale_stride = mlp->w_dense.n_out / 128;
    g1.dtype = mlp->w_dense.dtype; g1.n_in = pl.d; g1.n_out = pl.f; g1.nseg = 1;
    g1.idx = nullptr; g1.val = x; g1.k = pl.d; g1.out = a;
    g1.partial = reinterpret_cast<float*>(base + pl.off_part_dense); g1.counters = cnt_dense;
    g1.act = scheme == DIP_GATE_PRUNING ? 1 : 0;
    st = check_hip(launch_gemv(g1, pl.dense, hs, DIP_KERNEL_GEMV_DENSE), "dense GEMV");
    if (st) return st;

    // m = topK(|a|, k)
    SelectParams sp;
    std::memset(&sp, 0, sizeof(sp));
    sp.v = a; sp.n = pl.f; sp.k = k; sp.idx_out = idx; sp.mask_out = dbg ? dbg->mask : nullptr;
    st = check_hip(launch_select(sp, hs, DIP_KERNEL_SELECT_MID), "select");
    if (st) return st;

    // the other pre-activation for the kept neurons only, combined into h
    RowdotParams rp;
    std::memset(&rp, 0, sizeof(rp));
    rp.w = mlp->w_rows.data; rp.row_stride = mlp->w_rows.row_stride_bytes;
    rp.scales = static_cast<const uint16_t*>(mlp->w_rows.scales); rp.scale_stride = mlp->w_rows.n_out / 128;
    rp.dtype = mlp->w_rows.dtype; rp.n_rows = pl.f; rp.n_cols = pl.d;
    rp.idx = idx; rp.k = k; rp.x = x; rp.a = a; rp.mode = scheme == DIP_GATE_PRUNING ? 1 : 2; rp.out = hsel;
    st = check_hip(launch_rowdot(rp, hs, DIP_KERNEL_ROWDOT), "row-gathered dot products");
    if (st) return st;

    // y = sum over kept neurons of W^d[:, j] h_j
    GemvParams g2;
    std::memset(&g2, 0, sizeof(g2));
    g2.w = mlp->w_d.data; g2.row_stride = mlp->w_d.row_stride_bytes;
    g2.scales = static_cast<const uint16_t*>(mlp->w_d.scales); g2.scale_stride = mlp->w_d.n_out / 128;
    g2.dtype = mlp->w_d.dtype; g2.n_in = pl.f; g2.n_out = pl.d; g2.nseg = 1;
    g2.idx = idx; g2.val = hsel; g2.k = k; g2.out = y_out;
    g2.partial = reinterpret_cast<float*>(base + pl.off_part_dn); g2.counters = cnt_dn;
    return check_hip(launch_gemv(g2, pl.dn, hs, DIP_KERNEL_GEMV_DOWN), "gathered GEMV (down)");
}

// ---- two-tier residency ------------------------------------------------------------------------
namespace {
int32_t validate_tier(const dip_tiered_weight* tw, const dip_cache* cache, const char* name) {
    if (!tw) return fail(DIP_ERR_INVALID_ARG, "%s: null descriptor", name);
    int32_t st = validate_weight(&tw->full, name);
    if (st) return st;
    if (tw->full.dtype == DIP_INT4_G128) return fail(DIP_ERR_UNSUPPORTED, "%s: tiers hold F32 or BF16 matrices", name);
    if (tw->full.n_in > DIP_MAX_N) return fail(DIP_ERR_UNSUPPORTED, "%s: more than %d columns", name, DIP_MAX_N);
    if (!tw->slots || !tw->slot_of) return fail(DIP_ERR_INVALID_ARG, "%s: null slots or slot_of", name);
    if (!aligned(tw->slots, 16)) return fail(DIP_ERR_UNSUPPORTED, "%s: slots must be 16-byte aligned", name);
    if (tw->reserved != 0) return fail(DIP_ERR_INVALID_ARG, "%s: reserved must be 0", name);
    if (tw->capacity < 0 || tw->capacity > tw->full.n_in) return fail(DIP_ERR_INVALID_ARG, "%s: capacity outside [0, n_in]", name);
    if (!cache) return fail(DIP_ERR_INVALID_ARG, "%s: a tiered matrix needs its cache", name);
    if ((st = validate_cache(cache, tw->full.n_in, name))) return st;
    if (cache->capacity != tw->capacity) return fail(DIP_ERR_INVALID_ARG, "%s: cache and tier capacities differ", name);
    return DIP_OK;
}

struct TierScratch {   // per pruning point, inside the workspace
    size_t off_ev, off_ins, off_fcol, off_fslot, off_fcnt, off_src, bytes;
};
TierScratch plan_tier(int n, int capacity, int k) {
    TierScratch t;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    t.off_ev = take(sizeof(uint32_t) * ((n + 31) / 32));
    t.off_ins = take(sizeof(uint32_t) * ((n + 31) / 32));
    t.off_fcol = take(sizeof(int32_t) * (size_t)std::max(capacity, 1));
    t.off_fslot = take(sizeof(int32_t) * (size_t)std::max(capacity, 1));
    t.off_fcnt = take(sizeof(uint32_t));
    t.off_src = take(sizeof(int32_t) * (size_t)std::max(k, 1));
    t.bytes = o;
    return t;
}
dip_mlp as_mlp(const dip_tiered_mlp* m) {
    dip_mlp r;
    r.w_ug = m->w_ug.full;
    r.w_d = m->w_d.full;
    return r;
}
}  // namespace

size_t dip_tier_init_workspace_bytes(const dip_tiered_weight* tw) {
    if (!tw || tw->capacity < 0) return 0;
    return plan_tier(tw->full.n_in, tw->capacity, 1).bytes;
}

int32_t dip_tier_init(const dip_tiered_weight* tw, const dip_cache* cache, void* ws, size_t ws_bytes,
                      void* stream) {
    int32_t st = validate_tier(tw, cache, "dip_tier_init");
    if (st) return st;
    const TierScratch ts = plan_tier(tw->full.n_in, tw->capacity, 1);
    if (!ws || ws_bytes < ts.bytes || !aligned(ws, 256))
        return fail(DIP_ERR_WORKSPACE, "dip_tier_init: workspace must be 256-aligned and >= %zu bytes", ts.bytes);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    TierInitParams ip;
    ip.bits = cache->bits; ip.n = tw->full.n_in; ip.slot_of = tw->slot_of;
    ip.fill_col = reinterpret_cast<int32_t*>(base + ts.off_fcol);
    ip.fill_slot = reinterpret_cast<int32_t*>(base + ts.off_fslot);
    ip.fill_count = reinterpret_cast<uint32_t*>(base + ts.off_fcnt);
    if ((st = check_hip(launch_tier_init(ip, hs), "dip_tier_init: slot map"))) return st;
    TierFillParams fp;
    fp.host_rows = tw->full.data; fp.slots = tw->slots; fp.row_stride = tw->full.row_stride_bytes;
    fp.row_bytes = (int64_t)tw->full.n_out * elem_bits(tw->full.dtype) / 8;
    fp.fill_col = ip.fill_col; fp.fill_slot = ip.fill_slot; fp.fill_count = ip.fill_count;
    fp.max_rows = tw->capacity;
    return check_hip(launch_tier_fill(fp, hs, -1), "dip_tier_init: fill");
}

size_t dip_tiered_mlp_forward_workspace_bytes(const dip_tiered_mlp* mlp, int32_t k_in, int32_t k_mid) {
    if (!mlp) return 0;
    const dip_mlp m = as_mlp(mlp);
    if (validate_mlp(&m, k_in, k_mid)) return 0;
    return align_up(plan_forward(&m, k_in, k_mid).total, 256) +
           plan_tier(m.w_ug.n_in, mlp->w_ug.capacity, k_in).bytes +
           plan_tier(m.w_d.n_in, mlp->w_d.capacity, k_mid).bytes;
}

int32_t dip_tiered_mlp_forward(const dip_tiered_mlp* mlp, const float* x, int32_t k_in, int32_t k_mid,
                               const dip_cache* cache_in, const dip_cache* cache_mid, float gamma,
                               float* y_out, const dip_debug* dbg, void* ws, size_t ws_bytes,
                               void* stream) {
    if (!mlp) return fail(DIP_ERR_INVALID_ARG, "dip_tiered_mlp_forward: null mlp descriptor");
    if (!x || !y_out) return fail(DIP_ERR_INVALID_ARG, "dip_tiered_mlp_forward: null x or y_out");
    const dip_mlp m = as_mlp(mlp);
    int32_t st = validate_mlp(&m, k_in, k_mid);
    if (st) return st;
    if ((st = validate_tier(&mlp->w_ug, cache_in, "w_ug"))) return st;
    if ((st = validate_tier(&mlp->w_d, cache_mid, "w_d"))) return st;
    if ((st = validate_gamma(gamma))) return st;
    if (dbg && (!aligned(dbg->idx_in, 16) || !aligned(dbg->idx_mid, 16)))
        return fail(DIP_ERR_UNSUPPORTED, "dip_tiered_mlp_forward: debug index lists must be 16-byte aligned");
    const size_t need = dip_tiered_mlp_forward_workspace_bytes(mlp, k_in, k_mid);
    if (!ws || ws_bytes < need || !aligned(ws, 256))
        return fail(DIP_ERR_WORKSPACE, "dip_tiered_mlp_forward: workspace must be 256-aligned and >= %zu bytes", need);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const ForwardPlan pl = plan_forward(&m, k_in, k_mid);
    char* base = static_cast<char*>(ws);
    char* tbase[2];
    tbase[0] = base + align_up(pl.total, 256);
    const TierScratch ts[2] = {plan_tier(pl.d, mlp->w_ug.capacity, k_in), plan_tier(pl.f, mlp->w_d.capacity, k_mid)};
    tbase[1] = tbase[0] + ts[0].bytes;

    int32_t* idx[2] = {reinterpret_cast<int32_t*>(base + pl.off_idx1), reinterpret_cast<int32_t*>(base + pl.off_idx2)};
    float* val[2] = {reinterpret_cast<float*>(base + pl.off_val1), reinterpret_cast<float*>(base + pl.off_val2)};
    float* h = reinterpret_cast<float*>(base + pl.off_h);
    if (dbg && dbg->idx_in) idx[0] = dbg->idx_in;
    if (dbg && dbg->idx_mid) idx[1] = dbg->idx_mid;
    if (dbg && dbg->h) h = dbg->h;
    uint32_t* cnt_ug = reinterpret_cast<uint32_t*>(base + pl.off_cnt);
    uint32_t* cnt_dn = cnt_ug + pl.strips_ug;

    for (int pt = 0; pt < 2; ++pt) {
        const dip_tiered_weight& tw = pt == 0 ? mlp->w_ug : mlp->w_d;
        const dip_cache* cache = pt == 0 ? cache_in : cache_mid;
        const int n = pt == 0 ? pl.d : pl.f, k = pt == 0 ? k_in : k_mid;
        char* tb = tbase[pt];
        uint32_t* evw = reinterpret_cast<uint32_t*>(tb + ts[pt].off_ev);
        uint32_t* insw = reinterpret_cast<uint32_t*>(tb + ts[pt].off_ins);
        int32_t* fcol = reinterpret_cast<int32_t*>(tb + ts[pt].off_fcol);
        int32_t* fslot = reinterpret_cast<int32_t*>(tb + ts[pt].off_fslot);
        uint32_t* fcnt = reinterpret_cast<uint32_t*>(tb + ts[pt].off_fcnt);
        int32_t* src = reinterpret_cast<int32_t*>(tb + ts[pt].off_src);

        // Alg. 1 steps 1-3, plus the words of what the update evicted and inserted
        SelectParams sp;
        std::memset(&sp, 0, sizeof(sp));
        sp.v = pt == 0 ? x : h; sp.n = n; sp.k = k; sp.gamma = gamma;
        sp.s_out = dbg ? (pt == 0 ? dbg->s_in : dbg->s_mid) : nullptr;
        sp.mask_out = dbg ? (pt == 0 ? dbg->mask_in : dbg->mask_mid) : nullptr;
        sp.idx_out = idx[pt]; sp.val_out = val[pt];
        sp.score_bits = cache->bits; sp.c_bits = cache->bits; sp.c_stamp = cache->stamp; sp.c_meta = cache->meta;
        sp.capacity = cache->capacity; sp.policy = cache->policy;
        sp.evicted_out = evw; sp.inserted_out = insw;
        if (pt == 0) { sp.zero_ptr = cnt_ug; sp.zero_n = pl.strips_ug + pl.strips_dn; }
        if ((st = check_hip(launch_select(sp, hs, pt == 0 ? DIP_KERNEL_SELECT_IN : DIP_KERNEL_SELECT_MID), "select"))) return st;

        // slots for the inserted columns, rows to copy, rows to read
        TierParams tp;
        tp.evicted = evw; tp.inserted = insw; tp.meta = cache->meta; tp.n = n; tp.capacity = tw.capacity;
        tp.slot_of = tw.slot_of; tp.fill_col = fcol; tp.fill_slot = fslot; tp.fill_count = fcnt;
        tp.idx = idx[pt]; tp.k = k; tp.src = src;
        if ((st = check_hip(launch_tier_update(tp, hs), "tier update"))) return st;
        TierFillParams fp;
        fp.host_rows = tw.full.data; fp.slots = tw.slots; fp.row_stride = tw.full.row_stride_bytes;
        fp.row_bytes = (int64_t)tw.full.n_out * elem_bits(tw.full.dtype) / 8;
        fp.fill_col = fcol; fp.fill_slot = fslot; fp.fill_count = fcnt;
        fp.max_rows = std::min(k, tw.capacity);
        if ((st = check_hip(launch_tier_fill(fp, hs, DIP_KERNEL_TIER_FILL), "tier fill"))) return st;

        GemvParams g;
        std::memset(&g, 0, sizeof(g));
        g.w = tw.slots; g.n_in = tw.capacity; g.w_alt = tw.full.data; g.n_alt = n;
        g.row_stride = tw.full.row_stride_bytes; g.dtype = tw.full.dtype;
        g.idx = src; g.val = val[pt]; g.k = k;
        if (pt == 0) {
            g.n_out = pl.f; g.nseg = 2; g.out = h;
            g.partial = reinterpret_cast<float*>(base + pl.off_part_ug); g.counters = cnt_ug;
            // (the launch shapes of dip_swiglu_mlp_forward: the same sums in the same order)
            st = check_hip(launch_gemv(g, pl.fuse_ug ? pl.fug : pl.ug, hs, DIP_KERNEL_GEMV_UPGATE), "gathered GEMV (up/gate)");
        } else {
            g.n_out = pl.d; g.nseg = 1; g.out = y_out;
            g.partial = reinterpret_cast<float*>(base + pl.off_part_dn); g.counters = cnt_dn;
            st = check_hip(launch_gemv(g, pl.fuse_dn ? pl.fdn : pl.dn, hs, DIP_KERNEL_GEMV_DOWN), "gathered GEMV (down)");
        }
        if (st) return st;
    }
    return DIP_OK;
}

int32_t dip_gemv_launch_shape(const dip_weight* w, int32_t k, int32_t bundled, int32_t* shape_out) {
    int32_t st = validate_weight(w, "dip_gemv_launch_shape");
    if (st) return st;
    if (!shape_out) return fail(DIP_ERR_INVALID_ARG, "dip_gemv_launch_shape: null output");
    if (k < 1 || k > w->n_in) return fail(DIP_ERR_INVALID_ARG, "dip_gemv_launch_shape: k must be in [1, n_in]");
    if (bundled && (w->n_out % 2)) return fail(DIP_ERR_INVALID_ARG, "dip_gemv_launch_shape: bundled matrix needs an even n_out");
    const GemvShape s = bundled ? choose_gemv_shape(w->dtype, w->n_out / 2, 2, k)
                                : choose_gemv_shape(w->dtype, w->n_out, 1, k);
    shape_out[0] = s.lpr; shape_out[1] = s.waves; shape_out[2] = s.ksplit; shape_out[3] = s.unroll;
    return DIP_OK;
}

int32_t dip_set_fusion(int32_t on) {
    if (on != 0 && on != 1) return fail(DIP_ERR_INVALID_ARG, "dip_set_fusion: 0 or 1");
    g_fusion = on;
    return DIP_OK;
}

int32_t dip_fused_launch_shape(const dip_weight* w, int32_t k, int32_t bundled, int32_t* shape_out) {
    int32_t st = validate_weight(w, "dip_fused_launch_shape");
    if (st) return st;
    if (!shape_out) return fail(DIP_ERR_INVALID_ARG, "dip_fused_launch_shape: null output");
    if (k < 1 || k > w->n_in) return fail(DIP_ERR_INVALID_ARG, "dip_fused_launch_shape: k must be in [1, n_in]");
    if (bundled && (w->n_out % 2)) return fail(DIP_ERR_INVALID_ARG, "dip_fused_launch_shape: bundled matrix needs an even n_out");
    GemvShape s;
    if (!fused_shape(w->dtype, w->n_in, bundled ? w->n_out / 2 : w->n_out, bundled ? 2 : 1, k, &s))
        return fail(DIP_ERR_UNSUPPORTED, "dip_fused_launch_shape: selection and product are launched apart for this shape");
    shape_out[0] = s.lpr; shape_out[1] = s.waves; shape_out[2] = s.ksplit; shape_out[3] = s.unroll;
    return DIP_OK;
}

int32_t dip_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink) return fail(DIP_ERR_INVALID_ARG, "dip_stream_read: null pointer");
    if (bytes < 16 || bytes % 16 || !aligned(src, 16))
        return fail(DIP_ERR_INVALID_ARG, "dip_stream_read: buffer must be 16-byte aligned, a multiple of 16 bytes");
    return check_hip(launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream), DIP_KERNEL_STREAM_READ),
                     "dip_stream_read");
}

int32_t dip_profile_disable(void) {
    for (hipEvent_t e : g_prof.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_prof.stop) (void)hipEventDestroy(e);
    g_prof.start.clear();
    g_prof.stop.clear();
    g_prof.kind.clear();
    g_prof.used = 0;
    g_prof.on = false;
    return DIP_OK;
}

int32_t dip_profile_enable(int32_t max_launches) {
    if (max_launches < 1 || max_launches > (1 << 20))
        return fail(DIP_ERR_INVALID_ARG, "dip_profile_enable: max_launches must be in [1, 2^20]");
    dip_profile_disable();
    for (int i = 0; i < max_launches; ++i) {
        hipEvent_t a, b;
        int32_t st = check_hip(hipEventCreate(&a), "hipEventCreate");
        if (st) { dip_profile_disable(); return st; }
        g_prof.start.push_back(a);
        st = check_hip(hipEventCreate(&b), "hipEventCreate");
        if (st) { dip_profile_disable(); return st; }
        g_prof.stop.push_back(b);
        g_prof.kind.push_back(-1);
    }
    g_prof.on = true;
    return DIP_OK;
}

int32_t dip_profile_read(int32_t kind, double* total_ms, int32_t* launches) {
    if (!total_ms || !launches) return fail(DIP_ERR_INVALID_ARG, "dip_profile_read: null output");
    if (kind < 0 || kind >= DIP_KERNEL_KINDS) return fail(DIP_ERR_INVALID_ARG, "dip_profile_read: unknown kernel kind");
    double sum = 0.0;
    int32_t n = 0;
    for (size_t i = 0; i < g_prof.used; ++i) {
        if (g_prof.kind[i] != kind) continue;
        int32_t st = check_hip(hipEventSynchronize(g_prof.stop[i]), "hipEventSynchronize");
        if (st) return st;
        float ms = 0.f;
        st = check_hip(hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]), "hipEventElapsedTime");
        if (st) return st;
        sum += ms;
        ++n;
    }
    *total_ms = sum;
    *launches = n;
    return DIP_OK;
}

}  // extern "C"
