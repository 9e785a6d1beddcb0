// The C ABI: context, workspace bookkeeping, host helpers and argument
// validation.  Nothing here touches the GPU except hipSetDevice before a
// launch; every check runs on the host before anything is enqueued.
#include <math.h>
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "common.h"

using namespace lvlm;

namespace {

lvlm_status fail(lvlm_ctx *ctx, lvlm_status st, const char *fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

bool float_dtype(int dt) { return dt == LVLM_BF16 || dt == LVLM_F32; }
int elem_bytes(int dt) { return dt == LVLM_BF16 ? 2 : 4; }

// Upper limits of the size fields (include/lvlm.h states them): generous for any cache or sequence that fits a GPU,
// and tight enough that no size or grid computation in the library can overflow.
constexpr int kMaxBatch = 1 << 16, kMaxHeads = 1 << 10, kMaxTokens = 1 << 22, kMaxSlots = 1 << 24, kMaxRowElems = 1 << 20;
const char *kTooLarge = "size beyond the documented limits (B 65536, heads 1024, N 4194304, Lmax 16777216, row_elems 1048576)";

const char *check_score(const lvlm_score_desc *d) {
    if (!d) return "null descriptor";
    if (!float_dtype(d->dtype)) return "dtype must be LVLM_BF16 or LVLM_F32";
    if (d->hd != 64 && d->hd != 128) return "head dimension must be 64 or 128";
    if (d->B < 1 || d->N < 1 || d->T < 1 || d->Hq < 1 || d->Hkv < 1) return "sizes must be positive";
    if (d->B > kMaxBatch || d->N > kMaxTokens || d->Hq > kMaxHeads) return kTooLarge;
    if (d->Hq % d->Hkv != 0) return "Hq must be a multiple of Hkv";
    if ((long long)(d->Hq / d->Hkv) * d->T >= 65536) return "query rows per KV head (Hq/Hkv * T) must be below 65536";
    if (d->img_begin < 0 || d->n_img < 1 || (long long)d->img_begin + d->n_img > d->N) return "image span outside [0, N)";
    if (d->q_pos0 < 0) return "q_pos0 must be non-negative";
    if (!(d->scale >= 0.0f)) return "scale must be non-negative";
    const int vec = 16 / elem_bytes(d->dtype);
    const long long s[6] = {d->q_stride_b, d->q_stride_t, d->q_stride_h, d->k_stride_b, d->k_stride_n, d->k_stride_h};
    for (long long x : s)
        if (x < 0 || x % vec != 0) return "strides must be non-negative multiples of 16 bytes";
    if (d->q_stride_h < d->hd || d->k_stride_h < d->hd) return "head stride smaller than the head dimension";
    if ((d->sh_stride_b == 0) != (d->sh_stride_h == 0)) return "score_head strides must be both zero or both set";
    if (d->sh_stride_h != 0 && (d->sh_stride_h < d->n_img || d->sh_stride_b < d->sh_stride_h))
        return "score_head strides smaller than the rows they separate";
    return nullptr;
}

const char *check_prefill(const lvlm_prefill_desc *d) {
    if (!d) return "null descriptor";
    if (!float_dtype(d->dtype)) return "dtype must be LVLM_BF16 or LVLM_F32";
    if (d->hd != 64 && d->hd != 128) return "head dimension must be 64 or 128";
    if (d->B < 1 || d->N < 1 || d->Hq < 1 || d->Hkv < 1) return "sizes must be positive";
    if (d->B > kMaxBatch || d->N > kMaxTokens || d->Hq > kMaxHeads) return kTooLarge;
    if (d->Hq % d->Hkv != 0) return "Hq must be a multiple of Hkv";
    if (d->T < 0 || d->T > d->N) return "T must be in [0, N]";
    if (!(d->scale > 0.0f)) return "scale must be positive";
    const int vec = 16 / elem_bytes(d->dtype);
    const long long s[12] = {d->q_stride_b, d->q_stride_n, d->q_stride_h, d->k_stride_b, d->k_stride_n, d->k_stride_h,
                             d->v_stride_b, d->v_stride_n, d->v_stride_h, d->o_stride_b, d->o_stride_n, d->o_stride_h};
    for (long long x : s)
        if (x < 0 || x % vec != 0) return "strides must be non-negative multiples of 16 bytes";
    if (d->q_stride_h < d->hd || d->k_stride_h < d->hd || d->v_stride_h < d->hd || d->o_stride_h < d->hd)
        return "head stride smaller than the head dimension";
    if ((long long)d->B * d->Hq * ((d->N + 127) / 128) >= (1ll << 28) || (long long)d->B * d->Hq * d->N >= (1ll << 33))
        return "too many query blocks for one launch";
    if (d->dtype == LVLM_F32 && (d->B > 65535 || d->Hq > 65535)) return "fp32: B and Hq must be below 65536";
    if (d->T > 0) {
        const lvlm_score_desc sd = prefill_score_desc(*d);
        return check_score(&sd);
    }
    return nullptr;
}

const char *check_probs(const lvlm_probs_desc *d) {
    if (!d) return "null descriptor";
    if (!float_dtype(d->dtype)) return "dtype must be LVLM_BF16 or LVLM_F32";
    if (d->B < 1 || d->N < 1 || d->T < 1 || d->Hq < 1 || d->Hkv < 1) return "sizes must be positive";
    if (d->B > kMaxBatch || d->N > kMaxTokens || d->Hq > kMaxHeads) return kTooLarge;
    if (d->Hq % d->Hkv != 0) return "Hq must be a multiple of Hkv";
    if ((long long)(d->Hq / d->Hkv) * d->T >= 65536) return "query rows per KV head (Hq/Hkv * T) must be below 65536";
    if (d->img_begin < 0 || d->n_img < 1 || (long long)d->img_begin + d->n_img > d->N) return "image span outside [0, N)";
    if (d->p_stride_t < d->N || d->p_stride_h < d->p_stride_t || d->p_stride_b < d->p_stride_h)
        return "probs strides smaller than the rows they separate";
    if ((d->sh_stride_b == 0) != (d->sh_stride_h == 0)) return "score_head strides must be both zero or both set";
    if (d->sh_stride_h != 0 && (d->sh_stride_h < d->n_img || d->sh_stride_b < d->sh_stride_h))
        return "score_head strides smaller than the rows they separate";
    return nullptr;
}

const char *check_merge(const lvlm_merge_desc *d, const lvlm_plane *planes) {
    if (!d) return "null descriptor";
    if (d->B < 1 || d->N < 1) return "sizes must be positive";
    if (d->B > kMaxBatch || d->N > kMaxTokens) return kTooLarge;
    if (d->img_begin < 0 || d->n_img < 1 || (long long)d->img_begin + d->n_img > d->N) return "image span outside [0, N)";
    if (d->n_keep < 1 || d->n_keep > d->n_img) return "n_keep must be in [1, n_img]";
    if (d->n_planes < 1 || d->n_planes > LVLM_MAX_PLANES) return "n_planes must be in [1, LVLM_MAX_PLANES]";
    if (!planes) return "null plane table";
    const int r = d->n_img - d->n_keep;
    for (int i = 0; i < d->n_planes; ++i) {
        const lvlm_plane &p = planes[i];
        if (!p.src || !p.dst) return "null plane pointer";
        if (!aligned16(p.src) || !aligned16(p.dst)) return "plane pointers must be 16-byte aligned";
        if (p.row_elems < 1) return "row_elems must be positive";
        if (p.row_elems > kMaxRowElems) return kTooLarge;
        if (p.dtype != LVLM_BF16 && p.dtype != LVLM_F32 && p.dtype != LVLM_I32) return "unknown plane dtype";
        if (p.merge_rule != LVLM_RULE_WEIGHTED && p.merge_rule != LVLM_RULE_TOP) return "unknown merge rule";
        if (p.dtype == LVLM_I32 && p.merge_rule != LVLM_RULE_TOP) return "integer planes need LVLM_RULE_TOP";
        if (p.src_stride_b < (long long)d->N * p.row_elems) return "src_stride_b smaller than one sequence";
        if (p.dst_stride_b < (long long)(d->N - r) * p.row_elems) return "dst_stride_b smaller than one output sequence";
        const size_t eb = elem_bytes(p.dtype);
        const char *s0 = static_cast<const char *>(p.src);
        const char *d0 = static_cast<const char *>(p.dst);
        const char *s1 = s0 + ((size_t)(d->B - 1) * p.src_stride_b + (size_t)d->N * p.row_elems) * eb;
        const char *d1 = d0 + ((size_t)(d->B - 1) * p.dst_stride_b + (size_t)(d->N - r) * p.row_elems) * eb;
        if (s0 < d1 && d0 < s1) return "src and dst of a plane overlap";
    }
    return nullptr;
}

const char *check_kv(const lvlm_kv_desc *d) {
    if (!d) return "null descriptor";
    if (!float_dtype(d->dtype)) return "dtype must be LVLM_BF16 or LVLM_F32";
    if (d->hd != 64 && d->hd != 128) return "head dimension must be 64 or 128";
    if (d->B < 1 || d->Hkv < 1 || d->Lmax < 1) return "sizes must be positive";
    if (d->B > kMaxBatch || d->Hkv > kMaxHeads || d->Lmax > kMaxSlots) return kTooLarge;
    if (d->len_bound < 0 || d->len_bound > d->Lmax) return "len_bound must be in [0, Lmax]";
    if (d->mode != LVLM_KV_THRESHOLD && d->mode != LVLM_KV_BUDGET) return "unknown mode";
    if (d->order != LVLM_ORDER_STABLE && d->order != LVLM_ORDER_FILL) return "unknown order";
    if (d->mode == LVLM_KV_BUDGET && d->budget < 1) return "budget must be at least 1";
    if (d->mode == LVLM_KV_BUDGET && d->n_recent < 0) return "n_recent must be non-negative";
    if (d->mode == LVLM_KV_THRESHOLD && !(d->beta == d->beta)) return "beta is NaN";
    return nullptr;
}

const char *check_attn(const lvlm_attn_desc *d) {
    if (!d) return "null descriptor";
    if (!float_dtype(d->dtype)) return "dtype must be LVLM_BF16 or LVLM_F32";
    if (d->hd != 64 && d->hd != 128) return "head dimension must be 64 or 128";
    if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->Lmax < 1) return "sizes must be positive";
    if (d->B > kMaxBatch || d->Hq > kMaxHeads || d->Lmax > kMaxSlots) return kTooLarge;
    if (d->Hq % d->Hkv != 0) return "Hq must be a multiple of Hkv";
    if (d->len_bound < 0 || d->len_bound > d->Lmax) return "len_bound must be in [0, Lmax]";
    if (d->new_kind < 0 || d->new_kind > 255) return "new_kind out of range";
    if (d->evict_budget < 0 || d->evict_recent < 0) return "evict_budget and evict_recent must not be negative";
    return nullptr;
}

lvlm_status need_ws(lvlm_ctx *ctx, size_t bytes) {
    if (bytes == 0) return LVLM_OK;
    if (!ctx->ws) return fail(ctx, LVLM_ERR_WORKSPACE, "no workspace attached (need %zu bytes)", bytes);
    if (ctx->ws_bytes < bytes)
        return fail(ctx, LVLM_ERR_WORKSPACE, "workspace too small: have %zu bytes, need %zu", ctx->ws_bytes, bytes);
    return LVLM_OK;
}

lvlm_status after_launch(lvlm_ctx *ctx, hipError_t e) {
    if (e != hipSuccess) return fail(ctx, LVLM_ERR_HIP, "launch failed: %s", hipGetErrorString(e));
    return LVLM_OK;
}

lvlm_status bind_device(lvlm_ctx *ctx) {
    const hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail(ctx, LVLM_ERR_HIP, "hipSetDevice(%d): %s", ctx->device, hipGetErrorString(e));
    return LVLM_OK;
}

}  // namespace

extern "C" {

lvlm_status lvlm_create(lvlm_ctx **ctx, int device) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    *ctx = nullptr;
    if (device < 0) return LVLM_ERR_INVALID_ARG;
    lvlm_ctx *c = new (std::nothrow) lvlm_ctx();
    if (!c) return LVLM_ERR_HIP;
    c->device = device;
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->err[0] = '\0';
    c->prof_on = false;
    c->prof_open = c->prof_first = false;
    c->prof_n = c->prof_cap = 0;
    c->prof_ev = nullptr;
    c->prof_name = nullptr;
    *ctx = c;
    return LVLM_OK;
}

lvlm_status lvlm_destroy(lvlm_ctx *ctx) {
    if (ctx) {
        for (int i = 0; i < 2 * ctx->prof_cap; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
        delete[] ctx->prof_ev;
        delete[] ctx->prof_name;
    }
    delete ctx;
    return LVLM_OK;
}

lvlm_status lvlm_profile(lvlm_ctx *ctx, int enable) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (enable && ctx->prof_cap == 0) {
        constexpr int kCap = 4096;
        if (lvlm_status st = bind_device(ctx)) return st;
        ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * kCap];
        ctx->prof_name = new (std::nothrow) const char *[kCap];
        if (!ctx->prof_ev || !ctx->prof_name) return fail(ctx, LVLM_ERR_HIP, "out of host memory");
        for (int i = 0; i < 2 * kCap; ++i) {
            const hipError_t e = hipEventCreate(&ctx->prof_ev[i]);
            if (e != hipSuccess) return fail(ctx, LVLM_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
            ctx->prof_cap = (i + 1) / 2;
        }
    }
    ctx->prof_on = enable != 0;
    ctx->prof_open = false;
    if (enable) ctx->prof_n = 0;
    return LVLM_OK;
}

lvlm_status lvlm_profile_read(lvlm_ctx *ctx, lvlm_profile_entry *out, int max_entries, int *n_entries) {
    if (!ctx || !out || !n_entries || max_entries < 1) return LVLM_ERR_INVALID_ARG;
    int n = 0;
    for (int i = 0; i < ctx->prof_n; ++i) {
        hipError_t e = hipEventSynchronize(ctx->prof_ev[2 * i + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]);
        if (e != hipSuccess) return fail(ctx, LVLM_ERR_HIP, "profile read: %s", hipGetErrorString(e));
        int k = 0;
        while (k < n && strcmp(out[k].name, ctx->prof_name[i]) != 0) ++k;
        if (k == n) {
            if (n == max_entries) continue;
            strncpy(out[k].name, ctx->prof_name[i], sizeof(out[k].name) - 1);
            out[k].name[sizeof(out[k].name) - 1] = '\0';
            out[k].calls = 0;
            out[k].total_ms = 0.f;
            out[k].min_ms = ms;
            out[k].max_ms = ms;
            ++n;
        }
        out[k].calls += 1;
        out[k].total_ms += ms;
        if (ms < out[k].min_ms) out[k].min_ms = ms;
        if (ms > out[k].max_ms) out[k].max_ms = ms;
    }
    ctx->prof_n = 0;
    *n_entries = n;
    return LVLM_OK;
}

const char *lvlm_last_error(const lvlm_ctx *ctx) { return ctx ? ctx->err : "null context"; }

lvlm_status lvlm_workspace_bytes(const lvlm_ctx *ctx, lvlm_op op, const void *desc, size_t *bytes) {
    lvlm_ctx *c = const_cast<lvlm_ctx *>(ctx);
    if (!ctx || !desc || !bytes) return fail(c, LVLM_ERR_INVALID_ARG, "null argument");
    const char *why = nullptr;
    switch (op) {
        case LVLM_OP_SCORE: {
            const auto *d = static_cast<const lvlm_score_desc *>(desc);
            if ((why = check_score(d))) break;
            *bytes = score_ws(*d).total;
            return LVLM_OK;
        }
        case LVLM_OP_SCORE_PROBS: {
            const auto *d = static_cast<const lvlm_probs_desc *>(desc);
            if ((why = check_probs(d))) break;
            *bytes = probs_ws(*d).total;
            return LVLM_OK;
        }
        case LVLM_OP_PREFILL_ATTN: {
            const auto *d = static_cast<const lvlm_prefill_desc *>(desc);
            if ((why = check_prefill(d))) break;
            *bytes = prefill_ws(*d).total;
            return LVLM_OK;
        }
        case LVLM_OP_MERGE:
        case LVLM_OP_MERGE_SIMILAR: {
            // only shapes matter for the size: plane pointers are not inspected
            const auto *qy = static_cast<const lvlm_merge_query *>(desc);
            const lvlm_merge_desc *d = qy->desc;
            if (!d || !qy->planes) { why = "null merge query member"; break; }
            if (d->B < 1 || d->N < 1 || d->n_img < 1 || d->n_img > d->N || d->n_planes < 1 ||
                d->n_planes > LVLM_MAX_PLANES) { why = "bad merge descriptor"; break; }
            if (d->B > kMaxBatch || d->N > kMaxTokens) { why = kTooLarge; break; }
            for (int i = 0; i < d->n_planes; ++i) {
                if (qy->planes[i].row_elems < 1) why = "row_elems must be positive";
                else if (qy->planes[i].row_elems > kMaxRowElems) why = kTooLarge;
            }
            if (why) break;
            if (op == LVLM_OP_MERGE_SIMILAR) {
                if (d->n_keep < 1 || d->n_keep > d->n_img) { why = "n_keep must be in [1, n_img]"; break; }
                *bytes = sim_ws(*d).total;
            } else {
                *bytes = merge_ws(*d, qy->planes).total;
            }
            return LVLM_OK;
        }
        case LVLM_OP_KV_COMPRESS: {
            const auto *d = static_cast<const lvlm_kv_desc *>(desc);
            if ((why = check_kv(d))) break;
            *bytes = kv_ws(*d).total;
            return LVLM_OK;
        }
        case LVLM_OP_DECODE_ATTN: {
            const auto *d = static_cast<const lvlm_attn_desc *>(desc);
            if ((why = check_attn(d))) break;
            if (d->Hq / d->Hkv > 8) { why = "more than 8 query heads per KV head"; break; }
            *bytes = attn_ws(*d).total;
            return LVLM_OK;
        }
        default: why = "unknown op";
    }
    return fail(c, LVLM_ERR_INVALID_ARG, "%s", why);
}

lvlm_status lvlm_set_workspace(lvlm_ctx *ctx, void *dev_ptr, size_t bytes) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255u))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    ctx->ws = dev_ptr;
    ctx->ws_bytes = dev_ptr ? bytes : 0;
    return LVLM_OK;
}

lvlm_status lvlm_schedule(int n_img, double final_keep, int n_stages, int *n_keep_out) {
    if (n_img < 1 || n_stages < 1 || !n_keep_out || !(final_keep > 0.0) || final_keep > 1.0) return LVLM_ERR_INVALID_ARG;
    for (int s = 1; s <= n_stages; ++s) {
        const double v = floor((double)n_img * pow(final_keep, (double)s / (double)n_stages) + 0.5);
        int k = (int)v;
        if (k < 1) k = 1;
        if (k > n_img) k = n_img;
        n_keep_out[s - 1] = k;
    }
    return LVLM_OK;
}

lvlm_status lvlm_merge_weights(lvlm_merge_mode mode, int m, float *w) {
    if (m < 1 || !w) return LVLM_ERR_INVALID_ARG;
    switch (mode) {
        case LVLM_MERGE_LINEAR_RANK: {
            const double sum = (double)m * ((double)m + 1.0) / 2.0;
            for (int k = 0; k < m; ++k) w[k] = (float)((double)(m - k) / sum);
            return LVLM_OK;
        }
        case LVLM_MERGE_PAIRWISE:
            for (int k = 0; k < m; ++k) w[k] = (float)ldexp(1.0, -(k + 1));
            w[m - 1] = (float)ldexp(1.0, -(m - 1));
            return LVLM_OK;
        case LVLM_MERGE_LINEAR_RAW:
            for (int k = 0; k < m; ++k) w[k] = (float)(m - k);
            return LVLM_OK;
    }
    return LVLM_ERR_INVALID_ARG;
}

lvlm_status lvlm_score_plan(const lvlm_ctx *ctx, const lvlm_score_desc *d, int32_t *form) {
    lvlm_ctx *c = const_cast<lvlm_ctx *>(ctx);
    if (!ctx || !form) return fail(c, LVLM_ERR_INVALID_ARG, "score_plan: null argument");
    if (const char *why = check_score(d)) return fail(c, LVLM_ERR_INVALID_ARG, "score_plan: %s", why);
    const ScoreWs w = score_ws(*d);
    *form = w.shared_tiles ? (w.key_segs > 1 ? 3 : 2) : (w.single ? 1 : 0);
    return LVLM_OK;
}

lvlm_status lvlm_score_tokens(lvlm_ctx *ctx, void *stream, const lvlm_score_desc *d, const void *q, const void *k,
                              const float *row_lse, float *score_head, float *score_mean) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_score(d)) return fail(ctx, LVLM_ERR_INVALID_ARG, "score_tokens: %s", why);
    if (!q || !k || !score_head || !score_mean) return fail(ctx, LVLM_ERR_INVALID_ARG, "score_tokens: null pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(score_head) || !aligned4(score_mean) || !aligned16(row_lse))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "score_tokens: pointers must be 16-byte aligned (score_mean: 4)");
    const ScoreWs w = score_ws(*d);
    if (lvlm_status st = need_ws(ctx, w.total)) return st;
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_score(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, w, static_cast<char *>(ctx->ws), q, k,
                                          row_lse, score_head, score_mean));
}

lvlm_status lvlm_score_from_probs(lvlm_ctx *ctx, void *stream, const lvlm_probs_desc *d, const void *probs,
                                  float *score_head, float *score_mean) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_probs(d)) return fail(ctx, LVLM_ERR_INVALID_ARG, "score_from_probs: %s", why);
    if (!probs || !score_head || !score_mean) return fail(ctx, LVLM_ERR_INVALID_ARG, "score_from_probs: null pointer");
    if (!aligned16(probs) || !aligned16(score_head) || !aligned4(score_mean))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "score_from_probs: pointers must be 16-byte aligned (score_mean: 4)");
    const ProbsWs w = probs_ws(*d);
    if (lvlm_status st = need_ws(ctx, w.total)) return st;
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_score_probs(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, w,
                                                static_cast<char *>(ctx->ws), probs, score_head, score_mean));
}

lvlm_status lvlm_prefill_attn(lvlm_ctx *ctx, void *stream, const lvlm_prefill_desc *d, const void *q, const void *k,
                              const void *v, void *out, float *row_lse, float *score_head, float *score_mean) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_prefill(d)) return fail(ctx, LVLM_ERR_INVALID_ARG, "prefill_attn: %s", why);
    if (!q || !k || !v || !out || !row_lse) return fail(ctx, LVLM_ERR_INVALID_ARG, "prefill_attn: null pointer");
    if (d->T > 0 && (!score_head || !score_mean))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "prefill_attn: T > 0 needs score_head and score_mean");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(row_lse) || !aligned16(score_head) ||
        !aligned4(score_mean))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "prefill_attn: pointers must be 16-byte aligned (score_mean: 4)");
    const PrefillWs w = prefill_ws(*d);
    if (lvlm_status st = need_ws(ctx, w.total)) return st;
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_prefill_attn(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, w, static_cast<char *>(ctx->ws),
                                                 q, k, v, out, row_lse, score_head, score_mean));
}

lvlm_status lvlm_merge_compact(lvlm_ctx *ctx, void *stream, const lvlm_merge_desc *d, const float *score_mean,
                               const float *w, const lvlm_plane *planes, int32_t *keep_idx, int32_t *merged_idx) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_merge(d, planes)) return fail(ctx, LVLM_ERR_INVALID_ARG, "merge_compact: %s", why);
    if (!score_mean && d->n_keep < d->n_img) return fail(ctx, LVLM_ERR_INVALID_ARG, "merge_compact: null score_mean");
    if (!aligned4(score_mean) || !aligned16(w) || !aligned16(keep_idx) || !aligned16(merged_idx))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "merge_compact: pointers must be 16-byte aligned (score_mean: 4)");
    const MergeWs mw = merge_ws(*d, planes);
    if (lvlm_status st = need_ws(ctx, mw.total)) return st;
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_merge(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, mw, static_cast<char *>(ctx->ws),
                                          score_mean, w, planes, keep_idx, merged_idx));
}

lvlm_status lvlm_merge_similar(lvlm_ctx *ctx, void *stream, const lvlm_merge_desc *d, const float *score_mean,
                               const lvlm_plane *planes, const float *size_in, float *size_out, int32_t *keep_idx,
                               int32_t *assign) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_merge(d, planes)) return fail(ctx, LVLM_ERR_INVALID_ARG, "merge_similar: %s", why);
    if (!score_mean && d->n_keep < d->n_img) return fail(ctx, LVLM_ERR_INVALID_ARG, "merge_similar: null score_mean");
    if (!aligned4(score_mean) || !aligned16(size_in) || !aligned16(size_out) || !aligned16(keep_idx) ||
        !aligned16(assign))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "merge_similar: pointers must be 16-byte aligned (score_mean: 4)");
    if (!float_dtype(planes[0].dtype) || (planes[0].row_elems * elem_bytes(planes[0].dtype)) % 16 != 0 ||
        (planes[0].src_stride_b * elem_bytes(planes[0].dtype)) % 16 != 0)
        return fail(ctx, LVLM_ERR_UNSUPPORTED,
                    "merge_similar: planes[0] must be bf16 or fp32 with rows that are a multiple of 16 bytes");
    if ((long long)d->n_img * planes[0].row_elems * elem_bytes(planes[0].dtype) > 0x7fffffffll)
        return fail(ctx, LVLM_ERR_UNSUPPORTED, "merge_similar: the image rows of planes[0] must span less than 2 GiB");
    const SimWs w = sim_ws(*d);
    if (lvlm_status st = need_ws(ctx, w.total)) return st;
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_merge_similar(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, w,
                                                  static_cast<char *>(ctx->ws), score_mean, planes, size_in, size_out,
                                                  keep_idx, assign));
}

lvlm_status lvlm_kv_compress(lvlm_ctx *ctx, void *stream, const lvlm_kv_desc *d, void *k_cache, void *v_cache,
                             float *score, uint8_t *kind, int32_t *orig_pos, int32_t *len, int32_t *n_evicted) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_kv(d)) return fail(ctx, LVLM_ERR_INVALID_ARG, "kv_compress: %s", why);
    if (!k_cache || !v_cache || !score || !kind || !orig_pos || !len)
        return fail(ctx, LVLM_ERR_INVALID_ARG, "kv_compress: null pointer");
    if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(score) || !aligned16(kind) || !aligned16(orig_pos) ||
        !aligned16(len) || !aligned16(n_evicted))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "kv_compress: pointers must be 16-byte aligned");
    // A budget no head can exceed (the host-known bound on every length is within it) evicts nothing:
    // with no n_evicted to fill in there is nothing to launch.
    const int bound = d->len_bound > 0 ? d->len_bound : d->Lmax;
    if (d->mode == LVLM_KV_BUDGET && bound <= d->budget && n_evicted == nullptr) return LVLM_OK;
    const KvWs w = kv_ws(*d);
    if (lvlm_status st = need_ws(ctx, w.total)) return st;
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_kv_compress(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, w, static_cast<char *>(ctx->ws),
                                                k_cache, v_cache, score, kind, orig_pos, len, n_evicted));
}

static lvlm_status decode_attn_call(lvlm_ctx *ctx, bool static_scratch, void *stream, const lvlm_attn_desc *d, const void *q, const void *k_new,
                             const void *v_new, void *k_cache, void *v_cache, float *score, uint8_t *kind,
                             int32_t *orig_pos, int32_t *len, void *out) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (const char *why = check_attn(d)) return fail(ctx, LVLM_ERR_INVALID_ARG, "decode_attn: %s", why);
    if (d->Hq / d->Hkv > 8)
        return fail(ctx, LVLM_ERR_UNSUPPORTED, "decode_attn: more than 8 query heads per KV head");
    if (!q || !k_cache || !v_cache || !len || !out) return fail(ctx, LVLM_ERR_INVALID_ARG, "decode_attn: null pointer");
    if ((k_new == nullptr) != (v_new == nullptr))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "decode_attn: k_new and v_new must be given together");
    if (k_new && (!kind || !orig_pos))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "decode_attn: kind and orig_pos are needed to append");
    if (d->evict_budget > 0 && (!score || !kind || !orig_pos))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "decode_attn: score, kind and orig_pos are needed to evict");
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache) ||
        !aligned16(score) || !aligned16(kind) || !aligned16(orig_pos) || !aligned16(len) || !aligned16(out))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "decode_attn: pointers must be 16-byte aligned");
    const AttnWs w = attn_ws(*d);
    char *ws = static_cast<char *>(ctx->ws);
    if (static_scratch) {
        // the fixed array inside the library instead of the caller's workspace: nothing is allocated here
        if (w.total > (size_t)LVLM_STATIC_SCRATCH_BYTES)
            return fail(ctx, LVLM_ERR_WORKSPACE,
                        "decode_attn_static: this shape needs %zu bytes of scratch, the built-in array holds %zu "
                        "(use lvlm_decode_attn with a workspace)", w.total, (size_t)LVLM_STATIC_SCRATCH_BYTES);
        if (lvlm_status st = bind_device(ctx)) return st;
        size_t have = 0;
        const hipError_t e = attn_static_scratch(ctx->device, &ws, &have);
        if (e != hipSuccess) return fail(ctx, LVLM_ERR_HIP, "decode_attn_static: scratch array: %s", hipGetErrorString(e));
    } else {
        if (lvlm_status st = need_ws(ctx, w.total)) return st;
        if (lvlm_status st = bind_device(ctx)) return st;
    }
    return after_launch(ctx, launch_decode_attn(Prof{ctx, static_cast<hipStream_t>(stream)}, *d, w, ws,
                                                q, k_new, v_new, k_cache, v_cache, score, kind, orig_pos, len, out));
}

lvlm_status lvlm_stream_probe(lvlm_ctx *ctx, void *stream, const void *src, size_t bytes, int32_t n_workgroups,
                              uint32_t *sink) {
    if (!ctx) return LVLM_ERR_INVALID_ARG;
    if (!src || !sink || bytes < 16 || n_workgroups < 1 || n_workgroups > (1 << 20))
        return fail(ctx, LVLM_ERR_INVALID_ARG, "stream_probe: null pointer, fewer than 16 bytes or a workgroup count outside [1, 2^20]");
    if (!aligned16(src) || !aligned4(sink)) return fail(ctx, LVLM_ERR_INVALID_ARG, "stream_probe: src must be 16-byte aligned");
    if (lvlm_status st = bind_device(ctx)) return st;
    return after_launch(ctx, launch_stream_probe(Prof{ctx, static_cast<hipStream_t>(stream)}, src, bytes, n_workgroups, sink));
}

lvlm_status lvlm_decode_plan(const lvlm_ctx *ctx, const lvlm_attn_desc *d, int32_t *n_split, int32_t *split_len,
                             int32_t *form) {
    lvlm_ctx *c = const_cast<lvlm_ctx *>(ctx);
    if (!ctx || !n_split || !split_len || !form) return fail(c, LVLM_ERR_INVALID_ARG, "decode_plan: null argument");
    if (const char *why = check_attn(d)) return fail(c, LVLM_ERR_INVALID_ARG, "decode_plan: %s", why);
    const AttnWs w = attn_ws(*d);
    const int bound = d->len_bound > 0 ? d->len_bound : d->Lmax;
    *n_split = w.n_split;
    *split_len = w.split_len;
    *form = w.tail_entry ? 2 : ((w.split_len > 128 || w.n_split * w.split_len < bound) ? 1 : 0);
    return LVLM_OK;
}

lvlm_status lvlm_decode_attn(lvlm_ctx *ctx, void *stream, const lvlm_attn_desc *d, const void *q, const void *k_new,
                             const void *v_new, void *k_cache, void *v_cache, float *score, uint8_t *kind,
                             int32_t *orig_pos, int32_t *len, void *out) {
    return decode_attn_call(ctx, false, stream, d, q, k_new, v_new, k_cache, v_cache, score, kind, orig_pos, len, out);
}

lvlm_status lvlm_decode_attn_static(lvlm_ctx *ctx, void *stream, const lvlm_attn_desc *d, const void *q,
                                    const void *k_new, const void *v_new, void *k_cache, void *v_cache, float *score,
                                    uint8_t *kind, int32_t *orig_pos, int32_t *len, void *out) {
    return decode_attn_call(ctx, true, stream, d, q, k_new, v_new, k_cache, v_cache, score, kind, orig_pos, len, out);
}

}  // extern "C"
