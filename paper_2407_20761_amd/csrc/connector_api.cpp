// C ABI of the ViT -> LLM hand-over: validation and the composition of its forward / backward out
// of the row-wise kernels in connector.hip, the GEMM, the GELU and the column-sum kernels.
#include <vector>

#include "ob_internal.h"

using namespace ob;

namespace {

constexpr int MAX_TILES = 1 << 16;

struct CDims { int n_tok, Hv, W, Ht, g, n_tiles; };

struct Bump {
    size_t off = 0;
    size_t take(size_t bytes) { const size_t o = off; off += align_up(bytes, 256); return o; }
};
struct CSaved { size_t un, h, a, stats, total; };
struct CWork { size_t z, da, dh, dun, partial, gemm, gemm_bytes, total; };

CSaved saved_layout(const CDims &m) {
    Bump L; CSaved s; const size_t n = m.n_tok;
    s.un = L.take(n * m.W * 2); s.h = L.take(n * m.Ht * 2); s.a = L.take(n * m.Ht * 2); s.stats = L.take(n * 2 * 4);
    s.total = L.off;
    return s;
}
CWork work_layout(const CDims &m) {
    Bump L; CWork w; const size_t n = m.n_tok;
    w.z = L.take(n * m.Ht * 2);      // z in the forward, dz in the backward
    w.da = L.take(n * m.Ht * 2); w.dh = L.take(n * m.Ht * 2); w.dun = L.take(n * m.W * 2);
    const size_t p_norm = (size_t)subsample_wgrad_partials(m.n_tok) * 2 * m.W * 4;
    const size_t p_bias = (size_t)colsum_partials(m.n_tok) * m.Ht * 4;
    w.partial = L.take(p_norm > p_bias ? p_norm : p_bias);
    // slice sums of the GEMMs whose last round of tiles is split along K
    size_t g = 0;
    const int shapes[6][4] = {{0, m.n_tok, m.Ht, m.W}, {0, m.n_tok, m.Ht, m.Ht}, {2, m.Ht, m.Ht, m.n_tok},
                              {1, m.n_tok, m.Ht, m.Ht}, {2, m.Ht, m.W, m.n_tok}, {1, m.n_tok, m.W, m.Ht}};
    for (const auto &q : shapes) {
        const size_t b = gemm_workspace_bytes(q[0], q[1], q[2], q[3]);
        if (b > g) g = b;
    }
    w.gemm_bytes = g; w.gemm = L.take(g);
    w.total = L.off;
    return w;
}

int validate(const ob_connector_desc *d, int n_tiles, const char *who, CDims *out) {
    if (!d) return fail(OB_EINVAL, "%s: desc is null", who);
    if (d->dtype != OB_BF16 && d->dtype != OB_FP32) return fail(OB_EUNSUPPORTED, "%s: dtype must be OB_BF16 or OB_FP32", who);
    if (d->vit_hidden < 64 || d->llm_hidden < 64 || d->vit_hidden % 64 || d->llm_hidden % 64)
        return fail(OB_EUNSUPPORTED, "%s: vit_hidden and llm_hidden must be positive multiples of 64", who);
    if (4 * d->vit_hidden > subsample_max_width())
        return fail(OB_EUNSUPPORTED, "%s: 4 * vit_hidden > %d", who, subsample_max_width());
    if (d->grid < 2 || d->grid % 2 || d->grid > 1024) return fail(OB_EINVAL, "%s: grid must be even, 2 .. 1024", who);
    if (!(d->norm_eps >= 0.f)) return fail(OB_EINVAL, "%s: norm_eps must be >= 0", who);
    if (n_tiles < 1 || n_tiles > MAX_TILES) return fail(OB_EINVAL, "%s: n_tiles %d outside [1, %d]", who, n_tiles, MAX_TILES);
    const long n_tok = (long)n_tiles * (d->grid / 2) * (d->grid / 2);
    if (n_tok > (1 << 22)) return fail(OB_EINVAL, "%s: %ld sub-sampled tokens is too many", who, n_tok);
    if (out) *out = CDims{(int)n_tok, d->vit_hidden, 4 * d->vit_hidden, d->llm_hidden, d->grid, n_tiles};
    return OB_OK;
}

int validate_rows(const int32_t *rows_host, const int32_t *rows_dev, int n, int llm_tokens, const char *who) {
    if (!rows_host || !rows_dev) return fail(OB_EINVAL, "%s: dst_rows_host / dst_rows_dev is null", who);
    if (llm_tokens < n) return fail(OB_EINVAL, "%s: llm_tokens %d < %d visual tokens", who, llm_tokens, n);
    std::vector<bool> seen((size_t)llm_tokens, false);
    for (int i = 0; i < n; ++i) {
        const int r = rows_host[i];
        if (r < 0 || r >= llm_tokens) return fail(OB_EINVAL, "%s: dst_rows[%d] = %d outside [0, %d)", who, i, r, llm_tokens);
        if (seen[r]) return fail(OB_EINVAL, "%s: dst_rows[%d] = %d appears twice", who, i, r);
        seen[r] = true;
    }
    return OB_OK;
}

inline unsigned char *at(void *base, size_t off) { return (unsigned char *)base + off; }
inline const unsigned char *at(const void *base, size_t off) { return (const unsigned char *)base + off; }

}  // namespace

extern "C" size_t ob_connector_saved_bytes(const ob_connector_desc *desc, int n_tiles) {
    CDims m;
    if (validate(desc, n_tiles, "ob_connector_saved_bytes", &m)) return 0;
    if (desc->dtype == OB_FP32) return f32::connector_saved_bytes(m.n_tok, m.Hv, m.Ht);
    return saved_layout(m).total;
}

extern "C" size_t ob_connector_workspace_bytes(const ob_connector_desc *desc, int n_tiles) {
    CDims m;
    if (validate(desc, n_tiles, "ob_connector_workspace_bytes", &m)) return 0;
    if (desc->dtype == OB_FP32) return f32::connector_work_bytes(m.n_tok, m.Hv, m.Ht);
    return work_layout(m).total;
}

extern "C" int ob_connector_fwd(const ob_connector_desc *desc, const ob_connector_weights *w, const void *v,
                                int n_tiles, const int32_t *dst_rows_host, const int32_t *dst_rows_dev,
                                void *x_llm, int llm_tokens, void *saved, size_t saved_bytes, void *ws,
                                size_t ws_bytes, void *hip_stream) {
    const char *who = "ob_connector_fwd";
    CDims m;
    if (int rc = validate(desc, n_tiles, who, &m)) return rc;
    if (!v || !x_llm) return fail(OB_EINVAL, "%s: v / x_llm is null", who);
    if (!w || !w->n_g || !w->n_b || !w->w1 || !w->b1 || !w->w2 || !w->b2) return fail(OB_EINVAL, "%s: a weight pointer is null", who);
    if (int rc = validate_rows(dst_rows_host, dst_rows_dev, m.n_tok, llm_tokens, who)) return rc;
    if (desc->dtype == OB_FP32) {   // debug path: same steps, every tensor fp32
        if (!saved || saved_bytes < f32::connector_saved_bytes(m.n_tok, m.Hv, m.Ht))
            return fail(OB_EWORKSPACE, "%s: saved buffer too small (%zu bytes given)", who, saved_bytes);
        if (!ws || ws_bytes < f32::connector_work_bytes(m.n_tok, m.Hv, m.Ht))
            return fail(OB_EWORKSPACE, "%s: workspace too small (%zu bytes given)", who, ws_bytes);
        f32::connector_fwd(w, v, m.n_tok, m.g, m.Hv, m.Ht, desc->norm_eps, dst_rows_dev, x_llm, saved, ws,
                           (hipStream_t)hip_stream);
        return check_launch(who);
    }
    const CSaved sv = saved_layout(m);
    const CWork wk = work_layout(m);
    if (!saved || saved_bytes < sv.total) return fail(OB_EWORKSPACE, "%s: saved buffer too small (%zu bytes given)", who, saved_bytes);
    if (!ws || ws_bytes < wk.total) return fail(OB_EWORKSPACE, "%s: workspace too small (%zu bytes given)", who, ws_bytes);
    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char *un = at(saved, sv.un), *h = at(saved, sv.h), *a = at(saved, sv.a), *z = at(ws, wk.z);
    launch_subsample_norm_fwd(v, w->n_g, w->n_b, un, (float *)at(saved, sv.stats), m.n_tok, m.g, m.Hv, desc->norm_eps, s);
    void *gws = wk.gemm_bytes ? at(ws, wk.gemm) : nullptr;
    launch_gemm_nt(m.n_tok, m.Ht, m.W, un, m.W, w->w1, m.W, h, m.Ht, w->b1, nullptr, 0, s, 0, gws);
    launch_act_fwd(OB_GELU, h, a, m.n_tok, m.Ht, s);
    launch_gemm_nt(m.n_tok, m.Ht, m.Ht, a, m.Ht, w->w2, m.Ht, z, m.Ht, w->b2, nullptr, 0, s, 0, gws);
    launch_rows_scatter(z, x_llm, dst_rows_dev, m.n_tok, m.Ht, s);
    return check_launch(who);
}

extern "C" int ob_connector_bwd(const ob_connector_desc *desc, const ob_connector_weights *w,
                                const ob_connector_grads *g, int flags, const void *v, const void *dx_llm,
                                void *dv, int n_tiles, const int32_t *dst_rows_host,
                                const int32_t *dst_rows_dev, int llm_tokens, const void *saved,
                                size_t saved_bytes, void *ws, size_t ws_bytes, void *hip_stream) {
    const char *who = "ob_connector_bwd";
    CDims m;
    if (int rc = validate(desc, n_tiles, who, &m)) return rc;
    if (flags & ~OB_BWD_ACCUMULATE) return fail(OB_EINVAL, "%s: unknown flag bits %d", who, flags);
    if (!v || !dx_llm || !dv) return fail(OB_EINVAL, "%s: v / dx_llm / dv is null", who);
    if (!w || !w->n_g || !w->w1 || !w->w2) return fail(OB_EINVAL, "%s: a weight pointer is null", who);
    if (!g || !g->n_g || !g->n_b || !g->w1 || !g->b1 || !g->w2 || !g->b2) return fail(OB_EINVAL, "%s: a gradient pointer is null", who);
    if (int rc = validate_rows(dst_rows_host, dst_rows_dev, m.n_tok, llm_tokens, who)) return rc;
    if (desc->dtype == OB_FP32) {
        if (!saved || saved_bytes < f32::connector_saved_bytes(m.n_tok, m.Hv, m.Ht))
            return fail(OB_EWORKSPACE, "%s: saved buffer too small (%zu bytes given)", who, saved_bytes);
        if (!ws || ws_bytes < f32::connector_work_bytes(m.n_tok, m.Hv, m.Ht))
            return fail(OB_EWORKSPACE, "%s: workspace too small (%zu bytes given)", who, ws_bytes);
        f32::connector_bwd(w, g, flags & OB_BWD_ACCUMULATE ? 1 : 0, dx_llm, dv, m.n_tok, m.n_tiles, m.g, m.Hv, m.Ht,
                           dst_rows_dev, saved, ws, (hipStream_t)hip_stream);
        return check_launch(who);
    }
    const CSaved sv = saved_layout(m);
    const CWork wk = work_layout(m);
    if (!saved || saved_bytes < sv.total) return fail(OB_EWORKSPACE, "%s: saved buffer too small (%zu bytes given)", who, saved_bytes);
    if (!ws || ws_bytes < wk.total) return fail(OB_EWORKSPACE, "%s: workspace too small (%zu bytes given)", who, ws_bytes);
    hipStream_t s = (hipStream_t)hip_stream;
    const int acc = flags & OB_BWD_ACCUMULATE ? 1 : 0;
    const unsigned char *un = at(saved, sv.un), *h = at(saved, sv.h), *a = at(saved, sv.a);
    const float *stats = (const float *)at(saved, sv.stats);
    unsigned char *dz = at(ws, wk.z), *da = at(ws, wk.da), *dh = at(ws, wk.dh), *dun = at(ws, wk.dun);
    float *partial = (float *)at(ws, wk.partial);
    void *gws = at(ws, wk.gemm);
    const int ncs = colsum_partials(m.n_tok);
    int rc;
    launch_rows_gather(dz, dx_llm, dst_rows_dev, m.n_tok, m.Ht, s);
    // z = a W2^T + b2
    if ((rc = gemm_any(2, m.Ht, m.Ht, m.n_tok, dz, a, g->w2, nullptr, acc ? g->w2 : nullptr, gws, wk.gemm_bytes, s))) return rc;
    launch_colsum(dz, m.n_tok, m.Ht, m.Ht, partial, s);
    launch_reduce_partials(partial, ncs, m.Ht, g->b2, m.Ht, acc, s);
    if ((rc = gemm_any(1, m.n_tok, m.Ht, m.Ht, dz, w->w2, da, nullptr, nullptr, gws, wk.gemm_bytes, s))) return rc;
    // a = GELU(h), h = un W1^T + b1
    launch_act_bwd(OB_GELU, da, h, dh, m.n_tok, m.Ht, s);
    if ((rc = gemm_any(2, m.Ht, m.W, m.n_tok, dh, un, g->w1, nullptr, acc ? g->w1 : nullptr, gws, wk.gemm_bytes, s))) return rc;
    launch_colsum(dh, m.n_tok, m.Ht, m.Ht, partial, s);
    launch_reduce_partials(partial, ncs, m.Ht, g->b1, m.Ht, acc, s);
    if ((rc = gemm_any(1, m.n_tok, m.W, m.Ht, dh, w->w1, dun, nullptr, nullptr, gws, wk.gemm_bytes, s))) return rc;
    // un = LayerNorm(gather(v))
    launch_subsample_norm_bwd(dun, v, stats, w->n_g, dv, m.n_tok, m.n_tiles, m.g, m.Hv, s);
    launch_subsample_norm_wgrad(dun, v, stats, partial, m.n_tok, m.g, m.Hv, s);
    const int nwp = subsample_wgrad_partials(m.n_tok);
    launch_reduce_partials(partial, nwp, 2 * m.W, g->n_g, m.W, acc, s);
    launch_reduce_partials(partial + m.W, nwp, 2 * m.W, g->n_b, m.W, acc, s);
    return check_launch(who);
}
