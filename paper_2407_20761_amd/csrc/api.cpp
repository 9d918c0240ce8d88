// C ABI of the library: argument validation (host only, before anything is launched) and the
// composition of one transformer block's forward / backward out of the kernels.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "ob_internal.h"

namespace ob {

static thread_local char g_err[512] = "";

int fail(int status, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

int check_launch(const char *what) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(OB_EHIP, "%s: %s", what, hipGetErrorString(e));
    return OB_OK;
}

// ---- opt-in kernel timing ------------------------------------------------------------------
namespace {
struct ProfState {
    bool on = false;
    int used = 0;
    std::vector<hipEvent_t> start, stop;
    std::vector<int> cls;
    std::vector<double> work;
};
ProfState g_prof;
const char *const kClassNames[K_COUNT] = {
    "gemm", "attn_fwd", "attn_bwd_dq", "attn_bwd_dkv", "norm_fwd",
    "norm_bwd", "rotary", "act_fwd", "act_bwd", "colsum", "reduce_partials",
    "subsample_norm_fwd", "subsample_norm_bwd", "rows_copy"};
}  // namespace

ProfScope::ProfScope(int c, hipStream_t s, double work) : slot(-1), stream(s) {
    if (!g_prof.on || g_prof.used >= (int)g_prof.start.size()) return;
    slot = g_prof.used++;
    g_prof.cls[slot] = c;
    g_prof.work[slot] = work;
    (void)hipEventRecord(g_prof.start[slot], stream);
}
ProfScope::~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], stream);
}

namespace {

constexpr int MAX_TOKENS = 1 << 22;
constexpr int MAX_HIDDEN = 8192;  // row-wise kernels keep one row in registers

int validate_segments(const ob_segments *seg, const char *who) {
    if (!seg) return fail(OB_EINVAL, "%s: segments is null", who);
    if (!seg->cu_host || !seg->cu_dev) return fail(OB_EINVAL, "%s: cu_host / cu_dev is null", who);
    if (seg->n_seg < 1) return fail(OB_ESEGMENTS, "%s: n_seg must be >= 1", who);
    if (seg->total_tokens < 1 || seg->total_tokens > MAX_TOKENS)
        return fail(OB_EINVAL, "%s: total_tokens %d outside [1, %d]", who, seg->total_tokens, MAX_TOKENS);
    if (seg->cu_host[0] != 0) return fail(OB_ESEGMENTS, "%s: cu_seqlens[0] = %d, must be 0", who, seg->cu_host[0]);
    int longest = 0;
    for (int j = 0; j < seg->n_seg; ++j) {
        const long len = (long)seg->cu_host[j + 1] - seg->cu_host[j];
        if (len <= 0)
            return fail(OB_ESEGMENTS, "%s: segment %d has length %ld (offsets must strictly increase)", who, j, len);
        if (len > longest) longest = (int)len;
    }
    if (seg->cu_host[seg->n_seg] != seg->total_tokens)
        return fail(OB_ESEGMENTS, "%s: cu_seqlens[n_seg] = %d but total_tokens = %d", who,
                    seg->cu_host[seg->n_seg], seg->total_tokens);
    if (seg->max_seqlen < longest)
        return fail(OB_ESEGMENTS, "%s: max_seqlen %d < longest segment %d", who, seg->max_seqlen, longest);
    return OB_OK;
}

}  // namespace

int validate_attn(const ob_segments *seg, int nq, int nkv, int d, int ldq, int ldkv, int ldo,
                  int mask, int dtype, const char *who) {
    if (nq < 1 || nkv < 1 || nq % nkv != 0)
        return fail(OB_EINVAL, "%s: n_q_heads %d must be a positive multiple of n_kv_heads %d", who, nq, nkv);
    if (d != 64 && d != 128) return fail(OB_EUNSUPPORTED, "%s: head_dim %d not in {64, 128}", who, d);
    if (dtype != OB_BF16 && dtype != OB_FP32) return fail(OB_EINVAL, "%s: unknown dtype %d", who, dtype);
    if (mask != OB_MASK_SEG_BIDIR && mask != OB_MASK_SEG_CAUSAL) return fail(OB_EINVAL, "%s: unknown mask kind %d", who, mask);
    if (ldq < nq * d || ldo < nq * d || ldkv < nkv * d || ldq % 8 || ldkv % 8 || ldo % 8)
        return fail(OB_EINVAL, "%s: row strides must cover the heads and be multiples of 8 elements", who);
    return validate_segments(seg, who);
}

namespace {

int validate_desc(const ob_block_desc *dsc, const char *who) {
    if (!dsc) return fail(OB_EINVAL, "%s: desc is null", who);
    if (dsc->dtype != OB_BF16 && dsc->dtype != OB_FP32) return fail(OB_EINVAL, "%s: unknown dtype %d", who, dsc->dtype);
    if (dsc->hidden < 64 || dsc->mlp_dim < 64 || dsc->n_q_heads < 1 || dsc->n_kv_heads < 1)
        return fail(OB_EINVAL, "%s: non-positive dimension", who);
    if (dsc->n_q_heads % dsc->n_kv_heads)
        return fail(OB_EINVAL, "%s: n_q_heads %d not a multiple of n_kv_heads %d", who, dsc->n_q_heads, dsc->n_kv_heads);
    if (dsc->head_dim != 64 && dsc->head_dim != 128)
        return fail(OB_EUNSUPPORTED, "%s: head_dim %d not in {64, 128}", who, dsc->head_dim);
    if (dsc->hidden % 64 || dsc->mlp_dim % 64)
        return fail(OB_EUNSUPPORTED, "%s: hidden and mlp_dim must be multiples of 64", who);
    if (dsc->hidden > MAX_HIDDEN) return fail(OB_EUNSUPPORTED, "%s: hidden > %d", who, MAX_HIDDEN);
    if (dsc->norm != OB_LAYERNORM && dsc->norm != OB_RMSNORM) return fail(OB_EINVAL, "%s: unknown norm", who);
    if (dsc->mlp != OB_GELU && dsc->mlp != OB_SWIGLU) return fail(OB_EINVAL, "%s: unknown mlp kind", who);
    if (dsc->mask != OB_MASK_SEG_BIDIR && dsc->mask != OB_MASK_SEG_CAUSAL) return fail(OB_EINVAL, "%s: unknown mask", who);
    if (!(dsc->norm_eps >= 0.f)) return fail(OB_EINVAL, "%s: norm_eps must be >= 0", who);
    if (dsc->use_rotary && !(dsc->rotary_base > 1.f)) return fail(OB_EINVAL, "%s: rotary_base must be > 1", who);
    return OB_OK;
}

struct Dims {
    int T, H, nq, nkv, d, F, upF, Dqkv, HD;
};
Dims dims_of(const ob_block_desc *dsc, int T) {
    Dims m;
    m.T = T; m.H = dsc->hidden; m.nq = dsc->n_q_heads; m.nkv = dsc->n_kv_heads; m.d = dsc->head_dim;
    m.F = dsc->mlp_dim; m.upF = dsc->mlp == OB_SWIGLU ? 2 * dsc->mlp_dim : dsc->mlp_dim;
    m.Dqkv = (m.nq + 2 * m.nkv) * m.d; m.HD = m.nq * m.d;
    return m;
}

// bump layout of the saved-activation buffer and of the backward workspace
struct Layout {
    size_t off = 0;
    size_t take(size_t bytes) { const size_t o = off; off += align_up(bytes, 256); return o; }
};
size_t max4(size_t a, size_t b, size_t c, size_t d) { a = a > b ? a : b; c = c > d ? c : d; return a > c ? a : c; }
struct Saved { size_t h1, qkv, o, lse, x1, h2, up, act, stat1, stat2, gemm, gemm_bytes, total; };
Saved saved_layout(const Dims &m) {
    Layout L; Saved s; const size_t T = m.T;
    s.h1 = L.take(T * m.H * 2); s.qkv = L.take(T * m.Dqkv * 2); s.o = L.take(T * m.HD * 2);
    s.lse = L.take((size_t)m.nq * T * 4); s.x1 = L.take(T * m.H * 2); s.h2 = L.take(T * m.H * 2);
    s.up = L.take(T * m.upF * 2); s.act = L.take(T * m.F * 2);
    s.stat1 = L.take(T * 2 * 4); s.stat2 = L.take(T * 2 * 4);
    // scratch of the forward GEMMs (slice sums of a split contraction), not read by the backward pass
    s.gemm_bytes = max4(gemm_workspace_bytes(0, m.T, m.Dqkv, m.H), gemm_workspace_bytes(0, m.T, m.H, m.HD),
                        gemm_workspace_bytes(0, m.T, m.upF, m.H), gemm_workspace_bytes(0, m.T, m.H, m.F));
    s.gemm = L.take(s.gemm_bytes);
    s.total = L.off;
    return s;
}
struct Work { size_t dact, dup, dh, dx1, d_o, dqkv, delta, lse2, p_down, p_up, p_o, p_qkv, p_n2, p_n1, gemm, gemm_bytes, total; };
Work work_layout(const Dims &m) {
    Layout L; Work w; const size_t T = m.T;
    w.dact = L.take(T * m.F * 2); w.dup = L.take(T * m.upF * 2); w.dh = L.take(T * m.H * 2);
    w.dx1 = L.take(T * m.H * 2); w.d_o = L.take(T * m.HD * 2); w.dqkv = L.take(T * m.Dqkv * 2);
    w.delta = L.take((size_t)m.nq * T * 4); w.lse2 = L.take((size_t)m.nq * T * 4);
    // fp32 partial sums of the column reductions, one region each: they are all summed by one
    // launch at the end of the backward pass
    const size_t ncs = colsum_partials(m.T), nnb = norm_bwd_partials(m.T, m.H);
    // (b_down and b_o: column sums of dy and dx1, left by the second norm's backward next to its own partials)
    w.p_down = L.take(nnb * 2 * m.H * 4); w.p_up = L.take(ncs * m.upF * 4); w.p_o = 0;
    w.p_qkv = L.take(ncs * m.Dqkv * 4); w.p_n2 = L.take(nnb * 2 * m.H * 4); w.p_n1 = L.take(nnb * 2 * m.H * 4);
    size_t g = 0;
    auto upd = [&](int layout, int M, int N, int K) { const size_t b = gemm_workspace_bytes(layout, M, N, K); if (b > g) g = b; };
    upd(1, m.T, m.F, m.H);      // dact  = dy W_down
    // the four weight gradients (dy^T act, dup^T h2, dx1^T o, dqkv^T h1) go out as one group
    const GemmTN wg[4] = {{m.H, m.F, nullptr, nullptr, nullptr, nullptr}, {m.upF, m.H, nullptr, nullptr, nullptr, nullptr},
                          {m.H, m.HD, nullptr, nullptr, nullptr, nullptr}, {m.Dqkv, m.H, nullptr, nullptr, nullptr, nullptr}};
    { const size_t b = gemm_tn_group_workspace_bytes(4, wg, m.T); if (b > g) g = b; }
    upd(1, m.T, m.H, m.upF);    // dh2 = dup W_up
    upd(1, m.T, m.HD, m.H);     // d_o = dx1 W_o
    upd(1, m.T, m.H, m.Dqkv);   // dh1 = dqkv W_qkv
    w.gemm_bytes = g; w.gemm = L.take(g);
    w.total = L.off;
    return w;
}

inline unsigned char *at(void *base, size_t off) { return (unsigned char *)base + off; }
inline const unsigned char *at(const void *base, size_t off) { return (const unsigned char *)base + off; }

}  // namespace
}  // namespace ob

using namespace ob;

extern "C" const char *ob_last_error(void) { return g_err; }

extern "C" int ob_prof_num_classes(void) { return K_COUNT; }
extern "C" const char *ob_prof_class_name(int cls) { return cls >= 0 && cls < K_COUNT ? kClassNames[cls] : ""; }

extern "C" int ob_prof_begin(int max_launches) {
    if (g_prof.on) return fail(OB_EINVAL, "ob_prof_begin: already profiling");
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(OB_EINVAL, "ob_prof_begin: max_launches out of range");
    g_prof.start.assign(max_launches, nullptr);
    g_prof.stop.assign(max_launches, nullptr);
    g_prof.cls.assign(max_launches, 0);
    g_prof.work.assign(max_launches, 0.0);
    for (int i = 0; i < max_launches; ++i)
        if (hipEventCreate(&g_prof.start[i]) != hipSuccess || hipEventCreate(&g_prof.stop[i]) != hipSuccess)
            return fail(OB_EHIP, "ob_prof_begin: hipEventCreate failed");
    g_prof.used = 0;
    g_prof.on = true;
    return OB_OK;
}

extern "C" int ob_prof_end(double *ms_per_class, int64_t *launches_per_class, double *work_per_class,
                           int n_classes) {
    if (!g_prof.on) return fail(OB_EINVAL, "ob_prof_end: not profiling");
    if (!ms_per_class || !launches_per_class || !work_per_class || n_classes < K_COUNT)
        return fail(OB_EINVAL, "ob_prof_end: output arrays must hold ob_prof_num_classes() entries");
    g_prof.on = false;
    for (int c = 0; c < K_COUNT; ++c) { ms_per_class[c] = 0; launches_per_class[c] = 0; work_per_class[c] = 0; }
    int rc = OB_OK;
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess)
            rc = fail(OB_EHIP, "ob_prof_end: event query failed");
        ms_per_class[g_prof.cls[i]] += ms;
        launches_per_class[g_prof.cls[i]] += 1;
        work_per_class[g_prof.cls[i]] += g_prof.work[i];
    }
    const bool overflow = g_prof.used >= (int)g_prof.start.size();
    for (size_t i = 0; i < g_prof.start.size(); ++i) { (void)hipEventDestroy(g_prof.start[i]); (void)hipEventDestroy(g_prof.stop[i]); }
    g_prof.start.clear(); g_prof.stop.clear(); g_prof.used = 0;
    if (rc == OB_OK && overflow) return fail(OB_EWORKSPACE, "ob_prof_end: more launches than max_launches; totals are partial");
    return rc;
}
extern "C" int ob_has_device_code(void) { return 1; }

extern "C" int ob_varlen_attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
                                  int ldq, int ldkv, int ldo, const ob_segments *seg, int nq, int nkv,
                                  int d, float scale, int mask, int dtype, void *hip_stream) {
    if (!q || !k || !v || !o || !lse) return fail(OB_EINVAL, "ob_varlen_attn_fwd: null tensor pointer");
    if (int rc = validate_attn(seg, nq, nkv, d, ldq, ldkv, ldo, mask, dtype, "ob_varlen_attn_fwd")) return rc;
    if (dtype == OB_FP32)
        f32::attn_fwd(q, k, v, o, lse, ldq, ldkv, ldo, seg, nq, nkv, d, scale, mask, (hipStream_t)hip_stream);
    else
        launch_attn_fwd(q, k, v, o, lse, ldq, ldkv, ldo, seg, nq, nkv, d, scale, mask, (hipStream_t)hip_stream);
    return check_launch("ob_varlen_attn_fwd");
}

extern "C" size_t ob_varlen_attn_bwd_workspace_bytes(int total_tokens, int nq, int nkv, int d) {
    if (total_tokens < 1 || nq < 1 || nkv < 1 || d < 1 || nq % nkv) return 0;
    return 2 * align_up((size_t)total_tokens * nq * 4, 256);
}

extern "C" int ob_varlen_attn_bwd(const void *d_o, const void *q, const void *k, const void *v,
                                  const void *o, const float *lse, void *dq, void *dk, void *dv, int ldq,
                                  int ldkv, int ldo, const ob_segments *seg, int nq, int nkv, int d,
                                  float scale, int mask, int dtype, void *ws, size_t ws_bytes,
                                  void *hip_stream) {
    if (!d_o || !q || !k || !v || !o || !lse || !dq || !dk || !dv)
        return fail(OB_EINVAL, "ob_varlen_attn_bwd: null tensor pointer");
    if (int rc = validate_attn(seg, nq, nkv, d, ldq, ldkv, ldo, mask, dtype, "ob_varlen_attn_bwd")) return rc;
    if (!ws || ws_bytes < ob_varlen_attn_bwd_workspace_bytes(seg->total_tokens, nq, nkv, d))
        return fail(OB_EWORKSPACE, "ob_varlen_attn_bwd: workspace too small (%zu bytes given)", ws_bytes);
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == OB_FP32) {
        f32::attn_bwd(d_o, q, k, v, o, lse, dq, dk, dv, (float *)ws, ldq, ldkv, ldo, seg, nq, nkv, d, scale, mask, s);
        return check_launch("ob_varlen_attn_bwd");
    }
    const size_t rows = align_up((size_t)seg->total_tokens * nq * 4, 256);
    float *delta = (float *)ws, *lse2 = (float *)((unsigned char *)ws + rows);
    launch_attn_bwd(d_o, q, k, v, o, lse, lse2, delta, dq, dk, dv, ldq, ldkv, ldo, seg, nq, nkv, d, scale, mask, 0.f, s);
    return check_launch("ob_varlen_attn_bwd");
}

extern "C" size_t ob_block_saved_bytes(const ob_block_desc *desc, int total_tokens) {
    if (validate_desc(desc, "ob_block_saved_bytes") || total_tokens < 1 || total_tokens > MAX_TOKENS) return 0;
    if (desc->dtype == OB_FP32) return f32::saved_layout(desc, total_tokens).total;
    return saved_layout(dims_of(desc, total_tokens)).total;
}

extern "C" size_t ob_block_workspace_bytes(const ob_block_desc *desc, int total_tokens) {
    if (validate_desc(desc, "ob_block_workspace_bytes") || total_tokens < 1 || total_tokens > MAX_TOKENS) return 0;
    if (desc->dtype == OB_FP32) return f32::work_layout(desc, total_tokens).total;
    return work_layout(dims_of(desc, total_tokens)).total;
}

extern "C" size_t ob_block_saved_offset(const ob_block_desc *desc, int total_tokens, const char *name) {
    if (!name || validate_desc(desc, "ob_block_saved_offset") || total_tokens < 1) return (size_t)-1;
    Saved s = saved_layout(dims_of(desc, total_tokens));
    if (desc->dtype == OB_FP32) {
        const f32::SavedF32 f = f32::saved_layout(desc, total_tokens);
        s.h1 = f.h1; s.qkv = f.qkv; s.o = f.o; s.lse = f.lse; s.x1 = f.x1; s.h2 = f.h2; s.up = f.up; s.act = f.act;
        s.stat1 = f.stat1; s.stat2 = f.stat2;
    }
    const struct { const char *n; size_t o; } tab[] = {
        {"h1", s.h1}, {"qkv", s.qkv}, {"o", s.o}, {"lse", s.lse}, {"x1", s.x1}, {"h2", s.h2},
        {"up", s.up}, {"act", s.act}, {"stat1", s.stat1}, {"stat2", s.stat2}};
    for (const auto &e : tab)
        if (!strcmp(e.n, name)) return e.o;
    return (size_t)-1;
}

static int validate_block(const ob_block_desc *desc, const ob_block_weights *w, const ob_segments *seg,
                          const void *saved, size_t saved_bytes, const void *ws, size_t ws_bytes,
                          const char *who) {
    if (int rc = validate_desc(desc, who)) return rc;
    if (!w) return fail(OB_EINVAL, "%s: weights is null", who);
    if (!w->n1_g || !w->w_qkv || !w->w_o || !w->n2_g || !w->w_up || !w->w_down)
        return fail(OB_EINVAL, "%s: a required weight pointer is null", who);
    if (desc->has_bias) {
        if (!w->b_qkv || !w->b_o || !w->b_up || !w->b_down) return fail(OB_EINVAL, "%s: has_bias set but a bias pointer is null", who);
        if (desc->norm == OB_LAYERNORM && (!w->n1_b || !w->n2_b)) return fail(OB_EINVAL, "%s: has_bias set but a beta pointer is null", who);
    }
    if (int rc = validate_segments(seg, who)) return rc;
    if (!saved || saved_bytes < ob_block_saved_bytes(desc, seg->total_tokens))
        return fail(OB_EWORKSPACE, "%s: saved buffer too small (%zu bytes given)", who, saved_bytes);
    if (!ws || ws_bytes < ob_block_workspace_bytes(desc, seg->total_tokens))
        return fail(OB_EWORKSPACE, "%s: workspace too small (%zu bytes given)", who, ws_bytes);
    return OB_OK;
}

// forward of one bf16 block into `saved`; y == nullptr: everything but the last GEMM (the replay
// of the re-computation path, which has no use for the block output)
static void block_fwd_bf16(const ob_block_desc *desc, const ob_block_weights *w, const void *x, void *y,
                           void *saved, const ob_segments *seg, hipStream_t s) {
    const Dims m = dims_of(desc, seg->total_tokens);
    const Saved sv = saved_layout(m);
    const bool bias = desc->has_bias != 0;
    const bool beta = bias && desc->norm == OB_LAYERNORM;
    unsigned char *h1 = at(saved, sv.h1), *qkv = at(saved, sv.qkv), *o = at(saved, sv.o);
    unsigned char *x1 = at(saved, sv.x1), *h2 = at(saved, sv.h2), *up = at(saved, sv.up), *act = at(saved, sv.act);
    float *lse = (float *)at(saved, sv.lse);
    void *gws = sv.gemm_bytes ? at(saved, sv.gemm) : nullptr;
    const float scale = 1.0f / sqrtf((float)m.d);

    launch_norm_fwd(desc->norm, x, w->n1_g, beta ? w->n1_b : nullptr, h1, (float *)at(saved, sv.stat1), m.T, m.H, desc->norm_eps, s);
    launch_gemm_nt(m.T, m.Dqkv, m.H, h1, m.H, w->w_qkv, m.H, qkv, m.Dqkv, bias ? w->b_qkv : nullptr, nullptr, 0, s, 0, gws);
    if (desc->use_rotary)
        launch_rotary(qkv, m.Dqkv, m.T, m.nq + m.nkv, m.d, seg->cu_dev, seg->n_seg, desc->rotary_base, 1.0f, s);
    launch_attn_fwd(qkv, qkv + (size_t)m.nq * m.d * 2, qkv + (size_t)(m.nq + m.nkv) * m.d * 2, o, lse, m.Dqkv,
                    m.Dqkv, m.HD, seg, m.nq, m.nkv, m.d, scale, desc->mask, s);
    launch_gemm_nt(m.T, m.H, m.HD, o, m.HD, w->w_o, m.HD, x1, m.H, bias ? w->b_o : nullptr, x, m.H, s, 0, gws);
    launch_norm_fwd(desc->norm, x1, w->n2_g, beta ? w->n2_b : nullptr, h2, (float *)at(saved, sv.stat2), m.T, m.H, desc->norm_eps, s);
    launch_gemm_nt(m.T, m.upF, m.H, h2, m.H, w->w_up, m.H, up, m.upF, bias ? w->b_up : nullptr, nullptr, 0, s, 0, gws);
    launch_act_fwd(desc->mlp, up, act, m.T, m.F, s);
    if (y) launch_gemm_nt(m.T, m.H, m.F, act, m.F, w->w_down, m.F, y, m.H, bias ? w->b_down : nullptr, x1, m.H, s, 0, gws);
}

extern "C" int ob_block_fwd(const ob_block_desc *desc, const ob_block_weights *w, const void *x, void *y,
                            void *saved, size_t saved_bytes, const ob_segments *seg, void *ws,
                            size_t ws_bytes, void *hip_stream) {
    if (!x || !y) return fail(OB_EINVAL, "ob_block_fwd: x / y is null");
    if (int rc = validate_block(desc, w, seg, saved, saved_bytes, ws, ws_bytes, "ob_block_fwd")) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    if (desc->dtype == OB_FP32) f32::block_fwd(desc, w, x, y, saved, seg, s);
    else block_fwd_bf16(desc, w, x, y, saved, seg, s);
    return check_launch("ob_block_fwd");
}

extern "C" int ob_block_bwd(const ob_block_desc *desc, const ob_block_weights *w, const ob_block_grads *g,
                            int flags, const void *x, const void *dy, void *dx,
                            void *saved, size_t saved_bytes, const ob_segments *seg, void *ws,
                            size_t ws_bytes, void *hip_stream) {
    if (!x || !dy || !dx) return fail(OB_EINVAL, "ob_block_bwd: x / dy / dx is null");
    if (flags & ~(OB_BWD_ACCUMULATE | OB_BWD_RECOMPUTE)) return fail(OB_EINVAL, "ob_block_bwd: unknown flag bits %d", flags);
    const int accumulate_wgrad = flags & OB_BWD_ACCUMULATE;
    if (int rc = validate_block(desc, w, seg, saved, saved_bytes, ws, ws_bytes, "ob_block_bwd")) return rc;
    if (!g) return fail(OB_EINVAL, "ob_block_bwd: grads is null");
    if (!g->n1_g || !g->w_qkv || !g->w_o || !g->n2_g || !g->w_up || !g->w_down)
        return fail(OB_EINVAL, "ob_block_bwd: a required gradient pointer is null");
    const bool bias = desc->has_bias != 0;
    const bool beta = bias && desc->norm == OB_LAYERNORM;
    if (bias && (!g->b_qkv || !g->b_o || !g->b_up || !g->b_down)) return fail(OB_EINVAL, "ob_block_bwd: a bias gradient pointer is null");
    if (beta && (!g->n1_b || !g->n2_b)) return fail(OB_EINVAL, "ob_block_bwd: a beta gradient pointer is null");

    hipStream_t s = (hipStream_t)hip_stream;
    if (desc->dtype == OB_FP32) {
        if (flags & OB_BWD_RECOMPUTE) f32::block_fwd(desc, w, x, nullptr, saved, seg, s);
        f32::block_bwd(desc, w, g, accumulate_wgrad ? 1 : 0, x, dy, dx, saved, seg, ws, s);
        return check_launch("ob_block_bwd");
    }
    if (flags & OB_BWD_RECOMPUTE) block_fwd_bf16(desc, w, x, nullptr, saved, seg, s);
    const Dims m = dims_of(desc, seg->total_tokens);
    const Saved sv = saved_layout(m);
    const Work wk = work_layout(m);
    const int acc = accumulate_wgrad ? 1 : 0;
    const unsigned char *h1 = at(saved, sv.h1), *qkv = at(saved, sv.qkv), *o = at(saved, sv.o);
    const unsigned char *x1 = at(saved, sv.x1), *h2 = at(saved, sv.h2), *up = at(saved, sv.up), *act = at(saved, sv.act);
    const float *lse = (const float *)at(saved, sv.lse);
    unsigned char *dact = at(ws, wk.dact), *dup = at(ws, wk.dup), *dh = at(ws, wk.dh), *dx1 = at(ws, wk.dx1);
    unsigned char *d_o = at(ws, wk.d_o), *dqkv = at(ws, wk.dqkv), *gws = at(ws, wk.gemm);
    float *delta = (float *)at(ws, wk.delta);
    const float scale = 1.0f / sqrtf((float)m.d);
    const int ncs = colsum_partials(m.T), nnb = norm_bwd_partials(m.T, m.H);
    int rc;
    ReduceBatch sums;      // the column reductions' second halves, launched together at the end
    auto bias_grad = [&](const void *src, int C, size_t region, void *out) {
        float *partial = (float *)at(ws, region);
        launch_colsum(src, m.T, C, C, partial, s);
        sums.add(partial, ncs, C, out, C);
    };
    auto norm_grads = [&](size_t region, void *gamma_out, void *beta_out) {
        const float *partial = (const float *)at(ws, region);
        sums.add(partial, nnb, 2 * m.H, gamma_out, m.H);
        if (beta) sums.add(partial + m.H, nnb, 2 * m.H, beta_out, m.H);
    };

    // y = x1 + act W_down^T + b_down
    if ((rc = gemm_any(1, m.T, m.F, m.H, dy, w->w_down, dact, nullptr, nullptr, gws, wk.gemm_bytes, s))) return rc;
    launch_act_bwd(desc->mlp, dact, up, dup, m.T, m.F, s);
    if (bias) bias_grad(dup, m.upF, wk.p_up, g->b_up);
    if ((rc = gemm_any(1, m.T, m.H, m.upF, dup, w->w_up, dh, nullptr, nullptr, gws, wk.gemm_bytes, s))) return rc;
    // dx1 = dy + norm2_bwd(dh2)
    // (with biases the same pass leaves the column sums of dy and of dx1: the gradients of b_down and b_o)
    float *csum = bias ? (float *)at(ws, wk.p_down) : nullptr;
    launch_norm_bwd(desc->norm, dh, x1, (const float *)at(saved, sv.stat2), w->n2_g, dy, dx1, (float *)at(ws, wk.p_n2), m.T, m.H, s, csum);
    norm_grads(wk.p_n2, g->n2_g, g->n2_b);
    if (bias) {
        sums.add(csum, nnb, 2 * m.H, g->b_down, m.H);
        sums.add(csum + m.H, nnb, 2 * m.H, g->b_o, m.H);
    }
    // x1 = x + o W_o^T + b_o
    if ((rc = gemm_any(1, m.T, m.HD, m.H, dx1, w->w_o, d_o, nullptr, nullptr, gws, wk.gemm_bytes, s))) return rc;
    // attention
    float *lse2 = (float *)at(ws, wk.lse2);
    // (the rotary backward of dq and dk happens in the attention kernels' epilogues)
    launch_attn_bwd(d_o, qkv, qkv + (size_t)m.nq * m.d * 2, qkv + (size_t)(m.nq + m.nkv) * m.d * 2, o, lse, lse2, delta,
                    dqkv, dqkv + (size_t)m.nq * m.d * 2, dqkv + (size_t)(m.nq + m.nkv) * m.d * 2,
                    m.Dqkv, m.Dqkv, m.HD, seg, m.nq, m.nkv, m.d, scale, desc->mask,
                    desc->use_rotary ? desc->rotary_base : 0.f, s);
    // qkv = h1 W_qkv^T + b_qkv
    if (bias) bias_grad(dqkv, m.Dqkv, wk.p_qkv, g->b_qkv);
    if ((rc = gemm_any(1, m.T, m.H, m.Dqkv, dqkv, w->w_qkv, dh, nullptr, nullptr, gws, wk.gemm_bytes, s))) return rc;
    // dx = dx1 + norm1_bwd(dh1)
    launch_norm_bwd(desc->norm, dh, x, (const float *)at(saved, sv.stat1), w->n1_g, dx1, dx, (float *)at(ws, wk.p_n1), m.T, m.H, s);
    norm_grads(wk.p_n1, g->n1_g, g->n1_b);
    // The four weight gradients, dW = (upstream gradient)^T (layer input) over all tokens, in one launch:
    // their operands are all still in place (dy, the workspace members, `saved`), and dealt to the chip as
    // one list of tiles they leave one incomplete round instead of four.
    const GemmTN wgrads[4] = {{m.H, m.F, dy, act, g->w_down, acc ? g->w_down : nullptr},
                              {m.upF, m.H, dup, h2, g->w_up, acc ? g->w_up : nullptr},
                              {m.H, m.HD, dx1, o, g->w_o, acc ? g->w_o : nullptr},
                              {m.Dqkv, m.H, dqkv, h1, g->w_qkv, acc ? g->w_qkv : nullptr}};
    if ((rc = gemm_tn_group(4, wgrads, m.T, gws, wk.gemm_bytes, s))) return rc;
    if ((rc = launch_reduce_batch(sums, acc, s))) return rc;
    return check_launch("ob_block_bwd");
}

extern "C" size_t ob_gemm_workspace_bytes(int layout, int M, int N, int K) {
    if (layout < 0 || layout > 2 || M < 1 || N < 1 || K < 1) return 0;
    return gemm_workspace_bytes(layout, M, N, K);
}

extern "C" int ob_gemm_bf16(int layout, int M, int N, int K, const void *A, const void *B, void *C,
                            const void *bias, const void *R, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!A || !B || !C) return fail(OB_EINVAL, "ob_gemm_bf16: null matrix pointer");
    if (layout < 0 || layout > 2) return fail(OB_EINVAL, "ob_gemm_bf16: layout %d not in {0,1,2}", layout);
    if (M < 1 || N < 1 || K < 1) return fail(OB_EINVAL, "ob_gemm_bf16: non-positive size");
    if (N % 64) return fail(OB_EUNSUPPORTED, "ob_gemm_bf16: N = %d must be a multiple of 64", N);
    if (layout != 2 && K % 64) return fail(OB_EUNSUPPORTED, "ob_gemm_bf16: K = %d must be a multiple of 64 for layouts NT / NN", K);
    if (layout == 2 && M % 64) return fail(OB_EUNSUPPORTED, "ob_gemm_bf16: M = %d must be a multiple of 64 for layout TN", M);
    const size_t need = gemm_workspace_bytes(layout, M, N, K);
    if (need && ws && ws_bytes < need) return fail(OB_EWORKSPACE, "ob_gemm_bf16: workspace too small (%zu < %zu)", ws_bytes, need);
    return gemm_any(layout, M, N, K, A, B, C, bias, R, ws, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int ob_debug_materialize_mask(const ob_segments *seg, int mask, uint8_t *mask_dev, void *hip_stream) {
    if (!mask_dev) return fail(OB_EINVAL, "ob_debug_materialize_mask: null output");
    if (mask != OB_MASK_SEG_BIDIR && mask != OB_MASK_SEG_CAUSAL) return fail(OB_EINVAL, "ob_debug_materialize_mask: unknown mask kind");
    if (int rc = validate_segments(seg, "ob_debug_materialize_mask")) return rc;
    if (seg->total_tokens > 4096) return fail(OB_EUNSUPPORTED, "ob_debug_materialize_mask: T > 4096");
    launch_mask(seg->cu_dev, seg->n_seg, seg->total_tokens, mask, mask_dev, (hipStream_t)hip_stream);
    return check_launch("ob_debug_materialize_mask");
}
