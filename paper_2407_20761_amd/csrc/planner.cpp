// Host-side planning steps of the method that sit next to the hot path: the arithmetic of the
// adaptive re-computation procedure (Sec. 4.3, Step 4) and the balanced model partitioning search
// (Sec. 4.2: greedy anchor, radius-r candidates, VAR(fwd_time) + SUM(comm) ranking).  No GPU work.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "ob_internal.h"

using namespace ob;

// Sec. 4.3, Step 4.  With re-computation enabled everywhere a stage has `free_bytes` left (M_r);
// keeping one ViT / LLM layer's activations costs saved_bytes_vit / saved_bytes_llm (M_v / M_t)
// and saves that layer's forward replay.  Among the (keep_vit, keep_llm) pairs that fit, take the
// one that saves the most replay time (ties: fewer bytes, then fewer ViT layers).  Every failed
// trial run of the caller adds one to `extra_recompute`: one more kept layer is given up, the
// kind with the larger footprint first.
extern "C" int ob_recompute_plan(int64_t free_bytes, int n_vit, int64_t saved_bytes_vit, double fwd_ms_vit,
                                 int n_llm, int64_t saved_bytes_llm, double fwd_ms_llm, int extra_recompute,
                                 int *keep_vit, int *keep_llm) {
    if (!keep_vit || !keep_llm) return fail(OB_EINVAL, "ob_recompute_plan: null output");
    if (n_vit < 0 || n_llm < 0 || extra_recompute < 0 || free_bytes < 0)
        return fail(OB_EINVAL, "ob_recompute_plan: negative count or budget");
    if ((n_vit > 0 && saved_bytes_vit <= 0) || (n_llm > 0 && saved_bytes_llm <= 0))
        return fail(OB_EINVAL, "ob_recompute_plan: per-layer bytes must be positive");
    if (!(fwd_ms_vit >= 0) || !(fwd_ms_llm >= 0)) return fail(OB_EINVAL, "ob_recompute_plan: negative time");
    int best_v = 0, best_t = 0;
    double best_ms = -1.0;
    int64_t best_bytes = 0;
    for (int kv = 0; kv <= n_vit; ++kv) {
        const int64_t used_v = (int64_t)kv * saved_bytes_vit;
        if (used_v > free_bytes) break;
        // keeping a layer whose replay costs nothing only spends bytes
        const int kt = (n_llm == 0 || !(fwd_ms_llm > 0)) ? 0
                       : (int)std::min<int64_t>(n_llm, (free_bytes - used_v) / saved_bytes_llm);
        const double ms = kv * fwd_ms_vit + kt * fwd_ms_llm;
        const int64_t bytes = used_v + (int64_t)kt * saved_bytes_llm;
        if (ms > best_ms || (ms == best_ms && bytes < best_bytes)) {
            best_ms = ms; best_bytes = bytes; best_v = kv; best_t = kt;
        }
    }
    for (int e = 0; e < extra_recompute && best_v + best_t > 0; ++e) {
        const bool drop_vit = best_v > 0 && (best_t == 0 || saved_bytes_vit > saved_bytes_llm ||
                                             (saved_bytes_vit == saved_bytes_llm && fwd_ms_vit <= fwd_ms_llm));
        if (drop_vit) --best_v; else --best_t;
    }
    *keep_vit = best_v;
    *keep_llm = best_t;
    return OB_OK;
}

namespace {

int validate_bmp(const double *fwd, int L, int N, const char *who) {
    if (!fwd) return fail(OB_EINVAL, "%s: fwd_ms is null", who);
    if (N < 1 || L < N) return fail(OB_EINVAL, "%s: need 1 <= N <= L (L = %d, N = %d)", who, L, N);
    for (int i = 0; i < L; ++i)
        if (!(fwd[i] >= 0)) return fail(OB_EINVAL, "%s: fwd_ms[%d] is negative or NaN", who, i);
    return OB_OK;
}

// Anchor P+ (Sec. 4.2 "Partition Candidates"): layers are numbered 1..L, stage i holds layers
// P(i-1) <= l < P(i) with P(0) = 1, P(N) = L + 1.  Cut i goes where the running time is closest to
// i/N of the total, among the positions that leave every stage at least one layer.
void anchor(const double *fwd, int L, int N, int *P) {
    std::vector<double> cum(L + 1, 0.0);  // cum[j] = time of layers 1..j
    for (int j = 1; j <= L; ++j) cum[j] = cum[j - 1] + fwd[j - 1];
    int prev = 1;
    for (int i = 1; i < N; ++i) {
        const double target = cum[L] * i / N;
        int best = prev + 1;
        double best_d = INFINITY;
        for (int p = prev + 1; p <= L + 1 - (N - i); ++p) {  // stage i = layers prev .. p-1
            const double dist = std::fabs(cum[p - 1] - target);
            if (dist < best_d) { best_d = dist; best = p; }
        }
        P[i - 1] = best;
        prev = best;
    }
}

}  // namespace

extern "C" int ob_bmp_anchor(const double *fwd_ms, int L, int N, int *P_out) {
    if (int rc = validate_bmp(fwd_ms, L, N, "ob_bmp_anchor")) return rc;
    if (N > 1 && !P_out) return fail(OB_EINVAL, "ob_bmp_anchor: P_out is null");
    anchor(fwd_ms, L, N, P_out);
    return OB_OK;
}

// Candidates = every P with |P(i) - P+(i)| <= r that is strictly increasing inside (1, L + 1);
// score = sum_i (FWD(S_i) - mean)^2 + comm_weight * sum_{i<N} ACTIV(last layer of S_i)  (Eq. 4 + Eq. 5
// as printed: no 1/N); the top_k lowest scores are returned in ascending order (ties: lexicographic).
extern "C" int ob_bmp_search(const double *fwd_ms, const double *activ, int L, int N, int r, double comm_weight,
                             int top_k, int *cand_out, double *score_out, int64_t *n_candidates,
                             int *n_returned) {
    if (int rc = validate_bmp(fwd_ms, L, N, "ob_bmp_search")) return rc;
    if (!activ || !cand_out || !score_out || !n_candidates || !n_returned)
        return fail(OB_EINVAL, "ob_bmp_search: null pointer");
    if (r < 0 || top_k < 1) return fail(OB_EINVAL, "ob_bmp_search: r must be >= 0 and top_k >= 1");
    const int C = N - 1;
    double total = 1.0;
    for (int i = 0; i < C; ++i) total *= 2 * r + 1;
    if (total > 2e7) return fail(OB_EUNSUPPORTED, "ob_bmp_search: (2r+1)^(N-1) = %.3g candidates is too many", total);
    std::vector<int> base(std::max(C, 1)), off(std::max(C, 1), -r), P(std::max(C, 1));
    anchor(fwd_ms, L, N, base.data());
    std::vector<double> cum(L + 1, 0.0);
    for (int j = 1; j <= L; ++j) cum[j] = cum[j - 1] + fwd_ms[j - 1];
    struct Cand { double score; std::vector<int> P; };
    std::vector<Cand> all;
    int64_t valid = 0;
    for (;;) {
        bool ok = true;
        int prev = 1;
        for (int i = 0; i < C; ++i) {
            P[i] = base[i] + off[i];
            if (P[i] <= prev || P[i] > L) { ok = false; break; }   // every stage keeps >= 1 layer
            prev = P[i];
        }
        if (ok) {
            ++valid;
            double var = 0.0, comm = 0.0;
            const double mean = cum[L] / N;
            int lo = 1;
            for (int i = 0; i < N; ++i) {
                const int hi = i < C ? P[i] : L + 1;
                const double t = cum[hi - 1] - cum[lo - 1];
                var += (t - mean) * (t - mean);
                if (i < C) comm += activ[hi - 2];  // last layer of stage i+1 is layer hi-1 (1-based)
                lo = hi;
            }
            all.push_back({var + comm_weight * comm, std::vector<int>(P.begin(), P.begin() + C)});
        }
        int i = C - 1;  // odometer over the offsets, last cut fastest
        while (i >= 0 && off[i] == r) off[i--] = -r;
        if (i < 0) break;
        ++off[i];
    }
    std::stable_sort(all.begin(), all.end(), [](const Cand &a, const Cand &b) {
        return a.score < b.score || (a.score == b.score && a.P < b.P);
    });
    const int n = (int)std::min<size_t>(all.size(), (size_t)top_k);
    for (int k = 0; k < n; ++k) {
        for (int i = 0; i < C; ++i) cand_out[(size_t)k * C + i] = all[k].P[i];
        score_out[k] = all[k].score;
    }
    *n_candidates = valid;
    *n_returned = n;
    return OB_OK;
}
