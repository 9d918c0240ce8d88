// Host-side balanced dynamic mini-batch grouping (the paper's Alg. 1, "ISF") and its metrics
// (Eq. 1 PadRatio, Eq. 2 DistRatio).  Plain C++, no device involvement.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

#include "ob_internal.h"

namespace {

struct SplitMix64 {
    uint64_t s;
    explicit SplitMix64(uint64_t seed) : s(seed) {}
    uint64_t next() {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    // uniform in [0, n): draws in the top partial range [2^64 - 2^64 mod n, 2^64) are rejected
    uint64_t below(uint64_t n) {
        const uint64_t rem = (0 - n) % n;  // == 2^64 mod n
        for (;;) {
            const uint64_t r = next();
            if (rem == 0 || r < (uint64_t)0 - rem) return r % n;
        }
    }
};

// Fisher-Yates over `v` in place: i = n-1 .. 1, swap v[i] with v[j], j uniform in [0, i]
void shuffle(std::vector<int64_t> &v, uint64_t seed) {
    SplitMix64 rng(seed);
    for (int64_t i = (int64_t)v.size() - 1; i >= 1; --i) {
        const int64_t j = (int64_t)rng.below((uint64_t)i + 1);
        std::swap(v[i], v[j]);
    }
}

double spread_ratio(const int64_t *v, int64_t n) {
    if (!v || n <= 0) return -1.0;
    const int64_t mx = *std::max_element(v, v + n);
    if (mx <= 0) return -1.0;
    long double acc = 0;
    for (int64_t i = 0; i < n; ++i) acc += (long double)(mx - v[i]);
    return (double)(acc / ((long double)mx * (long double)n));
}

}  // namespace

extern "C" int ob_pack_isf(const int32_t *n_img, const int32_t *n_tok, int64_t n_samples,
                           int64_t Qv, int64_t Qt, int64_t Qv_min, int64_t Qt_min, int iters,
                           uint64_t seed, int64_t *group_offsets, int64_t *n_groups,
                           int64_t *sample_ids, int64_t *leftover_ids, int64_t *n_leftover,
                           int64_t *groups_per_iter) {
    if (!n_img || !n_tok || !group_offsets || !n_groups || !sample_ids || !leftover_ids ||
        !n_leftover)
        return ob::fail(OB_EINVAL, "ob_pack_isf: null pointer");
    if (n_samples < 0 || iters < 0 || Qv <= 0 || Qt <= 0)
        return ob::fail(OB_EINVAL, "ob_pack_isf: n_samples/iters must be >= 0, budgets > 0");
    for (int64_t i = 0; i < n_samples; ++i) {
        if (n_img[i] < 0 || n_tok[i] < 0)
            return ob::fail(OB_EINVAL, "ob_pack_isf: sample %lld has a negative size", (long long)i);
        if (n_img[i] > Qv || n_tok[i] > Qt)
            return ob::fail(OB_EINVAL, "ob_pack_isf: sample %lld alone exceeds a budget (%d tiles, %d tokens)",
                            (long long)i, n_img[i], n_tok[i]);
    }
    std::vector<int64_t> pool((size_t)n_samples);
    std::iota(pool.begin(), pool.end(), (int64_t)0);
    std::vector<char> taken((size_t)n_samples, 0);
    int64_t ng = 0, n_out = 0;
    group_offsets[0] = 0;
    for (int it = 0; it < iters; ++it) {
        if (groups_per_iter) groups_per_iter[it] = 0;
        if (pool.empty()) continue;
        std::vector<int64_t> order = pool;
        shuffle(order, seed + (uint64_t)it);
        // sampling + filtering fused per candidate: a candidate is complete when the next sample
        // would overflow either budget (or the walk ends); it is accepted iff it reaches Q'.
        size_t begin = 0;
        int64_t Iv = 0, It = 0;
        auto close = [&](size_t end) {
            if (end == begin) return;
            if (Iv >= Qv_min || It >= Qt_min) {
                for (size_t p = begin; p < end; ++p) {
                    sample_ids[n_out++] = order[p];
                    taken[(size_t)order[p]] = 1;
                }
                group_offsets[++ng] = n_out;
                if (groups_per_iter) groups_per_iter[it]++;
            }
        };
        for (size_t p = 0; p < order.size(); ++p) {
            const int64_t xi = n_img[order[p]], yi = n_tok[order[p]];
            if (p > begin && (Iv + xi > Qv || It + yi > Qt)) {
                close(p);
                begin = p;
                Iv = It = 0;
            }
            Iv += xi;
            It += yi;
        }
        close(order.size());
        std::vector<int64_t> rest;
        rest.reserve(pool.size());
        for (int64_t id : pool)
            if (!taken[(size_t)id]) rest.push_back(id);
        pool.swap(rest);
    }
    *n_groups = ng;
    *n_leftover = (int64_t)pool.size();
    std::copy(pool.begin(), pool.end(), leftover_ids);
    return OB_OK;
}

extern "C" int ob_pack_random(int64_t n_samples, int64_t B, uint64_t seed, int64_t *group_offsets,
                              int64_t *n_groups, int64_t *sample_ids, int64_t *leftover_ids,
                              int64_t *n_leftover) {
    if (!group_offsets || !n_groups || !sample_ids || !leftover_ids || !n_leftover)
        return ob::fail(OB_EINVAL, "ob_pack_random: null pointer");
    if (n_samples < 0 || B <= 0) return ob::fail(OB_EINVAL, "ob_pack_random: bad n_samples or B");
    std::vector<int64_t> perm((size_t)n_samples);
    std::iota(perm.begin(), perm.end(), (int64_t)0);
    shuffle(perm, seed);
    const int64_t full = n_samples / B;
    group_offsets[0] = 0;
    for (int64_t g = 0; g < full; ++g) {
        for (int64_t p = 0; p < B; ++p) sample_ids[g * B + p] = perm[(size_t)(g * B + p)];
        group_offsets[g + 1] = (g + 1) * B;
    }
    *n_groups = full;
    std::vector<int64_t> rest(perm.begin() + (size_t)(full * B), perm.end());
    std::sort(rest.begin(), rest.end());
    std::copy(rest.begin(), rest.end(), leftover_ids);
    *n_leftover = (int64_t)rest.size();
    return OB_OK;
}

// Sec. 5.4, method 2 ("Length-Group"): samples of similar size share a mini-batch.  Reading: sort
// by token count (ties by id), cut into consecutive runs of B, then shuffle the order of the
// mini-batches so that the ones a step hands to its devices are unrelated in size.
extern "C" int ob_pack_length_group(const int32_t *n_tok, int64_t n_samples, int64_t B, uint64_t seed,
                                    int64_t *group_offsets, int64_t *n_groups, int64_t *sample_ids,
                                    int64_t *leftover_ids, int64_t *n_leftover) {
    if (!n_tok || !group_offsets || !n_groups || !sample_ids || !leftover_ids || !n_leftover)
        return ob::fail(OB_EINVAL, "ob_pack_length_group: null pointer");
    if (n_samples < 0 || B <= 0) return ob::fail(OB_EINVAL, "ob_pack_length_group: bad n_samples or B");
    std::vector<int64_t> order((size_t)n_samples);
    std::iota(order.begin(), order.end(), (int64_t)0);
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return n_tok[a] < n_tok[b]; });
    const int64_t full = n_samples / B;
    std::vector<int64_t> batch((size_t)full);
    std::iota(batch.begin(), batch.end(), (int64_t)0);
    shuffle(batch, seed);
    group_offsets[0] = 0;
    for (int64_t g = 0; g < full; ++g) {
        for (int64_t p = 0; p < B; ++p) sample_ids[g * B + p] = order[(size_t)(batch[(size_t)g] * B + p)];
        group_offsets[g + 1] = (g + 1) * B;
    }
    *n_groups = full;
    std::vector<int64_t> rest(order.begin() + (size_t)(full * B), order.end());
    std::sort(rest.begin(), rest.end());
    std::copy(rest.begin(), rest.end(), leftover_ids);
    *n_leftover = (int64_t)rest.size();
    return OB_OK;
}

// Sec. 5.4, method 3 ("Device-Group"): the mini-batches one step hands to its devices are of
// similar size.  Reading: the random arm's mini-batches, ordered by their token totals (ties keep
// the random order), so that any run of consecutive mini-batches is close in size.
extern "C" int ob_pack_device_group(const int32_t *n_tok, int64_t n_samples, int64_t B, uint64_t seed,
                                    int64_t *group_offsets, int64_t *n_groups, int64_t *sample_ids,
                                    int64_t *leftover_ids, int64_t *n_leftover) {
    if (!n_tok) return ob::fail(OB_EINVAL, "ob_pack_device_group: null pointer");
    if (int rc = ob_pack_random(n_samples, B, seed, group_offsets, n_groups, sample_ids, leftover_ids, n_leftover))
        return rc;
    const int64_t full = *n_groups;
    std::vector<int64_t> total((size_t)full, 0), idx((size_t)full);
    for (int64_t g = 0; g < full; ++g)
        for (int64_t p = 0; p < B; ++p) total[(size_t)g] += n_tok[sample_ids[g * B + p]];
    std::iota(idx.begin(), idx.end(), (int64_t)0);
    std::stable_sort(idx.begin(), idx.end(), [&](int64_t a, int64_t b) { return total[(size_t)a] < total[(size_t)b]; });
    std::vector<int64_t> out((size_t)(full * B));
    for (int64_t g = 0; g < full; ++g)
        for (int64_t p = 0; p < B; ++p) out[(size_t)(g * B + p)] = sample_ids[idx[(size_t)g] * B + p];
    std::copy(out.begin(), out.end(), sample_ids);
    return OB_OK;
}

extern "C" int ob_build_cu_seqlens_llm(const int64_t *group_ids, int64_t n, const int32_t *n_tok,
                                       int32_t *cu_out, int32_t *max_seqlen_out) {
    if (!group_ids || !n_tok || !cu_out) return ob::fail(OB_EINVAL, "ob_build_cu_seqlens_llm: null pointer");
    if (n <= 0) return ob::fail(OB_EINVAL, "ob_build_cu_seqlens_llm: empty group");
    int64_t acc = 0;
    int32_t mx = 0;
    cu_out[0] = 0;
    for (int64_t p = 0; p < n; ++p) {
        const int32_t len = n_tok[group_ids[p]];
        if (len <= 0) return ob::fail(OB_ESEGMENTS, "ob_build_cu_seqlens_llm: sample %lld has no tokens",
                                      (long long)group_ids[p]);
        acc += len;
        if (acc > INT32_MAX) return ob::fail(OB_ESEGMENTS, "ob_build_cu_seqlens_llm: total exceeds int32");
        mx = std::max(mx, len);
        cu_out[p + 1] = (int32_t)acc;
    }
    if (max_seqlen_out) *max_seqlen_out = mx;
    return OB_OK;
}

extern "C" int ob_build_cu_seqlens_vit(int64_t n_tiles, int32_t tile_len, int32_t *cu_out) {
    if (!cu_out) return ob::fail(OB_EINVAL, "ob_build_cu_seqlens_vit: null pointer");
    if (n_tiles <= 0 || tile_len <= 0 || n_tiles * (int64_t)tile_len > INT32_MAX)
        return ob::fail(OB_EINVAL, "ob_build_cu_seqlens_vit: bad tile count or length");
    for (int64_t j = 0; j <= n_tiles; ++j) cu_out[j] = (int32_t)(j * tile_len);
    return OB_OK;
}

extern "C" double ob_pad_ratio(const int64_t *tokens_per_sample, int64_t n) {
    return spread_ratio(tokens_per_sample, n);
}
extern "C" double ob_dist_ratio(const int64_t *tokens_per_minibatch, int64_t n) {
    return spread_ratio(tokens_per_minibatch, n);
}
