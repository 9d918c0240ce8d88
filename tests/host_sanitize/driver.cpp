// Host-only driver for the AddressSanitizer / UBSan build of the library's host code: the packer
// (Alg. 1 and the other grouping arms), the partition search and re-computation plan, and every
// validation path of the device entry points (which must return before anything is launched; the
// launchers are stubs that abort).  Exits 0 when every check holds.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/omnibal.h"

static int failures = 0;
#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) { std::fprintf(stderr, "%s:%d: CHECK(%s) failed: %s\n", __FILE__, __LINE__, #cond, ob_last_error()); ++failures; } \
    } while (0)

static uint64_t lcg(uint64_t &s) { s = s * 6364136223846793005ull + 1442695040888963407ull; return s >> 33; }

static void packer_cases() {
    for (int n : {1, 2, 7, 64, 1000, 5000}) {
        for (uint64_t seed : {0ull, 5ull}) {
            uint64_t st = 17 * n + seed;
            std::vector<int32_t> img(n), tok(n);
            for (int i = 0; i < n; ++i) { img[i] = 1 + lcg(st) % 12; tok[i] = 256 * img[i] + 1 + lcg(st) % 4096; }
            std::vector<int64_t> off(n + 1), ids(n), left(n), per_iter(10);
            int64_t ng = 0, nl = 0;
            int rc = ob_pack_isf(img.data(), tok.data(), n, 42, 16384, 42, 16384 - 128, 10, seed, off.data(), &ng,
                                 ids.data(), left.data(), &nl, per_iter.data());
            CHECK(rc == OB_OK);
            CHECK(ng >= 0 && ng <= n && nl >= 0 && off[ng] + nl == n);
            std::vector<char> seen(n, 0);
            for (int64_t g = 0; g < ng; ++g) {
                int64_t iv = 0, it = 0;
                CHECK(off[g] < off[g + 1]);
                for (int64_t p = off[g]; p < off[g + 1]; ++p) {
                    CHECK(ids[p] >= 0 && ids[p] < n && !seen[ids[p]]);
                    seen[ids[p]] = 1; iv += img[ids[p]]; it += tok[ids[p]];
                }
                CHECK(iv <= 42 && it <= 16384 && (iv >= 42 || it >= 16384 - 128));
            }
            for (int64_t p = 0; p < nl; ++p) { CHECK(!seen[left[p]]); seen[left[p]] = 1; }
            // groups_per_iter may be null
            rc = ob_pack_isf(img.data(), tok.data(), n, 42, 16384, 42, 16384 - 128, 3, seed, off.data(), &ng,
                             ids.data(), left.data(), &nl, nullptr);
            CHECK(rc == OB_OK);
            for (int64_t B : {1, 3, 8}) {
                CHECK(ob_pack_random(n, B, seed, off.data(), &ng, ids.data(), left.data(), &nl) == OB_OK);
                CHECK(ng == n / B && nl == n % B);
                CHECK(ob_pack_length_group(tok.data(), n, B, seed, off.data(), &ng, ids.data(), left.data(), &nl) == OB_OK);
                CHECK(ng == n / B && nl == n % B);
                CHECK(ob_pack_device_group(tok.data(), n, B, seed, off.data(), &ng, ids.data(), left.data(), &nl) == OB_OK);
                CHECK(ng == n / B && nl == n % B);
            }
            if (ng > 0) {
                std::vector<int32_t> cu(off[1] - off[0] + 1);
                int32_t mx = 0;
                CHECK(ob_build_cu_seqlens_llm(ids.data(), off[1] - off[0], tok.data(), cu.data(), &mx) == OB_OK);
                CHECK(cu[0] == 0 && mx > 0);
            }
        }
    }
    // a sample that alone exceeds a budget is an input error
    int32_t img1[2] = {1, 50}, tok1[2] = {300, 300};
    int64_t off[3], ids[2], left[2], ng, nl;
    CHECK(ob_pack_isf(img1, tok1, 2, 42, 16384, 42, 16000, 2, 0, off, &ng, ids, left, &nl, nullptr) == OB_EINVAL);
    CHECK(ob_pack_isf(nullptr, tok1, 2, 42, 16384, 42, 16000, 2, 0, off, &ng, ids, left, &nl, nullptr) == OB_EINVAL);
    CHECK(ob_pack_random(2, 0, 0, off, &ng, ids, left, &nl) == OB_EINVAL);
    int32_t cu[13];
    CHECK(ob_build_cu_seqlens_vit(12, 1025, cu) == OB_OK && cu[12] == 12300);
    CHECK(ob_build_cu_seqlens_vit(0, 1025, cu) != OB_OK);
    int64_t v[4] = {1, 2, 3, 6};
    CHECK(ob_pad_ratio(v, 4) == 0.5 && ob_dist_ratio(v, 1) == 0.0);
}

static void planner_cases() {
    std::vector<double> fwd(20, 1.0), act(20, 2.0);
    int P[3];
    CHECK(ob_bmp_anchor(fwd.data(), 20, 4, P) == OB_OK && P[0] == 6 && P[1] == 11 && P[2] == 16);
    std::vector<int> cand(30 * 3);
    std::vector<double> score(30);
    int64_t n_cand = 0;
    int n_ret = 0;
    CHECK(ob_bmp_search(fwd.data(), act.data(), 20, 4, 1, 0.5, 30, cand.data(), score.data(), &n_cand, &n_ret) == OB_OK);
    CHECK(n_cand == 27 && n_ret == 27);
    CHECK(ob_bmp_search(fwd.data(), act.data(), 20, 4, 2, 0.5, 5, cand.data(), score.data(), &n_cand, &n_ret) == OB_OK);
    CHECK(n_ret == 5 && n_cand <= 125);
    CHECK(ob_bmp_search(fwd.data(), act.data(), 20, 1, 1, 0.5, 5, cand.data(), score.data(), &n_cand, &n_ret) == OB_OK);
    CHECK(ob_bmp_anchor(fwd.data(), 3, 4, P) == OB_EINVAL);
    CHECK(ob_bmp_anchor(nullptr, 20, 4, P) == OB_EINVAL);
    uint64_t st = 9;
    for (int t = 0; t < 50; ++t) {
        const int L = 2 + lcg(st) % 40, N = 1 + lcg(st) % (L < 8 ? L : 8), r = lcg(st) % 3;
        std::vector<double> f(L), a(L);
        for (int i = 0; i < L; ++i) { f[i] = 0.5 + (lcg(st) % 100) / 10.0; a[i] = 1 + lcg(st) % 50; }
        std::vector<int> anchor(N > 1 ? N - 1 : 1), c(8 * (N > 1 ? N - 1 : 1));
        std::vector<double> sc(8);
        CHECK(ob_bmp_anchor(f.data(), L, N, anchor.data()) == OB_OK);
        CHECK(ob_bmp_search(f.data(), a.data(), L, N, r, 0.01, 8, c.data(), sc.data(), &n_cand, &n_ret) == OB_OK);
        CHECK(n_ret >= 1 && n_ret <= 8);
        for (int k = 1; k < n_ret; ++k) CHECK(sc[k - 1] <= sc[k]);
    }
    int kv = -1, kt = -1;
    CHECK(ob_recompute_plan(100, 4, 30, 1.0, 4, 20, 1.0, 0, &kv, &kt) == OB_OK && 30 * kv + 20 * kt <= 100);
    CHECK(ob_recompute_plan(100, 4, 30, 1.0, 4, 20, 1.0, 100, &kv, &kt) == OB_OK && kv == 0 && kt == 0);
    CHECK(ob_recompute_plan(-1, 4, 30, 1.0, 4, 20, 1.0, 0, &kv, &kt) == OB_EINVAL);
    CHECK(ob_recompute_plan(100, 4, 0, 1.0, 4, 20, 1.0, 0, &kv, &kt) == OB_EINVAL);
}

static void validation_cases() {
    void *p = (void *)0x1000;   // never dereferenced: validation fails first
    int32_t cu_ok[3] = {0, 5, 9}, cu_bad0[3] = {1, 5, 9}, cu_empty[4] = {0, 5, 5, 9};
    ob_segments good{cu_ok, (const int32_t *)p, 2, 9, 5};
    ob_segments bad0{cu_bad0, (const int32_t *)p, 2, 9, 5};
    ob_segments empty{cu_empty, (const int32_t *)p, 3, 9, 5};
    ob_segments total{cu_ok, (const int32_t *)p, 2, 10, 5};
    ob_segments shortmax{cu_ok, (const int32_t *)p, 2, 9, 3};
    ob_segments nodev{cu_ok, nullptr, 2, 9, 5};
    auto fwd = [&](const ob_segments *s, int nq, int nkv, int d, int ldq, int mask, int dtype, void *q) {
        return ob_varlen_attn_fwd(q, p, p, p, (float *)p, ldq, 128, 256, s, nq, nkv, d, 0.125f, mask, dtype, nullptr);
    };
    CHECK(fwd(&good, 4, 2, 64, 256, 1, 0, nullptr) == OB_EINVAL);
    CHECK(fwd(&bad0, 4, 2, 64, 256, 1, 0, p) == OB_ESEGMENTS);
    CHECK(fwd(&empty, 4, 2, 64, 256, 1, 0, p) == OB_ESEGMENTS);
    CHECK(fwd(&total, 4, 2, 64, 256, 1, 0, p) == OB_ESEGMENTS);
    CHECK(fwd(&shortmax, 4, 2, 64, 256, 1, 0, p) == OB_ESEGMENTS);
    CHECK(fwd(&nodev, 4, 2, 64, 256, 1, 0, p) == OB_EINVAL);
    CHECK(fwd(nullptr, 4, 2, 64, 256, 1, 0, p) == OB_EINVAL);
    CHECK(fwd(&good, 4, 3, 64, 256, 1, 0, p) == OB_EINVAL);
    CHECK(fwd(&good, 4, 2, 96, 256, 1, 0, p) == OB_EUNSUPPORTED);
    CHECK(fwd(&good, 4, 2, 64, 100, 1, 0, p) == OB_EINVAL);
    CHECK(fwd(&good, 4, 2, 64, 256, 7, 0, p) == OB_EINVAL);
    CHECK(fwd(&good, 4, 2, 64, 256, 1, 7, p) == OB_EINVAL);
    CHECK(ob_varlen_attn_bwd(p, p, p, p, p, (const float *)p, p, p, p, 256, 128, 256, &good, 4, 2, 64, 0.125f, 1, 0, p,
                             16, nullptr) == OB_EWORKSPACE);
    CHECK(ob_varlen_attn_bwd_workspace_bytes(9, 4, 2, 64) >= 2u * 9 * 4 * 4);
    CHECK(ob_varlen_attn_bwd_workspace_bytes(9, 4, 3, 64) == 0);

    ob_block_desc d{256, 4, 4, 64, 1024, OB_LAYERNORM, OB_GELU, OB_MASK_SEG_CAUSAL, OB_BF16, 0, 10000.f, 1e-5f, 1};
    const size_t sb = ob_block_saved_bytes(&d, 9), wb = ob_block_workspace_bytes(&d, 9);
    CHECK(sb > 0 && wb > 0);
    CHECK(ob_block_saved_offset(&d, 9, "qkv") != (size_t)-1 && ob_block_saved_offset(&d, 9, "nope") == (size_t)-1);
    ob_block_weights w{p, p, p, p, p, p, p, p, p, p, p, p};
    ob_block_grads g{p, p, p, p, p, p, p, p, p, p, p, p};
    CHECK(ob_block_fwd(&d, &w, nullptr, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    CHECK(ob_block_fwd(&d, &w, p, p, p, sb - 1, &good, p, wb, nullptr) == OB_EWORKSPACE);
    CHECK(ob_block_fwd(&d, &w, p, p, p, sb, &good, p, wb - 1, nullptr) == OB_EWORKSPACE);
    CHECK(ob_block_fwd(&d, &w, p, p, p, sb, &bad0, p, wb, nullptr) == OB_ESEGMENTS);
    CHECK(ob_block_fwd(&d, nullptr, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    ob_block_weights w_nobias = w;
    w_nobias.b_up = nullptr;
    CHECK(ob_block_fwd(&d, &w_nobias, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    ob_block_desc bad = d;
    bad.head_dim = 96;
    CHECK(ob_block_fwd(&bad, &w, p, p, p, sb, &good, p, wb, nullptr) == OB_EUNSUPPORTED);
    bad = d; bad.hidden = 100;
    CHECK(ob_block_saved_bytes(&bad, 9) == 0);
    bad = d; bad.n_kv_heads = 3;
    CHECK(ob_block_fwd(&bad, &w, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    bad = d; bad.use_rotary = 1; bad.rotary_base = 0.5f;
    CHECK(ob_block_fwd(&bad, &w, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    CHECK(ob_block_bwd(&d, &w, &g, 4, p, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);      // unknown flag
    CHECK(ob_block_bwd(&d, &w, nullptr, 0, p, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    ob_block_grads g_nobias = g;
    g_nobias.b_o = nullptr;
    CHECK(ob_block_bwd(&d, &w, &g_nobias, 0, p, p, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);
    CHECK(ob_block_bwd(&d, &w, &g, 0, p, nullptr, p, p, sb, &good, p, wb, nullptr) == OB_EINVAL);

    CHECK(ob_gemm_bf16(3, 64, 64, 64, p, p, p, nullptr, nullptr, nullptr, 0, nullptr) == OB_EINVAL);
    CHECK(ob_gemm_bf16(0, 64, 100, 64, p, p, p, nullptr, nullptr, nullptr, 0, nullptr) == OB_EUNSUPPORTED);
    CHECK(ob_gemm_bf16(0, 64, 64, 100, p, p, p, nullptr, nullptr, nullptr, 0, nullptr) == OB_EUNSUPPORTED);
    CHECK(ob_gemm_bf16(2, 100, 64, 64, p, p, p, nullptr, nullptr, nullptr, 0, nullptr) == OB_EUNSUPPORTED);
    CHECK(ob_gemm_bf16(0, 0, 64, 64, p, p, p, nullptr, nullptr, nullptr, 0, nullptr) == OB_EINVAL);
    CHECK(ob_gemm_bf16(0, 64, 64, 64, nullptr, p, p, nullptr, nullptr, nullptr, 0, nullptr) == OB_EINVAL);
    CHECK(ob_debug_materialize_mask(&good, 5, (uint8_t *)p, nullptr) == OB_EINVAL);
    CHECK(ob_debug_materialize_mask(&good, 0, nullptr, nullptr) == OB_EINVAL);

    ob_connector_desc cd{128, 256, 8, OB_BF16, 1e-5f};
    ob_connector_weights cw{p, p, p, p, p, p};
    int32_t rows_ok[32], rows_dup[32], rows_out[32];
    for (int i = 0; i < 32; ++i) { rows_ok[i] = i; rows_dup[i] = i / 2; rows_out[i] = 40 + i; }
    const size_t csb = ob_connector_saved_bytes(&cd, 2), cwb = ob_connector_workspace_bytes(&cd, 2);
    CHECK(csb > 0 && cwb > 0);
    CHECK(ob_connector_fwd(&cd, &cw, p, 2, rows_dup, (const int32_t *)p, p, 64, p, csb, p, cwb, nullptr) != OB_OK);
    CHECK(ob_connector_fwd(&cd, &cw, p, 2, rows_out, (const int32_t *)p, p, 64, p, csb, p, cwb, nullptr) != OB_OK);
    CHECK(ob_connector_fwd(&cd, &cw, p, 2, rows_ok, (const int32_t *)p, p, 64, p, csb - 1, p, cwb, nullptr) == OB_EWORKSPACE);
    CHECK(ob_connector_fwd(&cd, &cw, nullptr, 2, rows_ok, (const int32_t *)p, p, 64, p, csb, p, cwb, nullptr) == OB_EINVAL);
    ob_connector_desc cbad = cd;
    cbad.grid = 7;
    CHECK(ob_connector_saved_bytes(&cbad, 2) == 0);

    double ms[32]; int64_t n[32]; double wk[32];
    CHECK(ob_prof_end(ms, n, wk, 32) == OB_EINVAL);     // not profiling
    CHECK(ob_prof_begin(0) == OB_EINVAL);
    CHECK(ob_prof_num_classes() > 0 && ob_prof_class_name(0)[0] != 0 && ob_prof_class_name(-1)[0] == 0);
}

int main() {
    packer_cases();
    planner_cases();
    validation_cases();
    if (failures) { std::fprintf(stderr, "%d checks failed\n", failures); return 1; }
    std::puts("host sanitizer driver: all checks passed");
    return 0;
}
