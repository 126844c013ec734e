// Sanitizer run of the CPU oracle.  TEST INFRASTRUCTURE ONLY.
//
// Built by tests/test_oracle_sanitized.py with -fsanitize=address,undefined and run as a program of its own: it
// drives every function of s3_oracle.cpp over the hand-computed case of tests/golden/tiny_case.json (values typed
// in below) and over random shapes with ragged sizes, so that an out-of-bounds access, a use after free, a signed
// overflow or a misaligned access in the oracle ends the run with a report instead of a silently wrong expectation.
#include "s3_oracle.cpp"

#include <cstdio>
#include <cstdlib>
#include <random>

#define CHECK(c)                                                          \
    do {                                                                  \
        if (!(c)) {                                                       \
            std::fprintf(stderr, "sanitize_check: %s failed (line %d)\n", #c, __LINE__); \
            return 1;                                                     \
        }                                                                 \
    } while (0)

static int hand_case() {
    // 6 tokens, d_head 2, 8 features, k 2 (Sec. 3.3 - 3.5 worked by hand)
    const float w[16] = {1, 0, 0, 1, -1, 0, 0, -1, 1, 1, 1, -1, -1, 1, -1, -1};
    const float b[8] = {0, 0, 0, 0.5f, 0, 0, 0, 0};
    const float x[12] = {2, 1, 1, 2, -1, -1, 1, -1, 1, 1, 0, 0};
    const int32_t want_ids[12] = {4, 0, 4, 1, 7, 3, 5, 3, 4, 0, 3, 0};
    const float want_vals[12] = {3, 2, 3, 2, 2, 1.5f, 2, 1.5f, 2, 1, 0.5f, 0};
    int32_t ids[12];
    float vals[12];
    double zsel[12], gap[6], z[48];
    CHECK(orc_encode_topk(x, 1, 6, 2, w, b, 8, 2, ids, vals, zsel, gap, z) == 0);
    for (int i = 0; i < 12; ++i) CHECK(ids[i] == want_ids[i] && vals[i] == want_vals[i]);
    double zat[12];
    CHECK(orc_preact_at(x, 1, 6, 2, w, b, 8, ids, 2, zat) == 0);
    for (int i = 0; i < 12; ++i) CHECK(zat[i] == zsel[i]);
    const int32_t pos[6] = {0, 1, 2, 3, 4, 5};
    void* ix = orc_index_new();
    CHECK(orc_index_append(ix, ids, pos, 6, 2) == 0 && orc_index_postings(ix) == 12);
    int32_t off[9], csr[12];
    const int32_t want_off[9] = {0, 3, 4, 4, 7, 10, 11, 11, 12};
    const int32_t want_csr[12] = {0, 4, 5, 1, 2, 3, 5, 0, 1, 4, 3, 2};
    CHECK(orc_index_export(ix, 8, off, csr) == 0);
    for (int i = 0; i < 9; ++i) CHECK(off[i] == want_off[i]);
    for (int i = 0; i < 12; ++i) CHECK(csr[i] == want_csr[i]);
    const int32_t qids[2] = {4, 0};
    const float qvals[2] = {3, 2};
    double S[6] = {0, 0, 0, 0, 0, 0};
    CHECK(orc_score_accumulate(ix, qids, qvals, 1, 2, 0, S, 6) == 0);
    const double idf3 = orc_idf(3), want_S[6] = {5, 3, 0, 0, 5, 2};
    for (int i = 0; i < 6; ++i) CHECK(std::fabs(S[i] - want_S[i] * idf3) < 1e-15);
    double W[5];
    CHECK(orc_pool(S, 6, 2, W) == 5);
    int32_t st[3];
    double sc[3];
    CHECK(orc_topb(W, 5, 2, 3, 1, st, sc) == 3 && st[0] == 0 && st[1] == 4 && st[2] == 2);
    orc_index_free(ix);
    return 0;
}

static int random_shapes() {
    std::mt19937 rng(7);
    std::normal_distribution<float> nd;
    const int shapes[4][4] = {{1, 1, 1, 1}, {37, 8, 50, 7}, {130, 64, 129, 64}, {5, 3, 9, 9}};   // T, d, n_feat, k
    for (auto& sh : shapes) {
        const int T = sh[0], d = sh[1], n_feat = sh[2], k = sh[3];
        std::vector<uint16_t> x((size_t)T * d), w((size_t)n_feat * d);
        std::vector<float> b(n_feat);
        auto bf16 = [&](float f) { uint32_t u; std::memcpy(&u, &f, 4); return (uint16_t)(u >> 16); };
        for (auto& v : x) v = bf16(nd(rng));
        for (auto& v : w) v = bf16(nd(rng));
        for (auto& v : b) v = nd(rng);
        std::vector<int32_t> ids((size_t)T * k), pos(T);
        std::vector<float> vals((size_t)T * k);
        std::vector<double> gap(T);
        CHECK(orc_encode_topk(x.data(), 0, T, d, w.data(), b.data(), n_feat, k, ids.data(), vals.data(), nullptr,
                              gap.data(), nullptr) == 0);
        for (int t = 0; t < T; ++t) pos[t] = 3 * t + 1;
        void* ix = orc_index_new();
        CHECK(orc_index_append(ix, ids.data(), pos.data(), T, k) == 0);
        std::vector<int32_t> off(n_feat + 1), csr((size_t)T * k);
        CHECK(orc_index_export(ix, n_feat, off.data(), csr.data()) == 0 && off[n_feat] == T * k);
        const int64_t L = 3 * (int64_t)T + 2;
        std::vector<double> S(L, 0.0), W(L);
        CHECK(orc_score_accumulate(ix, ids.data(), vals.data(), T, k, 5, S.data(), L) == 0);
        for (int len : {1, 4, (int)L, (int)L + 10}) {
            const int64_t nw = orc_pool(S.data(), L, len, W.data());
            CHECK(nw == L - std::min<int64_t>(len, L) + 1);
            std::vector<int32_t> st(nw + 2);
            std::vector<double> sc(nw + 2);
            const int found = orc_topb(W.data(), nw, len, (int)nw + 2, 1, st.data(), sc.data());
            CHECK(found >= 1 && found <= nw);
        }
        // Phase-2 tail and Phase-3 set operations on the same scores
        for (int K : {1, 8, 48}) {
            std::vector<double> g(K), D(L);
            CHECK(orc_smoothing_kernel(K % 3, K, g.data()) == 0);
            CHECK(orc_conv1d(S.data(), L, g.data(), K, D.data()) == 0);
            std::vector<int32_t> c(40), lo(40), hi(40);
            std::vector<double> pk(40);
            const int n = orc_nms_peaks(D.data(), L, 40, K / 2, c.data(), pk.data());
            for (int i = 0; i < n; ++i) orc_grow_span(D.data(), L, c[i], 0.5, 24, &lo[i], &hi[i]);
            std::vector<unsigned char> mask(L);
            std::vector<int32_t> idx(L);
            const int32_t extra[3] = {-1, 0, (int32_t)L + 4};
            const int64_t m = orc_fuse(L, lo.data(), hi.data(), n, extra, 3, 4, 4, mask.data(), idx.data());
            CHECK(m >= 1 && m <= L);
        }
        orc_index_free(ix);
    }
    return 0;
}

int main() {
    if (hand_case() || random_shapes()) return 1;
    std::puts("sanitize_check ok");
    return 0;
}
