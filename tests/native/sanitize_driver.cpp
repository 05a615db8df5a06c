// Sanitizer pass over the CPU oracle: built by tests/test_sanitize_oracle.py together with
// oracle/fsa_oracle.cpp under -fsanitize=address,undefined.  Every buffer is a heap array of
// exactly the size the oracle's header states, so any read or write past an end, any signed
// overflow or misaligned access inside the oracle aborts the run.  Cases: both indptr widths,
// the three table types, fanouts 1..64, rows of degree 0, below, at and far above the fanout,
// empty batches, saved-ID arrays with holes, all optional outputs present and absent.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../oracle/fsa_oracle.h"

static uint64_t state = 0x243F6A8885A308D3ull;
static uint32_t rnd() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(state >> 33); }
static double rndf() { return (double)rnd() / 2147483648.0 - 0.5; }

template <typename T> struct Exact {               // heap array of exactly n elements (never nullptr-by-accident)
    T* p; size_t n;
    explicit Exact(size_t n_) : p((T*)std::malloc(n_ ? n_ * sizeof(T) : 1)), n(n_) { std::memset(p, 0, n_ ? n_ * sizeof(T) : 1); }
    ~Exact() { std::free(p); }
    Exact(const Exact&) = delete;
};

#define REQUIRE(cond) do { if (!(cond)) { std::printf("FAILED %s at line %d (case %d)\n", #cond, __LINE__, case_no); return 1; } } while (0)

int main() {
    int case_no = 0;
    // generator and helpers
    {
        const uint32_t ctr[4] = {0, 0, 0, 0}, key[2] = {0, 0};
        uint32_t out[4];
        orc_philox4x32_10(ctr, key, out);
        REQUIRE(out[0] == 0x6627e8d5u);
        for (uint32_t n : {1u, 2u, 7u, 0x7fffffffu, 0xffffffffu}) REQUIRE(orc_draw(123, 5, 1, 3, n) < n);
        const double v[3] = {1.0, -2.5, 1e-40};
        uint16_t b16[3]; float f32[3];
        orc_round_to_bf16(v, 3, b16);
        orc_round_to_f32(v, 3, f32);
    }
    for (case_no = 1; case_no <= 60; ++case_no) {
        const int wide = case_no & 1, xdt = case_no % 3;
        const int64_t n = 40 + rnd() % 200;
        const int64_t D = 1 + rnd() % 9;
        const int k1 = case_no <= 6 ? (case_no <= 3 ? 1 : 64) : 1 + rnd() % 20;
        const int k2 = case_no <= 6 ? (case_no % 3 == 0 ? 64 : 1 + rnd() % 5) : 1 + rnd() % 12;
        const int k3 = 1 + rnd() % 4;
        const int64_t B = case_no == 7 ? 0 : 1 + rnd() % 30;
        // degrees: zeros, short rows, rows at the fanouts, one hub
        std::vector<int64_t> deg(n);
        for (int64_t i = 0; i < n; ++i) {
            const uint32_t r = rnd() % 10;
            deg[i] = r < 2 ? 0 : r < 6 ? rnd() % (k1 + 2) : rnd() % 40;
        }
        deg[0] = 0; deg[1] = k1; deg[2] = k1 + 1; deg[3] = 700; deg[4] = k2; deg[5] = 1;
        int64_t E = 0;
        for (int64_t d : deg) E += d;
        Exact<int32_t> ip32(n + 1); Exact<int64_t> ip64(n + 1);
        { int64_t a = 0; for (int64_t i = 0; i <= n; ++i) { ip32.p[i] = (int32_t)a; ip64.p[i] = a; if (i < n) a += deg[i]; } }
        Exact<int32_t> indices(E); Exact<float> ew(E);
        for (int64_t e = 0; e < E; ++e) { indices.p[e] = (int32_t)(rnd() % n); ew.p[e] = rnd() % 5 == 0 ? 0.0f : (float)(rnd() % 1000) / 1000.0f; }
        const void* indptr = wide ? (const void*)ip64.p : (const void*)ip32.p;
        Exact<float> xf(n * D); Exact<uint16_t> xb(n * D); Exact<double> xd(n * D);
        for (int64_t i = 0; i < n * D; ++i) { const double v = rndf(); xf.p[i] = (float)v; xd.p[i] = v; uint32_t u; float f = (float)v; std::memcpy(&u, &f, 4); xb.p[i] = (uint16_t)(u >> 16); }
        const void* x = xdt == ORC_X_F32 ? (const void*)xf.p : xdt == ORC_X_BF16 ? (const void*)xb.p : (const void*)xd.p;
        Exact<int32_t> seeds(B);
        for (int64_t b = 0; b < B; ++b) seeds.p[b] = b < 6 ? (int32_t)b : (int32_t)(rnd() % n);
        const int32_t fan[3] = {k1, k2, k3};

        // single rows
        { Exact<int64_t> pos(k1); Exact<int32_t> ids(k1);
          for (int64_t v = 0; v < 6; ++v) {
              const int32_t c = orc_sample_row(indptr, wide, indices.p, v, 0, k1, 77, pos.p, ids.p);
              REQUIRE(c == (deg[v] < k1 ? deg[v] : k1));
              for (int i = 0; i < c; ++i) REQUIRE(pos.p[i] >= 0 && pos.p[i] < deg[v]);
              REQUIRE(orc_sample_row(indptr, wide, indices.p, v, 1, k1, 77, nullptr, nullptr) == c);
          } }
        // 1-hop
        Exact<double> out(B * D); Exact<int32_t> ids1(B * k1);
        REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 1, 9, out.p, nullptr, ids1.p, nullptr) == 0);
        REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 1, 9, out.p, nullptr, nullptr, nullptr) == 0);
        REQUIRE(orc_mean_replay_fwd(x, xdt, D, n, ids1.p, nullptr, B, k1, 0, out.p, nullptr) == 0);
        Exact<double> g(B * D), gx(n * D);
        for (int64_t i = 0; i < B * D; ++i) g.p[i] = rndf();
        REQUIRE(orc_mean_bwd(g.p, nullptr, ids1.p, nullptr, B, k1, 0, D, gx.p, n) == 0);
        // 2-hop, all outputs, then none of the optional ones
        Exact<double> h1(B * k1 * D); Exact<int32_t> ids2(B * k1 * k2);
        REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 2, 9, out.p, h1.p, ids1.p, ids2.p) == 0);
        REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 2, 9, out.p, nullptr, nullptr, nullptr) == 0);
        for (int64_t i = 0; i < B * k1 * k2; ++i) REQUIRE(ids2.p[i] >= -1 && ids2.p[i] < n);
        // holes anywhere in the saved arrays
        for (int64_t i = 0; i < B * k1 * k2; ++i) if (rnd() % 7 == 0) ids2.p[i] = -1;
        for (int64_t i = 0; i < B * k1; ++i) if (rnd() % 9 == 0) ids1.p[i] = -1;
        REQUIRE(orc_mean_replay_fwd(x, xdt, D, n, ids1.p, ids2.p, B, k1, k2, out.p, h1.p) == 0);
        REQUIRE(orc_mean_replay_fwd(x, xdt, D, n, ids1.p, ids2.p, B, k1, k2, out.p, nullptr) == 0);
        Exact<double> gh(B * k1 * D);
        for (int64_t i = 0; i < B * k1 * D; ++i) gh.p[i] = rndf();
        REQUIRE(orc_mean_bwd(g.p, gh.p, ids1.p, ids2.p, B, k1, k2, D, gx.p, n) == 0);
        REQUIRE(orc_mean_bwd(g.p, nullptr, ids1.p, ids2.p, B, k1, k2, D, gx.p, n) == 0);
        // weighted
        Exact<float> w1(B * k1), w2(B * k1 * k2);
        REQUIRE(orc_sample_wmean_fwd(indptr, wide, indices.p, ew.p, n, x, xdt, D, seeds.p, B, fan, 1, 9, out.p, nullptr, ids1.p, nullptr, w1.p, nullptr) == 0);
        REQUIRE(orc_wmean_replay_fwd(x, xdt, D, n, ids1.p, nullptr, w1.p, nullptr, B, k1, 0, out.p, nullptr) == 0);
        REQUIRE(orc_wmean_bwd(g.p, nullptr, ids1.p, nullptr, w1.p, nullptr, B, k1, 0, D, gx.p, n) == 0);
        REQUIRE(orc_sample_wmean_fwd(indptr, wide, indices.p, ew.p, n, x, xdt, D, seeds.p, B, fan, 2, 9, out.p, h1.p, ids1.p, ids2.p, w1.p, w2.p) == 0);
        REQUIRE(orc_wmean_replay_fwd(x, xdt, D, n, ids1.p, ids2.p, w1.p, w2.p, B, k1, k2, out.p, h1.p) == 0);
        REQUIRE(orc_wmean_bwd(g.p, gh.p, ids1.p, ids2.p, w1.p, w2.p, B, k1, k2, D, gx.p, n) == 0);
        // three hops (smaller fanouts keep the pure loops short)
        if (k1 <= 20) {
            Exact<double> h2(B * k1 * k2 * D), m1(B * D);
            Exact<int32_t> ids3(B * k1 * k2 * k3), cnt2(B * k1);
            REQUIRE(orc_sample_mean3_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 9, out.p, h1.p, h2.p, m1.p, ids1.p, ids2.p, ids3.p, cnt2.p) == 0);
            REQUIRE(orc_sample_mean3_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 9, out.p, nullptr, nullptr, nullptr, ids1.p, ids2.p, ids3.p, nullptr) == 0);
            for (int64_t i = 0; i < B * k1 * k2 * k3; ++i) if (rnd() % 11 == 0) ids3.p[i] = -1;
            REQUIRE(orc_mean3_replay_fwd(x, xdt, D, n, ids1.p, ids2.p, ids3.p, B, k1, k2, k3, out.p, h1.p, h2.p, m1.p, cnt2.p) == 0);
            REQUIRE(orc_mean3_replay_fwd(x, xdt, D, n, ids1.p, ids2.p, ids3.p, B, k1, k2, k3, out.p, nullptr, nullptr, nullptr, nullptr) == 0);
            Exact<double> gh2(B * k1 * k2 * D);
            REQUIRE(orc_mean3_bwd(g.p, gh.p, gh2.p, g.p, ids1.p, ids2.p, ids3.p, B, k1, k2, k3, D, gx.p, n) == 0);
            REQUIRE(orc_mean3_bwd(g.p, nullptr, nullptr, nullptr, ids1.p, ids2.p, ids3.p, B, k1, k2, k3, D, gx.p, n) == 0);
        }
        // bad arguments are refused, not acted on
        REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 3, 9, out.p, nullptr, nullptr, nullptr) < 0);
        REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, 0, x, xdt, D, seeds.p, B, fan, 1, 9, out.p, nullptr, nullptr, nullptr) < 0);
        if (B > 0) {
            seeds.p[B - 1] = (int32_t)n;                     // a seed outside the graph
            REQUIRE(orc_sample_mean_fwd(indptr, wide, indices.p, n, x, xdt, D, seeds.p, B, fan, 1, 9, out.p, nullptr, nullptr, nullptr) < 0);
        }
    }
    std::printf("ok %d cases\n", case_no - 1);
    return 0;
}
