// Host-side plan builder and permutation search under AddressSanitizer and
// UndefinedBehaviorSanitizer (built and run by tests/test_host_sanitizers.py
// with g++; no GPU, no HIP).  Exercises ragged shapes, all three layouts, both
// weight types, both weight spaces, empty block rows, every error path, and
// the feed-back search, and checks the structural invariants of each plan.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <numeric>
#include <random>
#include <vector>

#include "pivot_internal.h"

namespace pivot {
// the device-side launcher is not part of this build: one slice, always
int fc_row_slices(const FcShape&, int, int) { return 1; }
const char* last_error();
}

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); std::exit(1); } } while (0)

static std::vector<int32_t> random_perm(int n, std::mt19937& rng) {
    std::vector<int32_t> p(n);
    std::iota(p.begin(), p.end(), 0);
    std::shuffle(p.begin(), p.end(), rng);
    return p;
}

static void one_plan(int M, int K, int bh, int bw, int wdtype, int layout, int w_space, int chunk_tiles, bool with_bias,
                     double keep, std::mt19937& rng) {
    const int nbr = (M + bh - 1) / bh, nbc = (K + bw - 1) / bw;
    std::vector<uint8_t> mask((size_t)nbr * nbc);
    std::bernoulli_distribution coin(keep);
    for (auto& m : mask) m = coin(rng) ? 1 : 0;
    if (nbr > 2) for (int j = 0; j < nbc; ++j) mask[(size_t)1 * nbc + j] = 0;      // an empty block row
    const size_t es = wdtype == PIVOT_F32 ? 4 : 2;
    std::vector<uint8_t> W((size_t)M * K * es);
    for (auto& b : W) b = (uint8_t)(rng() & 0x3F);
    auto prow = random_perm(M, rng), pcol = random_perm(K, rng);
    std::vector<float> bias(M, 0.5f);
    pivot_fc_desc d{};
    d.M = M; d.K = K; d.bh = bh; d.bw = bw; d.wdtype = wdtype; d.layout = layout; d.act = PIVOT_ACT_RELU;
    d.chunk_tiles = chunk_tiles; d.device = -1;
    pivot::HostPlan hp;
    const int rc = pivot::build_host_plan(d, W.data(), w_space, mask.data(), prow.data(), pcol.data(),
                                          with_bias ? bias.data() : nullptr, hp);
    REQUIRE(rc == PIVOT_OK);
    size_t T = 0;
    for (auto m : mask) T += m;
    REQUIRE((size_t)hp.T == T && hp.row_ptr.size() == (size_t)nbr + 1 && hp.row_ptr.back() == hp.T);
    REQUIRE(hp.vals.size() == T * bh * bw * es && hp.xidx.size() == T * bw);
    std::vector<int> covered(hp.T, 0);
    for (int c = 0; c < hp.nchunks; ++c) {
        const int32_t* q = &hp.chunks[4 * c];
        REQUIRE(q[0] >= 0 && q[0] < nbr && q[1] >= hp.row_ptr[q[0]] && q[2] <= hp.row_ptr[q[0] + 1] && q[2] - q[1] <= hp.chunk_tiles);
        for (int t = q[1]; t < q[2]; ++t) covered[t]++;
    }
    for (int t = 0; t < hp.T; ++t) REQUIRE(covered[t] == 1);
    for (int r = 0; r < M; ++r) REQUIRE(hp.invprow[prow[r]] == r);
    for (int c = 0; c < K; ++c) REQUIRE(hp.invpcol[pcol[c]] == c);
    for (size_t i = 0; i < hp.xidx.size(); ++i) REQUIRE(hp.xidx[i] >= -1 && hp.xidx[i] < K);
}

int main() {
    std::mt19937 rng(12345);
    const int shapes[][4] = {{37, 53, 8, 8}, {64, 64, 16, 16}, {100, 33, 32, 16}, {5, 7, 8, 64}, {129, 257, 64, 32}, {1, 1, 8, 8}};
    int n = 0;
    for (auto& s : shapes)
        for (int wd : {PIVOT_F32, PIVOT_F16})
            for (int layout : {PIVOT_BRC, PIVOT_BCR, PIVOT_CBR})
                for (int ws : {PIVOT_W_NATURAL, PIVOT_W_PIVOTED})
                    for (int ct : {0, 1, 3}) {
                        one_plan(s[0], s[1], s[2], s[3], wd, layout, ws, ct, (n & 1) != 0, n % 3 == 0 ? 1.0 : 0.4, rng);
                        ++n;
                    }
    // error paths: nothing may be read out of bounds, nothing leaked
    {
        pivot_fc_desc d{};
        d.M = 8; d.K = 8; d.bh = 8; d.bw = 8; d.wdtype = PIVOT_F32; d.layout = PIVOT_BRC; d.device = -1;
        std::vector<float> W(64, 1.f);
        uint8_t mask[1] = {1};
        std::vector<int32_t> id(8), bad(8);
        std::iota(id.begin(), id.end(), 0);
        bad = id; bad[3] = 2;
        pivot::HostPlan hp;
        REQUIRE(pivot::build_host_plan(d, W.data(), PIVOT_W_PIVOTED, mask, bad.data(), id.data(), nullptr, hp) == PIVOT_E_NOT_PERMUTATION);
        bad = id; bad[0] = 8;
        REQUIRE(pivot::build_host_plan(d, W.data(), PIVOT_W_PIVOTED, mask, id.data(), bad.data(), nullptr, hp) == PIVOT_E_NOT_PERMUTATION);
        bad[0] = -1;
        REQUIRE(pivot::build_host_plan(d, W.data(), PIVOT_W_PIVOTED, mask, id.data(), bad.data(), nullptr, hp) == PIVOT_E_NOT_PERMUTATION);
        REQUIRE(pivot::build_host_plan(d, nullptr, PIVOT_W_PIVOTED, mask, id.data(), id.data(), nullptr, hp) == PIVOT_E_NULL);
        d.layout = 7;
        REQUIRE(pivot::build_host_plan(d, W.data(), PIVOT_W_PIVOTED, mask, id.data(), id.data(), nullptr, hp) == PIVOT_E_UNSUPPORTED);
        REQUIRE(std::strlen(pivot::last_error()) > 0);
    }
    // feed-back search: ragged sizes, more levels than the matrix can be halved, bad starts
    for (auto mk : {std::pair<int, int>{1, 1}, {5, 3}, {37, 53}, {64, 48}}) {
        const int M = mk.first, K = mk.second;
        std::vector<float> A((size_t)M * K);
        std::uniform_real_distribution<float> u(0.f, 1.f);
        for (auto& v : A) v = u(rng);
        auto p0 = random_perm(M, rng), c0 = random_perm(K, rng);
        std::vector<int32_t> po(M), co(K);
        double mass = -1.0;
        for (int levels : {0, 1, 3, 20}) {
            REQUIRE(pivot_feedback_search(A.data(), M, K, levels, 50, p0.data(), c0.data(), po.data(), co.data(), &mass) == PIVOT_OK);
            std::vector<int> seen(M, 0);
            for (int r = 0; r < M; ++r) { REQUIRE(po[r] >= 0 && po[r] < M); seen[po[r]]++; }
            for (int r = 0; r < M; ++r) REQUIRE(seen[r] == 1);
            REQUIRE(mass >= 0.0);
        }
        if (M > 1) {
            auto bad = p0; bad[0] = bad[1];
            REQUIRE(pivot_feedback_search(A.data(), M, K, 1, 50, bad.data(), c0.data(), po.data(), co.data(), nullptr) == PIVOT_E_NOT_PERMUTATION);
        }
        REQUIRE(pivot_feedback_search(A.data(), M, K, 21, 50, p0.data(), c0.data(), po.data(), co.data(), nullptr) == PIVOT_E_SHAPE);
    }
    std::printf("host sanitizer run: %d plans built, all checks passed\n", n);
    return 0;
}
