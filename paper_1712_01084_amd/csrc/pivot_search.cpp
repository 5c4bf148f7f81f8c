// Feed-back PBP pruning (paper Section 3.2): given the magnitudes of a trained
// dense layer, pick row and column permutations that keep as much magnitude
// as possible inside a block-diagonal pattern, by recursive bisection.  Each
// level splits every block's rows and columns in halves so as to maximise the
// mass in the upper-left and lower-right sub-blocks (the off-diagonal
// sub-blocks are what pruning deletes: every level halves the fill-in), with a
// greedy alternating search started from the permutations handed in (the
// paper starts from random ones; the caller draws them).
//
// One level, for one block with row list R and column list C (current order):
//   halves R1|R2 and C1|C2 = first/second half of the lists (sizes floor, rest);
//   repeat (at most max_iter times, or until nothing moves):
//     rows:    gain(r) = mass(r, C1) - mass(r, C2); R1 := the |R1| rows of
//              largest gain (ties: earlier in the current list first), R2 := rest;
//              both halves keep the relative order of the current list;
//     columns: the same with rows and columns exchanged.
// Each half-step is optimal for its side given the other, so the captured mass
// never decreases.  Sums run in list order in double precision.
#include <algorithm>
#include <numeric>
#include <vector>

#include "pivot_internal.h"

namespace {

struct Ctx {
    const float* W; int M, K, max_iter;
};

// Reorders `own` (rows if rows_side) so that the `n1` entries with the largest
// gain against the other side's halves come first; returns true if it changed.
bool improve_side(const Ctx& c, std::vector<int>& own, int n1, const std::vector<int>& other, int o1, bool rows_side) {
    const int n = (int)own.size();
    std::vector<double> gain(n);
    for (int i = 0; i < n; ++i) {
        double a = 0.0, b = 0.0;
        for (int j = 0; j < (int)other.size(); ++j) {
            const size_t idx = rows_side ? (size_t)own[i] * c.K + other[j] : (size_t)other[j] * c.K + own[i];
            const double w = (double)c.W[idx];
            if (j < o1) a += w; else b += w;
        }
        gain[i] = a - b;
    }
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return gain[x] > gain[y]; });
    std::vector<char> first(n, 0);
    for (int k = 0; k < n1; ++k) first[order[k]] = 1;
    std::vector<int> out;
    out.reserve(n);
    for (int i = 0; i < n; ++i) if (first[i]) out.push_back(own[i]);
    for (int i = 0; i < n; ++i) if (!first[i]) out.push_back(own[i]);
    const bool changed = (out != own);
    own.swap(out);
    return changed;
}

void bisect(const Ctx& c, std::vector<int>& R, std::vector<int>& C, int levels) {
    if (levels == 0 || R.size() < 2 || C.size() < 2) return;
    const int r1 = (int)R.size() / 2, c1 = (int)C.size() / 2;
    for (int it = 0; it < c.max_iter; ++it) {
        const bool a = improve_side(c, R, r1, C, c1, true);
        const bool b = improve_side(c, C, c1, R, r1, false);
        if (!a && !b) break;
    }
    std::vector<int> Ra(R.begin(), R.begin() + r1), Rb(R.begin() + r1, R.end());
    std::vector<int> Ca(C.begin(), C.begin() + c1), Cb(C.begin() + c1, C.end());
    bisect(c, Ra, Ca, levels - 1);
    bisect(c, Rb, Cb, levels - 1);
    std::copy(Ra.begin(), Ra.end(), R.begin());
    std::copy(Rb.begin(), Rb.end(), R.begin() + r1);
    std::copy(Ca.begin(), Ca.end(), C.begin());
    std::copy(Cb.begin(), Cb.end(), C.begin() + c1);
}

// Mass inside the block-diagonal pattern the recursion leaves (same split sizes).
double captured(const Ctx& c, const int* R, int nr, const int* C, int nc, int levels) {
    if (levels == 0 || nr < 2 || nc < 2) {
        double s = 0.0;
        for (int i = 0; i < nr; ++i)
            for (int j = 0; j < nc; ++j) s += (double)c.W[(size_t)R[i] * c.K + C[j]];
        return s;
    }
    const int r1 = nr / 2, c1 = nc / 2;
    return captured(c, R, r1, C, c1, levels - 1) + captured(c, R + r1, nr - r1, C + c1, nc - c1, levels - 1);
}

bool is_perm(const int32_t* p, int n) {
    std::vector<char> seen(n, 0);
    for (int i = 0; i < n; ++i) {
        if (p[i] < 0 || p[i] >= n || seen[p[i]]) return false;
        seen[p[i]] = 1;
    }
    return true;
}

}  // namespace

extern "C" int pivot_feedback_search(const float* absW, int M, int K, int levels, int max_iter,
                                     const int32_t* prow0, const int32_t* pcol0,
                                     int32_t* prow_out, int32_t* pcol_out, double* captured_mass) {
    using namespace pivot;
    if (!absW || !prow0 || !pcol0 || !prow_out || !pcol_out) { set_error("absW, prow0, pcol0, prow_out and pcol_out are required"); return PIVOT_E_NULL; }
    if (M < 1 || K < 1 || levels < 0 || levels > 20 || max_iter < 1) { set_error("bad M, K, levels or max_iter"); return PIVOT_E_SHAPE; }
    if (!is_perm(prow0, M) || !is_perm(pcol0, K)) { set_error("the starting arrays are not permutations"); return PIVOT_E_NOT_PERMUTATION; }
    try {
        Ctx c{absW, M, K, max_iter};
        std::vector<int> R(prow0, prow0 + M), C(pcol0, pcol0 + K);
        bisect(c, R, C, levels);
        std::copy(R.begin(), R.end(), prow_out);
        std::copy(C.begin(), C.end(), pcol_out);
        if (captured_mass) *captured_mass = captured(c, R.data(), M, C.data(), K, levels);
    } catch (const std::bad_alloc&) {
        set_error("out of host memory");
        return PIVOT_E_ALLOC;
    }
    return PIVOT_OK;
}
