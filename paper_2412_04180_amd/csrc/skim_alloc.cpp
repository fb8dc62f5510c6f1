// Greedy mixed-precision bit allocation (Alg. 1) -- host code of libskim.
//
// Every row starts at bmin bits and the row with the largest error reduction is upgraded
// until the budget is spent.
//
// Unit costs (the algorithm as printed): the order in which the greedy loop takes the
// upgrades is known in closed form.  Upgrade j of a row becomes available when upgrade j-1
// has been taken, and is then taken at once if its reduction is at least that of j-1 (which
// was the largest on offer).  So upgrade j is taken when the running minimum
// k_j = min(g_1 .. g_j) of the row's reductions comes up, and the loop's order is all
// upgrades sorted by (k descending, row ascending, j ascending).  The first T of them are
// found by selection (std::nth_element): O(n) instead of n log n heap steps.
//
// Row costs (tables joining matrices of different width): a binary heap keyed by
// (reduction per unit cost, descending; row index, ascending); a row whose cost no longer
// fits the remaining budget can never fit later (the budget only shrinks) and is dropped.
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <queue>
#include <vector>

#include "skim.h"

namespace {
struct Cand {
    double gain;  // reduction / cost
    int64_t row;
};
struct Worse {
    bool operator()(const Cand &a, const Cand &b) const {
        if (a.gain != b.gain) return a.gain < b.gain;
        return a.row > b.row;
    }
};
struct Upgrade {
    double key;    // running minimum of the row's reductions up to this upgrade
    int32_t row;
    int32_t level;
};
struct Earlier {   // the order in which the greedy loop takes upgrades
    bool operator()(const Upgrade &a, const Upgrade &b) const {
        if (a.key != b.key) return a.key > b.key;
        if (a.row != b.row) return a.row < b.row;
        return a.level < b.level;
    }
};
}  // namespace

extern "C" skim_status skim_greedy_allocate(const double *E, const int64_t *row_cost, int64_t n, int bmin,
                                            int bmax, double avg_bits, uint8_t *bits_out, int64_t *spent_out,
                                            int64_t *budget_out) {
    if (!E || !bits_out || n < 1) return SKIM_ERR_ARG;
    if (bmin < 1 || bmax < bmin || bmax > 8) return SKIM_ERR_ARG;
    const int nb = bmax - bmin + 1;
    int64_t csum = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t c = row_cost ? row_cost[i] : 1;
        if (c < 1) return SKIM_ERR_ARG;
        csum += c;
    }
    const int64_t B = (int64_t)floor(avg_bits * (double)csum + 1e-9);
    if (B < (int64_t)bmin * csum || B > (int64_t)bmax * csum) return SKIM_ERR_BUDGET;
    int64_t spent = (int64_t)bmin * csum;

    if (!row_cost && n <= 0x7fffffff) {
        const int64_t T = B - spent;              // upgrades to hand out
        const int nu = nb - 1;
        for (int64_t i = 0; i < n; ++i) bits_out[i] = (uint8_t)bmin;
        if (T > 0 && nu > 0) {
            std::vector<Upgrade> up((size_t)n * nu);
            for (int64_t i = 0; i < n; ++i) {
                double k = 0.0;
                for (int j = 0; j < nu; ++j) {
                    const double g = E[i * nb + j] - E[i * nb + j + 1];
                    k = (j == 0 || g < k) ? g : k;
                    up[(size_t)i * nu + j] = {k, (int32_t)i, (int32_t)j};
                }
            }
            if ((size_t)T < up.size()) std::nth_element(up.begin(), up.begin() + T, up.end(), Earlier());
            const size_t take = std::min((size_t)T, up.size());
            for (size_t t = 0; t < take; ++t) bits_out[up[t].row] += 1;
        }
        if (spent_out) *spent_out = B;
        if (budget_out) *budget_out = B;
        return SKIM_OK;
    }

    std::vector<Cand> init;
    init.reserve((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        bits_out[i] = (uint8_t)bmin;
        if (bmin < bmax) {
            const int64_t c = row_cost ? row_cost[i] : 1;
            init.push_back({(E[i * nb] - E[i * nb + 1]) / (double)c, i});
        }
    }
    std::priority_queue<Cand, std::vector<Cand>, Worse> heap(Worse(), std::move(init));
    while (!heap.empty()) {
        const Cand top = heap.top();
        heap.pop();
        const int64_t i = top.row;
        const int64_t c = row_cost ? row_cost[i] : 1;
        if (c > B - spent) continue;  // does not fit now, never will
        bits_out[i] += 1;
        spent += c;
        if (bits_out[i] < bmax) {
            const int col = bits_out[i] - bmin;
            heap.push({(E[i * nb + col] - E[i * nb + col + 1]) / (double)c, i});
        }
    }
    if (spent_out) *spent_out = spent;
    if (budget_out) *budget_out = B;
    return SKIM_OK;
}

extern "C" int64_t skim_packed_words(const uint8_t *bits_host, int64_t n, int64_t m) {
    if (!bits_host || n < 0 || m < 0) return -1;
    int64_t words = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int b = bits_host[i];
        if (b < 1 || b > SKIM_MAX_BITS) return -1;
        words += (m * b + 31) / 32;
    }
    return words;
}

extern "C" int64_t skim_codebook_entries(const uint8_t *bits_host, int64_t n) {
    if (!bits_host || n < 0) return -1;
    int64_t e = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int b = bits_host[i];
        if (b < 1 || b > SKIM_MAX_BITS) return -1;
        e += (int64_t)1 << b;
    }
    return e;
}
