// Greedy mixed-precision bit allocation (Alg. 1) -- host code of libskim.
//
// Every row starts at bmin bits.  A binary heap keyed by (error reduction per
// unit cost, descending; row index, ascending) yields the row to upgrade; after
// an upgrade the row's next reduction is pushed.  A row whose cost no longer
// fits the remaining budget can never fit later (the budget only shrinks) and
// is dropped.  n rows, at most n*(bmax-bmin) upgrades: O(n log n).
#include <math.h>
#include <stdint.h>

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
