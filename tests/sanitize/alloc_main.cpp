// Drives the host functions of libskim (csrc/skim_alloc.cpp: Alg. 1 with unit and with row costs, the sizing
// helpers) under AddressSanitizer and UndefinedBehaviorSanitizer: both ends of the budget, tables full of
// ties, one row, non-integer budgets, bad arguments.  Built and run by tests/test_sanitizers.py.
#include <stdint.h>
#include <stdio.h>

#include <vector>

#include "../../paper_2412_04180_amd/csrc/skim_alloc.cpp"

static uint64_t st = 99;
static double uni() {
    st = st * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(st >> 11) / 9007199254740992.0;
}

int main() {
    const int64_t ns[] = {1, 2, 7, 100, 4097};
    const double avgs[] = {1.0, 1.5, 2.25, 3.2, 3.999, 4.0};
    for (int64_t n : ns)
        for (double avg : avgs)
            for (int kind = 0; kind < 3; ++kind) {
                std::vector<double> E((size_t)n * 4);
                for (int64_t i = 0; i < n; ++i) {
                    double e = uni();
                    for (int j = 3; j >= 0; --j) {
                        E[(size_t)i * 4 + j] = e;
                        e += kind == 0 ? uni() : (kind == 1 ? (double)(int)(uni() * 3) : uni() - 0.3);
                    }
                }
                std::vector<uint8_t> bits((size_t)n);
                std::vector<int64_t> cost((size_t)n);
                for (int64_t i = 0; i < n; ++i) cost[(size_t)i] = 1 + (int64_t)(uni() * 5);
                int64_t spent = -1, budget = -1;
                if (skim_greedy_allocate(E.data(), nullptr, n, 1, 4, avg, bits.data(), &spent, &budget) != SKIM_OK) return 1;
                int64_t sum = 0;
                for (int64_t i = 0; i < n; ++i) sum += bits[(size_t)i];
                if (sum != spent || spent != budget) return 2;
                if (skim_greedy_allocate(E.data(), cost.data(), n, 1, 4, avg, bits.data(), &spent, &budget) != SKIM_OK) return 3;
                if (spent > budget) return 4;
                if (skim_packed_words(bits.data(), n, 11008) < 0 || skim_codebook_entries(bits.data(), n) < 0) return 5;
            }
    double E1[4] = {4, 3, 2, 1};
    uint8_t b1;
    if (skim_greedy_allocate(E1, nullptr, 1, 1, 4, 5.0, &b1, nullptr, nullptr) != SKIM_ERR_BUDGET) return 6;
    if (skim_greedy_allocate(nullptr, nullptr, 1, 1, 4, 2.0, &b1, nullptr, nullptr) != SKIM_ERR_ARG) return 7;
    if (skim_greedy_allocate(E1, nullptr, 1, 1, 4, 2.0, &b1, nullptr, nullptr) != SKIM_OK || b1 != 2) return 8;
    printf("ok\n");
    return 0;
}
