// Host-only check of the planner under AddressSanitizer and UndefinedBehaviorSanitizer: built
// by tests/test_sanitizers.py from csrc/plan.cpp (no GPU code) and oracle/oracle.c, it plans
// random chains through the C ABI, compares every plan with the oracle's exhaustive search
// and walks the error paths.  Exit status 0 = everything agreed and the sanitizers saw nothing.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "../include/mom.h"

extern "C" {
int oracle_plan_bruteforce(int32_t n, const int64_t *dims, const int32_t *props, int32_t elide, uint64_t *cost,
                           int32_t *n_eff, int32_t *out_splits, int32_t *result_prop, int64_t *num_trees);
int oracle_plan_bruteforce_time(int32_t n, const int64_t *dims, const int32_t *props, uint64_t *time_ps, uint64_t *mults,
                                int32_t *n_eff, int32_t *out_splits);
int32_t oracle_transposed_property(int32_t p);
}

static int failures = 0;
#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::printf("check failed at line %d: %s\n", __LINE__, #cond); \
            ++failures;                                                    \
        }                                                                  \
    } while (0)

int main()
{
    std::mt19937 rng(12345);
    const int64_t pool[] = {1, 5, 32, 33, 64, 65, 128, 130, 300, 1000};
    for (int trial = 0; trial < 1500; ++trial) {
        const int n = 1 + (int)(rng() % 8);
        std::vector<int64_t> dims(n + 1);
        std::vector<int32_t> props(n), trans(n), chain(n);
        dims[0] = pool[rng() % 10];
        for (int i = 0; i < n; ++i) {
            props[i] = (int32_t)(rng() % 5);
            trans[i] = (int32_t)(rng() % 2);
            dims[i + 1] = props[i] == MOM_GENERAL ? pool[rng() % 10] : dims[i];
            chain[i] = trans[i] ? oracle_transposed_property(props[i]) : props[i];
        }
        for (int objective = 0; objective < 2; ++objective) {
            mom_plan_t *plan = nullptr;
            CHECK(mom_chain_plan_ex(dims.data(), props.data(), trans.data(), n, objective, nullptr, &plan) == MOM_OK);
            if (!plan) continue;
            uint64_t cost = 0, time_ps = 0, mults = 0;
            int32_t n_eff = 0, rprop = 0;
            int64_t trees = 0;
            std::vector<int32_t> want(n + 1), got(n + 1);
            if (objective == MOM_PLAN_MIN_MULTS) {
                CHECK(oracle_plan_bruteforce(n, dims.data(), chain.data(), 1, &cost, &n_eff, want.data(), &rprop, &trees) == 0);
                CHECK(mom_plan_cost_mults(plan) == cost);
                int32_t p = -1;
                CHECK(mom_plan_result(plan, nullptr, nullptr, &p) == MOM_OK && p == rprop);
            } else {
                CHECK(oracle_plan_bruteforce_time(n, dims.data(), chain.data(), &time_ps, &mults, &n_eff, want.data()) == 0);
                CHECK(mom_plan_cost_time_ps(plan) == time_ps && mom_plan_cost_mults(plan) == mults);
            }
            const int32_t k = mom_plan_num_products(plan);
            CHECK(k == (n_eff > 0 ? n_eff - 1 : 0));
            CHECK(mom_plan_splits(plan, got.data(), k) == MOM_OK);
            CHECK(std::memcmp(got.data(), want.data(), sizeof(int32_t) * k) == 0);
            CHECK(k == 0 || mom_plan_splits(plan, got.data(), k - 1) == MOM_ERR_BUFFER_TOO_SMALL);
            char text[512];
            CHECK(mom_plan_string(plan, text, sizeof text) == MOM_OK);
            const size_t len = std::strlen(text);
            std::vector<char> exact(len + 1);
            CHECK(mom_plan_string(plan, exact.data(), len + 1) == MOM_OK);
            CHECK(mom_plan_string(plan, exact.data(), len) == MOM_ERR_BUFFER_TOO_SMALL);
            uint64_t sum = 0;
            for (int32_t i = 0; i < k; ++i) {
                int64_t shape[3];
                int32_t pr[3], level;
                uint64_t m;
                CHECK(mom_plan_product(plan, i, shape, pr, &m, &level) == MOM_OK);
                sum += m;
            }
            CHECK(sum == mom_plan_cost_mults(plan));
            CHECK(mom_plan_product(plan, k, nullptr, nullptr, nullptr, nullptr) == MOM_ERR_BAD_N);
            CHECK(mom_plan_num_launches(plan) >= 1);
            // evaluation argument checks that fail before anything touches a GPU
            CHECK(mom_chain_eval(plan, nullptr, nullptr, nullptr, 0, nullptr, 0, 0, nullptr) == MOM_ERR_NULL);
            // the same tree again as a forced tree
            mom_plan_t *again = nullptr;
            CHECK(mom_chain_plan_ex(dims.data(), props.data(), trans.data(), n, objective, got.data(), &again) == MOM_OK);
            CHECK(again && mom_plan_cost_mults(again) == mom_plan_cost_mults(plan));
            mom_plan_destroy(again);
            mom_plan_destroy(plan);
        }
        // a sum of this chain and a plain matrix of its shape
        if (trial % 10 == 0) {
            std::vector<int64_t> d2(dims);
            d2.push_back(dims[0]); d2.push_back(dims[n]);
            std::vector<int32_t> p2(props), t2(trans);
            p2.push_back(MOM_GENERAL); t2.push_back(0);
            const int32_t lens[2] = {n, 1};
            mom_equation_t *eq = nullptr;
            CHECK(mom_equation_plan(d2.data(), p2.data(), t2.data(), lens, 2, 0, &eq) == MOM_OK);
            int64_t r = 0, c = 0;
            int32_t p = -1;
            CHECK(mom_equation_result(eq, &r, &c, &p) == MOM_OK && r == dims[0] && c == dims[n] && p == MOM_GENERAL);
            CHECK(mom_equation_num_chains(eq) == 2 && mom_equation_chain(eq, 2) == nullptr && mom_equation_chain(eq, 0) != nullptr);
            mom_equation_destroy(eq);
        }
    }
    // error paths
    mom_plan_t *plan = reinterpret_cast<mom_plan_t *>(1);
    const int64_t d3[] = {4, 4, 4, 4};
    const int32_t g3[] = {0, 0, 0}, bad_split[] = {2, 0}, bad_prop[] = {0, 9, 0}, lower_rect[] = {1};
    const int64_t rect[] = {4, 5};
    CHECK(mom_chain_plan(nullptr, g3, 3, &plan) == MOM_ERR_NULL && plan == nullptr);
    CHECK(mom_chain_plan(d3, g3, 0, &plan) == MOM_ERR_BAD_N);
    CHECK(mom_chain_plan(d3, bad_prop, 3, &plan) == MOM_ERR_BAD_PROP);
    CHECK(mom_chain_plan(rect, lower_rect, 1, &plan) == MOM_ERR_NOT_SQUARE);
    CHECK(mom_plan_from_splits(d3, g3, 3, bad_split, &plan) == MOM_ERR_BAD_SPLITS);
    CHECK(mom_chain_plan_ex(d3, g3, bad_prop, 3, 0, nullptr, &plan) == MOM_ERR_BAD_TRANS);
    CHECK(mom_chain_plan_ex(d3, g3, nullptr, 3, 7, nullptr, &plan) == MOM_ERR_BAD_FLAGS);
    const int64_t huge[] = {2147483392, 2147483392, 2147483392, 2147483392, 2147483392};
    const int32_t g4[] = {0, 0, 0, 0};
    CHECK(mom_chain_plan(huge, g4, 4, &plan) == MOM_ERR_OVERFLOW && plan == nullptr);
    mom_plan_destroy(nullptr);
    mom_equation_destroy(nullptr);
    CHECK(std::strlen(mom_status_string(MOM_ERR_NOMEM)) > 0);
    std::printf("%s (%d failures)\n", failures ? "FAILED" : "ok", failures);
    return failures ? 1 : 0;
}
