// Driver for a sanitizer build of the host-side partitioner (tests/test_sanitizers.py compiles this file together
// with paper_2605_08962_amd/csrc/va_partition.hip, as plain C++, under -fsanitize=address,undefined and runs it).
// Buffers have exactly the documented sizes; results are checked for what any correct partition satisfies.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../include/varlen_attn.h"

static int fails = 0;
static void expect(bool cond, const char* what) {
    if (!cond) { std::printf("FAILED: %s\n", what); ++fails; }
}

static void run(const std::vector<int32_t>& len, int bins, int method, int equal_counts) {
    const int n = (int)len.size();
    std::vector<int32_t> bin_of(n);
    std::vector<double> cost(bins);
    const double lin = 1.0, quad = 0.01;
    const int rc = varlen_attn_balance_partition(n ? len.data() : nullptr, n, bins, method, equal_counts, lin, quad,
                                                 n ? bin_of.data() : nullptr, cost.data());
    expect(rc == VA_OK, "partition returns VA_OK");
    if (rc != VA_OK || n == 0) return;
    std::vector<double> sum(bins, 0.0);
    std::vector<int> count(bins, 0);
    for (int i = 0; i < n; ++i) {
        expect(bin_of[i] >= 0 && bin_of[i] < bins, "bin in range");
        if (bin_of[i] < 0 || bin_of[i] >= bins) return;
        sum[bin_of[i]] += lin * len[i] + quad * (double)len[i] * len[i];
        ++count[bin_of[i]];
    }
    int lo = n, hi = 0;
    for (int b = 0; b < bins; ++b) {
        expect(std::fabs(sum[b] - cost[b]) <= 1e-9 * (1.0 + sum[b]), "bin_cost is the sum of its samples' costs");
        lo = count[b] < lo ? count[b] : lo;
        hi = count[b] > hi ? count[b] : hi;
    }
    if (equal_counts) expect(hi - lo <= 1, "equal_counts: bin sizes differ by at most one");
}

int main() {
    uint64_t s = 0x9E3779B97F4A7C15ull;
    auto rnd = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; };
    for (int method = 0; method < 2; ++method)
        for (int eq = 0; eq < 2; ++eq) {
            run({}, 4, method, eq);
            run({7}, 1, method, eq);
            run({7}, 5, method, eq);                       // more bins than samples
            run({0, 0, 0, 5, 0}, 3, method, eq);           // empty samples
            run({9, 9, 9, 9, 9, 9, 9}, 3, method, eq);     // all ties
            for (int n : {2, 17, 64, 257, 1000})
                for (int bins : {1, 2, 7, 8, 64}) {
                    std::vector<int32_t> len(n);
                    for (auto& x : len) x = (int32_t)(rnd() % 9216);
                    len[n / 2] = 65536;                    // one very long sample
                    run(len, bins, method, eq);
                }
        }
    // rejected arguments
    int32_t one[1] = {3}, out[1];
    expect(varlen_attn_balance_partition(one, 1, 0, 0, 0, 1.0, 0.0, out, nullptr) == VA_ERR_BAD_SHAPE, "bins < 1");
    expect(varlen_attn_balance_partition(one, 1, 2, 7, 0, 1.0, 0.0, out, nullptr) == VA_ERR_BAD_SHAPE, "unknown method");
    expect(varlen_attn_balance_partition(one, -1, 2, 0, 0, 1.0, 0.0, out, nullptr) == VA_ERR_BAD_SHAPE, "negative count");
    one[0] = -3;
    expect(varlen_attn_balance_partition(one, 1, 2, 0, 0, 1.0, 0.0, out, nullptr) == VA_ERR_BAD_SHAPE, "negative length");
    one[0] = 3;
    expect(varlen_attn_balance_partition(one, 1, 2, 0, 0, -1.0, 0.0, out, nullptr) == VA_ERR_BAD_SCALE, "negative cost");
    expect(varlen_attn_balance_partition(one, 1, 2, 0, 0, 1.0, NAN, out, nullptr) == VA_ERR_BAD_SCALE, "NaN cost");
    expect(varlen_attn_balance_partition(nullptr, 1, 2, 0, 0, 1.0, 0.0, out, nullptr) == VA_ERR_NULL_PTR, "null lengths");
    expect(varlen_attn_balance_partition(one, 1, 2, 0, 0, 1.0, 0.0, nullptr, nullptr) == VA_ERR_NULL_PTR, "null bin_of");
    if (fails) return 1;
    std::printf("ok\n");
    return 0;
}
