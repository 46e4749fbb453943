// Host-side length-balanced partitioner: splits the samples of a group of ranks into one bin per
// rank so that the most expensive bin is cheap.  This is the step in front of the attention kernels
// in the paper's pipeline (Section 5.1, decentralized grouped reordering: the sample sizes of a group
// are gathered, the samples reordered "using the Karp algorithm", then redistributed); the paper
// gives no detail, so the method is the k-way Karmarkar-Karp largest differencing method, with greedy
// longest-processing-time-first scheduling offered beside it.  Pure host code, no GPU work.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <queue>
#include <vector>

#include "../../include/varlen_attn.h"

namespace {

struct Slot {
    double cost;
    int32_t head, tail;  // singly linked list of the samples in this slot (-1: empty)
};

// A partial solution: `bins` slots sorted by cost, descending.
struct Partial {
    double spread;
    int64_t created;
    std::vector<Slot> slots;
};

struct BySpread {
    const std::vector<Partial>* pool;
    bool operator()(int32_t a, int32_t b) const {  // "a comes after b" for the max-heap
        const Partial &x = (*pool)[a], &y = (*pool)[b];
        if (x.spread != y.spread) return x.spread < y.spread;
        return x.created > y.created;
    }
};

std::vector<int32_t> by_decreasing_cost(const std::vector<double>& c) {
    std::vector<int32_t> order(c.size());
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return c[a] > c[b]; });
    return order;
}

void differencing(const std::vector<double>& c, int bins, bool equal_counts, int32_t* bin_of) {
    const int32_t n = (int32_t)c.size();
    if (n == 0) return;
    std::vector<int32_t> next(n, -1);  // links of the member lists
    const std::vector<int32_t> order = by_decreasing_cost(c);
    std::vector<Partial> pool;
    pool.reserve(2 * (size_t)n);
    auto finish = [&](Partial& p) {
        p.spread = p.slots.front().cost - p.slots.back().cost;
        p.created = (int64_t)pool.size();
    };
    if (equal_counts) {
        for (int32_t g = 0; g < n; g += bins) {
            Partial p;
            p.slots.assign(bins, Slot{0.0, -1, -1});
            for (int j = 0; j < bins && g + j < n; ++j) p.slots[j] = Slot{c[order[g + j]], order[g + j], order[g + j]};
            finish(p);
            pool.push_back(std::move(p));
        }
    } else {
        for (int32_t i : order) {
            Partial p;
            p.slots.assign(bins, Slot{0.0, -1, -1});
            p.slots[0] = Slot{c[i], i, i};
            finish(p);
            pool.push_back(std::move(p));
        }
    }
    std::priority_queue<int32_t, std::vector<int32_t>, BySpread> heap(BySpread{&pool});
    for (int32_t i = 0; i < (int32_t)pool.size(); ++i) heap.push(i);
    while (heap.size() > 1) {
        const int32_t ia = heap.top(); heap.pop();
        const int32_t ib = heap.top(); heap.pop();
        Partial m;
        m.slots.resize(bins);
        for (int j = 0; j < bins; ++j) {
            const Slot& a = pool[ia].slots[j];
            const Slot& b = pool[ib].slots[bins - 1 - j];
            Slot s{a.cost + b.cost, a.head, a.tail};
            if (b.head >= 0) {  // append b's members behind a's
                if (s.head < 0) { s.head = b.head; } else { next[s.tail] = b.head; }
                s.tail = b.tail;
            }
            m.slots[j] = s;
        }
        std::stable_sort(m.slots.begin(), m.slots.end(), [](const Slot& x, const Slot& y) { return x.cost > y.cost; });
        pool[ia].slots.clear(); pool[ia].slots.shrink_to_fit();
        pool[ib].slots.clear(); pool[ib].slots.shrink_to_fit();
        finish(m);
        pool.push_back(std::move(m));  // reserve() above keeps the heap's pointer to the pool valid
        heap.push((int32_t)pool.size() - 1);
    }
    const Partial& last = pool[heap.top()];
    for (int b = 0; b < bins; ++b)
        for (int32_t i = last.slots[b].head; i >= 0; i = next[i]) bin_of[i] = b;
}

void greedy(const std::vector<double>& c, int bins, bool equal_counts, int32_t* bin_of) {
    const int32_t n = (int32_t)c.size();
    const int32_t lo = n / bins, extra = n % bins;
    std::vector<double> total(bins, 0.0);
    std::vector<int32_t> count(bins, 0);
    int32_t full_bins = 0;  // bins holding lo + 1 samples
    for (int32_t i : by_decreasing_cost(c)) {
        int best = -1;
        for (int b = 0; b < bins; ++b) {
            const bool room = !equal_counts || count[b] < lo || (count[b] == lo && full_bins < extra);
            if (room && (best < 0 || total[b] < total[best])) best = b;
        }
        bin_of[i] = best;
        total[best] += c[i];
        if (++count[best] == lo + 1) ++full_bins;
    }
}

}  // namespace

extern "C" int varlen_attn_balance_partition(const int32_t* lengths, int32_t num_seqs, int32_t bins, int32_t method,
                                             int32_t equal_counts, double lin_cost, double quad_cost,
                                             int32_t* bin_of, double* bin_cost) {
    if (num_seqs < 0 || bins < 1 || (method != VA_PARTITION_KARMARKAR_KARP && method != VA_PARTITION_LPT) ||
        (equal_counts != 0 && equal_counts != 1))
        return VA_ERR_BAD_SHAPE;
    if (!std::isfinite(lin_cost) || !std::isfinite(quad_cost) || lin_cost < 0.0 || quad_cost < 0.0) return VA_ERR_BAD_SCALE;
    if (num_seqs > 0 && (!lengths || !bin_of)) return VA_ERR_NULL_PTR;
    std::vector<double> c((size_t)num_seqs);
    for (int32_t i = 0; i < num_seqs; ++i) {
        if (lengths[i] < 0) return VA_ERR_BAD_SHAPE;
        const double L = (double)lengths[i];
        c[i] = lin_cost * L + (quad_cost * L) * L;
    }
    if (method == VA_PARTITION_KARMARKAR_KARP)
        differencing(c, bins, equal_counts != 0, bin_of);
    else
        greedy(c, bins, equal_counts != 0, bin_of);
    if (bin_cost) {
        for (int b = 0; b < bins; ++b) bin_cost[b] = 0.0;
        for (int32_t i = 0; i < num_seqs; ++i) bin_cost[bin_of[i]] += c[i];
    }
    return VA_OK;
}
