// Token-balanced dispatch on the host: which data-parallel rank (or GPU) gets which prompt group.
//
// The paper balances the tokens its workers process by treating the assignment as one-dimensional bin packing
// and solving it with the Karmarkar-Karp algorithm: equal sample counts per data-parallel group with a small
// spread of token totals, the count constraint relaxed for pipeline stages (Sec. 4.4; effect in Sec. 7.4).
// This is that algorithm in its k-way form (largest differencing method) and its count-balanced variant.
// The decode path of this library needs no exchange between GPUs, so this is all a multi-GPU run adds: each
// GPU runs the attention kernels on the groups it is dealt here.
#include "../../include/rollout_attn.h"

#include <algorithm>
#include <cstdint>
#include <limits>
#include <new>
#include <queue>
#include <vector>

namespace {

struct Part {            // one set of a partial solution: a chain of items
    int64_t sum;
    int64_t first_index; // smallest item index in the set; max() when empty (orders equal sums)
    int64_t head, tail;  // chain through next[]; -1 when empty
};

struct Solution {        // k sets in order of decreasing sum
    int64_t spread;
    int64_t created;
    std::vector<Part> parts;
};

struct LaterFirst {      // priority queue: largest spread on top, the older solution on a tie
    bool operator()(const Solution *a, const Solution *b) const
    {
        if (a->spread != b->spread) return a->spread < b->spread;
        return a->created > b->created;
    }
};

void order_parts(std::vector<Part> &p)
{
    std::sort(p.begin(), p.end(), [](const Part &x, const Part &y) {
        if (x.sum != y.sum) return x.sum > y.sum;
        return x.first_index < y.first_index;
    });
}

} // namespace

extern "C" ra_status rollout_attn_balance(const int64_t *weights, int64_t n, int32_t k, int32_t equal_count, int32_t *part,
                                          int64_t *part_sums)
{
    if (n < 0 || k < 1 || (n > 0 && (!weights || !part))) return RA_ERR_INVALID_ARG;
    for (int64_t i = 0; i < n; i++)
        if (weights[i] < 0) return RA_ERR_INVALID_ARG;
    if (part_sums) std::fill(part_sums, part_sums + k, (int64_t)0);
    if (n == 0) return RA_OK;
    const int64_t kEmpty = std::numeric_limits<int64_t>::max();
    try {
        std::vector<int64_t> next((size_t)n, -1);
        std::vector<Solution> pool;
        pool.reserve((size_t)(2 * n + 2));
        std::priority_queue<Solution *, std::vector<Solution *>, LaterFirst> heap;
        auto single = [&](int64_t i) { return i < 0 ? Part{0, kEmpty, -1, -1} : Part{weights[i], i, i, i}; };
        auto push = [&](std::vector<Part> &&parts) {
            order_parts(parts);
            pool.push_back(Solution{parts.front().sum - parts.back().sum, (int64_t)pool.size(), std::move(parts)});
            heap.push(&pool.back());
        };
        if (!equal_count) {
            for (int64_t i = 0; i < n; i++) {
                std::vector<Part> parts((size_t)k, single(-1));
                parts[0] = single(i);
                push(std::move(parts));
            }
        } else {
            std::vector<int64_t> order((size_t)n);
            for (int64_t i = 0; i < n; i++) order[(size_t)i] = i;
            std::stable_sort(order.begin(), order.end(), [&](int64_t x, int64_t y) { return weights[x] > weights[y]; });
            for (int64_t t = 0; t < n; t += k) {
                std::vector<Part> parts;
                for (int64_t j = t; j < t + k; j++) parts.push_back(single(j < n ? order[(size_t)j] : -1));
                push(std::move(parts));
            }
        }
        while (heap.size() > 1) {
            Solution *a = heap.top();
            heap.pop();
            Solution *b = heap.top();
            heap.pop();
            std::vector<Part> parts((size_t)k);
            for (int32_t j = 0; j < k; j++) {
                const Part &x = a->parts[(size_t)j], &y = b->parts[(size_t)(k - 1 - j)];
                Part m{x.sum + y.sum, std::min(x.first_index, y.first_index), x.head, x.tail};
                if (x.head < 0) {
                    m.head = y.head, m.tail = y.tail;
                } else if (y.head >= 0) {
                    next[(size_t)x.tail] = y.head;
                    m.tail = y.tail;
                }
                parts[(size_t)j] = m;
            }
            push(std::move(parts));
        }
        const Solution *last = heap.top();
        for (int32_t p = 0; p < k; p++) {
            if (part_sums) part_sums[p] = last->parts[(size_t)p].sum;
            for (int64_t i = last->parts[(size_t)p].head; i >= 0; i = next[(size_t)i]) part[i] = p;
        }
    } catch (const std::bad_alloc &) {
        return RA_ERR_DEVICE;
    }
    return RA_OK;
}
