// Host-side load balancing for ODC: Karmarkar-Karp k-way partitioning, the LB-Mini and
// LB-Micro plans of paper Section 4 / Appendix C, and the runtime / bubble-rate estimate
// (Eq. 1, Appendix F).  Plain C++, no GPU.
#include "../../include/odc_packing.h"

#include "../../include/odc.h"

#include <algorithm>
#include <limits>
#include <new>
#include <queue>
#include <vector>

namespace {

constexpr int64_t kMax = std::numeric_limits<int64_t>::max();

struct Subset {
    int64_t sum = 0;
    std::vector<int> items;  // ascending
    int first() const { return items.empty() ? std::numeric_limits<int>::max() : items.front(); }
};

// A partial solution: k subsets, largest sum first (ties: smaller first index first).
struct Partial {
    std::vector<Subset> sets;
    int64_t spread() const { return sets.front().sum - sets.back().sum; }
    void order()
    {
        std::sort(sets.begin(), sets.end(), [](const Subset &a, const Subset &b) {
            if (a.sum != b.sum) return a.sum > b.sum;
            return a.first() < b.first();
        });
    }
};

struct HeapEntry {
    int64_t spread;
    int64_t serial;
    int index;  // into the pool of partial solutions
};

struct HeapLess {  // priority_queue pops the LARGEST: larger spread, then smaller serial
    bool operator()(const HeapEntry &a, const HeapEntry &b) const
    {
        if (a.spread != b.spread) return a.spread < b.spread;
        return a.serial > b.serial;
    }
};

// Largest differencing method, k-way.  Returns the final partial solution's subsets.
int kk(const int64_t *costs, int n, int k, bool equal_size, std::vector<Subset> *out)
{
    if (!costs && n > 0) return ODC_ERR_INVALID_ARG;
    if (n < 0 || k < 1) return ODC_ERR_INVALID_ARG;
    if (equal_size && n % k != 0) return ODC_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        if (costs[i] < 0) return ODC_ERR_INVALID_ARG;
        if (costs[i] > kMax - total) return ODC_ERR_OVERFLOW;
        total += costs[i];
    }
    out->assign(static_cast<size_t>(k), Subset{});
    if (n == 0) return ODC_OK;

    std::vector<Partial> pool;
    std::priority_queue<HeapEntry, std::vector<HeapEntry>, HeapLess> heap;
    int64_t serial = 0;
    auto push = [&](Partial &&p) {
        p.order();
        heap.push(HeapEntry{p.spread(), serial++, static_cast<int>(pool.size())});
        pool.push_back(std::move(p));
    };
    if (equal_size) {
        std::vector<int> idx(static_cast<size_t>(n));
        for (int i = 0; i < n; ++i) idx[static_cast<size_t>(i)] = i;
        std::sort(idx.begin(), idx.end(), [&](int a, int b) {
            if (costs[a] != costs[b]) return costs[a] > costs[b];
            return a < b;
        });
        for (int g = 0; g < n; g += k) {
            Partial p;
            p.sets.resize(static_cast<size_t>(k));
            for (int j = 0; j < k; ++j) {
                const int item = idx[static_cast<size_t>(g + j)];
                p.sets[static_cast<size_t>(j)].sum = costs[item];
                p.sets[static_cast<size_t>(j)].items = {item};
            }
            push(std::move(p));
        }
    } else {
        for (int i = 0; i < n; ++i) {
            Partial p;
            p.sets.resize(static_cast<size_t>(k));
            p.sets[0].sum = costs[i];
            p.sets[0].items = {i};
            push(std::move(p));
        }
    }
    while (heap.size() > 1) {
        const HeapEntry ea = heap.top();
        heap.pop();
        const HeapEntry eb = heap.top();
        heap.pop();
        Partial &a = pool[static_cast<size_t>(ea.index)];
        Partial &b = pool[static_cast<size_t>(eb.index)];
        Partial m;
        m.sets.resize(static_cast<size_t>(k));
        for (int i = 0; i < k; ++i) {  // i-th largest of a with i-th smallest of b
            Subset &sa = a.sets[static_cast<size_t>(i)];
            Subset &sb = b.sets[static_cast<size_t>(k - 1 - i)];
            Subset &dst = m.sets[static_cast<size_t>(i)];
            dst.sum = sa.sum + sb.sum;
            dst.items.resize(sa.items.size() + sb.items.size());
            std::merge(sa.items.begin(), sa.items.end(), sb.items.begin(), sb.items.end(), dst.items.begin());
        }
        a.sets.clear();
        b.sets.clear();
        push(std::move(m));
    }
    *out = std::move(pool[static_cast<size_t>(heap.top().index)].sets);
    return ODC_OK;
}

int costs_of(const int64_t *seqlens, const std::vector<int> &ids, int64_t hidden, std::vector<int64_t> *costs)
{
    costs->resize(ids.size());
    for (size_t j = 0; j < ids.size(); ++j) {
        const int64_t c = odc_compute_cost(seqlens[ids[j]], hidden);
        if (c < 0) return seqlens[ids[j]] < 0 ? ODC_ERR_INVALID_ARG : ODC_ERR_OVERFLOW;
        (*costs)[j] = c;
    }
    return ODC_OK;
}

// Partition one device's samples into k microbatches; reports whether any exceeds the cap.
int micro_parts(const int64_t *seqlens, const std::vector<int> &ids, int k, int64_t hidden, int64_t max_tokens,
                std::vector<Subset> *parts, bool *oom)
{
    std::vector<int64_t> costs;
    int rc = costs_of(seqlens, ids, hidden, &costs);
    if (rc != ODC_OK) return rc;
    rc = kk(costs.data(), static_cast<int>(ids.size()), k, false, parts);
    if (rc != ODC_OK) return rc;
    *oom = false;
    for (const Subset &s : *parts) {
        int64_t tokens = 0;
        for (int j : s.items) tokens += seqlens[ids[static_cast<size_t>(j)]];
        if (tokens > max_tokens && s.items.size() > 1) *oom = true;  // a lone oversize sample is accepted
    }
    return ODC_OK;
}

}  // namespace

extern "C" {

int64_t odc_compute_cost(int64_t seqlen, int64_t hidden)
{
    if (seqlen < 0 || hidden < 0) return -1;
    if (hidden > kMax / 6) return -1;
    const int64_t h6 = 6 * hidden;
    if (seqlen > kMax - h6) return -1;
    const int64_t f = seqlen + h6;
    if (seqlen != 0 && f > kMax / seqlen) return -1;
    return seqlen * f;
}

int odc_kk_partition(const int64_t *costs, int n, int k, int equal_size, int *part_of)
{
    if (!part_of && n > 0) return ODC_ERR_INVALID_ARG;
    try {
        std::vector<Subset> sets;
        const int rc = kk(costs, n, k, equal_size != 0, &sets);
        if (rc != ODC_OK) return rc;
        for (int p = 0; p < k; ++p)
            for (int item : sets[static_cast<size_t>(p)].items) part_of[item] = p;
        return ODC_OK;
    } catch (const std::bad_alloc &) {
        return ODC_ERR_NOMEM;
    }
}

int odc_plan_minibatch(const int64_t *seqlens, int n, int world, int64_t max_tokens, int64_t hidden, int mode,
                       int *device_of, int *micro_of, int *micro_count)
{
    if (!seqlens || !device_of || !micro_of || !micro_count || n < 1 || world < 1 || max_tokens < 1 ||
        hidden < 0 || mode < 0 || mode > 2)
        return ODC_ERR_INVALID_ARG;
    if (mode != 0 && n % world != 0) return ODC_ERR_INVALID_ARG;
    try {
        std::vector<int> all(static_cast<size_t>(n));
        for (int i = 0; i < n; ++i) {
            if (seqlens[i] < 0) return ODC_ERR_INVALID_ARG;
            all[static_cast<size_t>(i)] = i;
        }
        if (mode == 2) {
            // LocalSort: the minibatch is dealt to the devices in the order given; each device
            // sorts its samples by length (longest first, ties by index) and runs them one per
            // microbatch.  No balancing, no packing.
            const int per_device = n / world;
            for (int d = 0; d < world; ++d) {
                std::vector<int> ids(all.begin() + static_cast<std::ptrdiff_t>(d) * per_device,
                                     all.begin() + static_cast<std::ptrdiff_t>(d + 1) * per_device);
                std::stable_sort(ids.begin(), ids.end(), [&](int a, int b) { return seqlens[a] > seqlens[b]; });
                for (int m = 0; m < per_device; ++m) {
                    device_of[ids[static_cast<size_t>(m)]] = d;
                    micro_of[ids[static_cast<size_t>(m)]] = m;
                }
                micro_count[d] = per_device;
            }
            return ODC_OK;
        }
        std::vector<int64_t> costs;
        int rc = costs_of(seqlens, all, hidden, &costs);
        if (rc != ODC_OK) return rc;
        std::vector<Subset> devices;
        rc = kk(costs.data(), n, world, mode == 1, &devices);
        if (rc != ODC_OK) return rc;

        if (mode == 0) {
            for (int d = 0; d < world; ++d) {
                const std::vector<int> &ids = devices[static_cast<size_t>(d)].items;
                micro_count[d] = 0;
                if (ids.empty()) continue;
                std::vector<Subset> parts;
                for (int k = 1;; ++k) {
                    bool oom = false;
                    rc = micro_parts(seqlens, ids, k, hidden, max_tokens, &parts, &oom);
                    if (rc != ODC_OK) return rc;
                    if (!oom || k >= static_cast<int>(ids.size())) break;
                }
                int m = 0;
                for (const Subset &s : parts) {
                    if (s.items.empty()) continue;
                    for (int j : s.items) {
                        device_of[ids[static_cast<size_t>(j)]] = d;
                        micro_of[ids[static_cast<size_t>(j)]] = m;
                    }
                    ++m;
                }
                micro_count[d] = m;
            }
            return ODC_OK;
        }
        // LB-Micro: one k for all devices
        const int per_device = n / world;
        std::vector<std::vector<Subset>> parts(static_cast<size_t>(world));
        for (int k = 1;; ++k) {
            bool any_oom = false;
            for (int d = 0; d < world; ++d) {
                bool oom = false;
                rc = micro_parts(seqlens, devices[static_cast<size_t>(d)].items, k, hidden, max_tokens,
                                 &parts[static_cast<size_t>(d)], &oom);
                if (rc != ODC_OK) return rc;
                any_oom = any_oom || oom;
            }
            if (!any_oom || k >= per_device) {
                for (int d = 0; d < world; ++d) {
                    const std::vector<int> &ids = devices[static_cast<size_t>(d)].items;
                    for (int m = 0; m < k; ++m)
                        for (int j : parts[static_cast<size_t>(d)][static_cast<size_t>(m)].items) {
                            device_of[ids[static_cast<size_t>(j)]] = d;
                            micro_of[ids[static_cast<size_t>(j)]] = m;
                        }
                    micro_count[d] = k;
                }
                return ODC_OK;
            }
        }
    } catch (const std::bad_alloc &) {
        return ODC_ERR_NOMEM;
    }
}

int odc_plan_runtime(const int64_t *seqlens, int n, int world, int64_t hidden, const int *device_of,
                     const int *micro_of, int64_t *t_collective, int64_t *t_odc, int64_t *busy,
                     double *bubble_collective, double *bubble_odc)
{
    if (!seqlens || !device_of || !micro_of || !t_collective || !t_odc || n < 0 || world < 1 || hidden < 0)
        return ODC_ERR_INVALID_ARG;
    try {
        std::vector<std::vector<int64_t>> cost(static_cast<size_t>(world));
        for (int i = 0; i < n; ++i) {
            const int d = device_of[i], m = micro_of[i];
            if (d < 0 || d >= world || m < 0) return ODC_ERR_INVALID_ARG;
            const int64_t c = odc_compute_cost(seqlens[i], hidden);
            if (c < 0) return seqlens[i] < 0 ? ODC_ERR_INVALID_ARG : ODC_ERR_OVERFLOW;
            std::vector<int64_t> &row = cost[static_cast<size_t>(d)];
            if (row.size() <= static_cast<size_t>(m)) row.resize(static_cast<size_t>(m) + 1, 0);
            if (c > kMax - row[static_cast<size_t>(m)]) return ODC_ERR_OVERFLOW;
            row[static_cast<size_t>(m)] += c;
        }
        size_t steps = 0;
        for (const auto &row : cost) steps = std::max(steps, row.size());
        int64_t tc = 0, to = 0, sum_busy = 0;
        for (size_t m = 0; m < steps; ++m) {
            int64_t worst = 0;
            for (const auto &row : cost)
                if (m < row.size()) worst = std::max(worst, row[m]);
            if (worst > kMax - tc) return ODC_ERR_OVERFLOW;
            tc += worst;
        }
        for (int d = 0; d < world; ++d) {
            int64_t b = 0;
            for (int64_t c : cost[static_cast<size_t>(d)]) {
                if (c > kMax - b) return ODC_ERR_OVERFLOW;
                b += c;
            }
            if (busy) busy[d] = b;
            to = std::max(to, b);
            if (b > kMax - sum_busy) return ODC_ERR_OVERFLOW;
            sum_busy += b;
        }
        *t_collective = tc;
        *t_odc = to;
        if (bubble_collective)
            *bubble_collective = tc > 0 ? 1.0 - static_cast<double>(sum_busy) / (static_cast<double>(world) * static_cast<double>(tc)) : 0.0;
        if (bubble_odc)
            *bubble_odc = to > 0 ? 1.0 - static_cast<double>(sum_busy) / (static_cast<double>(world) * static_cast<double>(to)) : 0.0;
        return ODC_OK;
    } catch (const std::bad_alloc &) {
        return ODC_ERR_NOMEM;
    }
}

}  // extern "C"
