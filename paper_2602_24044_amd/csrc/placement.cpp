// Adapter placement over GPUs (paper Sec. 7: the greedy caching algorithm and its feasibility test).  Host code
// only.  The predictors of throughput and starvation are the caller's (the paper trains ML models for them); the
// library walks the allocation.
//
// What makes the walk simple: the adapter queue is the priority order, a GPU takes adapters from its head, and
// what a failed test rolls back returns to the head.  So every GPU ends up with one contiguous range of the
// priority order, only the GPU at the head of the GPU queue ever holds provisional adapters, and the whole state
// is a cursor into the order plus, for the open GPU, where its range starts, how far it is committed and its
// current A_max.  A GPU whose test fails leaves the queue for good; one whose test passes stays at its head.
#include "../../include/lora_mi355.h"

#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

namespace {

constexpr int32_t kTestingPoints[] = {8, 16, 32, 64, 96, 128, 160, 192, 256, 320, 384};
constexpr int kNumTestingPoints = sizeof(kTestingPoints) / sizeof(kTestingPoints[0]);

bool is_testing_point(int32_t count)
{
    return std::binary_search(kTestingPoints, kTestingPoints + kNumTestingPoints, count);
}

// next candidate A_max after p in the list of counts (the last one stays)
int32_t next_config(int32_t p)
{
    const int32_t* it = std::upper_bound(kTestingPoints, kTestingPoints + kNumTestingPoints, p);
    return it == kTestingPoints + kNumTestingPoints ? kTestingPoints[kNumTestingPoints - 1] : *it;
}

bool valid_workload(int32_t n, const int32_t* size, const double* rate)
{
    if (n < 0 || (n > 0 && (!size || !rate))) return false;
    for (int32_t a = 0; a < n; ++a)
        if (size[a] <= 0 || !(rate[a] >= 0.0) || !std::isfinite(rate[a])) return false;
    return true;
}

// Largest size first; inside one size the arrival rates alternate high, low, second highest, second lowest, ...
void priority_order(int32_t n, const int32_t* size, const double* rate, std::vector<int32_t>& order)
{
    std::vector<int32_t> by_rate(n);
    std::iota(by_rate.begin(), by_rate.end(), 0);
    std::sort(by_rate.begin(), by_rate.end(), [&](int32_t a, int32_t b) {
        if (size[a] != size[b]) return size[a] > size[b];
        if (rate[a] != rate[b]) return rate[a] > rate[b];
        return a < b;
    });
    order.clear();
    order.reserve(n);
    for (int32_t first = 0; first < n;) {
        int32_t last = first;
        while (last + 1 < n && size[by_rate[last + 1]] == size[by_rate[first]]) ++last;
        for (int32_t lo = first, hi = last, k = 0; lo <= hi; ++k) order.push_back(by_rate[(k & 1) ? hi-- : lo++]);
        first = last + 1;
    }
}

}  // namespace

extern "C" {

lora_status lora_priority_sorting(int32_t n_adapters, const int32_t* size, const double* rate, int32_t* order_out)
{
    if (!valid_workload(n_adapters, size, rate) || (n_adapters > 0 && !order_out)) return LORA_ERR_INVALID_ARG;
    std::vector<int32_t> order;
    priority_order(n_adapters, size, rate, order);
    std::copy(order.begin(), order.end(), order_out);
    return LORA_OK;
}

lora_status lora_place_adapters(int32_t n_adapters, const int32_t* size, const double* rate, int32_t n_gpus,
                                lora_throughput_fn predict_throughput, lora_starvation_fn predict_starvation,
                                void* user, int32_t* gpu_of, int32_t* a_max_of)
{
    if (!valid_workload(n_adapters, size, rate) || n_gpus < 0 || !predict_throughput || !predict_starvation ||
        (n_adapters > 0 && !gpu_of) || (n_gpus > 0 && !a_max_of))
        return LORA_ERR_INVALID_ARG;
    std::vector<int32_t> order;
    priority_order(n_adapters, size, rate, order);
    std::vector<int32_t> sizes(n_adapters);
    std::vector<double> rates(n_adapters);
    for (int32_t k = 0; k < n_adapters; ++k) {
        sizes[k] = size[order[k]];
        rates[k] = rate[order[k]];
    }
    std::fill(a_max_of, a_max_of + n_gpus, 0);

    // feasibility test of the open GPU's range [start, end) of the order under its configuration p:
    // returns the configuration to commit, or 0 when starvation is predicted
    auto test = [&](int32_t start, int32_t end, int32_t p) -> int32_t {
        const int32_t cnt = end - start, p_next = next_config(p);
        int32_t best = p_next;
        if (p > 0) {
            const double t_now = predict_throughput(user, cnt, sizes.data() + start, rates.data() + start, p);
            const double t_next = predict_throughput(user, cnt, sizes.data() + start, rates.data() + start, p_next);
            if (t_now > t_next) best = p;
        }
        return predict_starvation(user, cnt, sizes.data() + start, rates.data() + start, best) ? 0 : best;
    };

    std::vector<int32_t> range_end(n_gpus, 0);      // GPU g holds order[range_end[g-1], range_end[g])
    int32_t g = 0, start = 0, committed = 0, pos = 0, p = 0;
    while (pos < n_adapters) {
        if (g == n_gpus) return LORA_ERR_STARVATION;
        ++pos;                                      // provisional include
        if (!is_testing_point(pos - start)) continue;
        const int32_t best = test(start, pos, p);
        if (best > 0) {
            committed = pos;
            p = best;
        } else {                                    // roll back, the GPU leaves the queue with what it has
            a_max_of[g] = p;
            range_end[g] = committed;
            pos = start = committed;
            p = 0;
            ++g;
        }
    }
    if (pos > committed) {                          // what is still provisional on the open GPU
        const int32_t best = test(start, pos, p);
        if (best == 0) return LORA_ERR_STARVATION;
        p = best;
        committed = pos;
    }
    if (g < n_gpus) {
        a_max_of[g] = p;
        range_end[g] = committed;
        for (int32_t k = g + 1; k < n_gpus; ++k) range_end[k] = committed;
    }
    for (int32_t k = 0, gpu = 0; k < n_adapters; ++k) {
        while (k >= range_end[gpu]) ++gpu;
        gpu_of[order[k]] = gpu;
    }
    return LORA_OK;
}

}  // extern "C"
