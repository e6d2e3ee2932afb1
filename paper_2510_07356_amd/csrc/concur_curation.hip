// Host-only implementation of include/concur_curation.h (Equations 1-3, Sections 3.5, 4.2 and 6 of
// the paper).  Compiled into the same shared library; touches no device.
#include "../../include/concur_curation.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <unordered_map>
#include <vector>

extern "C" {

int concur_speedup(int64_t n, const double* t_torch, const double* t_kernel, const uint8_t* correct,
                   double* speedup) {
    if (n < 0 || !t_torch || !t_kernel || !correct || !speedup) return -1;
    for (int64_t i = 0; i < n; ++i) {
        if (correct[i] && !(t_kernel[i] > 0.0)) return -1;
        speedup[i] = correct[i] ? t_torch[i] / t_kernel[i] : 0.0;
    }
    return 0;
}

double concur_fast_p(int64_t n_tasks, const double* speedup, double p) {
    if (n_tasks <= 0 || !speedup) return std::numeric_limits<double>::quiet_NaN();
    int64_t hits = 0;
    for (int64_t i = 0; i < n_tasks; ++i) hits += speedup[i] > p;
    return (double)hits / (double)n_tasks;
}

double concur_exec_pass_at_k(int64_t n_tasks, int32_t k, const uint8_t* correct) {
    if (n_tasks <= 0 || k <= 0 || !correct) return std::numeric_limits<double>::quiet_NaN();
    int64_t pass = 0;
    for (int64_t t = 0; t < n_tasks; ++t) {
        bool any = false;
        for (int32_t j = 0; j < k; ++j) any = any || correct[t * k + j] != 0;
        pass += any;
    }
    return (double)pass / (double)n_tasks;
}

double concur_fast1_pass_at_k(int64_t n_tasks, int32_t k, const double* speedup) {
    if (n_tasks <= 0 || k <= 0 || !speedup) return std::numeric_limits<double>::quiet_NaN();
    int64_t pass = 0;
    for (int64_t t = 0; t < n_tasks; ++t) {
        bool any = false;
        for (int32_t j = 0; j < k; ++j) any = any || speedup[t * k + j] > 1.0;
        pass += any;
    }
    return (double)pass / (double)n_tasks;
}

double concur_arl(int64_t n_tasks, int32_t m, const int32_t* lengths) {
    if (n_tasks <= 0 || m <= 0 || !lengths) return std::numeric_limits<double>::quiet_NaN();
    long double sum = 0.0L;
    for (int64_t i = 0; i < n_tasks * m; ++i) sum += lengths[i];
    return (double)(sum / ((long double)n_tasks * m));
}

int concur_difficulty_bins(int64_t n_tasks, const double* task_arl, double lo, double hi, int32_t* bin) {
    if (n_tasks < 0 || !task_arl || !bin || !(lo <= hi)) return -1;
    for (int64_t i = 0; i < n_tasks; ++i) bin[i] = task_arl[i] < lo ? 0 : (task_arl[i] > hi ? 2 : 1);
    return 0;
}

int64_t concur_select(int64_t n, const int64_t* task_id, const double* speedup, const int32_t* reasoning_len,
                      const uint8_t* single_op, double speedup_threshold, int64_t single_op_quota,
                      uint8_t* selected, int64_t counts[3]) {
    if (n < 0 || !task_id || !speedup || !reasoning_len || !single_op || !selected || single_op_quota < 0) return -1;
    std::fill(selected, selected + n, (uint8_t)0);
    // (a) shortest trace of each task, kept iff it also has the task's highest speedup
    struct Best { int64_t shortest; double max_speedup; };
    std::unordered_map<int64_t, Best> tasks;
    tasks.reserve((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        auto it = tasks.find(task_id[i]);
        if (it == tasks.end()) {
            tasks.emplace(task_id[i], Best{i, speedup[i]});
        } else {
            if (reasoning_len[i] < reasoning_len[it->second.shortest]) it->second.shortest = i;
            it->second.max_speedup = std::max(it->second.max_speedup, speedup[i]);
        }
    }
    for (const auto& kv : tasks) {
        const int64_t i = kv.second.shortest;
        if (speedup[i] > 0.0 && speedup[i] >= kv.second.max_speedup) selected[i] |= 1;
    }
    // (b) high-performance kernels
    for (int64_t i = 0; i < n; ++i)
        if (speedup[i] > speedup_threshold) selected[i] |= 2;
    // (c) correct single-operator samples not yet taken, shortest reasoning first
    std::vector<int64_t> pool;
    for (int64_t i = 0; i < n; ++i)
        if (single_op[i] && speedup[i] > 0.0 && selected[i] == 0) pool.push_back(i);
    std::stable_sort(pool.begin(), pool.end(),
                     [&](int64_t x, int64_t y) { return reasoning_len[x] < reasoning_len[y]; });
    for (int64_t j = 0; j < (int64_t)pool.size() && j < single_op_quota; ++j) selected[pool[j]] |= 4;
    int64_t ca = 0, cb = 0, cc = 0, total = 0;
    for (int64_t i = 0; i < n; ++i) {
        ca += (selected[i] & 1) != 0;
        cb += (selected[i] & 3) == 2;
        cc += (selected[i] & 4) != 0;
        total += selected[i] != 0;
    }
    if (counts) { counts[0] = ca; counts[1] = cb; counts[2] = cc; }
    return total;
}

}  // extern "C"
