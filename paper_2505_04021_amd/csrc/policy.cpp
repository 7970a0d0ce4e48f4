// The two CPU policies that drive the balloons (host code only, no device work):
//   * slack-aware request arbitration on one GPU (paper Sec. 5.2, Alg. 2: Moore-Hodgson on
//     prefill deadlines) decides which waiting requests are admitted, and in which order;
//   * model placement by KV pressure ratio (paper Sec. 5.1, Alg. 1) decides which GPU's pool a
//     model balloons in.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <queue>
#include <vector>

#pragma GCC visibility push(default)      // the library is built with hidden visibility
#include "../../include/prism_kv.h"
#pragma GCC visibility pop

extern "C" {

int arbitrate_requests(int n, const double *arrival, const double *ttft_slo, const double *prompt_len,
                       const double *prefill_speed, double now, int32_t *accepted) {
    if (n < 0 || (n > 0 && (!arrival || !ttft_slo || !prompt_len || !prefill_speed || !accepted))) return PKV_E_ARG;
    for (int i = 0; i < n; ++i)
        if (!(prefill_speed[i] > 0.0) || !(prompt_len[i] >= 0.0) || !std::isfinite(arrival[i] + ttft_slo[i])) return PKV_E_ARG;
    std::vector<int> order((size_t)n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return arrival[a] + ttft_slo[a] < arrival[b] + ttft_slo[b]; });
    // S as a max-heap on (execution time, earliest position first) plus a removed flag per position
    struct Item {
        double e;
        int pos;
        bool operator<(const Item &o) const { return e < o.e || (e == o.e && pos > o.pos); }
    };
    std::priority_queue<Item> heap;
    std::vector<char> in_s((size_t)n, 0);
    double t = now;
    for (int k = 0; k < n; ++k) {
        const int r = order[(size_t)k];
        const double e = prompt_len[r] / prefill_speed[r];
        heap.push(Item{e, k});
        in_s[(size_t)k] = 1;
        t += e;
        if (t > arrival[r] + ttft_slo[r]) {          // the newcomer would miss: drop the longest of S
            const Item top = heap.top();
            heap.pop();
            in_s[(size_t)top.pos] = 0;
            t -= top.e;
        }
    }
    int m = 0;
    for (int k = 0; k < n; ++k)
        if (in_s[(size_t)k]) accepted[m++] = order[(size_t)k];
    return m;
}

int place_models(int n_gpus, double capacity, double tau, int n_models, const double *token_rate, const double *token_size,
                 const double *slo, const double *weight, const int32_t *current_gpu, const int32_t *tp_group,
                 int32_t *gpu_out) {
    if (n_gpus <= 0 || n_models < 0 || !(capacity > 0.0) || !(tau >= 0.0)) return PKV_E_ARG;
    if (n_models > 0 && (!token_rate || !token_size || !slo || !weight || !gpu_out)) return PKV_E_ARG;
    for (int j = 0; j < n_models; ++j) {
        if (!(slo[j] > 0.0) || !(token_rate[j] >= 0.0) || !(token_size[j] >= 0.0) || !(weight[j] >= 0.0)) return PKV_E_ARG;
        if (current_gpu && (current_gpu[j] < -1 || current_gpu[j] >= n_gpus)) return PKV_E_ARG;
    }
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<double> demand((size_t)n_models);
    for (int j = 0; j < n_models; ++j) demand[(size_t)j] = token_rate[j] * token_size[j] / slo[j];
    std::vector<int> order((size_t)n_models);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return demand[(size_t)a] > demand[(size_t)b]; });
    std::vector<double> shared((size_t)n_gpus, capacity), rate((size_t)n_gpus, 0.0);
    auto kvpr = [&](int i) { return shared[(size_t)i] > 0.0 ? rate[(size_t)i] / shared[(size_t)i] : inf; };
    for (int k = 0; k < n_models; ++k) {
        const int j = order[(size_t)k];
        // GPUs that already hold a part of the same tensor-parallel model are not candidates
        auto taken = [&](int i) {
            if (!tp_group || tp_group[j] < 0) return false;
            for (int q = 0; q < k; ++q) {
                const int o = order[(size_t)q];
                if (tp_group[o] == tp_group[j] && gpu_out[o] == i) return true;
            }
            return false;
        };
        int best = -1;
        double best_r = inf;
        for (int i = 0; i < n_gpus; ++i) {
            if (taken(i)) continue;
            const double r = kvpr(i);
            if (best < 0 || r < best_r) { best = i; best_r = r; }
        }
        if (best < 0) return PKV_E_RANGE;            // more parts than GPUs
        int target = best;
        const int cur = current_gpu ? current_gpu[j] : -1;
        if (cur >= 0 && !taken(cur)) {
            const double cur_r = kvpr(cur);
            if (!(cur_r - best_r > tau)) target = cur;        // the move is not worth a migration
        }
        gpu_out[j] = target;
        rate[(size_t)target] += demand[(size_t)j];
        shared[(size_t)target] -= weight[j];
    }
    return n_models;
}

}  // extern "C"
