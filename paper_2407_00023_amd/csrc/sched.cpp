// Scheduling decisions on the host, as plain functions over numbers the caller holds.
//
// Sec. 3.3 ("waiting queue request ordering") and Algorithm 3: priority groups by cached share and a batch that
// takes from the groups in proportion to their numbers.  Sec. 3.2 with Algorithms 1 and 2: the load cost L + M + P
// of a GPU for a request, and the exploit / explore decision.  The regression coefficients, ImbalR and the form of
// the decode ratio are not printed in the paper: they are parameters, and the choices are stated in the header.
#include <algorithm>
#include <cstdint>
#include <deque>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "common.h"

namespace pa {

static inline int32_t group_of(int32_t cached_len, int32_t prompt_len, int32_t P) {
    if (prompt_len <= 0 || cached_len <= 0) return 0;
    const int64_t c = std::min(cached_len, prompt_len);
    return static_cast<int32_t>(std::min<int64_t>(P, c * P / prompt_len));
}

static inline double prefill_time(const pa_cost_model& m, double n) {
    return n > 0 ? m.prefill_per_token * n + m.prefill_base : 0.0;
}
static inline double decode_time(const pa_cost_model& m, double n) {
    return n > 0 ? m.decode_per_token * n + m.decode_base : 0.0;
}

// Shares of `total` in proportion to weight[p], by largest remainder; equal remainders go to the higher index.
// All in integers: share = floor(total * w / W), remainder = (total * w) mod W.
static void apportion(int64_t total, const std::vector<int64_t>& weight, std::vector<int64_t>& share) {
    const size_t n = weight.size();
    share.assign(n, 0);
    int64_t W = 0;
    for (int64_t w : weight) W += w;
    if (W == 0 || total == 0) return;
    std::vector<std::pair<int64_t, size_t>> rem(n);
    int64_t given = 0;
    for (size_t p = 0; p < n; ++p) {
        const __int128 x = static_cast<__int128>(total) * weight[p];
        share[p] = static_cast<int64_t>(x / W);
        rem[p] = {static_cast<int64_t>(x % W), p};
        given += share[p];
    }
    std::sort(rem.begin(), rem.end(), [](const auto& a, const auto& b) { return a > b; });
    for (int64_t k = 0; k < total - given; ++k) ++share[rem[static_cast<size_t>(k)].second];
}

}  // namespace pa

extern "C" int pa_priority_group(int32_t cached_len, int32_t prompt_len, int32_t P, int32_t* group) {
    PA_REQUIRE(group != nullptr && P >= 1, "pa_priority_group: bad argument (P=%d)", P);
    PA_REQUIRE(cached_len >= 0 && prompt_len >= 0, "pa_priority_group: negative length");
    *group = pa::group_of(cached_len, prompt_len, P);
    return PA_OK;
}

extern "C" int pa_priority_select(const int32_t* cached_len, const int32_t* prompt_len, int64_t n_waiting, int32_t P,
                                  int64_t n_pick, int32_t* picked, int64_t* n_picked) {
    PA_REQUIRE(n_picked != nullptr && P >= 1 && n_waiting >= 0 && n_pick >= 0, "pa_priority_select: bad argument");
    PA_REQUIRE(n_waiting <= INT32_MAX, "pa_priority_select: queue too long for int32 indices");
    PA_REQUIRE(n_waiting == 0 || (cached_len && prompt_len), "pa_priority_select: NULL queue");
    int64_t left = std::min(n_pick, n_waiting);
    PA_REQUIRE(left == 0 || picked, "pa_priority_select: picked is NULL");
    try {
        const size_t G = static_cast<size_t>(P) + 1;
        std::vector<std::vector<int32_t>> groups(G);
        for (int64_t i = 0; i < n_waiting; ++i) {
            PA_REQUIRE(cached_len[i] >= 0 && prompt_len[i] >= 0, "pa_priority_select: negative length at %lld",
                       static_cast<long long>(i));
            groups[pa::group_of(cached_len[i], prompt_len[i], P)].push_back(static_cast<int32_t>(i));
        }
        std::vector<int64_t> taken(G, 0), weight(G), share;
        while (left > 0) {
            int64_t W = 0;
            for (size_t p = 0; p < G; ++p) {
                weight[p] = taken[p] < static_cast<int64_t>(groups[p].size()) ? static_cast<int64_t>(p) : 0;
                W += weight[p];
            }
            if (W == 0) break;
            pa::apportion(left, weight, share);
            for (size_t p = 0; p < G; ++p) {
                const int64_t k = std::min(share[p], static_cast<int64_t>(groups[p].size()) - taken[p]);
                taken[p] += k;
                left -= k;
            }
        }
        taken[0] += std::min(left, static_cast<int64_t>(groups[0].size()) - taken[0]);
        int64_t n = 0;
        for (size_t p = G; p-- > 0;)
            for (int64_t k = 0; k < taken[p]; ++k) picked[n++] = groups[p][static_cast<size_t>(k)];
        *n_picked = n;
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_priority_select: out of host memory");
    }
    return PA_OK;
}

extern "C" int pa_e2_load_cost(const pa_cost_model* model, const int32_t* hist_missed_len, int64_t n_hist,
                               double avg_output_len, const int32_t* evict_tokens, const int32_t* evict_sharers,
                               int64_t n_evict, int64_t n_requests, int32_t missed_len_k, double* L, double* M,
                               double* P) {
    PA_REQUIRE(model != nullptr, "pa_e2_load_cost: model is NULL");
    PA_REQUIRE(n_hist >= 0 && (n_hist == 0 || hist_missed_len), "pa_e2_load_cost: bad history");
    PA_REQUIRE(n_evict >= 0 && (n_evict == 0 || (evict_tokens && evict_sharers)), "pa_e2_load_cost: bad eviction set");
    PA_REQUIRE(n_requests >= 0 && missed_len_k >= 0, "pa_e2_load_cost: negative count");
    double l = 0.0, m = 0.0;
    for (int64_t r = 0; r < n_hist; ++r) {
        l += pa::prefill_time(*model, hist_missed_len[r]);
        l += pa::decode_time(*model, avg_output_len);
    }
    for (int64_t j = 0; j < n_evict; ++j) {
        const double share = n_requests > 0 ? static_cast<double>(evict_sharers[j]) / static_cast<double>(n_requests) : 0.0;
        m += pa::prefill_time(*model, evict_tokens[j]) * share;
    }
    if (L) *L = l;
    if (M) *M = m;
    if (P) *P = pa::prefill_time(*model, missed_len_k);
    return PA_OK;
}

extern "C" int pa_e2_schedule(int32_t prompt_len, int32_t cached_len, const uint8_t* on_longest_node,
                              const double* cost, const double* decode_ratio, double imbal_r, int32_t n_gpus,
                              int32_t* gpu, int32_t* mode) {
    PA_REQUIRE(n_gpus >= 1 && on_longest_node && cost && decode_ratio && gpu, "pa_e2_schedule: bad argument");
    PA_REQUIRE(prompt_len >= 0 && cached_len >= 0 && cached_len <= prompt_len, "pa_e2_schedule: bad lengths %d / %d",
               cached_len, prompt_len);
    const int32_t missed_len = prompt_len - cached_len;
    if (missed_len < cached_len) {
        int32_t best = -1;
        for (int32_t i = 0; i < n_gpus; ++i)
            if (on_longest_node[i] && (best < 0 || cost[i] < cost[best])) best = i;
        if (best >= 0) {
            *gpu = best;
            if (mode) *mode = PA_EXPLOIT;
            return PA_OK;
        }
    }
    int32_t top = 0, low = 0;
    for (int32_t i = 1; i < n_gpus; ++i) {
        if (decode_ratio[i] > decode_ratio[top]) top = i;
        if (cost[i] < cost[low]) low = i;
    }
    if (decode_ratio[top] > imbal_r) {
        *gpu = top;
        if (mode) *mode = PA_EXPLORE_DECODE;
    } else {
        *gpu = low;
        if (mode) *mode = PA_EXPLORE_COST;
    }
    return PA_OK;
}

extern "C" int pa_e2_longest_piece(const int32_t* cached_len, int32_t n_gpus, uint8_t* on_longest_node) {
    PA_REQUIRE(n_gpus >= 1 && cached_len && on_longest_node, "pa_e2_longest_piece: bad argument");
    try {
        std::vector<int32_t> cuts;
        for (int32_t i = 0; i < n_gpus; ++i) {
            PA_REQUIRE(cached_len[i] >= 0, "pa_e2_longest_piece: negative length");
            if (cached_len[i] > 0) cuts.push_back(cached_len[i]);
        }
        std::sort(cuts.begin(), cuts.end());
        cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
        int32_t prev = 0, best_len = 0, best_end = -1;
        for (int32_t cut : cuts) {  // the first of the longest pieces wins
            if (cut - prev > best_len) {
                best_len = cut - prev;
                best_end = cut;
            }
            prev = cut;
        }
        for (int32_t i = 0; i < n_gpus; ++i) on_longest_node[i] = best_end >= 0 && cached_len[i] >= best_end;
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_e2_longest_piece: out of host memory");
    }
    return PA_OK;
}

struct pa_history {
    struct Gpu {
        std::deque<std::pair<int64_t, int32_t>> assigned;  // (time, missed_len)
        std::deque<std::pair<int64_t, int32_t>> finished;  // (time, output_len)
    };
    std::vector<Gpu> gpus;
    int64_t window = 0;
    pa_cost_model model{};
    std::mutex mu;
};

extern "C" int pa_history_create(int32_t n_gpus, int64_t window, const pa_cost_model* model, pa_history** out) {
    PA_REQUIRE(out && model && n_gpus >= 1 && window >= 1, "pa_history_create: bad argument");
    pa_history* h = new (std::nothrow) pa_history();
    if (!h) return pa::fail(PA_ENOMEM, "pa_history_create: out of host memory");
    try {
        h->gpus.resize(static_cast<size_t>(n_gpus));
    } catch (const std::bad_alloc&) {
        delete h;
        return pa::fail(PA_ENOMEM, "pa_history_create: out of host memory");
    }
    h->window = window;
    h->model = *model;
    *out = h;
    return PA_OK;
}

extern "C" int pa_history_destroy(pa_history* h) {
    delete h;
    return PA_OK;
}

extern "C" int pa_history_assign(pa_history* h, int32_t gpu, int64_t now, int32_t missed_len) {
    PA_REQUIRE(h && gpu >= 0 && gpu < static_cast<int32_t>(h->gpus.size()) && missed_len >= 0, "pa_history_assign: bad argument");
    std::lock_guard<std::mutex> lk(h->mu);
    auto& q = h->gpus[static_cast<size_t>(gpu)].assigned;
    PA_REQUIRE(q.empty() || now >= q.back().first, "pa_history_assign: time went backwards");
    try {
        q.emplace_back(now, missed_len);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_history_assign: out of host memory");
    }
    return PA_OK;
}

extern "C" int pa_history_complete(pa_history* h, int32_t gpu, int64_t now, int32_t output_len) {
    PA_REQUIRE(h && gpu >= 0 && gpu < static_cast<int32_t>(h->gpus.size()) && output_len >= 0, "pa_history_complete: bad argument");
    std::lock_guard<std::mutex> lk(h->mu);
    auto& q = h->gpus[static_cast<size_t>(gpu)].finished;
    PA_REQUIRE(q.empty() || now >= q.back().first, "pa_history_complete: time went backwards");
    try {
        q.emplace_back(now, output_len);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_history_complete: out of host memory");
    }
    return PA_OK;
}

extern "C" int pa_history_gpu_load(pa_history* h, int32_t gpu, int64_t now, double* L, double* decode_ratio,
                                   int64_t* n_requests, double* avg_output_len) {
    PA_REQUIRE(h && gpu >= 0 && gpu < static_cast<int32_t>(h->gpus.size()), "pa_history_gpu_load: bad argument");
    std::lock_guard<std::mutex> lk(h->mu);
    auto& g = h->gpus[static_cast<size_t>(gpu)];
    const bool bounded = now > INT64_MIN + h->window;
    const int64_t horizon = bounded ? now - h->window : INT64_MIN;  // entries at or before it are outside the window
    while (bounded && !g.assigned.empty() && g.assigned.front().first <= horizon) g.assigned.pop_front();
    while (bounded && !g.finished.empty() && g.finished.front().first <= horizon) g.finished.pop_front();
    double out_sum = 0.0;
    int64_t out_n = 0;
    for (const auto& e : g.finished)
        if (e.first <= now) {
            out_sum += e.second;
            ++out_n;
        }
    const double avg = out_n ? out_sum / static_cast<double>(out_n) : h->model.default_output_len;
    double pt = 0.0, dt = 0.0;
    int64_t n = 0;
    for (const auto& e : g.assigned)
        if (e.first <= now) {
            pt += pa::prefill_time(h->model, e.second);
            dt += pa::decode_time(h->model, avg);
            ++n;
        }
    if (L) *L = pt + dt;
    if (decode_ratio) *decode_ratio = pt + dt > 0 ? dt / (pt + dt) : 0.0;
    if (n_requests) *n_requests = n;
    if (avg_output_len) *avg_output_len = avg;
    return PA_OK;
}
