// Request scheduler (eMoE Section 3.5: the expected-latency model of Eq. 3 and the greedy admission
// of Algorithm 1).  Host code only: a few numbers per request.
#include <algorithm>
#include <vector>

#include "common.h"

using namespace emoe;

namespace {

// n_i: running requests that will finish after request i (strictly more tokens left to generate)
int finishes_after(const std::vector<emoe_request>& run, size_t i) {
    int n = 0;
    for (size_t j = 0; j < run.size(); ++j)
        if (j != i && run[j].g_remaining > run[i].g_remaining) ++n;
    return n;
}

// Eq. 3: t_i = dE + (W + n_i G_i) c + r_i; without a new request dE = 0 and W = 0
double expected_latency(const std::vector<emoe_request>& run, size_t i, double c, const emoe_request* fresh) {
    const double d_e = fresh ? fresh->delta_e : 0.0;
    const double w = fresh ? (double)fresh->input_tokens : 0.0;
    return d_e + (w + (double)finishes_after(run, i) * (double)run[i].g_remaining) * c + run[i].run_time;
}

}  // namespace

extern "C" {

int emoe_expected_latency(int32_t n_running, const emoe_request* running, int32_t i, double c,
                          const emoe_request* new_request, double* latency) {
    if (!running || !latency) return EMOE_ERR_NULL;
    if (n_running <= 0 || i < 0 || i >= n_running) return EMOE_ERR_SHAPE;
    std::vector<emoe_request> run(running, running + n_running);
    *latency = expected_latency(run, (size_t)i, c, new_request);
    return EMOE_OK;
}

int emoe_schedule(int32_t n_waiting, const emoe_request* waiting, int32_t n_scheduled, const emoe_request* scheduled,
                  int64_t t_max, double c, int32_t* admitted, int32_t* n_admitted) {
    if (n_waiting < 0 || n_scheduled < 0) return EMOE_ERR_SHAPE;
    if (!n_admitted || (n_waiting > 0 && (!waiting || !admitted)) || (n_scheduled > 0 && !scheduled))
        return EMOE_ERR_NULL;
    std::vector<emoe_request> run(scheduled, scheduled + n_scheduled);
    int64_t tokens = 0;
    for (const auto& s : run) tokens += s.input_tokens;
    std::vector<int32_t> order(n_waiting);
    for (int32_t i = 0; i < n_waiting; ++i) order[i] = i;
    // most stringent first: the earliest first-token deadline; equal deadlines keep queue order
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return waiting[a].first_token_slo < waiting[b].first_token_slo; });
    int32_t count = 0;
    for (int32_t i : order) {
        const emoe_request& r = waiting[i];
        if (!(r.input_tokens + tokens < t_max)) continue;  // the engine cannot take its tokens now
        bool ok = true;
        for (size_t j = 0; j < run.size() && ok; ++j)
            if (expected_latency(run, j, c, nullptr) < run[j].slo)  // a request that meets its SLO now ...
                ok = expected_latency(run, j, c, &r) < run[j].slo;  // ... must still meet it
        if (!ok) continue;
        emoe_request joined = r;
        joined.run_time = 0.0;
        run.push_back(joined);
        tokens += r.input_tokens;
        admitted[count++] = i;
    }
    *n_admitted = count;
    return EMOE_OK;
}

int emoe_generation_tick(emoe_request* request, int32_t completed, double reset_fraction) {
    if (!request) return EMOE_ERR_NULL;
    if (reset_fraction < 0.0) return EMOE_ERR_SHAPE;
    int32_t g = request->g_remaining > 0 ? request->g_remaining - 1 : 0;
    if (g == 0 && !completed) {
        g = (int32_t)((double)request->g_initial * reset_fraction);
        if (g < 1) g = 1;
    }
    request->g_remaining = g;
    return EMOE_OK;
}

}  // extern "C"
