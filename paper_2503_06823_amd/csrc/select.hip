// Choice of the resident experts of one layer (eMoE Section 3.4, Eq. 2; Section 3.2.2, last
// paragraph).  Host code only: the inputs are a handful of numbers per expert and per request, and
// the result (a list of (expert, slot) pairs) is what emoe_load_experts consumes.
#include <algorithm>
#include <vector>

#include "common.h"

using namespace emoe;

extern "C" {

int emoe_expected_tokens(int32_t E, int32_t n_tasks, const double* freq, int32_t n_requests,
                         const int32_t* request_task, const int64_t* request_tokens, const double* w_out,
                         const int32_t* sensitive, double* expected) {
    if (E <= 0 || n_tasks <= 0 || n_requests < 0) return EMOE_ERR_SHAPE;
    if (!freq || !w_out || !sensitive || !expected || (n_requests > 0 && (!request_task || !request_tokens)))
        return EMOE_ERR_NULL;
    for (int32_t j = 0; j < n_requests; ++j)
        if (request_task[j] < 0 || request_task[j] >= n_tasks || request_tokens[j] < 0) return EMOE_ERR_SHAPE;
    // per task type: running requests T and their input tokens sum_j W_j
    std::vector<double> sum_w(n_tasks, 0.0);
    std::vector<int64_t> count(n_tasks, 0);
    for (int32_t j = 0; j < n_requests; ++j) {
        sum_w[request_task[j]] += (double)request_tokens[j];
        count[request_task[j]] += 1;
    }
    for (int32_t i = 0; i < E; ++i) expected[i] = 0.0;
    for (int32_t t = 0; t < n_tasks; ++t) {  // N_i = (sum_j W_j + T W_o) s f_i, added over the task types
        const double load = sum_w[t] + (double)count[t] * w_out[t];
        const double s = sensitive[t] ? 1.0 : 0.0;
        for (int32_t i = 0; i < E; ++i) expected[i] += load * s * freq[(size_t)t * E + i];
    }
    return EMOE_OK;
}

int emoe_select_experts(int32_t E, const double* expected, int32_t L, int32_t* selected) {
    if (E <= 0 || L <= 0 || L > E) return EMOE_ERR_SHAPE;
    if (!expected || !selected) return EMOE_ERR_NULL;
    std::vector<int32_t> order(E);
    for (int32_t i = 0; i < E; ++i) order[i] = i;
    // descending expected tokens; equal values keep ascending index order
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return expected[a] > expected[b]; });
    for (int32_t i = 0; i < L; ++i) selected[i] = order[i];
    return EMOE_OK;
}

int emoe_plan_load(int32_t E, int32_t S, int32_t k, const int32_t* expert_of_slot_host, int32_t L,
                   const int32_t* selected, int32_t* expert_ids, int32_t* slot_ids, int32_t* n) {
    if (E <= 0 || S <= 0 || S > E || k <= 0 || L <= 0) return EMOE_ERR_SHAPE;
    if (!expert_of_slot_host || !selected || !expert_ids || !slot_ids || !n) return EMOE_ERR_NULL;
    if (L > S || L < k) return EMOE_ERR_RESIDENT;  // does not fit the slots / would leave fewer than k resident
    std::vector<char> keep(E, 0), resident(E, 0);
    for (int32_t i = 0; i < L; ++i) {
        if (selected[i] < 0 || selected[i] >= E || keep[selected[i]]) return EMOE_ERR_RESIDENT;
        keep[selected[i]] = 1;
    }
    std::vector<int32_t> eos(expert_of_slot_host, expert_of_slot_host + S);
    for (int32_t s = 0; s < S; ++s) {
        if (eos[s] < -1 || eos[s] >= E) return EMOE_ERR_RESIDENT;
        if (eos[s] >= 0) {
            if (resident[eos[s]]) return EMOE_ERR_RESIDENT;
            resident[eos[s]] = 1;
        }
    }
    int32_t count = 0;
    int32_t next = 0;  // slots below `next` hold selected experts
    for (int32_t i = 0; i < L; ++i) {  // the selection is in descending workload order: higher workload loads first
        const int32_t e = selected[i];
        if (resident[e]) continue;
        while (next < S && eos[next] >= 0 && keep[eos[next]]) ++next;
        if (next >= S) return EMOE_ERR_RESIDENT;  // cannot happen with L <= S
        eos[next] = e;
        expert_ids[count] = e;
        slot_ids[count] = next;
        ++count;
    }
    for (int32_t s = 0; s < S; ++s) {  // experts that were not selected leave the GPU
        if (eos[s] >= 0 && !keep[eos[s]]) {
            expert_ids[count] = -1;
            slot_ids[count] = s;
            ++count;
        }
    }
    *n = count;
    return EMOE_OK;
}

}  // extern "C"
