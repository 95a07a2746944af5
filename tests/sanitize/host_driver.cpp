// Drives every host-only path of libemoe (argument validation of all entry points, workspace
// arithmetic, Section 3.4 selection, Section 3.3 prompt rule, Section 3.5 scheduler) with seeded
// random and deliberately bad arguments.  Built by tests/test_sanitize.py from the library's sources
// with AddressSanitizer and UndefinedBehaviorSanitizer on the host side and run without a GPU: no
// path taken here enqueues anything.  Exit status 0 = every invariant held and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "emoe.h"

static uint64_t rng_state = 0x2503068230ull;
static uint32_t rnd() {  // splitmix64, upper half
    uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return (uint32_t)((z ^ (z >> 31)) >> 32);
}
static int rint_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
static double runit() { return rnd() / 4294967296.0; }

#define REQUIRE(cond)                                                        \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                    \
        }                                                                    \
    } while (0)

static void selection_round() {
    const int E = rint_in(1, 64), n_tasks = rint_in(1, 6), n_req = rint_in(0, 40);
    std::vector<double> freq((size_t)n_tasks * E), w_out(n_tasks), expected(E);
    std::vector<int32_t> sens(n_tasks), task(n_req);
    std::vector<int64_t> tokens(n_req);
    for (auto& f : freq) f = rnd() % 4 == 0 ? 0.0 : runit();  // repeated zeros: equal expected values
    for (int t = 0; t < n_tasks; ++t) { w_out[t] = rint_in(0, 300); sens[t] = rnd() % 3 != 0; }
    for (int j = 0; j < n_req; ++j) { task[j] = rint_in(0, n_tasks - 1); tokens[j] = rint_in(0, 4000); }
    REQUIRE(emoe_expected_tokens(E, n_tasks, freq.data(), n_req, task.data(), tokens.data(), w_out.data(), sens.data(),
                                 expected.data()) == EMOE_OK);
    for (double v : expected) REQUIRE(v >= 0.0);
    const int L = rint_in(1, E);
    std::vector<int32_t> selected(L);
    REQUIRE(emoe_select_experts(E, expected.data(), L, selected.data()) == EMOE_OK);
    std::vector<char> seen(E, 0);
    for (int i = 0; i < L; ++i) {
        REQUIRE(selected[i] >= 0 && selected[i] < E && !seen[selected[i]]);
        seen[selected[i]] = 1;
        if (i > 0) {
            const double a = expected[selected[i - 1]], b = expected[selected[i]];
            REQUIRE(a > b || (a == b && selected[i - 1] < selected[i]));
        }
    }
    // plan against a random resident map
    const int S = rint_in(L, E), k = rint_in(1, L);
    std::vector<int32_t> eos(S, -1), ids(S), slots(S);
    std::vector<char> used(E, 0);
    for (int s = 0; s < S; ++s)
        if (rnd() % 3 != 0) {
            int e = rint_in(0, E - 1);
            if (!used[e]) { used[e] = 1; eos[s] = e; }
        }
    int32_t n = -1;
    REQUIRE(emoe_plan_load(E, S, k, eos.data(), L, selected.data(), ids.data(), slots.data(), &n) == EMOE_OK);
    REQUIRE(n >= 0 && n <= S);
    std::vector<char> slot_named(S, 0);
    std::vector<int32_t> after(eos);
    for (int i = 0; i < n; ++i) {
        REQUIRE(slots[i] >= 0 && slots[i] < S && !slot_named[slots[i]]);
        slot_named[slots[i]] = 1;
        REQUIRE(ids[i] >= -1 && ids[i] < E);
        after[slots[i]] = ids[i];
    }
    int resident = 0;  // afterwards exactly the selection is resident
    for (int s = 0; s < S; ++s)
        if (after[s] >= 0) { REQUIRE(seen[after[s]]); ++resident; }
    REQUIRE(resident == L);
    // bad arguments
    REQUIRE(emoe_plan_load(E, S, k, eos.data(), S + 1, selected.data(), ids.data(), slots.data(), &n) != EMOE_OK);
    REQUIRE(emoe_select_experts(E, expected.data(), E + 1, selected.data()) == EMOE_ERR_SHAPE);
    REQUIRE(emoe_select_experts(E, nullptr, L, selected.data()) == EMOE_ERR_NULL);
    if (n_req > 0) {
        task[0] = n_tasks;
        REQUIRE(emoe_expected_tokens(E, n_tasks, freq.data(), n_req, task.data(), tokens.data(), w_out.data(),
                                     sens.data(), expected.data()) == EMOE_ERR_SHAPE);
    }
}

static emoe_request random_request() {
    emoe_request r{};
    r.input_tokens = rint_in(1, 2000);
    r.g_initial = rint_in(1, 500);
    r.g_remaining = rint_in(0, r.g_initial);
    r.slo = runit() * 50.0;
    r.first_token_slo = rnd() % 4 == 0 ? 1.0 : runit() * 5.0;  // repeated values: equal stringency
    r.run_time = runit() * 10.0;
    r.delta_e = rnd() % 2 ? runit() : 0.0;
    return r;
}

static void scheduling_round() {
    const int nw = rint_in(0, 30), ns = rint_in(0, 20);
    std::vector<emoe_request> waiting(nw), sched(ns);
    for (auto& r : waiting) r = random_request();
    for (auto& r : sched) r = random_request();
    std::vector<int32_t> admitted(nw > 0 ? nw : 1);
    int32_t n = -1;
    const int64_t t_max = rint_in(0, 40000);
    REQUIRE(emoe_schedule(nw, waiting.data(), ns, sched.data(), t_max, 0.001 * runit(), admitted.data(), &n) == EMOE_OK);
    REQUIRE(n >= 0 && n <= nw);
    int64_t tokens = 0;
    for (const auto& r : sched) tokens += r.input_tokens;
    std::vector<char> seen(nw > 0 ? nw : 1, 0);
    for (int i = 0; i < n; ++i) {
        REQUIRE(admitted[i] >= 0 && admitted[i] < nw && !seen[admitted[i]]);
        seen[admitted[i]] = 1;
        tokens += waiting[admitted[i]].input_tokens;
        if (i > 0) REQUIRE(waiting[admitted[i - 1]].first_token_slo <= waiting[admitted[i]].first_token_slo);
    }
    REQUIRE(n == 0 || tokens < t_max);
    if (ns > 0) {
        double lat = -1.0;
        const int i = rint_in(0, ns - 1);
        REQUIRE(emoe_expected_latency(ns, sched.data(), i, 0.01, nw > 0 ? &waiting[0] : nullptr, &lat) == EMOE_OK);
        REQUIRE(lat >= sched[i].run_time);
        REQUIRE(emoe_expected_latency(ns, sched.data(), ns, 0.01, nullptr, &lat) == EMOE_ERR_SHAPE);
    }
    emoe_request r = random_request();
    for (int step = 0; step < 3 * r.g_initial + 3; ++step) {
        REQUIRE(emoe_generation_tick(&r, 0, 0.05) == EMOE_OK);
        REQUIRE(r.g_remaining >= 1 && r.g_remaining <= r.g_initial);
    }
    r.g_remaining = 1;
    REQUIRE(emoe_generation_tick(&r, 1, 0.05) == EMOE_OK && r.g_remaining == 0);
    REQUIRE(emoe_generation_tick(nullptr, 0, 0.05) == EMOE_ERR_NULL);
    REQUIRE(emoe_schedule(nw, waiting.data(), ns, sched.data(), t_max, 0.0, admitted.data(), nullptr) == EMOE_ERR_NULL);
}

// Every forward-path entry point must reject a bad description or a missing pointer on the host,
// before any HIP call (this process has no GPU to call).
static void validation_round() {
    emoe_layer_desc d{};
    d.T = rint_in(0, 2000); d.d_model = 8 * rint_in(1, 600); d.d_ff = 8 * rint_in(1, 1000);
    d.E = rint_in(1, 64); d.S = rint_in(1, d.E); d.k = rint_in(1, d.S);
    d.dtype = rnd() % 2; d.act = rnd() % 2;
    size_t pws = 0, fws = 0;
    REQUIRE(emoe_workspace_bytes(&d, &pws, &fws) == EMOE_OK);
    REQUIRE(pws >= (size_t)d.S * 4 && pws % 256 == 0);
    REQUIRE(fws >= (size_t)d.T * d.k * d.d_ff * (d.dtype == EMOE_F32 ? 4 : 2));
    int32_t dummy_i[4] = {0, 0, 0, 0};
    float dummy_f[4] = {0, 0, 0, 0};
    void* p = dummy_i;  // never dereferenced: every call below fails validation first
    REQUIRE(emoe_route(&d, nullptr, p, nullptr, dummy_i, dummy_i, dummy_f, nullptr) == EMOE_ERR_NULL);
    REQUIRE(emoe_route_observe(&d, p, p, nullptr, dummy_i, dummy_i, dummy_f, nullptr, nullptr) == EMOE_ERR_NULL);
    REQUIRE(emoe_permute(&d, p, dummy_i, dummy_i, dummy_i, dummy_i, dummy_i, dummy_i, p, p, pws - 1, nullptr) ==
            EMOE_ERR_WORKSPACE);
    REQUIRE(emoe_permute(&d, nullptr, dummy_i, dummy_i, dummy_i, dummy_i, dummy_i, dummy_i, p, p, pws, nullptr) ==
            EMOE_ERR_NULL);
    REQUIRE(emoe_permute_static(&d, nullptr, dummy_i, dummy_i, dummy_i, dummy_i, dummy_i, dummy_i, p, nullptr) ==
            EMOE_ERR_NULL);
    const void* w3 = d.act == EMOE_ACT_SWIGLU ? p : nullptr;
    REQUIRE(emoe_expert_ffn(&d, p, dummy_i, p, w3, p, p, p, fws - 1, nullptr) == EMOE_ERR_WORKSPACE);
    REQUIRE(emoe_expert_ffn(&d, p, dummy_i, p, d.act == EMOE_ACT_SWIGLU ? nullptr : p, p, p, p, fws, nullptr) != EMOE_OK);
    REQUIRE(emoe_expert_ffn_pass(&d, 3, p, dummy_i, p, w3, p, p, p, fws, nullptr) == EMOE_ERR_SHAPE);
    REQUIRE(emoe_expert_ffn_gather(&d, p, nullptr, dummy_i, p, w3, p, p, p, fws, nullptr) == EMOE_ERR_NULL);
    REQUIRE(emoe_expert_ffn_gather_pass(&d, 0, p, dummy_i, dummy_i, p, w3, p, p, p, fws, nullptr) == EMOE_ERR_SHAPE);
    REQUIRE(emoe_combine(&d, p, dummy_i, nullptr, p, nullptr) == EMOE_ERR_NULL);
    REQUIRE(emoe_layer_forward(&d, p, p, nullptr, dummy_i, p, w3, p, dummy_i, dummy_f, dummy_i, dummy_i, dummy_i, dummy_i,
                               p, p, p, pws, p, fws - 1, nullptr) == EMOE_ERR_WORKSPACE);
    emoe_layer_desc bad = d;
    switch (rnd() % 6) {
        case 0: bad.E = 65; bad.S = bad.S; break;
        case 1: bad.k = bad.S + 1; break;
        case 2: bad.d_model += 4; break;
        case 3: bad.dtype = 7; break;
        case 4: bad.T = -1; break;
        default: bad.S = bad.E + 1; break;
    }
    REQUIRE(emoe_workspace_bytes(&bad, &pws, &fws) != EMOE_OK);
    REQUIRE(emoe_route(&bad, p, p, nullptr, dummy_i, dummy_i, dummy_f, nullptr) != EMOE_OK);
    // emoe_load_experts: validation against the caller's mirror happens before anything is enqueued
    const int S = d.S, E = d.E;
    std::vector<int32_t> mirror(S, -1), before;
    std::vector<const void*> hw(E, p);
    std::vector<int32_t> ids = {E}, slots = {0};  // expert id out of range
    before = mirror;
    REQUIRE(emoe_load_experts(&d, 1, ids.data(), slots.data(), hw.data(), hw.data(), hw.data(), p, p, p, dummy_i, dummy_i,
                              mirror.data(), nullptr, nullptr, nullptr) == EMOE_ERR_RESIDENT);
    ids[0] = 0; slots[0] = S;                      // slot out of range
    REQUIRE(emoe_load_experts(&d, 1, ids.data(), slots.data(), hw.data(), hw.data(), hw.data(), p, p, p, dummy_i, dummy_i,
                              mirror.data(), nullptr, nullptr, nullptr) == EMOE_ERR_RESIDENT);
    if (d.k > 1) {                                 // one expert is fewer than k residents
        slots[0] = 0;
        REQUIRE(emoe_load_experts(&d, 1, ids.data(), slots.data(), hw.data(), hw.data(), hw.data(), p, p, p, dummy_i,
                                  dummy_i, mirror.data(), nullptr, nullptr, nullptr) == EMOE_ERR_RESIDENT);
    }
    REQUIRE(mirror == before);
    REQUIRE(emoe_status_string(EMOE_ERR_RESIDENT) != nullptr && emoe_status_string(12345) != nullptr);
    // Section 3.3's rule
    REQUIRE(emoe_prompt_action(0, 40, 1) == EMOE_PROMPT_LOAD_ALL);
    REQUIRE(emoe_prompt_action(0, 40, 0) == EMOE_PROMPT_PREDICT);
    const int64_t idx = 1 + rnd() % 1000;
    const int period = rint_in(1, 60);
    REQUIRE(emoe_prompt_action(idx, period, 1) == (idx % period == 0 ? EMOE_PROMPT_PREDICT : EMOE_PROMPT_REUSE));
    REQUIRE(emoe_prompt_action(-1, period, 1) < 0 && emoe_prompt_action(idx, 0, 1) < 0);
}

int main(int argc, char** argv) {
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 300;
    for (int i = 0; i < rounds; ++i) {
        selection_round();
        scheduling_round();
        validation_round();
    }
    std::printf("host driver: %d rounds ok\n", rounds);
    return 0;
}
