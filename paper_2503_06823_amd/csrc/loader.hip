// Periodic, layer-after-layer expert loading for a stack of MoE layers (eMoE Section 3.3: the
// request index and the period p; Section 4: every layer's load is tied to that layer's
// computation in both directions, and layer i+1's load starts only after layer i's has finished).
//
// One process and one GPU, so the paper's per-layer lock and event become stream order:
//   * all loads of all layers are enqueued on ONE side stream, in layer order, so they are
//     serialised and never compete for the host link;
//   * per layer, a `loaded` event is recorded after its load; the compute stream waits for it
//     before the layer's forward (no stale weights);
//   * per layer, a `released` event is recorded on the compute stream after the layer's forward;
//     the layer's next load waits for it before overwriting a slot (the lock).
// The object owns the side stream, the events and the host mirrors of the slot maps; weights,
// slot buffers and device maps stay the caller's.
#include <new>
#include <vector>

#include "common.h"

using namespace emoe;

struct emoe_loader {
    struct Layer {
        emoe_loader_layer io;
        std::vector<int32_t> expert_of_slot;  // host mirror
        hipEvent_t loaded = nullptr, released = nullptr;
        bool load_pending = false;     // a load was enqueued that the compute stream has not yet been told to wait for
        bool release_recorded = false;
    };
    std::vector<Layer> layers;
    hipStream_t side = nullptr;
    int32_t period = 1;
    int64_t next_index = 0;
    int device = 0;
};

namespace {

bool all_experts_fit(const emoe_loader* ld) {
    for (const auto& l : ld->layers)
        if (l.io.desc.S != l.io.desc.E) return false;
    return true;
}

// enqueue one layer's change on the side stream
int load_layer(emoe_loader* ld, int i, int32_t n, const int32_t* experts, const int32_t* slots) {
    emoe_loader::Layer& l = ld->layers[i];
    int rc = emoe_load_experts(&l.io.desc, n, experts, slots, l.io.host_w1, l.io.host_w3, l.io.host_w2, l.io.w1_slots,
                               l.io.w3_slots, l.io.w2_slots, l.io.slot_of_expert, l.io.expert_of_slot,
                               l.expert_of_slot.data(), ld->side, l.release_recorded ? l.released : nullptr, l.loaded);
    if (rc == EMOE_OK) l.load_pending = true;
    return rc;
}

}  // namespace

extern "C" {

int emoe_prompt_action(int64_t prompt_index, int32_t period, int32_t all_experts_fit) {
    if (prompt_index < 0 || period <= 0) return EMOE_ERR_SHAPE;
    if (prompt_index == 0) return all_experts_fit ? EMOE_PROMPT_LOAD_ALL : EMOE_PROMPT_PREDICT;
    return prompt_index % period == 0 ? EMOE_PROMPT_PREDICT : EMOE_PROMPT_REUSE;
}

int emoe_loader_create(int32_t n_layers, const emoe_loader_layer* layers, int32_t period, emoe_loader** out) {
    if (!layers || !out) return EMOE_ERR_NULL;
    if (n_layers <= 0 || period <= 0) return EMOE_ERR_SHAPE;
    for (int i = 0; i < n_layers; ++i) {
        const emoe_loader_layer& l = layers[i];
        int rc = validate_desc(&l.desc);
        if (rc != EMOE_OK) return rc;
        const bool swiglu = l.desc.act == EMOE_ACT_SWIGLU;
        if (!l.host_w1 || !l.host_w2 || !l.w1_slots || !l.w2_slots || !l.slot_of_expert || !l.expert_of_slot ||
            (swiglu && (!l.host_w3 || !l.w3_slots)))
            return EMOE_ERR_NULL;
    }
    emoe_loader* ld = new (std::nothrow) emoe_loader;
    if (!ld) return EMOE_ERR_DEVICE;
    ld->period = period;
    ld->layers.resize(n_layers);
    bool ok = hipGetDevice(&ld->device) == hipSuccess &&
              hipStreamCreateWithFlags(&ld->side, hipStreamNonBlocking) == hipSuccess;  // default priority
    for (int i = 0; ok && i < n_layers; ++i) {
        emoe_loader::Layer& l = ld->layers[i];
        l.io = layers[i];
        l.expert_of_slot.assign(layers[i].desc.S, -1);
        ok = hipEventCreateWithFlags(&l.loaded, hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&l.released, hipEventDisableTiming) == hipSuccess;
    }
    if (!ok) {
        emoe_loader_destroy(ld);
        return EMOE_ERR_DEVICE;
    }
    *out = ld;
    return EMOE_OK;
}

int emoe_loader_destroy(emoe_loader* ld) {
    if (!ld) return EMOE_ERR_NULL;
    if (ld->side) (void)hipStreamSynchronize(ld->side);  // no copy may outlive the caller's buffers unnoticed
    for (auto& l : ld->layers) {
        if (l.loaded) (void)hipEventDestroy(l.loaded);
        if (l.released) (void)hipEventDestroy(l.released);
    }
    if (ld->side) (void)hipStreamDestroy(ld->side);
    delete ld;
    return EMOE_OK;
}

int emoe_loader_next_prompt(emoe_loader* ld, int64_t* prompt_index, int32_t* action) {
    if (!ld || !action) return EMOE_ERR_NULL;
    const int64_t index = ld->next_index;
    const int act = emoe_prompt_action(index, ld->period, all_experts_fit(ld) ? 1 : 0);
    if (act < 0) return act;
    if (act == EMOE_PROMPT_LOAD_ALL) {  // first prompt: every expert goes to the slot of its own number
        int32_t ids[kMaxExperts];
        for (int e = 0; e < kMaxExperts; ++e) ids[e] = e;
        for (size_t i = 0; i < ld->layers.size(); ++i) {
            int rc = load_layer(ld, (int)i, ld->layers[i].io.desc.E, ids, ids);
            if (rc != EMOE_OK) return rc;
        }
    }
    ld->next_index = index + 1;
    if (prompt_index) *prompt_index = index;
    *action = act;
    return EMOE_OK;
}

int emoe_loader_update(emoe_loader* ld, const int32_t* const* selected, const int32_t* L) {
    if (!ld || !selected || !L) return EMOE_ERR_NULL;
    const int n_layers = (int)ld->layers.size();
    // plan every layer before anything is enqueued, so a bad selection changes nothing
    std::vector<std::vector<int32_t>> ids(n_layers), slots(n_layers);
    std::vector<int32_t> count(n_layers, 0);
    for (int i = 0; i < n_layers; ++i) {
        const emoe_layer_desc& d = ld->layers[i].io.desc;
        if (!selected[i]) return EMOE_ERR_NULL;
        ids[i].resize(d.S);
        slots[i].resize(d.S);
        int rc = emoe_plan_load(d.E, d.S, d.k, ld->layers[i].expert_of_slot.data(), L[i], selected[i], ids[i].data(),
                                slots[i].data(), &count[i]);
        if (rc != EMOE_OK) return rc;
    }
    for (int i = 0; i < n_layers; ++i) {  // layer after layer on the one side stream
        if (count[i] == 0) continue;
        int rc = load_layer(ld, i, count[i], ids[i].data(), slots[i].data());
        if (rc != EMOE_OK) return rc;
    }
    return EMOE_OK;
}

int emoe_loader_layer_begin(emoe_loader* ld, int32_t layer, void* compute_stream) {
    if (!ld) return EMOE_ERR_NULL;
    if (layer < 0 || layer >= (int)ld->layers.size()) return EMOE_ERR_SHAPE;
    emoe_loader::Layer& l = ld->layers[layer];
    if (l.load_pending) {
        if (hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), l.loaded, 0) != hipSuccess)
            return EMOE_ERR_DEVICE;
        l.load_pending = false;
    }
    return EMOE_OK;
}

int emoe_loader_layer_end(emoe_loader* ld, int32_t layer, void* compute_stream) {
    if (!ld) return EMOE_ERR_NULL;
    if (layer < 0 || layer >= (int)ld->layers.size()) return EMOE_ERR_SHAPE;
    emoe_loader::Layer& l = ld->layers[layer];
    if (hipEventRecord(l.released, static_cast<hipStream_t>(compute_stream)) != hipSuccess) return EMOE_ERR_DEVICE;
    l.release_recorded = true;
    return EMOE_OK;
}

int emoe_loader_layer_ready(const emoe_loader* ld, int32_t layer, int32_t* ready) {
    if (!ld || !ready) return EMOE_ERR_NULL;
    if (layer < 0 || layer >= (int)ld->layers.size()) return EMOE_ERR_SHAPE;
    const hipError_t e = hipEventQuery(ld->layers[layer].loaded);  // never recorded counts as complete
    if (e != hipSuccess && e != hipErrorNotReady) return EMOE_ERR_DEVICE;
    *ready = e == hipSuccess ? 1 : 0;
    return EMOE_OK;
}

int emoe_loader_residents(const emoe_loader* ld, int32_t layer, int32_t* expert_of_slot_host) {
    if (!ld || !expert_of_slot_host) return EMOE_ERR_NULL;
    if (layer < 0 || layer >= (int)ld->layers.size()) return EMOE_ERR_SHAPE;
    const auto& m = ld->layers[layer].expert_of_slot;
    for (size_t s = 0; s < m.size(); ++s) expert_of_slot_host[s] = m[s];
    return EMOE_OK;
}

int emoe_loader_synchronize(emoe_loader* ld) {
    if (!ld) return EMOE_ERR_NULL;
    return hipStreamSynchronize(ld->side) == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

}  // extern "C"
