// C ABI of libemoe: host-side argument checks, workspace layout, dispatch to the kernels.
// The operations are documented in include/emoe.h.
#include <string.h>

#include "common.h"

#include <mutex>

namespace emoe {

namespace {
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

constexpr int kMaxDevices = 64;
std::mutex shape_mutex;
DeviceShape shape_of_device[kMaxDevices] = {};
size_t elem_bytes(const emoe_layer_desc& d) { return d.dtype == EMOE_F32 ? 4 : 2; }
}  // namespace

hipError_t device_shape(DeviceShape* out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(shape_mutex);
    DeviceShape& s = shape_of_device[dev];
    if (s.cus == 0) {
        int cus = 0, xcds = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds < 1) xcds = 1;
        if (cus < 1) return hipErrorInvalidDevice;
        if (cus % xcds != 0) xcds = 1;  // ids then map to themselves
        int groups = cus < kMaxGroups ? cus : kMaxGroups;
        groups -= groups % xcds;
        if (groups < xcds) { xcds = 1; groups = cus < kMaxGroups ? cus : kMaxGroups; }
        s.xcds = xcds;
        s.groups = groups;
        s.cus = cus;
    }
    *out = s;
    return hipSuccess;
}

int validate_desc(const emoe_layer_desc* d) {
    if (d == nullptr) return EMOE_ERR_NULL;
    if (d->dtype != EMOE_F32 && d->dtype != EMOE_BF16) return EMOE_ERR_UNSUPPORTED;
    if (d->act != EMOE_ACT_SWIGLU && d->act != EMOE_ACT_RELU) return EMOE_ERR_UNSUPPORTED;
    if (d->T < 0 || d->d_model <= 0 || d->d_ff <= 0 || d->E <= 0 || d->k <= 0 || d->S <= 0) return EMOE_ERR_SHAPE;
    if (d->k > d->S || d->S > d->E) return EMOE_ERR_SHAPE;
    if (d->E > kMaxExperts) return EMOE_ERR_UNSUPPORTED;
    if (d->d_model % 8 != 0 || d->d_ff % 8 != 0) return EMOE_ERR_UNSUPPORTED;
    const long long A = (long long)d->T * d->k;
    const long long widest = d->d_model > d->d_ff ? d->d_model : d->d_ff;
    // 32-bit byte offsets into the activation buffers, with room for one more row past the end (the
    // kernels address "out of range" as buffer size + an offset within a row)
    if ((A + 2) * widest > (1ll << 31)) return EMOE_ERR_SHAPE;
    // and into one slot's weight matrix
    if ((long long)d->d_model * d->d_ff >= (1ll << 31)) return EMOE_ERR_SHAPE;
    return EMOE_OK;
}

PermuteWs permute_ws_layout(const emoe_layer_desc& d) {
    PermuteWs w;
    const long long A = (long long)d.T * d.k;
    const long long n_blocks = (A + kPermuteChunk - 1) / kPermuteChunk;
    w.block_counts = 0;
    w.total = align256((size_t)(n_blocks > 0 ? n_blocks : 1) * d.S * sizeof(int32_t));
    return w;
}

FfnWs ffn_ws_layout(const emoe_layer_desc& d) {
    FfnWs w;
    const size_t A = (size_t)d.T * d.k;
    w.h = 0;
    w.partials = align256((A > 0 ? A : 1) * d.d_ff * elem_bytes(d));
    w.total = w.partials;
    if (d.dtype == EMOE_BF16 && ffn_bf16_path(d) == kFfnTiled) w.total += kTiledPartialBytes;
    if (d.dtype == EMOE_BF16 && ffn_bf16_path(d) == kFfnMid) w.total += kMidPartialBytes;
    return w;
}

// Row counts live on the device, so the choice goes by the average number of rows per slot.
// Few rows per slot: reading the weights dominates, use the streaming kernels.  They take 32 rows
// of a slot per pass over its weights, so they win only while every slot fits one pass, and lose
// a fifth as soon as one does not: at the Mixtral shape, 8 slots of 16-31 rows 454 us against the
// 64-row tiles' 455 us, but 16-35 rows 535 against 450 us; 6 slots of 15-26 rows 357 against
// 361 us, 18-35 rows 428 against 369 us.  With 22 rows per slot on average a slot of more than 32
// is rare under even routing.  Up to kMidRowsPerSlot rows per slot the tiles of 128 (up to 48: 64)
// token rows are used: they keep more weight bytes in flight than the tiles of 256 token rows
// (Mixtral shape, 8 slots, whole FFN: 493 us against the large tiles' 538 us at 64 rows per slot,
// 527 against 552 us at 96), but they lose once many slots need a second tile (128 rows per slot:
// 723 against 563 us).
constexpr long long kStreamRowsPerSlot = 22;
constexpr long long kMidRowsPerSlot = 100;
// A small layer (all resident slots' weights stream in some 60 us) is bound by how well its tiles
// fill the chip, not by the weight stream, and around 256 rows per slot the 128-row tiles fill it
// better: half the slots then need a second 256-row tile for a few rows.  Measured (FFN, us, 256-row
// against 128-row tiles): d = 768, f = 3072, 16 slots of 214-291 rows 120 / 86; 32 slots of 195-315
// rows 177 / 145; d = 2048, f = 1408, 8 slots of 182-206 rows 100 / 72; d = 2048, f = 8192, 2 slots
// of 256 rows 134 / 102, 3 slots of 238-266 rows 172 / 148.  Below about 170 rows per slot the
// 256-row tiles win or are level there too (16 slots of 99-148 rows: 104 / 123), and so they do at
// any number of rows once the weights are large (Mixtral shape, 8 slots of 232-278 rows: 863 / 998).
constexpr long long kSmallLayerWeightBytes = 320ll << 20;
constexpr long long kSmallLayerMidFrom = 170, kSmallLayerMidTo = 300;  // rows per slot
FfnPath ffn_bf16_path(const emoe_layer_desc& d) {
    const long long A = (long long)d.T * d.k;
    if (A <= kStreamRowsPerSlot * d.S) return kFfnStream;
    if (A <= kMidRowsPerSlot * d.S) return kFfnMid;
    const long long weight_bytes = (long long)d.S * (d.act == EMOE_ACT_SWIGLU ? 3 : 2) * d.d_model * d.d_ff * 2;
    if (weight_bytes <= kSmallLayerWeightBytes && A >= kSmallLayerMidFrom * d.S && A <= kSmallLayerMidTo * d.S)
        return kFfnMid;
    return kFfnTiled;
}

}  // namespace emoe

using namespace emoe;

extern "C" {

const char* emoe_status_string(int status) {
    switch (status) {
        case EMOE_OK: return "ok";
        case EMOE_ERR_NULL: return "a required pointer is NULL";
        case EMOE_ERR_SHAPE: return "an extent is out of range or inconsistent";
        case EMOE_ERR_UNSUPPORTED: return "unsupported dtype, activation or extent";
        case EMOE_ERR_RESIDENT: return "bad expert or slot id, duplicate, or fewer than k resident experts";
        case EMOE_ERR_WORKSPACE: return "workspace missing or too small";
        case EMOE_ERR_DEVICE: return "a HIP runtime call failed";
        default: return "unknown status";
    }
}

int emoe_workspace_bytes(const emoe_layer_desc* desc, size_t* permute_ws_bytes, size_t* ffn_ws_bytes) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (permute_ws_bytes) *permute_ws_bytes = permute_ws_layout(*desc).total;
    if (ffn_ws_bytes) *ffn_ws_bytes = ffn_ws_layout(*desc).total;
    return EMOE_OK;
}

int emoe_route(const emoe_layer_desc* desc, const void* x, const void* w_gate, const float* gate_bias,
               const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight, void* stream) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!x || !w_gate || !slot_of_expert || !topk_expert || !topk_weight) return EMOE_ERR_NULL;
    if (desc->T == 0) return EMOE_OK;
    hipError_t e = launch_route(*desc, x, w_gate, gate_bias, slot_of_expert, topk_expert, topk_weight, nullptr,
                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_route_observe(const emoe_layer_desc* desc, const void* x, const void* w_gate, const float* gate_bias,
                       const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                       int64_t* expert_tokens, void* stream) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!x || !w_gate || !slot_of_expert || !topk_expert || !topk_weight || !expert_tokens) return EMOE_ERR_NULL;
    if (desc->T == 0) return EMOE_OK;
    hipError_t e = launch_route(*desc, x, w_gate, gate_bias, slot_of_expert, topk_expert, topk_weight,
                                reinterpret_cast<unsigned long long*>(expert_tokens),
                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_permute(const emoe_layer_desc* desc, const void* x, const int32_t* topk_expert,
                 const int32_t* slot_of_expert, int32_t* slot_counts, int32_t* slot_offsets, int32_t* perm,
                 int32_t* inv_perm, void* x_perm, void* ws, size_t ws_bytes, void* stream) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!topk_expert || !slot_of_expert || !slot_counts || !slot_offsets || !perm || !inv_perm) return EMOE_ERR_NULL;
    if (x_perm && !x) return EMOE_ERR_NULL;  // x_perm == NULL: indices only, no row copy
    if (!ws || ws_bytes < permute_ws_layout(*desc).total) return EMOE_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (desc->T == 0) {  // no assignments: every slot is empty
        hipError_t z1 = launch_fill_i32(slot_counts, desc->S, 0, st);
        hipError_t z2 = launch_fill_i32(slot_offsets, desc->S + 1, 0, st);
        return (z1 == hipSuccess && z2 == hipSuccess) ? EMOE_OK : EMOE_ERR_DEVICE;
    }
    hipError_t e = launch_permute(*desc, x, topk_expert, slot_of_expert, slot_counts, slot_offsets, perm, inv_perm,
                                  x_perm, ws, st);
    return e == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

static int expert_ffn_passes(const emoe_layer_desc* desc, int passes, const void* x_perm, const int32_t* perm,
                             const int32_t* out_perm, const int32_t* slot_offsets, const void* w1_slots, const void* w3_slots,
                             const void* w2_slots, void* y_perm, void* ws, size_t ws_bytes, void* stream) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!x_perm || !slot_offsets || !w1_slots || !w2_slots || !y_perm) return EMOE_ERR_NULL;
    if (desc->act == EMOE_ACT_SWIGLU && !w3_slots) return EMOE_ERR_NULL;
    if (desc->act == EMOE_ACT_RELU && w3_slots) return EMOE_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < ffn_ws_layout(*desc).total) return EMOE_ERR_WORKSPACE;
    if (desc->T == 0) return EMOE_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const RowGather gather{perm, desc->k, desc->T, out_perm};  // perm == nullptr: x_perm holds the grouped rows themselves
    hipError_t e;
    if (desc->dtype == EMOE_F32)
        e = launch_ffn_f32(*desc, x_perm, gather, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, passes, st);
    else if (ffn_bf16_path(*desc) == kFfnStream)
        e = launch_ffn_bf16_stream(*desc, x_perm, gather, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, passes, st);
    else if (ffn_bf16_path(*desc) == kFfnMid)
        e = launch_ffn_bf16_mid(*desc, x_perm, gather, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, passes, st);
    else
        e = launch_ffn_bf16_tiled(*desc, x_perm, gather, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, passes, st);
    return e == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_expert_ffn(const emoe_layer_desc* desc, const void* x_perm, const int32_t* slot_offsets,
                    const void* w1_slots, const void* w3_slots, const void* w2_slots, void* y_perm, void* ws,
                    size_t ws_bytes, void* stream) {
    return expert_ffn_passes(desc, 3, x_perm, nullptr, nullptr, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes,
                             stream);
}

int emoe_expert_ffn_pass(const emoe_layer_desc* desc, int32_t pass, const void* x_perm, const int32_t* slot_offsets,
                         const void* w1_slots, const void* w3_slots, const void* w2_slots, void* y_perm, void* ws,
                         size_t ws_bytes, void* stream) {
    if (pass != 1 && pass != 2) return EMOE_ERR_SHAPE;
    return expert_ffn_passes(desc, pass == 1 ? 1 : 2, x_perm, nullptr, nullptr, slot_offsets, w1_slots, w3_slots, w2_slots,
                             y_perm, ws, ws_bytes, stream);
}

int emoe_expert_ffn_gather(const emoe_layer_desc* desc, const void* x, const int32_t* perm,
                           const int32_t* slot_offsets, const void* w1_slots, const void* w3_slots,
                           const void* w2_slots, void* y_perm, void* ws, size_t ws_bytes, void* stream) {
    if (!perm) return EMOE_ERR_NULL;
    return expert_ffn_passes(desc, 3, x, perm, nullptr, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes,
                             stream);
}

int emoe_expert_ffn_gather_pass(const emoe_layer_desc* desc, int32_t pass, const void* x, const int32_t* perm,
                                const int32_t* slot_offsets, const void* w1_slots, const void* w3_slots,
                                const void* w2_slots, void* y_perm, void* ws, size_t ws_bytes, void* stream) {
    if (pass != 1 && pass != 2) return EMOE_ERR_SHAPE;
    if (!perm) return EMOE_ERR_NULL;
    return expert_ffn_passes(desc, pass == 1 ? 1 : 2, x, perm, nullptr, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws,
                             ws_bytes, stream);
}

int emoe_expert_ffn_gather_combine(const emoe_layer_desc* desc, const void* x, const int32_t* perm,
                                   const int32_t* inv_perm, const int32_t* slot_offsets, const void* w1_slots,
                                   const void* w3_slots, const void* w2_slots, const float* topk_weight, void* y_perm,
                                   void* out, void* ws, size_t ws_bytes, void* stream) {
    if (!perm || !inv_perm || !topk_weight || !out) return EMOE_ERR_NULL;
    if (desc != nullptr && desc->k == 1)
        // one expert per token: its gate weight is exactly 1 and the combine is the inverse of the row
        // permutation, so the second product stores row r as out[perm[r]] and the fifth launch disappears
        return expert_ffn_passes(desc, 3, x, perm, perm, slot_offsets, w1_slots, w3_slots, w2_slots, out, ws, ws_bytes, stream);
    if (!y_perm) return EMOE_ERR_NULL;
    int rc = expert_ffn_passes(desc, 3, x, perm, nullptr, slot_offsets, w1_slots, w3_slots, w2_slots, y_perm, ws, ws_bytes,
                               stream);
    if (rc != EMOE_OK) return rc;
    return emoe_combine(desc, y_perm, inv_perm, topk_weight, out, stream);
}

int emoe_combine(const emoe_layer_desc* desc, const void* y_perm, const int32_t* inv_perm, const float* topk_weight,
                 void* out, void* stream) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!y_perm || !inv_perm || !topk_weight || !out) return EMOE_ERR_NULL;
    if (desc->T == 0) return EMOE_OK;
    hipError_t e = launch_combine(*desc, y_perm, inv_perm, topk_weight, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_layer_forward(const emoe_layer_desc* desc, const void* x, const void* w_gate, const float* gate_bias,
                       const int32_t* slot_of_expert, const void* w1_slots, const void* w3_slots,
                       const void* w2_slots, int32_t* topk_expert, float* topk_weight, int32_t* slot_counts,
                       int32_t* slot_offsets, int32_t* perm, int32_t* inv_perm, void* y_perm, void* out,
                       void* permute_ws, size_t permute_ws_bytes, void* ffn_ws, size_t ffn_ws_bytes, void* stream) {
    // everything the four calls would reject, before anything is enqueued
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!x || !w_gate || !slot_of_expert || !w1_slots || !w2_slots || !topk_expert || !topk_weight || !slot_counts ||
        !slot_offsets || !perm || !inv_perm || !y_perm || !out)
        return EMOE_ERR_NULL;
    if (desc->act == EMOE_ACT_SWIGLU && !w3_slots) return EMOE_ERR_NULL;
    if (desc->act == EMOE_ACT_RELU && w3_slots) return EMOE_ERR_UNSUPPORTED;
    if (!permute_ws || permute_ws_bytes < permute_ws_layout(*desc).total) return EMOE_ERR_WORKSPACE;
    if (!ffn_ws || ffn_ws_bytes < ffn_ws_layout(*desc).total) return EMOE_ERR_WORKSPACE;
    rc = emoe_route(desc, x, w_gate, gate_bias, slot_of_expert, topk_expert, topk_weight, stream);
    if (rc != EMOE_OK) return rc;
    rc = emoe_permute(desc, x, topk_expert, slot_of_expert, slot_counts, slot_offsets, perm, inv_perm, nullptr, permute_ws,
                      permute_ws_bytes, stream);
    if (rc != EMOE_OK) return rc;
    return emoe_expert_ffn_gather_combine(desc, x, perm, inv_perm, slot_offsets, w1_slots, w3_slots, w2_slots, topk_weight,
                                          y_perm, out, ffn_ws, ffn_ws_bytes, stream);
}

int emoe_load_experts(const emoe_layer_desc* desc, int32_t n, const int32_t* expert_ids, const int32_t* slot_ids,
                      const void* const* host_w1, const void* const* host_w3, const void* const* host_w2,
                      void* w1_slots, void* w3_slots, void* w2_slots, int32_t* slot_of_expert,
                      int32_t* expert_of_slot, int32_t* expert_of_slot_host, void* side_stream, void* wait_event,
                      void* done_event) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (n < 0 || n > desc->S) return EMOE_ERR_SHAPE;
    if (!slot_of_expert || !expert_of_slot || !expert_of_slot_host || !w1_slots || !w2_slots) return EMOE_ERR_NULL;
    if (n > 0 && (!expert_ids || !slot_ids || !host_w1 || !host_w2)) return EMOE_ERR_NULL;
    const bool swiglu = desc->act == EMOE_ACT_SWIGLU;
    if (swiglu && (!w3_slots || (n > 0 && !host_w3))) return EMOE_ERR_NULL;
    const int E = desc->E, S = desc->S;

    // ---- validate the change against the caller's mirror, on a copy -------------------------
    int32_t eos[kMaxExperts], soe[kMaxExperts];
    bool slot_named[kMaxExperts] = {}, expert_named[kMaxExperts] = {};
    for (int s = 0; s < S; ++s) {
        eos[s] = expert_of_slot_host[s];
        if (eos[s] < -1 || eos[s] >= E) return EMOE_ERR_RESIDENT;
    }
    for (int i = 0; i < n; ++i) {
        const int e = expert_ids[i], s = slot_ids[i];
        if (s < 0 || s >= S || e < -1 || e >= E) return EMOE_ERR_RESIDENT;
        if (slot_named[s]) return EMOE_ERR_RESIDENT;
        slot_named[s] = true;
        if (e >= 0) {
            if (expert_named[e]) return EMOE_ERR_RESIDENT;
            expert_named[e] = true;
            if (!host_w1[e] || !host_w2[e] || (swiglu && !host_w3[e])) return EMOE_ERR_NULL;
        }
    }
    for (int i = 0; i < n; ++i) {
        const int e = expert_ids[i], s = slot_ids[i];
        if (e >= 0)
            for (int s2 = 0; s2 < S; ++s2)
                if (eos[s2] == e) eos[s2] = -1;  // the expert moves: its old slot empties
        eos[s] = e;
    }
    int resident = 0;
    for (int e = 0; e < E; ++e) soe[e] = -1;
    for (int s = 0; s < S; ++s)
        if (eos[s] >= 0) {
            if (soe[eos[s]] >= 0) return EMOE_ERR_RESIDENT;  // mirror held an expert twice
            soe[eos[s]] = s;
            ++resident;
        }
    if (resident < desc->k) return EMOE_ERR_RESIDENT;

    // ---- enqueue: wait, copies in list order, maps, event -------------------------------------
    hipStream_t st = static_cast<hipStream_t>(side_stream);
    if (wait_event && hipStreamWaitEvent(st, static_cast<hipEvent_t>(wait_event), 0) != hipSuccess)
        return EMOE_ERR_DEVICE;
    const size_t mat_bytes = (size_t)desc->d_model * desc->d_ff * elem_bytes(*desc);
    for (int i = 0; i < n; ++i) {
        const int e = expert_ids[i], s = slot_ids[i];
        if (e < 0) continue;
        uint8_t* d1 = static_cast<uint8_t*>(w1_slots) + (size_t)s * mat_bytes;
        uint8_t* d2 = static_cast<uint8_t*>(w2_slots) + (size_t)s * mat_bytes;
        if (hipMemcpyAsync(d1, host_w1[e], mat_bytes, hipMemcpyHostToDevice, st) != hipSuccess) return EMOE_ERR_DEVICE;
        if (swiglu) {
            uint8_t* d3 = static_cast<uint8_t*>(w3_slots) + (size_t)s * mat_bytes;
            if (hipMemcpyAsync(d3, host_w3[e], mat_bytes, hipMemcpyHostToDevice, st) != hipSuccess)
                return EMOE_ERR_DEVICE;
        }
        if (hipMemcpyAsync(d2, host_w2[e], mat_bytes, hipMemcpyHostToDevice, st) != hipSuccess) return EMOE_ERR_DEVICE;
    }
    if (launch_write_maps(soe, E, eos, S, slot_of_expert, expert_of_slot, st) != hipSuccess) return EMOE_ERR_DEVICE;
    if (done_event && hipEventRecord(static_cast<hipEvent_t>(done_event), st) != hipSuccess) return EMOE_ERR_DEVICE;
    memcpy(expert_of_slot_host, eos, sizeof(int32_t) * S);
    return EMOE_OK;
}

}  // extern "C"
