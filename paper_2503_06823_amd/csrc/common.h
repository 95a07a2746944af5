// Internal declarations shared by the HIP sources of libemoe (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "emoe.h"

namespace emoe {

constexpr int kWave = 64;
constexpr int kMaxExperts = 64;
// The chip the kernels are written for is MI355X: 256 compute units in 8 XCDs (workgroup ids are
// dealt round-robin to the XCDs, each with its own L2).  The launch shapes take both numbers from
// the device at run time (device_shape()); nothing depends on them for correctness: no kernel waits
// for another workgroup.  kMaxGroups bounds the persistent launches, whose partial-sum workspaces
// are sized for that many workgroups.
constexpr int kMaxGroups = 256;
struct DeviceShape {
    int cus;     // compute units
    int xcds;    // XCDs the workgroup ids are dealt to, round-robin
    int groups;  // workgroups of a persistent launch: one per CU, at most kMaxGroups, a multiple of xcds
};
// Shape of the current device, queried once per device.
hipError_t device_shape(DeviceShape* out);

typedef uint16_t bf16_t;  // storage pattern of a bfloat16

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_f32(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f32(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_from_f32(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_from_f32(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// Workspace layout (all offsets multiples of 256 bytes).
struct PermuteWs {
    size_t block_counts;  // int32 [n_blocks][S]
    size_t total;
};
struct FfnWs {
    size_t h;         // dtype [A][f]
    size_t partials;  // fp32 K pieces of tiles cut along K (the two tiled bf16 paths, else 0 bytes)
    size_t total;
};
constexpr size_t kTiledPlanBytes = 256;  // the tiled kernel leaves its work plan here for the fix-up kernel
constexpr size_t kTiledPartialBytes = kTiledPlanBytes + (size_t)256 * 256 * 256 * sizeof(float);  // + 256 pieces of a 256x256 tile
constexpr size_t kMidPartialBytes = (size_t)512 * 128 * 128 * sizeof(float);  // the 128-row-tile kernel: two pieces of a 128x128 tile per CU
constexpr int kPermuteChunk = 1024;  // assignments per workgroup in the counting sort
PermuteWs permute_ws_layout(const emoe_layer_desc& d);
FfnWs ffn_ws_layout(const emoe_layer_desc& d);

// Which kernels the bf16 FFN runs: weight streaming (few rows per slot), tiles of 128 token rows
// (up to a few hundred rows per slot) or tiles of 256 token rows.
enum FfnPath { kFfnStream = 0, kFfnMid = 1, kFfnTiled = 2 };
FfnPath ffn_bf16_path(const emoe_layer_desc& d);

// Host-side checks common to the entry points; returns EMOE_OK or an error.
int validate_desc(const emoe_layer_desc* d);

// `passes` of the FFN launchers: bit 0 = pass 1 (x_perm -> h), bit 1 = pass 2 (h -> y_perm).
// Kernel launchers (each returns a hipError_t converted to emoe_status by the caller).
hipError_t launch_route_bf16(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                             const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                             unsigned long long* expert_tokens, hipStream_t st);
// expert_tokens: nullptr, or [E] counters that receive each token's k experts under ordinary routing
hipError_t launch_route(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                        const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                        unsigned long long* expert_tokens, hipStream_t st);
hipError_t launch_permute(const emoe_layer_desc& d, const void* x, const int32_t* topk_expert,
                          const int32_t* slot_of_expert, int32_t* counts, int32_t* offsets, int32_t* perm,
                          int32_t* inv_perm, void* x_perm, void* ws, hipStream_t st);
hipError_t launch_combine(const emoe_layer_desc& d, const void* y_perm, const int32_t* inv_perm,
                          const float* topk_weight, void* out, hipStream_t st);
// Where pass 1 finds the token row of grouped row r: in x_perm[r] (perm == nullptr), or in
// x[perm[r] / k] (the gather folded into the operand load; `rows` = T bounds the buffer).
// out_perm (pass 2 only): nullptr, or, with the combine folded into the second product of a layer
// with one expert per token, the permutation by which result row r is stored as row out_perm[r] of
// the output (the token it belongs to) instead of row r.
struct RowGather {
    const int32_t* perm;
    int k;
    int rows;
    const int32_t* out_perm;
};

hipError_t launch_ffn_f32(const emoe_layer_desc& d, const void* x_perm, RowGather gather, const int32_t* offsets, const void* w1,
                          const void* w3, const void* w2, void* y_perm, void* ws, int passes, hipStream_t st);
hipError_t launch_ffn_bf16_tiled(const emoe_layer_desc& d, const void* x_perm, RowGather gather, const int32_t* offsets,
                                 const void* w1, const void* w3, const void* w2, void* y_perm, void* ws,
                                 int passes, hipStream_t st);
hipError_t launch_ffn_bf16_mid(const emoe_layer_desc& d, const void* x_perm, RowGather gather, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, void* y_perm, void* ws, int passes,
                               hipStream_t st);
hipError_t launch_ffn_bf16_stream(const emoe_layer_desc& d, const void* x_perm, RowGather gather, const int32_t* offsets,
                                  const void* w1, const void* w3, const void* w2, void* y_perm, void* ws,
                                  int passes, hipStream_t st);
hipError_t launch_fill_i32(int32_t* p, int n, int32_t value, hipStream_t st);
hipError_t launch_write_maps(const int32_t* slot_of_expert_new, int E, const int32_t* expert_of_slot_new, int S,
                             int32_t* slot_of_expert_dev, int32_t* expert_of_slot_dev, hipStream_t st);

}  // namespace emoe
