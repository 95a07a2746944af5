// Small device-side writers used by emoe_load_experts and by the T == 0 case of emoe_permute.
// The new expert<->slot maps travel by value in the kernel arguments, so updating them needs no
// staging buffer and is ordered on the stream after the weight copies (eMoE Section 4: the layer
// waits on an event recorded after its load, so it never sees new maps with stale weights).
#include "common.h"

namespace emoe {
namespace {

struct Maps {
    int32_t slot_of_expert[kMaxExperts];
    int32_t expert_of_slot[kMaxExperts];
};

__global__ void write_maps_kernel(Maps m, int E, int S, int32_t* __restrict__ slot_of_expert,
                                  int32_t* __restrict__ expert_of_slot) {
    const int i = threadIdx.x;
    if (i < E) slot_of_expert[i] = m.slot_of_expert[i];
    if (i < S) expert_of_slot[i] = m.expert_of_slot[i];
}

__global__ void fill_i32_kernel(int32_t* __restrict__ p, int n, int32_t value) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

}  // namespace

hipError_t launch_write_maps(const int32_t* slot_of_expert_new, int E, const int32_t* expert_of_slot_new, int S,
                             int32_t* slot_of_expert_dev, int32_t* expert_of_slot_dev, hipStream_t st) {
    Maps m;
    for (int i = 0; i < kMaxExperts; ++i) {
        m.slot_of_expert[i] = i < E ? slot_of_expert_new[i] : -1;
        m.expert_of_slot[i] = i < S ? expert_of_slot_new[i] : -1;
    }
    write_maps_kernel<<<1, kMaxExperts, 0, st>>>(m, E, S, slot_of_expert_dev, expert_of_slot_dev);
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* p, int n, int32_t value, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    fill_i32_kernel<<<(n + 255) / 256, 256, 0, st>>>(p, n, value);
    return hipGetLastError();
}

}  // namespace emoe
