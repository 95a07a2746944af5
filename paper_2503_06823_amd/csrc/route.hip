// Gate logits and resident-restricted top-k (eMoE Section 1: the gate; Section 3.2.2, last
// paragraph: a token whose expert is not on the GPU goes to its next-best expert that is).
//
// One wavefront owns one token at a time.  Its 64 lanes split the d_model axis (16 bytes per
// lane per step, so a step reads 1 KiB of the token row contiguously); every lane keeps one
// partial sum per expert.  A butterfly reduce-scatter then leaves expert e's complete logit in
// lane e*(64/EP): 63 shuffles for 64 experts instead of 64 full reductions.  Top-k is k rounds
// of a wave-wide arg-max on (logit, lower index wins); softmax over the k winners.
// The summation order is fixed by the code, so results are reproducible run to run.
#include "common.h"

namespace emoe {
namespace {

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, float (&v)[8]) {
        uint4 r = *reinterpret_cast<const uint4*>(p);
        uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, float (&v)[4]) {
        float4 r = *reinterpret_cast<const float4*>(p);
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
};

// EP = number of experts rounded up to a power of two (1..64).
template <typename T, int EP>
__global__ __launch_bounds__(256) void route_kernel(const T* __restrict__ x, const T* __restrict__ w_gate,
                                                    const float* __restrict__ bias,
                                                    const int32_t* __restrict__ slot_of_expert,
                                                    int32_t* __restrict__ topk_expert,
                                                    float* __restrict__ topk_weight, int T_, int d, int E, int k) {
    constexpr int VN = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    // expert whose logit this lane ends up holding
    const int my_e = lane / (64 / EP);
    const bool resident = my_e < E && slot_of_expert[my_e] >= 0;
    const float my_bias = (bias != nullptr && my_e < E) ? bias[my_e] : 0.0f;

    for (int t = wave; t < T_; t += n_waves) {
        float acc[EP];
#pragma unroll
        for (int e = 0; e < EP; ++e) acc[e] = 0.0f;
        const T* xr = x + (size_t)t * d;
        for (int c = lane * VN; c < d; c += 64 * VN) {
            float xv[VN];
            Vec<T>::load(xr + c, xv);
#pragma unroll
            for (int e = 0; e < EP; ++e) {
                if (e < E) {
                    float wv[VN];
                    Vec<T>::load(w_gate + (size_t)e * d + c, wv);
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[e] = fmaf(xv[i], wv[i], acc[e]);
                }
            }
        }
        // butterfly reduce-scatter over the lanes
        int n = EP;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            if (n > 1) {
                const int half = n / 2;
                const bool upper = (lane & m) != 0;
#pragma unroll
                for (int i = 0; i < half; ++i) {
                    float send = upper ? acc[i] : acc[i + half];
                    float keep = upper ? acc[i + half] : acc[i];
                    acc[i] = keep + __shfl_xor(send, m);
                }
                n = half;
            } else {
                acc[0] += __shfl_xor(acc[0], m);
            }
        }
        const float logit = acc[0] + my_bias;

        // k rounds of arg-max over resident experts not taken yet
        bool avail = resident;
        float sel_v = 0.0f, top_v = 0.0f;
        int sel_e = 0;
        for (int j = 0; j < k; ++j) {
            float bv = logit;
            int be = my_e;
            bool bo = avail;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                float ov = __shfl_xor(bv, m);
                int oe = __shfl_xor(be, m);
                bool oo = __shfl_xor((int)bo, m) != 0;
                bool take = oo && (!bo || ov > bv || (ov == bv && oe < be));
                if (take) { bv = ov; be = oe; bo = true; }
            }
            if (!bo) {  // fewer than k resident experts: precondition broken, stay defined
                be = 0;
                bv = 0.0f;
            }
            if (my_e == be) avail = false;
            if (j == 0) top_v = bv;
            if (lane == j) { sel_v = bv; sel_e = be; }
        }
        float p = lane < k ? expf(sel_v - top_v) : 0.0f;
        float sum = p;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m);
        if (lane < k) {
            topk_expert[(size_t)t * k + lane] = sel_e;
            topk_weight[(size_t)t * k + lane] = p / sum;
        }
    }
}

template <typename T, int EP>
hipError_t launch_ep(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                     const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight, hipStream_t st) {
    const int waves_per_block = 4;
    int blocks = (d.T + waves_per_block - 1) / waves_per_block;
    if (blocks > 256 * 16) blocks = 256 * 16;
    route_kernel<T, EP><<<blocks, 64 * waves_per_block, 0, st>>>(
        static_cast<const T*>(x), static_cast<const T*>(w_gate), bias, slot_of_expert, topk_expert, topk_weight,
        d.T, d.d_model, d.E, d.k);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_t(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                    const int32_t* soe, int32_t* te, float* tw, hipStream_t st) {
    if (d.E <= 1) return launch_ep<T, 1>(d, x, w_gate, bias, soe, te, tw, st);
    if (d.E <= 2) return launch_ep<T, 2>(d, x, w_gate, bias, soe, te, tw, st);
    if (d.E <= 4) return launch_ep<T, 4>(d, x, w_gate, bias, soe, te, tw, st);
    if (d.E <= 8) return launch_ep<T, 8>(d, x, w_gate, bias, soe, te, tw, st);
    if (d.E <= 16) return launch_ep<T, 16>(d, x, w_gate, bias, soe, te, tw, st);
    if (d.E <= 32) return launch_ep<T, 32>(d, x, w_gate, bias, soe, te, tw, st);
    return launch_ep<T, 64>(d, x, w_gate, bias, soe, te, tw, st);
}

}  // namespace

hipError_t launch_route(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                        const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight, hipStream_t st) {
    if (d.dtype == EMOE_F32) return launch_t<float>(d, x, w_gate, bias, slot_of_expert, topk_expert, topk_weight, st);
    return launch_t<bf16_t>(d, x, w_gate, bias, slot_of_expert, topk_expert, topk_weight, st);
}

}  // namespace emoe
