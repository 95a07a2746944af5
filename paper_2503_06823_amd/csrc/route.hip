// Gate logits and resident-restricted top-k (eMoE Section 1: the gate; Section 3.2.2, last
// paragraph: a token whose expert is not on the GPU goes to its next-best expert that is):
// fp32 inputs, and bf16 inputs when there are few tokens, few experts and long rows (a decode step
// of a Mixtral-shaped layer).  Other bf16 batches take the matrix-core kernel of route_mfma.hip,
// which puts 32 tokens on a workgroup: with 64 tokens it runs on two CUs, bound by the latency of
// their walk along d_model.
//
// One wavefront (or, when there are few tokens, four) owns one token at a time.  Its 64 lanes
// split the d_model axis (16 bytes per lane per step, so a step reads 1 KiB of the token row
// contiguously); every lane keeps one
// partial sum per expert.  A butterfly reduce-scatter then leaves expert e's complete logit in
// lanes e*(64/EP) .. +64/EP-1: 63 shuffles for 64 experts instead of 64 full reductions.  The logits
// are then read into scalar registers and top-k is k rounds of compares that every lane performs
// on the same values (lower index wins a tie); softmax over the k winners.
// The summation order is fixed by the code, so results are reproducible run to run.
#include "common.h"

namespace emoe {
namespace {

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, float (&v)[8]) {
        const uint4 r = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
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
// SPLIT = wavefronts that share one token (1 or 4).  With few tokens (a decode step) one wavefront
// per token would leave most of the chip idle and make each wavefront walk the whole row alone, so
// four wavefronts split the row and add their partial logits through LDS in wavefront order.
template <typename T, int EP, int SPLIT>
__global__ __launch_bounds__(256) void route_kernel(const T* __restrict__ x, const T* __restrict__ w_gate,
                                                    const float* __restrict__ bias,
                                                    const int32_t* __restrict__ slot_of_expert,
                                                    int32_t* __restrict__ topk_expert,
                                                    float* __restrict__ topk_weight,
                                                    unsigned long long* __restrict__ expert_tokens, int T_, int d,
                                                    int E, int k) {
    constexpr int VN = Vec<T>::N;
    __shared__ float partial[SPLIT > 1 ? 4 * 64 : 1];
    const int lane = threadIdx.x & 63;
    const int wib = threadIdx.x >> 6;  // wavefront in block
    const int tokens_per_block = 4 / SPLIT;
    const int part = SPLIT > 1 ? wib : 0;  // which share of the row this wavefront sums
    // expert whose logit this lane ends up holding
    const int my_e = lane / (64 / EP);
    const bool resident = my_e < E && slot_of_expert[my_e] >= 0;
    const float my_bias = (bias != nullptr && my_e < E) ? bias[my_e] : 0.0f;

    for (int t0 = blockIdx.x * tokens_per_block; t0 < T_; t0 += gridDim.x * tokens_per_block) {
        const int t = t0 + (SPLIT > 1 ? 0 : wib);
        const bool live = t < T_;  // uniform per wavefront
        float acc[EP];
#pragma unroll
        for (int e = 0; e < EP; ++e) acc[e] = 0.0f;
        if (live) {
            const T* xr = x + (size_t)t * d;
            // two row pieces per trip, both requested before either is used
            int c = (part * 64 + lane) * VN;
            const int step = SPLIT * 64 * VN;
            for (; c + step < d; c += 2 * step) {
                float xa[VN], xb[VN];
                Vec<T>::load(xr + c, xa);
                Vec<T>::load(xr + c + step, xb);
                // Rows past the last expert repeat that expert's row (their sums are never looked at):
                // without a branch around them the loads of all rows are independent and go out together
                // instead of one memory round trip per expert.
#pragma unroll
                for (int e = 0; e < EP; ++e) {
                    const T* wp = w_gate + (size_t)(e < E ? e : E - 1) * d + c;
                    float wa[VN], wb[VN];
                    Vec<T>::load(wp, wa);
                    Vec<T>::load(wp + step, wb);
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[e] = fmaf(xa[i], wa[i], acc[e]);
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[e] = fmaf(xb[i], wb[i], acc[e]);
                }
            }
            if (c < d) {
                float xa[VN];
                Vec<T>::load(xr + c, xa);
#pragma unroll
                for (int e = 0; e < EP; ++e) {
                    const T* wp = w_gate + (size_t)(e < E ? e : E - 1) * d + c;
                    float wa[VN];
                    Vec<T>::load(wp, wa);
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[e] = fmaf(xa[i], wa[i], acc[e]);
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
        float logit = acc[0];
        if (SPLIT > 1) {  // the four shares of the row meet in LDS, added in wavefront order
            partial[wib * 64 + lane] = logit;
            __syncthreads();
            logit = ((partial[lane] + partial[64 + lane]) + partial[128 + lane]) + partial[192 + lane];
            __syncthreads();
            if (wib != 0) continue;
        }
        if (!live) continue;
        logit += my_bias;

        // Every lane of a group holds its expert's logit.  One lane per expert is read into scalar
        // registers, so that the k rounds of "largest logit among the resident experts not taken yet,
        // lower index on a tie" are plain compares on values every lane already has - no exchange
        // between lanes, whose latency would otherwise be paid 18 times per round.
        float lg[EP];
#pragma unroll
        for (int e = 0; e < EP; ++e)
            lg[e] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(logit), e * (64 / EP)));
        const unsigned long long res_lanes = __ballot(resident);
        unsigned long long avail = 0;  // bit e: expert e is resident and not taken yet
#pragma unroll
        for (int e = 0; e < EP; ++e) avail |= ((res_lanes >> (e * (64 / EP))) & 1ull) << e;
        float sel_v = 0.0f, top_v = 0.0f, sum = 0.0f;
        int sel_e = 0;
        for (int j = 0; j < k; ++j) {
            float bv = 0.0f;
            int be = -1;
#pragma unroll
            for (int e = 0; e < EP; ++e) {
                const bool ok = (avail >> e) & 1ull;
                if (ok && (be < 0 || lg[e] > bv)) { bv = lg[e]; be = e; }
            }
            if (be < 0) {  // fewer than k resident experts: precondition broken, stay defined
                be = 0;
                bv = 0.0f;
            } else {
                avail &= ~(1ull << be);
            }
            if (j == 0) top_v = bv;
            sum += expf(bv - top_v);
            if (lane == j) { sel_v = bv; sel_e = be; }
        }
        if (lane < k) {
            topk_expert[(size_t)t * k + lane] = sel_e;
            topk_weight[(size_t)t * k + lane] = expf(sel_v - top_v) / sum;
        }
        // Workload (Section 3.2.2: the number of tokens an expert receives): the same k rounds over
        // all E experts, resident or not.  Integer counts: the accumulated result has no order.
        if (expert_tokens != nullptr) {
            unsigned long long left = E >= 64 ? ~0ull : (1ull << E) - 1ull;
            int obs_e = -1;
            for (int j = 0; j < k; ++j) {
                float bv = 0.0f;
                int be = -1;
#pragma unroll
                for (int e = 0; e < EP; ++e) {
                    const bool ok = (left >> e) & 1ull;
                    if (ok && (be < 0 || lg[e] > bv)) { bv = lg[e]; be = e; }
                }
                if (be >= 0) left &= ~(1ull << be);
                if (lane == j) obs_e = be;
            }
            if (lane < k && obs_e >= 0) atomicAdd(&expert_tokens[obs_e], 1ull);
        }
    }
}

constexpr int kWaveRouteTokens = 256;

template <typename T, int EP>
hipError_t launch_ep(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                     const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                     unsigned long long* expert_tokens, hipStream_t st) {
    const T* xp = static_cast<const T*>(x);
    const T* wg = static_cast<const T*>(w_gate);
    if (d.T <= 2048) {  // fewer than two wavefronts per SIMD otherwise: share each token among four
        int blocks = d.T < 256 * 16 ? d.T : 256 * 16;
        route_kernel<T, EP, 4><<<blocks, 256, 0, st>>>(xp, wg, bias, slot_of_expert, topk_expert, topk_weight,
                                                       expert_tokens, d.T, d.d_model, d.E, d.k);
    } else {
        int blocks = (d.T + 3) / 4;
        if (blocks > 256 * 16) blocks = 256 * 16;
        route_kernel<T, EP, 1><<<blocks, 256, 0, st>>>(xp, wg, bias, slot_of_expert, topk_expert, topk_weight,
                                                       expert_tokens, d.T, d.d_model, d.E, d.k);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_t(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                    const int32_t* soe, int32_t* te, float* tw, unsigned long long* et, hipStream_t st) {
    if (d.E <= 1) return launch_ep<T, 1>(d, x, w_gate, bias, soe, te, tw, et, st);
    if (d.E <= 2) return launch_ep<T, 2>(d, x, w_gate, bias, soe, te, tw, et, st);
    if (d.E <= 4) return launch_ep<T, 4>(d, x, w_gate, bias, soe, te, tw, et, st);
    if (d.E <= 8) return launch_ep<T, 8>(d, x, w_gate, bias, soe, te, tw, et, st);
    if (d.E <= 16) return launch_ep<T, 16>(d, x, w_gate, bias, soe, te, tw, et, st);
    if (d.E <= 32) return launch_ep<T, 32>(d, x, w_gate, bias, soe, te, tw, et, st);
    return launch_ep<T, 64>(d, x, w_gate, bias, soe, te, tw, et, st);
}

}  // namespace

hipError_t launch_route(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                        const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                        unsigned long long* expert_tokens, hipStream_t st) {
    if (d.dtype == EMOE_F32)
        return launch_t<float>(d, x, w_gate, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
    // bf16: the matrix-core kernel runs T / 32 workgroups, each bound by the latency of its walk along
    // d_model (11 us at d_model = 4096 however few the tokens); one workgroup per token takes 6-8 us
    // with up to 16 experts (19 us with 64, where the matrix-core kernel stays the better one)
    if (d.T <= kWaveRouteTokens && d.E <= 16 && d.d_model >= 2048)
        return launch_t<bf16_t>(d, x, w_gate, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
    return launch_route_bf16(d, x, w_gate, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
}

}  // namespace emoe
