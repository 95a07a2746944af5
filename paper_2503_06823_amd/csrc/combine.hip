// Gate-weighted combine back to token order (eMoE Section 1: the layer output mixes the chosen
// experts' outputs with the gate's weights):
//   out[t,:] = sum_{j<k} topk_weight[t,j] * y_perm[inv_perm[t*k+j], :]   (j ascending, fp32, one rounding)
// One wavefront handles one (token, 16-byte-per-lane column chunk) unit; every load is a contiguous
// 1 KiB piece of a y_perm row.  An assignment with inv_perm < 0 (left out by the permutation)
// contributes nothing.
#include "common.h"

namespace emoe {
namespace {

template <typename T> struct Pack;
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
template <> struct Pack<bf16_t> {
    static constexpr int N = 8;
    template <bool ONCE>
    __device__ static void load(const bf16_t* p, float (&v)[8]) {
        uint32_t w[4];
        if (ONCE) {  // rows that will not be read again soon and do not fit the caches anyway: non-temporal
            const uintx4 r = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(p));
            w[0] = r.x; w[1] = r.y; w[2] = r.z; w[3] = r.w;
        } else {
            const uint4 r = *reinterpret_cast<const uint4*>(p);
            w[0] = r.x; w[1] = r.y; w[2] = r.z; w[3] = r.w;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static void store(bf16_t* p, const float (&v)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
        *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct Pack<float> {
    static constexpr int N = 4;
    template <bool ONCE>
    __device__ static void load(const float* p, float (&v)[4]) {
        float4 r = *reinterpret_cast<const float4*>(p);
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
    __device__ static void store(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};

template <typename T, bool ONCE>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ y_perm, const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ topk_weight, T* __restrict__ out,
                                                      int T_, int d, int k, int chunks) {
    constexpr int N = Pack<T>::N;
    const int lane = threadIdx.x & 63;
    const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const long long n_waves = ((long long)gridDim.x * blockDim.x) >> 6;
    const long long units = (long long)T_ * chunks;
    for (long long u = wave; u < units; u += n_waves) {
        const int t = (int)(u / chunks);
        const int c = (int)(u % chunks) * 64 * N + lane * N;
        // lane j fetches the row number and the weight of the token's j-th expert (k <= 64), so that the
        // rows' addresses are known at once and their loads go out together instead of one dependent
        // pair of loads per expert
        int my_r = -1;
        float my_w = 0.0f;
        if (lane < k) {
            my_r = inv_perm[(size_t)t * k + lane];
            my_w = topk_weight[(size_t)t * k + lane];
        }
        float acc[N];
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = 0.0f;
        for (int j0 = 0; j0 < k; j0 += 4) {  // four rows in flight, added in ascending j
            float v[4][N];
            float w[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int j = j0 + jj < k ? j0 + jj : k - 1;
                const int r = __builtin_amdgcn_readlane(my_r, j);
                const bool ok = j0 + jj < k && r >= 0;  // r < 0: an assignment the permutation left out
                w[jj] = ok ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), j)) : 0.0f;
#pragma unroll
                for (int i = 0; i < N; ++i) v[jj][i] = 0.0f;
                if (ok && c < d) Pack<T>::template load<ONCE>(y_perm + (size_t)r * d + c, v[jj]);
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if (j0 + jj < k) {
#pragma unroll
                    for (int i = 0; i < N; ++i) acc[i] = fmaf(w[jj], v[jj][i], acc[i]);
                }
            }
        }
        if (c < d) Pack<T>::store(out + (size_t)t * d + c, acc);
    }
}

template <typename T>
hipError_t launch_t(const emoe_layer_desc& d, const void* y_perm, const int32_t* inv_perm, const float* w, void* out,
                    hipStream_t st) {
    constexpr int N = Pack<T>::N;
    const int chunks = (d.d_model + 64 * N - 1) / (64 * N);
    long long units = (long long)d.T * chunks;
    long long blocks = (units + 3) / 4;
    if (blocks > 256 * 32) blocks = 256 * 32;
    // y_perm larger than half the 256 MB Infinity Cache: its rows come from HBM whatever is done, and without the
    // non-temporal hint they push each other through the caches (fine-grained layer, 201 MB: 47 -> 44 us); a smaller
    // one is still cached from the second product that wrote it (prefill layer, 67 MB: 22.6 us, 23.8 with the hint)
    const bool once = (size_t)d.T * d.k * d.d_model * sizeof(T) > ((size_t)128 << 20);
    if (once)
        combine_kernel<T, true><<<(int)blocks, 256, 0, st>>>(static_cast<const T*>(y_perm), inv_perm, w, static_cast<T*>(out),
                                                             d.T, d.d_model, d.k, chunks);
    else
        combine_kernel<T, false><<<(int)blocks, 256, 0, st>>>(static_cast<const T*>(y_perm), inv_perm, w, static_cast<T*>(out),
                                                              d.T, d.d_model, d.k, chunks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_combine(const emoe_layer_desc& d, const void* y_perm, const int32_t* inv_perm,
                          const float* topk_weight, void* out, hipStream_t st) {
    if (d.dtype == EMOE_F32) return launch_t<float>(d, y_perm, inv_perm, topk_weight, out, st);
    return launch_t<bf16_t>(d, y_perm, inv_perm, topk_weight, out, st);
}

}  // namespace emoe
