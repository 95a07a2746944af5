// Expert FFN for fp32 layers (eMoE Section 1: the experts; only slots that received rows are
// touched).  fp32 layers are the small verification shape, so this is a plain LDS-tiled FMA
// grouped GEMM: 64x64 output tile, 256 threads, 4x4 outputs per thread.  The fast paths are the
// bf16 MFMA kernels.
//   pass 1: h[r, n] = act(x_perm[r,:] . W1_s[n,:]) (* x_perm[r,:] . W3_s[n,:])
//   pass 2: y_perm[r, n] = h[r,:] . W2_s[n,:]
#include "common.h"

namespace emoe {
namespace {

constexpr int BM = 64, BN = 64, BK = 16;
enum Epilogue { kPlain = 0, kSwiglu = 1, kRelu = 2 };

// Finds the slot and the first row of M-tile `mt` in the ragged list of slot groups.
__device__ __forceinline__ bool find_group(const int32_t* __restrict__ offsets, int S, int bm, int mt, int& slot,
                                           int& row0, int& row_end) {
    for (int s = 0; s < S; ++s) {
        const int b = offsets[s], e = offsets[s + 1];
        const int tiles = (e - b + bm - 1) / bm;
        if (mt < tiles) {
            slot = s;
            row0 = b + mt * bm;
            row_end = e;
            return true;
        }
        mt -= tiles;
    }
    return false;
}

template <int EPI>
__global__ __launch_bounds__(256) void grouped_gemm_f32(const float* __restrict__ a, RowGather gather,
                                                        const int32_t* __restrict__ offsets,
                                                        const float* __restrict__ b0, const float* __restrict__ b1,
                                                        float* __restrict__ c, int S, int N, int K) {
    __shared__ float As[BK][BM + 4];
    __shared__ float B0s[BK][BN + 4];
    __shared__ float B1s[EPI == kSwiglu ? BK : 1][BN + 4];
    int slot, row0, row_end;
    if (!find_group(offsets, S, BM, blockIdx.y, slot, row0, row_end)) return;
    const int n0 = blockIdx.x * BN;
    const float* w0 = b0 + (size_t)slot * N * K;
    const float* w1 = EPI == kSwiglu ? b1 + (size_t)slot * N * K : nullptr;

    const int tid = threadIdx.x;
    const int lr = tid >> 2, lk = (tid & 3) * 4;  // loader: row within tile, k offset
    const int tx = tid & 15, ty = tid >> 4;       // compute: 4 columns tx*4.., 4 rows ty*4..
    float acc0[4][4] = {}, acc1[4][4] = {};
    int a_row = row0 + lr;  // row of `a` this thread loads
    if (gather.perm != nullptr && a_row < row_end) a_row = gather.perm[a_row] / gather.k;

    for (int k0 = 0; k0 < K; k0 += BK) {
        float4 va = make_float4(0, 0, 0, 0), vb0 = va, vb1 = va;
        const bool kok = k0 + lk < K;
        if (kok && row0 + lr < row_end) va = *reinterpret_cast<const float4*>(a + (size_t)a_row * K + k0 + lk);
        if (kok && n0 + lr < N) {
            vb0 = *reinterpret_cast<const float4*>(w0 + (size_t)(n0 + lr) * K + k0 + lk);
            if (EPI == kSwiglu) vb1 = *reinterpret_cast<const float4*>(w1 + (size_t)(n0 + lr) * K + k0 + lk);
        }
        __syncthreads();
        As[lk + 0][lr] = va.x; As[lk + 1][lr] = va.y; As[lk + 2][lr] = va.z; As[lk + 3][lr] = va.w;
        B0s[lk + 0][lr] = vb0.x; B0s[lk + 1][lr] = vb0.y; B0s[lk + 2][lr] = vb0.z; B0s[lk + 3][lr] = vb0.w;
        if (EPI == kSwiglu) {
            B1s[lk + 0][lr] = vb1.x; B1s[lk + 1][lr] = vb1.y; B1s[lk + 2][lr] = vb1.z; B1s[lk + 3][lr] = vb1.w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float av[4], bv0[4], bv1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                av[i] = As[kk][ty * 4 + i];
                bv0[i] = B0s[kk][tx * 4 + i];
                if (EPI == kSwiglu) bv1[i] = B1s[kk][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(av[i], bv0[j], acc0[i][j]);
                    if (EPI == kSwiglu) acc1[i][j] = fmaf(av[i], bv1[j], acc1[i][j]);
                }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = row0 + ty * 4 + i;
        if (r >= row_end) continue;
        const int dr = (EPI == kPlain && gather.out_perm != nullptr) ? gather.out_perm[r] : r;  // combine folded in: the token's row
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc0[i][j];
            if (EPI == kSwiglu) v = v / (1.0f + expf(-v)) * acc1[i][j];
            if (EPI == kRelu) v = fmaxf(v, 0.0f);
            c[(size_t)dr * N + n] = v;
        }
    }
}

}  // namespace

hipError_t launch_ffn_f32(const emoe_layer_desc& d, const void* x_perm, RowGather gather, const int32_t* offsets, const void* w1,
                          const void* w3, const void* w2, void* y_perm, void* ws, int passes, hipStream_t st) {
    const int A = d.T * d.k;
    float* h = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + ffn_ws_layout(d).h);
    const int m_tiles = (A + BM - 1) / BM + d.S;
    dim3 g1((d.d_ff + BN - 1) / BN, m_tiles), g2((d.d_model + BN - 1) / BN, m_tiles);
    const float* xp = static_cast<const float*>(x_perm);
    if (!(passes & 1)) {
    } else if (d.act == EMOE_ACT_SWIGLU)
        grouped_gemm_f32<kSwiglu><<<g1, 256, 0, st>>>(xp, gather, offsets, static_cast<const float*>(w1),
                                                      static_cast<const float*>(w3), h, d.S, d.d_ff, d.d_model);
    else
        grouped_gemm_f32<kRelu><<<g1, 256, 0, st>>>(xp, gather, offsets, static_cast<const float*>(w1), nullptr, h, d.S,
                                                    d.d_ff, d.d_model);
    if (passes & 2)
        grouped_gemm_f32<kPlain><<<g2, 256, 0, st>>>(h, RowGather{nullptr, 1, 0, gather.out_perm}, offsets, static_cast<const float*>(w2), nullptr,
                                                     static_cast<float*>(y_perm), d.S, d.d_model, d.d_ff);
    return hipGetLastError();
}

}  // namespace emoe
