// Expert FFN for bf16 layers with few rows per slot (a decode step): the cost is reading each
// resident, non-empty slot's weights from HBM exactly once (eMoE Section 5.1: fewer experts
// means fewer global-memory reads), so the kernels are shaped for streaming, not for MFMA rate.
//
// A work unit is 32 consecutive weight rows of one slot.  The weight rows are the MFMA's row
// operand (v_mfma_f32_32x32x16_bf16), up to 64 of the slot's tokens are the column operand, so a
// weight element is loaded once and used for every token.  Operands go from global memory
// straight into registers: weights are used once (nothing to share through LDS) and the slot's
// few token rows stay in L2.  A slot with no rows exits at once and its weights are never read.
// Latency is hidden by occupancy: every unit of the launch is resident at the same time.
//   pass 1 (K = d_model): one wavefront per unit, gate and up rows together, activation in
//                          registers, h rounded to bf16.
//   pass 2 (K = d_ff)   : four wavefronts per unit split K, partial sums meet in LDS (fixed
//                          order, so the result is reproducible), y rounded to bf16.
#include "common.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

enum Epilogue { kPlain = 0, kSwiglu = 1, kRelu = 2 };
constexpr int RB = 32;   // weight rows per unit
constexpr int KC = 64;   // K elements per loop step (four MFMA steps)

__device__ __forceinline__ bf16x8 load8(const bf16_t* p, bool ok) {
    if (!ok) {
        bf16x8 z;
#pragma unroll
        for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
        return z;
    }
    return *reinterpret_cast<const bf16x8*>(p);
}

// Accumulates rows [row_begin, row_begin + 32*NTB) of the slot against this unit's weight rows
// over K chunks [ch0, ch1).  GUARD: K is not a multiple of KC, pieces past K read as zero.
template <int EPI, int NTB, bool GUARD>
__device__ __forceinline__ void accumulate(const bf16_t* __restrict__ a, const bf16_t* __restrict__ wr0,
                                           const bf16_t* __restrict__ wr1, int row_begin, int row_end, int K, int ch0,
                                           int ch1, int lane, floatx16 (&acc0)[NTB], floatx16 (&acc1)[NTB]) {
    const int kq = (lane >> 5) * 8;
    const bf16_t* xr[NTB];
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
        int r = row_begin + tb * 32 + (lane & 31);
        r = r < row_end ? r : row_end - 1;
        xr[tb] = a + (size_t)r * K + kq;
    }
    for (int ch = ch0; ch < ch1; ++ch) {
        const int k0 = ch * KC;
        bf16x8 wf0[4], wf1[4], xf[NTB][4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bool ok = !GUARD || (k0 + ks * 16 + kq < K);
            wf0[ks] = load8(wr0 + k0 + ks * 16, ok);
            if (EPI == kSwiglu) wf1[ks] = load8(wr1 + k0 + ks * 16, ok);
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) xf[tb][ks] = load8(xr[tb] + k0 + ks * 16, ok);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) {
                acc0[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf0[ks], xf[tb][ks], acc0[tb], 0, 0, 0);
                if (EPI == kSwiglu)
                    acc1[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf1[ks], xf[tb][ks], acc1[tb], 0, 0, 0);
            }
    }
}

template <int EPI, int KW, int NTB, bool GUARD>
__device__ __forceinline__ void unit_body(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w0,
                                          const bf16_t* __restrict__ w1, bf16_t* __restrict__ c, int row_begin,
                                          int row_end, int n0, int N, int K, float* red) {
    const int lane = threadIdx.x & 63;
    const int kw = threadIdx.x >> 6;
    int n = n0 + (lane & 31);
    n = n < N ? n : N - 1;
    const bf16_t* wr0 = w0 + (size_t)n * K + (lane >> 5) * 8;
    const bf16_t* wr1 = EPI == kSwiglu ? w1 + (size_t)n * K + (lane >> 5) * 8 : nullptr;
    const int chunks = (K + KC - 1) / KC;
    const int ch0 = (int)((long long)chunks * kw / KW), ch1 = (int)((long long)chunks * (kw + 1) / KW);

    floatx16 acc0[NTB], acc1[NTB];
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc0[tb][v] = 0.0f; acc1[tb][v] = 0.0f; }
    accumulate<EPI, NTB, GUARD>(a, wr0, wr1, row_begin, row_end, K, ch0, ch1, lane, acc0, acc1);

    if (KW > 1) {  // partial sums of the K splits meet in LDS; wave 0 adds them in split order
        if (kw > 0) {
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((kw - 1) * NTB * 16 + tb * 16 + v) * 64 + lane] = acc0[tb][v];
        }
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int w = 1; w < KW; ++w)
#pragma unroll
                for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc0[tb][v] += red[((w - 1) * NTB * 16 + tb * 16 + v) * 64 + lane];
        }
        __syncthreads();  // red[] is reused by the next token chunk
        if (kw != 0) return;
    }
    // lane holds token lane%32 of each block and weight rows 8g + 4*(lane/32) + 0..3
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
        const int r = row_begin + tb * 32 + (lane & 31);
        if (r >= row_end) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nn = n0 + 8 * g + (lane >> 5) * 4;
            if (nn >= N) continue;
            floatx4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float t = acc0[tb][4 * g + q];
                if (EPI == kSwiglu) t = t / (1.0f + __expf(-t)) * acc1[tb][4 * g + q];
                if (EPI == kRelu) t = fmaxf(t, 0.0f);
                v[q] = t;
            }
            *reinterpret_cast<bf16x4*>(c + (size_t)r * N + nn) = __builtin_convertvector(v, bf16x4);
        }
    }
}

// grid.x = S * ceil(N / 32) units; blockDim.x = 64 * KW.
template <int EPI, int KW, bool GUARD>
__global__ __launch_bounds__(64 * KW) void stream_gemm_bf16(const bf16_t* __restrict__ a,
                                                             const int32_t* __restrict__ offsets,
                                                             const bf16_t* __restrict__ b0,
                                                             const bf16_t* __restrict__ b1, bf16_t* __restrict__ c,
                                                             int N, int K, int n_rb) {
    __shared__ float red[KW > 1 ? (KW - 1) * 2 * 16 * 64 : 1];
    const int slot = blockIdx.x / n_rb;
    const int n0 = (blockIdx.x % n_rb) * RB;
    const int row0 = offsets[slot], row_end = offsets[slot + 1];
    if (row_end <= row0) return;  // empty slot: its weights are never touched
    const bf16_t* w0 = b0 + (size_t)slot * N * K;
    const bf16_t* w1 = EPI == kSwiglu ? b1 + (size_t)slot * N * K : nullptr;
    int r = row0;
    // whole chunks of 64 tokens, then a last chunk of at most 64 (one block if it fits in 32)
    while (row_end - r > 64) {
        unit_body<EPI, KW, 2, GUARD>(a, w0, w1, c, r, row_end, n0, N, K, red);
        r += 64;
    }
    if (row_end - r > 32)
        unit_body<EPI, KW, 2, GUARD>(a, w0, w1, c, r, row_end, n0, N, K, red);
    else
        unit_body<EPI, KW, 1, GUARD>(a, w0, w1, c, r, row_end, n0, N, K, red);
}

template <int EPI, int KW>
hipError_t launch_one(const bf16_t* a, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c, int S,
                      int N, int K, hipStream_t st) {
    const int n_rb = (N + RB - 1) / RB;
    const unsigned blocks = (unsigned)(S * n_rb);
    if (K % KC == 0)
        stream_gemm_bf16<EPI, KW, false><<<blocks, 64 * KW, 0, st>>>(a, offsets, b0, b1, c, N, K, n_rb);
    else
        stream_gemm_bf16<EPI, KW, true><<<blocks, 64 * KW, 0, st>>>(a, offsets, b0, b1, c, N, K, n_rb);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_bf16_stream(const emoe_layer_desc& d, const void* x_perm, const int32_t* offsets,
                                  const void* w1, const void* w3, const void* w2, void* y_perm, void* ws,
                                  int passes, hipStream_t st) {
    bf16_t* h = reinterpret_cast<bf16_t*>(static_cast<uint8_t*>(ws) + ffn_ws_layout(d).h);
    const bf16_t* xp = static_cast<const bf16_t*>(x_perm);
    hipError_t e = hipSuccess;
    if (!(passes & 1)) {
    } else if (d.act == EMOE_ACT_SWIGLU)
        e = launch_one<kSwiglu, 1>(xp, offsets, static_cast<const bf16_t*>(w1), static_cast<const bf16_t*>(w3), h,
                                   d.S, d.d_ff, d.d_model, st);
    else
        e = launch_one<kRelu, 1>(xp, offsets, static_cast<const bf16_t*>(w1), nullptr, h, d.S, d.d_ff, d.d_model, st);
    if (e != hipSuccess || !(passes & 2)) return e;
    return launch_one<kPlain, 4>(h, offsets, static_cast<const bf16_t*>(w2), nullptr, static_cast<bf16_t*>(y_perm),
                                 d.S, d.d_model, d.d_ff, st);
}

}  // namespace emoe
