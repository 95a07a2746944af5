// Measurement aids, not steps of the layer: two kernels that show what this GPU sustains on the
// resources that bound the expert FFN, so that a roofline fraction can be quoted against a measured
// ceiling next to the datasheet one.
//
//   matrix loop : every workgroup copies a 256 x 64 tile of each of two caller-supplied bf16 operand
//                 buffers (the workload's own token rows and weights, so the matrix cores switch the
//                 same bit patterns as in the GEMM) into LDS once and then issues
//                 v_mfma_f32_32x32x16_bf16 back to back, four wavefronts of 4 x 4 blocks like the
//                 tiled FFN kernel, with (lds_reads = 1) or without the GEMM's LDS fragment reads and
//                 with no global memory traffic at all.  Flop per launch = workgroups * 4 wavefronts *
//                 iters * 4 K-steps * 16 MFMAs * 32768.
//   read stream : a grid-stride read of a buffer with 16-byte loads, eight in flight per lane,
//                 nothing written: the rate at which HBM delivers a stream that is read once.
//   copy stream : a plain copy, the kernel of known traffic for scaling hardware-counter readings.
//   scatter combine : the gate-weighted combine by atomic adds into an fp32 image, what folding the
//                 combine into the second product costs when a token has several experts.
#include "common.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kRowElems = 72;                      // 64 K elements + 8 of padding: conflict-free fragment reads
constexpr int kTileRows = 256;
constexpr int kLoopLds = 2 * kTileRows * kRowElems * 2;  // both operand tiles, bytes

template <bool LDS_READS>
__global__ __launch_bounds__(256) void mfma_loop_kernel(const bf16_t* __restrict__ a, size_t a_elems,
                                                        const bf16_t* __restrict__ b, size_t b_elems, int iters,
                                                        float* __restrict__ sink) {
    extern __shared__ __align__(16) bf16_t tile[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // operand tiles: 256 rows of 64 consecutive elements, taken from a different place per workgroup
    const size_t a_tiles = a_elems / (kTileRows * 64), b_tiles = b_elems / (kTileRows * 64);
    const bf16_t* asrc = a + (size_t)(blockIdx.x % a_tiles) * (kTileRows * 64);
    const bf16_t* bsrc = b + (size_t)((blockIdx.x * 7u + 3u) % b_tiles) * (kTileRows * 64);
    for (int i = threadIdx.x; i < kTileRows * 64; i += 256) {
        tile[(i / 64) * kRowElems + i % 64] = asrc[i];
        tile[(kTileRows + i / 64) * kRowElems + i % 64] = bsrc[i];
    }
    __syncthreads();
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    int xr[4], wr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        xr[i] = ((wave & 1) * 128 + i * 32 + (lane & 31)) * kRowElems + (lane >> 5) * 8;
        wr[i] = (kTileRows + (wave >> 1) * 128 + i * 32 + (lane & 31)) * kRowElems + (lane >> 5) * 8;
    }
    bf16x8 xf[2][4], wf[2][4];
    auto load_frags = [&](int buf, int kk) {
#pragma unroll
        for (int i = 0; i < 4; ++i) xf[buf][i] = *reinterpret_cast<const bf16x8*>(tile + xr[i] + kk * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) wf[buf][i] = *reinterpret_cast<const bf16x8*>(tile + wr[i] + kk * 16);
    };
    load_frags(0, 0);
    load_frags(1, 1);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (LDS_READS) load_frags((kk + 1) & 1, (kk + 1) & 3);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk & 1][ni], xf[kk & 1][mi], acc[ni][mi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

constexpr int kReadUnroll = 8;
__global__ __launch_bounds__(256) void read_stream_kernel(const uintx4* __restrict__ src, size_t n16, uintx4* __restrict__ sink) {
    size_t i = (size_t)blockIdx.x * 256 * kReadUnroll + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256 * kReadUnroll;
    uintx4 acc = {0u, 0u, 0u, 0u};
    for (; i + 256 * (kReadUnroll - 1) < n16; i += stride) {
        uintx4 v[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) acc ^= v[u];
    }
    // the data decide whether anything is written (it practically never is), so the loads cannot be dropped
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc;
}

// Plain grid-stride copy: a kernel of known traffic (bytes read, bytes written) by which hardware
// counter readings of the other kernels in the same profiler run are scaled.
__global__ __launch_bounds__(256) void copy_stream_kernel(const uintx4* __restrict__ src, uintx4* __restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// The combine done the way a second product with the combine folded into its epilogue has to do it
// when a token has several experts: the token's k rows come out of different output tiles at
// different times, so each is added into an fp32 image of the output with atomics (the image cleared
// before, converted to the storage type afterwards).  Three kernels: clear, scatter-add one grouped row
// per wavefront (256 contiguous bytes of atomics per instruction), convert.  Measured against
// combine_kernel, which reads the k rows of a token and writes the result once.
__global__ __launch_bounds__(256) void clear_f32_kernel(float4* __restrict__ p, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256)
        p[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}
__global__ __launch_bounds__(256) void scatter_add_kernel(const bf16_t* __restrict__ y_perm, const int32_t* __restrict__ perm,
                                                          const float* __restrict__ topk_weight, float* __restrict__ image,
                                                          int A, int d, int k) {
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = (gridDim.x * 256) >> 6;
    for (int r = wave; r < A; r += n_waves) {
        const int a = perm[r];
        const float w = topk_weight[a];
        float* dst = image + (size_t)(a / k) * d;
        const bf16_t* src = y_perm + (size_t)r * d;
        for (int c = lane; c < d; c += 64) unsafeAtomicAdd(dst + c, w * bf16_to_f32(src[c]));
    }
}
__global__ __launch_bounds__(256) void convert_f32_kernel(const float4* __restrict__ image, uint2* __restrict__ out, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        const float4 v = image[i];
        out[i] = make_uint2((uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16),
                            (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16));
    }
}

}  // namespace
}  // namespace emoe

using namespace emoe;

extern "C" {

int emoe_measure_mfma_loop(const void* a, size_t a_elems, const void* b, size_t b_elems, int32_t lds_reads,
                           int32_t workgroups, int32_t iters, float* sink, double* flop, void* stream) {
    if (!a || !b || !sink) return EMOE_ERR_NULL;
    if (a_elems < (size_t)kTileRows * 64 || b_elems < (size_t)kTileRows * 64 || workgroups <= 0 || iters <= 0)
        return EMOE_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (lds_reads) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_loop_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLoopLds);
        if (e != hipSuccess) return EMOE_ERR_DEVICE;
        mfma_loop_kernel<true><<<workgroups, 256, kLoopLds, st>>>(static_cast<const bf16_t*>(a), a_elems,
                                                                  static_cast<const bf16_t*>(b), b_elems, iters, sink);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_loop_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLoopLds);
        if (e != hipSuccess) return EMOE_ERR_DEVICE;
        mfma_loop_kernel<false><<<workgroups, 256, kLoopLds, st>>>(static_cast<const bf16_t*>(a), a_elems,
                                                                   static_cast<const bf16_t*>(b), b_elems, iters, sink);
    }
    if (flop) *flop = (double)workgroups * 4.0 * iters * 4.0 * 16.0 * 32768.0;
    return hipGetLastError() == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_measure_read_stream(const void* src, size_t bytes, int32_t workgroups, void* sink, void* stream) {
    if (!src || !sink) return EMOE_ERR_NULL;
    if (bytes == 0 || bytes % (16 * 256 * kReadUnroll) != 0 || workgroups <= 0) return EMOE_ERR_SHAPE;
    read_stream_kernel<<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uintx4*>(src), bytes / 16,
                                                                                  static_cast<uintx4*>(sink));
    return hipGetLastError() == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_measure_copy_stream(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream) {
    if (!src || !dst) return EMOE_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || workgroups <= 0) return EMOE_ERR_SHAPE;
    copy_stream_kernel<<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uintx4*>(src),
                                                                                  static_cast<uintx4*>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

int emoe_measure_scatter_combine(const emoe_layer_desc* desc, const void* y_perm, const int32_t* perm,
                                 const float* topk_weight, float* image, void* out, void* stream) {
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!y_perm || !perm || !topk_weight || !image || !out) return EMOE_ERR_NULL;
    if (desc->dtype != EMOE_BF16 || desc->d_model % 4 != 0) return EMOE_ERR_UNSUPPORTED;
    if (desc->T == 0) return EMOE_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t n4 = (size_t)desc->T * desc->d_model / 4;
    const int A = desc->T * desc->k;
    clear_f32_kernel<<<2048, 256, 0, st>>>(reinterpret_cast<float4*>(image), n4);
    scatter_add_kernel<<<2048, 256, 0, st>>>(static_cast<const bf16_t*>(y_perm), perm, topk_weight, image, A, desc->d_model,
                                             desc->k);
    convert_f32_kernel<<<2048, 256, 0, st>>>(reinterpret_cast<const float4*>(image), static_cast<uint2*>(out), n4);
    return hipGetLastError() == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}

}  // extern "C"
