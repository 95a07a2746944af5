// Expert FFN for bf16 layers with many rows per slot: grouped GEMM on the gfx950 matrix cores
// (eMoE Section 1: the experts; Section 5.1: only resident, non-empty slots cost compute and
// memory reads).
//
//   pass 1: h[r, n]      = act(x_perm[r,:] . W1_s[n,:]) (* x_perm[r,:] . W3_s[n,:])   K = d_model
//   pass 2: y_perm[r, n] = h[r,:] . W2_s[n,:]                                         K = d_ff
//
// Both operands are K-contiguous, so every MFMA operand is one 16-byte LDS read.  A workgroup of
// four wavefronts (2 x 2) owns a 256-token x 256-weight-row tile; each wavefront accumulates a
// 128 x 128 sub-tile as 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 in fp32.  In the SwiGLU pass the
// 256 weight rows are 128 rows of W1 and the SAME 128 rows of W3, laid out so that a lane holds the
// gate and the up value of the same output element and the activation is applied in registers.
// The weight rows go on the MFMA's row operand: a lane then owns four consecutive output columns
// of one token and stores them as one 8-byte write.
//
// Ragged groups: group sizes live on the device.  The launch covers an upper bound of M-tiles
// (ceil(A/256) + S); every workgroup finds its (slot, m-tile, n-tile) from slot_offsets and
// surplus workgroups exit.  Workgroup ids are dealt round-robin to the 8 XCDs, so ids are
// remapped: each XCD walks a contiguous range of the (slot, n-tile, m-tile) order with the
// m-tile fastest, which keeps one weight panel (and the slot's token panels) in that XCD's L2.
#include "common.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256;            // tokens per tile
constexpr int BR = 256;            // weight rows per tile (SwiGLU: 128 of W1 + 128 of W3)
constexpr int BK = 64;             // K step
constexpr int LDS_ROW = BK + 8;    // bf16 elements per LDS row: 144 bytes, conflict-free 16-byte reads
constexpr int TILE_ELEMS = BM * LDS_ROW;
constexpr int STAGE_ELEMS = 2 * TILE_ELEMS;  // token tile + weight tile
constexpr size_t LDS_BYTES = 2 * STAGE_ELEMS * sizeof(bf16_t);
constexpr int XCDS = 8;

enum Epilogue { kPlain = 0, kSwiglu = 1, kRelu = 2 };

template <int EPI>
__global__ __launch_bounds__(256, 1) void grouped_gemm_bf16(const bf16_t* __restrict__ a,
                                                            const int32_t* __restrict__ offsets,
                                                            const bf16_t* __restrict__ b0,
                                                            const bf16_t* __restrict__ b1, bf16_t* __restrict__ c,
                                                            int S, int N, int K, int n_tiles) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;  // output columns per tile
    extern __shared__ __align__(16) bf16_t lds[];

    // ---- which tile is mine -------------------------------------------------------------
    const int per_xcd = gridDim.x / XCDS;
    int rem = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS;
    int slot = -1, row0 = 0, row_end = 0, nt = 0;
    for (int s = 0; s < S; ++s) {
        const int b = offsets[s], e = offsets[s + 1];
        const int tiles = (e - b + BM - 1) / BM;
        const int span = tiles * n_tiles;
        if (rem < span) {
            slot = s;
            nt = rem / tiles;
            row0 = b + (rem % tiles) * BM;
            row_end = e;
            break;
        }
        rem -= span;
    }
    if (slot < 0) return;
    const int n0 = nt * BNO;
    const bf16_t* w0 = b0 + (size_t)slot * N * K;
    const bf16_t* w1 = EPI == kSwiglu ? b1 + (size_t)slot * N * K : nullptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global -> register staging: thread loads 16-byte chunk `lc` of rows lr + 32*i -----
    const int lc = tid & 7, lr = tid >> 3;
    const bf16_t* a_src[8];
    const bf16_t* b_src[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int r = row0 + lr + 32 * i;
        r = r < row_end ? r : row_end - 1;
        a_src[i] = a + (size_t)r * K + lc * 8;
        int n;
        const bf16_t* wb = w0;
        if (EPI == kSwiglu) {
            n = n0 + lr + 32 * (i & 3);
            if (i >= 4) wb = w1;
        } else {
            n = n0 + lr + 32 * i;
        }
        n = n < N ? n : N - 1;
        b_src[i] = wb + (size_t)n * K + lc * 8;
    }
    uint4 a_reg[8], b_reg[8];
    auto load_global = [&](int k0) {
        const bool ok = k0 + lc * 8 < K;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a_reg[i] = ok ? *reinterpret_cast<const uint4*>(a_src[i] + k0) : make_uint4(0, 0, 0, 0);
            b_reg[i] = ok ? *reinterpret_cast<const uint4*>(b_src[i] + k0) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int stage) {
        bf16_t* at = lds + stage * STAGE_ELEMS;
        bf16_t* bt = at + TILE_ELEMS;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<uint4*>(at + (lr + 32 * i) * LDS_ROW + lc * 8) = a_reg[i];
            *reinterpret_cast<uint4*>(bt + (lr + 32 * i) * LDS_ROW + lc * 8) = b_reg[i];
        }
    };

    // ---- fragment addresses ----------------------------------------------------------------
    // token block mi: tile rows wm*128 + mi*32 + lane%32; weight block ni: see header comment
    const int frag_k = (lane >> 5) * 8;
    int x_row[4], w_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x_row[i] = (wm * 128 + i * 32 + (lane & 31)) * LDS_ROW + frag_k;
        int rr;
        if (EPI == kSwiglu)
            rr = (i < 2) ? wn * 64 + i * 32 : 128 + wn * 64 + (i - 2) * 32;
        else
            rr = wn * 128 + i * 32;
        w_row[i] = (rr + (lane & 31)) * LDS_ROW + frag_k;
    }

    floatx16 acc[4][4];  // [weight block][token block]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int k_tiles = (K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < k_tiles; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < k_tiles;
        if (more) load_global((kt + 1) * BK);
        const bf16_t* at = lds + cur * STAGE_ELEMS;
        const bf16_t* bt = at + TILE_ELEMS;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 xf[4], wf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xf[i] = *reinterpret_cast<const bf16x8*>(at + x_row[i] + kk * 16);
                wf[i] = *reinterpret_cast<const bf16x8*>(bt + w_row[i] + kk * 16);
            }
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
        }
        if (more) store_lds(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds, per block, token lane%32 and weight rows 8g + 4*(lane/32) + 0..3 ---
    constexpr int NB = EPI == kSwiglu ? 2 : 4;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int r = row0 + wm * 128 + mi * 32 + (lane & 31);
        if (r >= row_end) continue;
        bf16_t* crow = c + (size_t)r * N;
#pragma unroll
        for (int ni = 0; ni < NB; ++ni) {
            const int nb = n0 + (EPI == kSwiglu ? wn * 64 : wn * 128) + ni * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = nb + 8 * g;
                if (n >= N) continue;
                floatx4 v;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float t = acc[ni][mi][4 * g + q];
                    if (EPI == kSwiglu) t = t / (1.0f + __expf(-t)) * acc[ni + 2][mi][4 * g + q];
                    if (EPI == kRelu) t = fmaxf(t, 0.0f);
                    v[q] = t;
                }
                bf16x4 o = __builtin_convertvector(v, bf16x4);
                *reinterpret_cast<bf16x4*>(crow + n) = o;
            }
        }
    }
}

template <int EPI>
hipError_t launch_one(const bf16_t* a, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c, int A,
                      int S, int N, int K, hipStream_t st) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    const int n_tiles = (N + BNO - 1) / BNO;
    const int m_tiles = (A + BM - 1) / BM + S;
    long long blocks = (long long)n_tiles * m_tiles;
    blocks = (blocks + XCDS - 1) / XCDS * XCDS;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&grouped_gemm_bf16<EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    grouped_gemm_bf16<EPI><<<(unsigned)blocks, 256, LDS_BYTES, st>>>(a, offsets, b0, b1, c, S, N, K, n_tiles);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_bf16_tiled(const emoe_layer_desc& d, const void* x_perm, const int32_t* offsets,
                                 const void* w1, const void* w3, const void* w2, void* y_perm, void* ws,
                                 int passes, hipStream_t st) {
    const int A = d.T * d.k;
    bf16_t* h = reinterpret_cast<bf16_t*>(static_cast<uint8_t*>(ws) + ffn_ws_layout(d).h);
    const bf16_t* xp = static_cast<const bf16_t*>(x_perm);
    hipError_t e = hipSuccess;
    if (!(passes & 1)) {
    } else if (d.act == EMOE_ACT_SWIGLU)
        e = launch_one<kSwiglu>(xp, offsets, static_cast<const bf16_t*>(w1), static_cast<const bf16_t*>(w3), h, A,
                                d.S, d.d_ff, d.d_model, st);
    else
        e = launch_one<kRelu>(xp, offsets, static_cast<const bf16_t*>(w1), nullptr, h, A, d.S, d.d_ff, d.d_model, st);
    if (e != hipSuccess || !(passes & 2)) return e;
    return launch_one<kPlain>(h, offsets, static_cast<const bf16_t*>(w2), nullptr, static_cast<bf16_t*>(y_perm), A,
                              d.S, d.d_model, d.d_ff, st);
}

}  // namespace emoe
