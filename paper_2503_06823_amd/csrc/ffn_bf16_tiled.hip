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
#include <type_traits>

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

// WM x WN wavefronts; each owns (BM/WM) tokens x (BR/WN) weight rows.  KTAIL: K is not a multiple
// of BK, 16-byte pieces past K are read as zeros.
template <int EPI, int WM, int WN, bool KTAIL>
__global__ __launch_bounds__(64 * WM * WN) void grouped_gemm_bf16(const bf16_t* __restrict__ a,
                                                                  const int32_t* __restrict__ offsets,
                                                                  const bf16_t* __restrict__ b0,
                                                                  const bf16_t* __restrict__ b1,
                                                                  bf16_t* __restrict__ c, int S, int N, int K,
                                                                  int n_tiles) {
    constexpr int NT = 64 * WM * WN;                   // threads
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;  // output columns per tile
    constexpr int TB = BM / WM / 32;                   // token blocks per wavefront
    constexpr int WB = BR / WN / 32;                   // weight-row blocks per wavefront
    constexpr int LROWS = NT / 8;                      // tile rows covered by one load round
    constexpr int LN = BM / LROWS;                     // load rounds per operand tile
    static_assert(EPI != kSwiglu || WB % 2 == 0, "gate and up blocks come in pairs");
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
    const int wm = wave / WN, wn = wave % WN;

    // ---- global -> register staging --------------------------------------------------------
    // A tile needs 2*LN 16-byte items per thread: items 0..LN-1 are chunk `lc` of token rows
    // lr + LROWS*i, items LN..2LN-1 the same of the weight rows.  Addresses are a uniform base
    // (advanced by one K tile per iteration) plus a 32-bit per-thread byte offset.
    const int lc = tid & 7, lr = tid >> 3;
    constexpr int NI = 2 * LN;
    uint32_t off[NI];
#pragma unroll
    for (int i = 0; i < LN; ++i) {
        const int tr = lr + LROWS * i;  // row of the tile
        int r = row0 + tr;
        r = r < row_end ? r : row_end - 1;
        off[i] = ((uint32_t)r * (uint32_t)K + lc * 8) * 2u;
        int n = n0 + (EPI == kSwiglu ? tr % (BR / 2) : tr);  // SwiGLU: second half = same rows of W3
        n = n < N ? n : N - 1;
        off[LN + i] = ((uint32_t)n * (uint32_t)K + lc * 8) * 2u;
    }
    const char* a_base = reinterpret_cast<const char*>(a);
    const char* w0_base = reinterpret_cast<const char*>(w0);
    const char* w1_base = reinterpret_cast<const char*>(EPI == kSwiglu ? w1 : w0);
    // Two register sets: tile t travels through set t&1.  A set is refilled (tile t+2) right
    // after it has been written to LDS (tile t), so two tiles are in flight from global memory
    // at any time: a load that misses L2 takes longer than one K tile of matrix work.
    uint4 reg[2][NI];
    // item j of the tile that starts at element k0 -> register set `set`
    auto load_item = [&](int set, int j, int k0) {
        const bool ok = !KTAIL || (k0 + lc * 8 < K);
        const char* base = j < LN ? a_base : ((EPI == kSwiglu && (j - LN) * LROWS >= BR / 2) ? w1_base : w0_base);
        reg[set][j] = ok ? *reinterpret_cast<const uint4*>(base + (size_t)k0 * 2 + off[j]) : make_uint4(0, 0, 0, 0);
    };
    // item j of register set `set` -> LDS buffer `stage`
    auto store_item = [&](int set, int j, int stage) {
        bf16_t* t = lds + stage * STAGE_ELEMS + (j < LN ? 0 : TILE_ELEMS);
        const int i = j < LN ? j : j - LN;
        *reinterpret_cast<uint4*>(t + (lr + LROWS * i) * LDS_ROW + lc * 8) = reg[set][j];
    };

    // ---- fragment addresses ----------------------------------------------------------------
    // SwiGLU: weight blocks 0..WB/2-1 are gate rows, WB/2..WB-1 the matching up rows
    const int frag_k = (lane >> 5) * 8;
    int x_row[TB], w_row[WB];
#pragma unroll
    for (int i = 0; i < TB; ++i) x_row[i] = (wm * (BM / WM) + i * 32 + (lane & 31)) * LDS_ROW + frag_k;
#pragma unroll
    for (int i = 0; i < WB; ++i) {
        int rr;
        if (EPI == kSwiglu)
            rr = (i < WB / 2) ? wn * (BR / 2 / WN) + i * 32 : BR / 2 + wn * (BR / 2 / WN) + (i - WB / 2) * 32;
        else
            rr = wn * (BR / WN) + i * 32;
        w_row[i] = (rr + (lane & 31)) * LDS_ROW + frag_k;
    }

    floatx16 acc[WB][TB];  // [weight block][token block]
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // ---- main loop ----------------------------------------------------------------------------
    // Software pipeline, one barrier per K tile.  While tile kt is multiplied out of LDS buffer
    // kt&1 in four 16-wide steps:
    //   steps 0-2: a third of tile kt+1 (in registers, requested two iterations ago) is written
    //           to the other buffer and the freed registers are refilled from global memory with
    //           tile kt+3, so the memory pipes see a steady trickle instead of a burst
    //   after step 2: every wavefront waits for its LDS traffic and meets at the barrier: tile
    //           kt+1 is now visible, buffer kt&1 is free
    //   step 3: the first fragments of tile kt+1 are requested
    // Each step requests the next step's fragments before its own MFMAs are issued, so LDS and
    // global latency hide behind matrix work; the scheduling barriers pin that order.
    const int k_tiles = (K + BK - 1) / BK;
    bf16x8 xf[2][TB], wf[2][WB];
    auto load_frags = [&](int buf, int stage, int kk) {
        const bf16_t* at = lds + stage * STAGE_ELEMS;
        const bf16_t* bt = at + TILE_ELEMS;
#pragma unroll
        for (int i = 0; i < TB; ++i) xf[buf][i] = *reinterpret_cast<const bf16x8*>(at + x_row[i] + kk * 16);
#pragma unroll
        for (int i = 0; i < WB; ++i) wf[buf][i] = *reinterpret_cast<const bf16x8*>(bt + w_row[i] + kk * 16);
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int ni = 0; ni < WB; ++ni)
#pragma unroll
            for (int mi = 0; mi < TB; ++mi)
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][ni], xf[buf][mi], acc[ni][mi], 0, 0, 0);
    };

#pragma unroll
    for (int j = 0; j < NI; ++j) load_item(0, j, 0);
#pragma unroll
    for (int j = 0; j < NI; ++j) store_item(0, j, 0);
    {
        const int k_last0 = (k_tiles - 1) * BK;
#pragma unroll
        for (int j = 0; j < NI; ++j) load_item(1, j, BK < k_last0 ? BK : k_last0);
#pragma unroll
        for (int j = 0; j < NI; ++j) load_item(0, j, 2 * BK < k_last0 ? 2 * BK : k_last0);
    }
    __syncthreads();
    load_frags(0, 0, 0);
    // items moved per step (steps 0..2): set (kt+1)&1 -> LDS as tile kt+1, then refilled with tile kt+3
    constexpr int PER = (NI + 2) / 3;
    // ODD (parity of kt) is compile-time so the register sets and LDS buffers are addressed
    // statically, and the body has no branches (a branch would make the compiler drain every
    // outstanding load).  Near the end of K the body still moves data: the loads are clamped to
    // the last tile and the surplus lands in an LDS buffer nobody reads any more.
    const int k_last = (k_tiles - 1) * BK;
    auto iteration = [&](auto odd_c, int kt) {
        constexpr int ODD = decltype(odd_c)::value;
        constexpr int cur = ODD, nxt = ODD ^ 1;  // LDS buffer of tile kt / of tile kt+1 (= its register set)
        int k3 = (kt + 3) * BK;
        k3 = k3 < k_last ? k3 : k_last;
        auto move_items = [&](int step) {
#pragma unroll
            for (int j = step * PER; j < (step + 1) * PER && j < NI; ++j) {
                store_item(nxt, j, nxt);
                load_item(nxt, j, k3);
            }
        };
        // step 0
        load_frags(1, cur, 1);
        move_items(0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(0);
        __builtin_amdgcn_sched_barrier(0);
        // step 1
        load_frags(0, cur, 2);
        move_items(1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(1);
        __builtin_amdgcn_sched_barrier(0);
        // step 2
        load_frags(1, cur, 3);
        move_items(2);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(0);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        // step 3
        load_frags(0, nxt, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(1);
        __builtin_amdgcn_sched_barrier(0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    int kt = 0;
    for (; kt + 1 < k_tiles; kt += 2) {
        iteration(I0{}, kt);
        iteration(I1{}, kt + 1);
    }
    if (kt < k_tiles) iteration(I0{}, kt);

    // ---- epilogue: lane holds, per block, token lane%32 and weight rows 8g + 4*(lane/32) + 0..3 ---
    constexpr int NB = EPI == kSwiglu ? WB / 2 : WB;
    const int col0 = n0 + wn * (BNO / WN) + (lane >> 5) * 4;
#pragma unroll
    for (int mi = 0; mi < TB; ++mi) {
        const int r = row0 + wm * (BM / WM) + mi * 32 + (lane & 31);
        if (r >= row_end) continue;
        bf16_t* crow = c + (size_t)r * N;
#pragma unroll
        for (int ni = 0; ni < NB; ++ni) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = col0 + ni * 32 + 8 * g;
                if (n >= N) continue;
                floatx4 v;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float t = acc[ni][mi][4 * g + q];
                    if (EPI == kSwiglu) t = t / (1.0f + __expf(-t)) * acc[ni + NB][mi][4 * g + q];
                    if (EPI == kRelu) t = fmaxf(t, 0.0f);
                    v[q] = t;
                }
                bf16x4 o = __builtin_convertvector(v, bf16x4);
                *reinterpret_cast<bf16x4*>(crow + n) = o;
            }
        }
    }
}

constexpr int kWavesM = 2, kWavesN = 2;

template <int EPI, bool KTAIL>
hipError_t launch_cfg(const bf16_t* a, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c,
                      unsigned blocks, int S, int N, int K, int n_tiles, hipStream_t st) {
    auto kern = grouped_gemm_bf16<EPI, kWavesM, kWavesN, KTAIL>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    kern<<<blocks, 64 * kWavesM * kWavesN, LDS_BYTES, st>>>(a, offsets, b0, b1, c, S, N, K, n_tiles);
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_one(const bf16_t* a, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c, int A,
                      int S, int N, int K, hipStream_t st) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    const int n_tiles = (N + BNO - 1) / BNO;
    const int m_tiles = (A + BM - 1) / BM + S;
    long long blocks = (long long)n_tiles * m_tiles;
    blocks = (blocks + XCDS - 1) / XCDS * XCDS;
    if (K % BK == 0) return launch_cfg<EPI, false>(a, offsets, b0, b1, c, (unsigned)blocks, S, N, K, n_tiles, st);
    return launch_cfg<EPI, true>(a, offsets, b0, b1, c, (unsigned)blocks, S, N, K, n_tiles, st);
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
