// Gate logits and resident-restricted top-k for bf16 inputs (eMoE Section 1: the gate; Section
// 3.2.2, last paragraph: a token whose expert is not on the GPU goes to its next-best expert that
// is), with the logits of 32 tokens computed together on the matrix cores.
//
// A workgroup of four wavefronts owns 32 tokens.  logit[t, e] = sum_i x[t, i] * Wg[e, i] is a
// 32-token x (16, 32 or 64)-expert product with K = d_model: the gate rows go on the row operand
// of v_mfma_f32_32x32x16_bf16 and the token rows on the column operand, so every gate row fetched
// is used for 32 tokens (a wavefront per token re-reads the whole gate matrix per token, which at
// 64 experts costs several times the read of x).
// K is walked in tiles of 128 elements.  A tile (32 token row pieces and the gate row pieces, 256
// bytes each) goes from global memory straight into LDS with buffer_load_dwordx4 ... lds, 1 KiB
// of whole row pieces per instruction, so memory is read in full cache lines; a lane-per-row
// register load would touch 32 rows per instruction and is bound by the L1's tag rate instead.
// In LDS the 16-byte chunk c of row r sits at chunk position c ^ (r & 15), which makes the MFMA
// fragment reads (32 rows x one chunk) bank-conflict free.  The kernel is bound by the latency of
// the x stream, so as many tile stages as fit in LDS are kept in flight.
// The four wavefronts split the eight MFMA steps of a tile; their partial logits meet in LDS and
// are added in wavefront order: fp32 accumulation, summation order fixed by the code.
//
// Wavefront 0 then holds, per lane, token lane%32 and 16 (or 32) of its logits, the other half
// being in lane^32.  Top-k is k rounds of: best available logit of this lane (ascending expert
// order, strict comparison, so the lower index wins a tie), one exchange with the partner lane,
// winner marked taken.  Weights are the softmax over the k winners.
#include <atomic>

#include "common.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int TOK = 32;                   // tokens per workgroup
constexpr int BK = 128;                   // K elements per tile
constexpr int ROW_BYTES = BK * 2;         // 256
constexpr int X_BYTES = TOK * ROW_BYTES;  // 8 KiB
constexpr int CPR = ROW_BYTES / 16;       // 16-byte chunks per tile row
constexpr int RPI = 1024 / ROW_BYTES;     // tile rows filled by one load instruction
constexpr int SPW = BK / 16 / 4;          // MFMA steps per wavefront and tile
constexpr int LX = X_BYTES / 1024 / 4;    // token load instructions per wavefront and tile
constexpr unsigned kRotation = 21;        // K-tile rotation per workgroup

// s_waitcnt immediate: vmcnt <= n and all LDS traffic done (vmcnt[3:0] | [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int wait_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0x0 << 8); }

// Workgroup barrier that leaves up to N global->LDS loads of this wavefront pending
// (__syncthreads() would drain them all).
template <int N>
__device__ __forceinline__ void barrier_keep_loads() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(wait_imm(N));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// WR = gate rows in a tile (16, 32 or 64 >= E; rows past E repeat row E-1 and are masked out).
template <int WR, int STAGES, bool KTAIL>
__global__ __launch_bounds__(256) void route_mfma_kernel(const bf16_t* __restrict__ x,
                                                         const bf16_t* __restrict__ w_gate,
                                                         const float* __restrict__ bias,
                                                         const int32_t* __restrict__ slot_of_expert,
                                                         int32_t* __restrict__ topk_expert,
                                                         float* __restrict__ topk_weight,
                                                         unsigned long long* __restrict__ expert_tokens, int T_,
                                                         int K, int E, int k) {
    constexpr int NB = WR == 64 ? 2 : 1;             // MFMA row blocks
    constexpr int W_BYTES = WR * ROW_BYTES;
    constexpr int STAGE_BYTES = W_BYTES + X_BYTES;
    constexpr int LW = W_BYTES / 1024 / 4;           // gate load instructions per wavefront and tile
    constexpr int LOADS = LW + LX;
    static_assert(LW >= 1 && (STAGES - 1) * LOADS < 64, "vmcnt counts at most 63 loads");
    static_assert(3 * NB * 16 * 64 * 4 <= STAGES * STAGE_BYTES, "the reduction reuses the tile stages");
    extern __shared__ __align__(16) char lds[];
    float* s_bias = reinterpret_cast<float*>(lds + STAGES * STAGE_BYTES);
    int* s_resident = reinterpret_cast<int*>(s_bias + kMaxExperts);
    int* s_hist = s_resident + kMaxExperts;  // this workgroup's tokens per expert under ordinary routing
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (threadIdx.x < kMaxExperts) {
        const int e = threadIdx.x;
        s_bias[e] = (bias != nullptr && e < E) ? bias[e] : 0.0f;
        s_resident[e] = (e < E && slot_of_expert[e] >= 0) ? 1 : 0;
        s_hist[e] = 0;
    }
    const int t0 = blockIdx.x * TOK;

    // ---- global -> LDS: instruction (w, i) fills RPI tile rows; lane l lands in row l/CPR, chunk
    //      position l%CPR and fetches global chunk (l%CPR) ^ (row&15) ------------------------------
    const int l_rin = lane / CPR, l_pos = lane % CPR;
    const uint32_t x_bytes = (uint32_t)T_ * (uint32_t)K * 2u;
    const uint32_t w_bytes = (uint32_t)E * (uint32_t)K * 2u;
    uint32_t w_voff[LW], x_voff[LX];
    int w_chunk[LW], x_chunk[LX];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int tr = (LW * wave + i) * RPI + l_rin;  // row of the gate tile
        w_chunk[i] = l_pos ^ (tr & 15);
        const int e = tr < E ? tr : E - 1;
        w_voff[i] = ((uint32_t)e * (uint32_t)K + w_chunk[i] * 8) * 2u;
    }
#pragma unroll
    for (int i = 0; i < LX; ++i) {
        const int tr = (LX * wave + i) * RPI + l_rin;  // row of the token tile
        x_chunk[i] = l_pos ^ (tr & 15);
        int t = t0 + tr;
        t = t < T_ ? t : T_ - 1;  // repeats of the last token, never written out
        x_voff[i] = ((uint32_t)t * (uint32_t)K + x_chunk[i] * 8) * 2u;
    }
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(x), 0, (int)x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(w_gate), 0, (int)w_bytes, 0x00020000);
    auto issue_tile = [&](int stage, int k0) {
        char* base = lds + stage * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            uint32_t v = w_voff[i];
            if (KTAIL && k0 + w_chunk[i] * 8 >= K) v = w_bytes;  // out of range: zeros
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (lds_void*)(base + (LW * wave + i) * 1024), 16, (int)v,
                                                     k0 * 2, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            uint32_t v = x_voff[i];
            if (KTAIL && k0 + x_chunk[i] * 8 >= K) v = x_bytes;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (lds_void*)(base + W_BYTES + (LX * wave + i) * 1024), 16,
                                                     (int)v, k0 * 2, 0, 0);
        }
    };

    // ---- fragment addresses: lane holds row lane%32 and, for MFMA step s, chunk 2s + lane/32 ------
    const int c = lane & 31;
    const int h = lane >> 5;
    const int w_row = WR == 16 ? (c & 15) : c;
    floatx16 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;

    const int k_tiles = (K + BK - 1) / BK;
    // Workgroups walk K from different starting tiles: token rows are a power-of-two-ish stride
    // apart, so workgroups marching through K in step would all pull from the same few HBM channels
    // at once.  The order is fixed per workgroup, so results stay reproducible.
    const int k_rot = (int)((blockIdx.x * kRotation) % (unsigned)k_tiles);
    auto k_of = [&](int t) {
        int tt = t + k_rot;
        return (tt >= k_tiles ? tt - k_tiles : tt) * BK;
    };
#pragma unroll
    for (int t = 0; t < STAGES - 1; ++t)
        if (t < k_tiles) issue_tile(t, k_of(t));
    // loads are counted per wavefront and retire in order: with `pending` tiles issued after tile t,
    // tile t has landed once at most pending * LOADS loads are outstanding
    int stage = 0;
    for (int t = 0; t < k_tiles; ++t) {
        if (t + STAGES - 2 < k_tiles) barrier_keep_loads<(STAGES - 2) * LOADS>();
        else barrier_keep_loads<0>();
        // everyone has finished tile t-1: its stage can take tile t+STAGES-1
        if (t + STAGES - 1 < k_tiles) issue_tile(stage == 0 ? STAGES - 1 : stage - 1, k_of(t + STAGES - 1));
        const char* wt = lds + stage * STAGE_BYTES;
        const char* xt = wt + W_BYTES;
#pragma unroll
        for (int s2 = 0; s2 < SPW; ++s2) {
            const int ch = 2 * (SPW * wave + s2) + h;  // this wavefront's MFMA steps of the tile
            const bf16x8 xf = *reinterpret_cast<const bf16x8*>(xt + c * ROW_BYTES + ((ch ^ (c & 15)) * 16));
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const bf16x8 wf = *reinterpret_cast<const bf16x8*>(wt + (32 * b + w_row) * ROW_BYTES +
                                                                   ((ch ^ (w_row & 15)) * 16));
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[b], 0, 0, 0);
            }
        }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
    }

    // the wavefronts' shares of K meet in LDS (the tile stages, all consumed), added in wavefront order
    barrier_keep_loads<0>();
    float* red = reinterpret_cast<float*>(lds);  // [wavefront - 1][NB * 16][64]
    if (wave > 0) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[((wave - 1) * NB * 16 + b * 16 + v) * 64 + lane] = acc[b][v];
    }
    __syncthreads();
    if (wave > 0) return;

    // Register i = 16 b + 4 g + r of this lane is the logit of expert 32 b + 8 g + 4 h + r.
    float logit[NB * 16];
#pragma unroll
    for (int i = 0; i < NB * 16; ++i) logit[i] = acc[i >> 4][i & 15];
#pragma unroll 1
    for (int w = 0; w < 3; ++w) {
#pragma unroll
        for (int i = 0; i < NB * 16; ++i) logit[i] += red[(w * NB * 16 + i) * 64 + lane];
    }
    const int t = t0 + c;
    const bool live = t < T_;
    uint32_t avail = 0, exists = 0;
#pragma unroll
    for (int i = 0; i < NB * 16; ++i) {
        const int e = 32 * (i >> 4) + 8 * ((i >> 2) & 3) + 4 * h + (i & 3);
        logit[i] += s_bias[e];
        if (s_resident[e]) avail |= 1u << i;
        if (e < E) exists |= 1u << i;
    }

    constexpr int kNone = 0x7fffffff;
    float top_v = 0.0f, sum = 0.0f;
    const size_t out0 = (size_t)t * k;
    for (int j = 0; j < k; ++j) {
        float bv = 0.0f;
        int bi = -1;
#pragma unroll
        for (int i = 0; i < NB * 16; ++i) {  // ascending expert order within the lane
            const bool ok = (avail >> i) & 1u;
            if (ok && (bi < 0 || logit[i] > bv)) { bv = logit[i]; bi = i; }
        }
        const int be = bi < 0 ? kNone : 32 * (bi >> 4) + 8 * ((bi >> 2) & 3) + 4 * h + (bi & 3);
        const float ov = __shfl_xor(bv, 32);
        const int oe = __shfl_xor(be, 32);
        const bool mine = be != kNone && (oe == kNone || bv > ov || (bv == ov && be < oe));
        float win_v = mine ? bv : ov;
        int win_e = mine ? be : oe;
        if (win_e == kNone) {  // fewer than k resident experts: precondition broken, stay defined
            win_e = 0;
            win_v = 0.0f;
        }
        if (mine) avail &= ~(1u << bi);
        if (j == 0) top_v = win_v;
        const float p = expf(win_v - top_v);
        sum += p;
        if (live && h == 0) {
            topk_expert[out0 + j] = win_e;
            topk_weight[out0 + j] = p;  // divided by the sum below
        }
    }
    if (live && h == 0) {
        for (int j = 0; j < k; ++j) topk_weight[out0 + j] = topk_weight[out0 + j] / sum;
    }

    // Workload (Section 3.2.2: the number of tokens an expert receives): the same k rounds over all
    // E experts, resident or not; integer counts, so the accumulated result does not depend on order.
    if (expert_tokens == nullptr) return;
    for (int j = 0; j < k; ++j) {
        float bv = 0.0f;
        int bi = -1;
#pragma unroll
        for (int i = 0; i < NB * 16; ++i) {
            const bool ok = (exists >> i) & 1u;
            if (ok && (bi < 0 || logit[i] > bv)) { bv = logit[i]; bi = i; }
        }
        const int be = bi < 0 ? kNone : 32 * (bi >> 4) + 8 * ((bi >> 2) & 3) + 4 * h + (bi & 3);
        const float ov = __shfl_xor(bv, 32);
        const int oe = __shfl_xor(be, 32);
        const bool mine = be != kNone && (oe == kNone || bv > ov || (bv == ov && be < oe));
        const int win_e = mine ? be : oe;
        if (mine) exists &= ~(1u << bi);
        if (live && h == 0 && win_e != kNone) atomicAdd(&s_hist[win_e], 1);
    }
    // one wavefront: its LDS operations complete in program order
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    if (lane < E) {
        const int n = s_hist[lane];
        if (n > 0) atomicAdd(&expert_tokens[lane], (unsigned long long)n);
    }
}

}  // namespace

namespace {

template <int WR, int STAGES, bool KTAIL>
hipError_t launch_cfg(const emoe_layer_desc& d, const bf16_t* x, const bf16_t* wg, const float* bias,
                      const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                      unsigned long long* expert_tokens, hipStream_t st) {
    constexpr int kLds = STAGES * (WR * ROW_BYTES + X_BYTES) + kMaxExperts * 12;
    static_assert(kLds <= 160 * 1024, "LDS of one CU");
    auto kern = route_mfma_kernel<WR, STAGES, KTAIL>;
    static std::atomic<bool> attr_set{false};  // set once per kernel; setting it twice from two threads is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    kern<<<(d.T + TOK - 1) / TOK, 256, kLds, st>>>(x, wg, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, d.T,
                                                  d.d_model, d.E, d.k);
    return hipGetLastError();
}

template <int WR, int STAGES>
hipError_t launch_wr(const emoe_layer_desc& d, const bf16_t* x, const bf16_t* wg, const float* bias,
                     const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                      unsigned long long* expert_tokens, hipStream_t st) {
    if (d.d_model % BK == 0)
        return launch_cfg<WR, STAGES, false>(d, x, wg, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
    return launch_cfg<WR, STAGES, true>(d, x, wg, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
}

}  // namespace

hipError_t launch_route_bf16(const emoe_layer_desc& d, const void* x, const void* w_gate, const float* bias,
                             const int32_t* slot_of_expert, int32_t* topk_expert, float* topk_weight,
                             unsigned long long* expert_tokens, hipStream_t st) {
    const bf16_t* xp = static_cast<const bf16_t*>(x);
    const bf16_t* wg = static_cast<const bf16_t*>(w_gate);
    // as many stages as LDS holds (12 / 16 / 24 KiB each), within the 63 loads vmcnt can count
    if (d.E <= 16) return launch_wr<16, 13>(d, xp, wg, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
    if (d.E <= 32) return launch_wr<32, 9>(d, xp, wg, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
    return launch_wr<64, 6>(d, xp, wg, bias, slot_of_expert, topk_expert, topk_weight, expert_tokens, st);
}

}  // namespace emoe
