// Expert FFN for bf16 layers with few rows per slot (a decode step): the cost is reading each
// resident, non-empty slot's weights from HBM exactly once (eMoE Section 5.1: fewer experts
// means fewer global-memory reads), so the kernels are shaped for streaming, not for MFMA rate.
//
// A workgroup (4 wavefronts, two workgroups per CU) owns 64 weight rows of one slot - in the
// SwiGLU pass 32 rows of W1 and the same 32 rows of W3 - and walks K in tiles of 128.  A tile goes
// from global memory straight into LDS with buffer_load_dwordx4 ... lds: every load instruction
// reads 1 KiB that is contiguous in LDS and consists of whole 256-byte row pieces in memory, so
// HBM is read in full cache lines no matter what layout the MFMA wants.  Three LDS stages per
// workgroup keep two tiles in flight; with two workgroups per CU that is 64 KiB of weights in flight
// per CU, enough to cover HBM latency at full bandwidth.  The slot's token rows (at most 32 per
// pass, they live in L2) ride along in the same tiles.
// In LDS the 16-byte chunk c of row r sits at chunk position c ^ (r & 15): the MFMA fragment reads
// (32 rows x one chunk) are then bank-conflict free.
// The weight rows are the MFMA's row operand (v_mfma_f32_32x32x16_bf16), the tokens its column
// operand, so a weight element is used for every token.  The four wavefronts split the eight MFMA
// K-steps of a tile; their partial sums meet in LDS at the end, added in wavefront order, so the
// result is reproducible.  A slot with no rows exits before it touches its weights; a slot with more
// than 32 rows is processed 32 rows at a time (the repeated weight reads come from cache).
#include "common.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

enum Epilogue { kPlain = 0, kSwiglu = 1, kRelu = 2 };
// weight rows per workgroup: template parameter WR, 64 (two MFMA row blocks) or 32 (one; plain and
// ReLU passes only, used when 64-row units would give fewer workgroups than the chip can hold).
// A 32-row unit's stage is half token rows, so it gets five stages instead of three (80 KiB, still
// two workgroups per CU): 64 KiB of weights in flight per CU like the 64-row units, where three
// workgroups of three stages hold 48 (second product of the Mixtral decode step: 126 -> 120 us).
constexpr int TOK = 32;                     // token rows per pass
constexpr int BK = 128;                     // K elements per tile
constexpr int ROW_BYTES = BK * 2;           // 256
constexpr int X_BYTES = TOK * ROW_BYTES;    // 8 KiB
constexpr int kMinStages = 3;               // LDS stages of one K tile each: 3 at 64 weight rows, 5 at 32
constexpr int CPR = ROW_BYTES / 16;         // 16-byte chunks per tile row
constexpr int RPI = 1024 / ROW_BYTES;       // tile rows filled by one load instruction
constexpr int SPW = BK / 16 / 4;            // MFMA steps per wavefront and tile
constexpr int LX = X_BYTES / 1024 / 4;      // token load instructions per wavefront and tile
// cache policy of the weight loads: every weight byte is read once per launch (non-temporal: bit 1 of the aux operand)
constexpr int kStreamOnce = 2;
constexpr unsigned kRotation = 21;           // K-tile rotation per workgroup (measured best of 1..29)
constexpr int RED_BYTES = 3 * 32 * 64 * 4;  // partial sums of wavefronts 1..3
static_assert(RED_BYTES <= kMinStages * (32 * ROW_BYTES + X_BYTES), "the reduction reuses the tile stages");

// s_waitcnt immediate: vmcnt <= n and all LDS traffic done (vmcnt[3:0] | [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int wait_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0x0 << 8); }

// Workgroup barrier that leaves up to N global->LDS loads of this wavefront pending
// (__syncthreads() would drain them all).  The empty asm statements keep the compiler from moving
// LDS accesses across it.
template <int N>
__device__ __forceinline__ void barrier_keep_loads() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(wait_imm(N));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// grid.x = S * ceil(N / BNO) workgroups, BNO = output columns per workgroup (32 SwiGLU, else 64).
template <int EPI, int WR, bool KTAIL>
__global__ __launch_bounds__(256, 2) void stream_gemm_bf16(const bf16_t* __restrict__ a, RowGather gather,
                                                           const int32_t* __restrict__ offsets,
                                                           const bf16_t* __restrict__ b0,
                                                           const bf16_t* __restrict__ b1, bf16_t* __restrict__ c,
                                                           int S, int N, int K, int n_units) {
    constexpr int BNO = EPI == kSwiglu ? WR / 2 : WR;
    constexpr int W_BYTES = WR * ROW_BYTES;          // 16 KiB at WR = 64
    constexpr int STAGE_BYTES = W_BYTES + X_BYTES;
    constexpr int LW = W_BYTES / 1024 / 4;           // weight load instructions per wavefront and tile
    constexpr int LOADS = LW + LX;
    constexpr int NBLK = WR / 32;                    // MFMA row blocks
    static_assert(WR == 64 || (WR == 32 && EPI != kSwiglu), "unsupported unit shape");
    constexpr int STAGES = WR == 64 ? 3 : 5;
    __shared__ __align__(16) char lds[STAGES * STAGE_BYTES];
    const int slot = blockIdx.x / n_units;
    const int n0 = (blockIdx.x % n_units) * BNO;
    const int row0 = offsets[slot], row_end = offsets[slot + 1];
    if (row_end <= row0) return;  // empty slot: its weights are never touched
    const int rows_total = offsets[S];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // ---- global -> LDS: instruction (w, i) fills RPI tile rows; lane l lands in row l/CPR, chunk
    //      position l%CPR and fetches global chunk (l%CPR) ^ (row&15) ------------------------------
    const int l_rin = lane / CPR, l_pos = lane % CPR;
    const uint32_t a_bytes = (uint32_t)(gather.perm != nullptr ? gather.rows : rows_total) * (uint32_t)K * 2u;
    const uint32_t b_bytes = (uint32_t)N * (uint32_t)K * 2u;
    uint32_t w_voff[LW];
    int w_chunk[LW];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int tr = (LW * wave + i) * RPI + l_rin;  // row of the weight tile
        w_chunk[i] = l_pos ^ (tr & 15);
        int n = n0 + (EPI == kSwiglu ? tr % (WR / 2) : tr);  // SwiGLU: rows 32..63 = same rows of W3
        n = n < N ? n : N - 1;
        w_voff[i] = ((uint32_t)n * (uint32_t)K + w_chunk[i] * 8) * 2u;
    }
    const bf16_t* wsel = (EPI == kSwiglu && wave >= 2) ? b1 : b0;  // wavefronts 2,3 load the W3 half
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a), 0, (int)a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(wsel + (size_t)slot * N * K), 0, (int)b_bytes, 0x00020000);

    // ---- fragment addresses: lane holds row lane%32 and, for MFMA step s, chunk 2s + lane/32 ------
    const int f_row = lane & 31;
    const int f_half = lane >> 5;
    const int k_tiles = (K + BK - 1) / BK;
    // Workgroups walk K from different starting tiles.  Rows are a power-of-two-ish stride apart, so
    // workgroups marching through K in step would all pull from the same few HBM channels at once;
    // the rotation spreads them (4.8 -> 5.7 TB/s at the Mixtral decode shape).  The order is fixed
    // per workgroup, so results stay reproducible.
    const int k_rot = (int)((blockIdx.x * kRotation) % (unsigned)k_tiles);
    auto k_of = [&](int t) {
        int tt = t + k_rot;
        return (tt >= k_tiles ? tt - k_tiles : tt) * BK;
    };

    for (int tok0 = row0; tok0 < row_end; tok0 += TOK) {  // 32 tokens per pass over the weights
        uint32_t x_voff[LX];
        int x_chunk[LX];
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            const int tr = (LX * wave + i) * RPI + l_rin;  // row of the token tile
            x_chunk[i] = l_pos ^ (tr & 15);
            int r = tok0 + tr;
            const bool past = r >= row_end;  // rows past the slot's end: out of range, zeros without memory traffic
            r = past ? row_end - 1 : r;
            if (gather.perm != nullptr) r = gather.perm[r] / gather.k;  // the token's row of x, not a copy of it
            x_voff[i] = past ? a_bytes : ((uint32_t)r * (uint32_t)K + x_chunk[i] * 8) * 2u;
        }
        auto issue_tile = [&](int stage, int k0) {
            char* base = lds + stage * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < LW; ++i) {
                uint32_t v = w_voff[i];
                if (KTAIL && k0 + w_chunk[i] * 8 >= K) v = b_bytes;  // out of range: zeros
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_void*)(base + (LW * wave + i) * 1024), 16, (int)v,
                                                         k0 * 2, 0, kStreamOnce);
            }
#pragma unroll
            for (int i = 0; i < LX; ++i) {
                uint32_t v = x_voff[i];
                if (KTAIL && k0 + x_chunk[i] * 8 >= K) v = a_bytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void*)(base + W_BYTES + (LX * wave + i) * 1024), 16,
                                                         (int)v, k0 * 2, 0, 0);
            }
        };

        floatx16 acc0, acc1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc0[v] = 0.0f; acc1[v] = 0.0f; }

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
                const int s = SPW * wave + s2;  // this wavefront's MFMA steps of the tile
                const int ch = 2 * s + f_half;
                const bf16x8 xf = *reinterpret_cast<const bf16x8*>(xt + f_row * ROW_BYTES + ((ch ^ (f_row & 15)) * 16));
                const bf16x8 w0f = *reinterpret_cast<const bf16x8*>(wt + f_row * ROW_BYTES + ((ch ^ (f_row & 15)) * 16));
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0f, xf, acc0, 0, 0, 0);
                if (NBLK == 2) {
                    const bf16x8 w1f =
                        *reinterpret_cast<const bf16x8*>(wt + (32 + f_row) * ROW_BYTES + ((ch ^ (f_row & 15)) * 16));
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1f, xf, acc1, 0, 0, 0);
                }
            }
            stage = stage + 1 == STAGES ? 0 : stage + 1;
        }

        // ---- partial sums of the four K splits meet in LDS; wavefront 0 adds them in order -----------
        barrier_keep_loads<0>();  // all tiles consumed: the stages can be reused
        float* red = reinterpret_cast<float*>(lds);
        if (wave > 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                red[((wave - 1) * 32 + v) * 64 + lane] = acc0[v];
                if (NBLK == 2) red[((wave - 1) * 32 + 16 + v) * 64 + lane] = acc1[v];
            }
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int w = 0; w < 3; ++w)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    acc0[v] += red[(w * 32 + v) * 64 + lane];
                    if (NBLK == 2) acc1[v] += red[(w * 32 + 16 + v) * 64 + lane];
                }
            // lane holds token lane%32 and weight rows 8g + 4*(lane/32) + 0..3 of each 32-row block
            const int r = tok0 + (lane & 31);
            if (r < row_end) {
                const int dr = (EPI == kPlain && gather.out_perm != nullptr) ? gather.out_perm[r] : r;  // combine folded in: the token's row
#pragma unroll
                for (int blk = 0; blk < (EPI == kSwiglu ? 1 : NBLK); ++blk) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int nn = n0 + blk * 32 + 8 * g + (lane >> 5) * 4;
                        if (nn >= N) continue;
                        floatx4 v;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float tv = blk == 0 ? acc0[4 * g + q] : acc1[4 * g + q];
                            if (EPI == kSwiglu) tv = tv / (1.0f + __expf(-tv)) * acc1[4 * g + q];
                            if (EPI == kRelu) tv = fmaxf(tv, 0.0f);
                            v[q] = tv;
                        }
                        *reinterpret_cast<bf16x4*>(c + (size_t)dr * N + nn) = __builtin_convertvector(v, bf16x4);
                    }
                }
            }
        }
        __syncthreads();  // the reduction buffer is tile memory again for the next 32 tokens
    }
}

template <int EPI, int WR>
hipError_t launch_wr(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c, int S,
                     int N, int K, hipStream_t st) {
    constexpr int BNO = EPI == kSwiglu ? WR / 2 : WR;
    const int n_units = (N + BNO - 1) / BNO;
    const unsigned blocks = (unsigned)(S * n_units);
    if (K % BK == 0)
        stream_gemm_bf16<EPI, WR, false><<<blocks, 256, 0, st>>>(a, gather, offsets, b0, b1, c, S, N, K, n_units);
    else
        stream_gemm_bf16<EPI, WR, true><<<blocks, 256, 0, st>>>(a, gather, offsets, b0, b1, c, S, N, K, n_units);
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_one(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c, int S,
                      int N, int K, hipStream_t st) {
    if constexpr (EPI != kSwiglu) {
        // fewer 64-row units than workgroup slots (2 per CU): halve the unit so the whole chip streams
        DeviceShape shape;
        hipError_t es = device_shape(&shape);
        if (es != hipSuccess) return es;
        if ((long long)S * ((N + 63) / 64) < 2 * shape.cus) return launch_wr<EPI, 32>(a, gather, offsets, b0, b1, c, S, N, K, st);
    }
    return launch_wr<EPI, 64>(a, gather, offsets, b0, b1, c, S, N, K, st);
}

}  // namespace

hipError_t launch_ffn_bf16_stream(const emoe_layer_desc& d, const void* x_perm, RowGather gather,
                                  const int32_t* offsets,
                                  const void* w1, const void* w3, const void* w2, void* y_perm, void* ws,
                                  int passes, hipStream_t st) {
    bf16_t* h = reinterpret_cast<bf16_t*>(static_cast<uint8_t*>(ws) + ffn_ws_layout(d).h);
    const bf16_t* xp = static_cast<const bf16_t*>(x_perm);
    hipError_t e = hipSuccess;
    if (!(passes & 1)) {
    } else if (d.act == EMOE_ACT_SWIGLU)
        e = launch_one<kSwiglu>(xp, gather, offsets, static_cast<const bf16_t*>(w1), static_cast<const bf16_t*>(w3), h, d.S,
                                d.d_ff, d.d_model, st);
    else
        e = launch_one<kRelu>(xp, gather, offsets, static_cast<const bf16_t*>(w1), nullptr, h, d.S, d.d_ff, d.d_model, st);
    if (e != hipSuccess || !(passes & 2)) return e;
    return launch_one<kPlain>(h, RowGather{nullptr, 1, 0, gather.out_perm}, offsets, static_cast<const bf16_t*>(w2), nullptr, static_cast<bf16_t*>(y_perm), d.S,
                              d.d_model, d.d_ff, st);
}

}  // namespace emoe
