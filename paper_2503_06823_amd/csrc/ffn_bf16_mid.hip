// Expert FFN for bf16 layers with a few dozen to a few hundred rows per slot: a prompt or two in
// prefill, a large decode batch (eMoE Section 5.5 measures prompts of 512 tokens, which leaves
// 128 rows per expert at top-2 of 8).  In this range the layer is bound by reading the resident
// experts' weights (Section 5.1: fewer experts, fewer global-memory reads) or sits near the ridge
// between that and the matrix cores, and tiles of 256 token rows waste both: a slot of 130 rows
// fills half a tile, a slot of 260 rows takes two.
//
//   pass 1: h[r, n]      = act(x_perm[r,:] . W1_s[n,:]) (* x_perm[r,:] . W3_s[n,:])   K = d_model
//   pass 2: y_perm[r, n] = h[r,:] . W2_s[n,:]                                         K = d_ff
//
// Tile: 128 token rows x 256 weight rows per workgroup (SwiGLU: 128 rows of W1 and the same 128 of
// W3, so the activation is applied in registers); four wavefronts (2 x 2), each 64 tokens x 128
// weight rows = 2 x 4 blocks of v_mfma_f32_32x32x16_bf16, fp32 accumulation.  The weight rows are
// the MFMA's row operand, so a lane ends up with four consecutive output columns of one token.
//
// Data movement: K is walked in tiles of 64 (a tile row = one 128-byte line).  A stage of LDS holds
// the token rows (16 KiB) and the weight rows (32 KiB) of one K tile; both go from global memory
// straight into LDS (buffer_load_dwordx4 ... lds, 1 KiB per instruction, eight rows of 128 bytes).
// Three stages: while tile t is multiplied, tiles t+1 and t+2 are on their way, 64 KiB of weights
// in flight per CU, which is what it takes to keep HBM busy at its latency.  The narrow token tile
// is what buys the third stage: with 256 token rows only two and a half stages fit.
// Up to 48 rows per slot on average the token tile is 64 rows (one row of four wavefronts, each 64
// tokens x 64 weight rows): a stage is 8 + 32 KiB, four stages fit, 96 KiB of weights in flight,
// and the weight panel of a slot of one m-tile is loaded with the non-temporal hint (first
// product at the Mixtral shape, 8 slots of 22-38 rows: 345 -> 310 us, 6.1 TB/s).  With 128 weight
// rows (plain and ReLU products) the 64-row arrangement has six stages of 8 + 16 KiB, 80 KiB of
// weights in flight (second product at the same shape: 171 -> 149 us, 6.3 TB/s).
// The 16-byte chunk c of row r sits at chunk position c ^ ((r >> 1) & 7), chosen by which global
// chunk a lane fetches, so the MFMA fragment reads (32 rows x one chunk) have no bank conflicts.
// Chunks past K (when K is not a multiple of 64), rows past the slot's end and weight rows past N
// are addressed out of range of their buffer: zeros arrive and no memory is touched.
//
// Work distribution.  Group sizes live on the device; everything is derived from slot_offsets there.
// Tiles are numbered slot by slot, and inside a slot all m-tiles of an n-tile are consecutive;
// workgroup ids go round-robin over the 8 XCDs and are remapped so that an XCD works on consecutive
// tiles: the m-tiles that share a weight panel run at the same time behind the same L2, and the
// panel is fetched from HBM once.
//  - Tiles of 256 weight rows: one workgroup per output tile, not persistent (tiles are short, at most
//    64 K tiles of half the work of the large kernel's, and the hardware's dispatcher balances
//    them); the launch covers an upper bound of tiles and surplus workgroups exit.
//  - Tiles of 128 weight rows (five stages; taken when tiles of 256 would number no more than the
//    CUs): the same with a short K; with a long one (64 K tiles or more) a persistent launch, one
//    workgroup per CU.  With clearly fewer tiles than CUs (a decode batch over two resident experts
//    at the Mixtral shape: 64) a workgroup per tile would leave CUs idle while the others each walk
//    a long K; instead all tiles' K tiles, in tile order, form one sequence that is cut into equal
//    consecutive shares, one per workgroup.  A share covers the end of one tile and the start of
//    the next: each piece leaves its fp32 accumulators in the workspace, and a second kernel adds
//    the pieces of a tile in K order (deterministic) and applies the epilogue.  That is done only
//    when it spares every workgroup a walk of 48 K tiles: the pieces are extra traffic.  Otherwise
//    the workgroups take whole tiles and nothing is cut.
#include <atomic>
#include <type_traits>

#include "common.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kTileRows = 128;             // token rows per tile (64 in the variant for slots of few rows)
constexpr int BK = 64;                     // K elements per tile
constexpr int ROW_BYTES = BK * 2;          // 128
constexpr int NW = 4;                      // wavefronts: 2 (tokens) x 2 (weight rows)
constexpr int TB = 2;                      // 32-token blocks per wavefront
constexpr unsigned kRotation = 21;          // K-tile rotation per slot (best of 5, 21, 37 and an even spread)

enum Epilogue { kPlain = 0, kSwiglu = 1, kRelu = 2 };

// s_waitcnt immediate: vmcnt <= n, all LDS traffic done (vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int wait_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0x0 << 8); }

// Workgroup barrier that leaves up to N of this wavefront's global->LDS loads pending (loads retire
// in order, so "at most N pending" means everything older has landed) and waits for its LDS reads.
template <int N>
__device__ __forceinline__ void barrier_keep_loads() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(wait_imm(N));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

constexpr int kGroups = kMaxGroups;  // the persistent launch has one workgroup per CU, at most this many
constexpr int kMinShare = 8;     // K tiles per workgroup, at least, when tiles are cut
constexpr int kMinSpared = 48;   // tiles are cut only if that shortens every workgroup's K walk by this many K tiles
constexpr long long kRowsPerSlot64 = 48;  // up to that many rows per slot on average: token tiles of 64 rows
constexpr int kMinPersistK = 64; // K tiles from which on the persistent launch (which may cut) is used at all

// The tiles of a launch and how a persistent launch shares them out, derived from slot_offsets by
// every wavefront: lane s holds slot s's rows and the number of its first tile.
struct Work {
    int s_begin, s_end, s_mtiles, first;  // per lane (= slot)
    int tiles;                            // all output tiles
    int kt;                               // K tiles per output tile
    long long units;                      // tiles * kt: the sequence that is cut into shares
    int sharers;                          // > 0: tiles are cut, that many workgroups take equal shares; 0: whole tiles
};
__device__ __forceinline__ Work make_work(const int32_t* __restrict__ offsets, int S, int n_tiles, int K, int lane, int G,
                                          int bm) {
    Work w;
    w.s_begin = lane < S ? offsets[lane] : 0;
    w.s_end = lane < S ? offsets[lane + 1] : 0;
    w.s_mtiles = (w.s_end - w.s_begin + bm - 1) / bm;
    const int span = w.s_mtiles * n_tiles;
    int incl = span;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    w.first = incl - span;
    w.tiles = __builtin_amdgcn_readlane(incl, 63);
    w.kt = (K + BK - 1) / BK;
    w.units = (long long)w.tiles * w.kt;
    // Cutting pays when it spares every workgroup a K walk of some length: the pieces are extra traffic
    // and the second kernel has work to do (a fine-grained layer with K = 2048, 176 tiles: 57 -> 72 us
    // when cut regardless).
    long long p = w.units / kMinShare;
    p = p < G ? p : G;
    const long long share = p > 0 ? (w.units + p - 1) / p : 0;
    w.sharers = (p > w.tiles && w.kt - share >= kMinSpared) ? (int)p : 0;
    return w;
}
// first unit of share g (g = 0 .. sharers; share g is [share_begin(g), share_begin(g + 1)); from sharers on: empty)
__device__ __forceinline__ long long share_begin(const Work& w, int g) {
    return g >= w.sharers ? w.units : w.units * g / w.sharers;
}
// the share that holds unit u: the largest g with share_begin(g) <= u
__device__ __forceinline__ int share_of(const Work& w, long long u) {
    return (int)(((u + 1) * w.sharers + w.units - 1) / w.units) - 1;
}
// tile number -> slot, first row, end of the slot's rows, n-tile
__device__ __forceinline__ void decode_tile(const Work& w, int S, int lane, int L, int bm, int& slot, int& row0,
                                            int& row_end, int& nt, int& mtiles) {
    // an empty slot starts where its successor does: the last slot that starts at or before L holds it
    slot = __popcll(__ballot(lane < S && w.first <= L)) - 1;
    const int rem = L - __builtin_amdgcn_readlane(w.first, slot);
    mtiles = __builtin_amdgcn_readlane(w.s_mtiles, slot);
    const int mt = rem % mtiles;
    nt = rem / mtiles;
    row0 = __builtin_amdgcn_readlane(w.s_begin, slot) + mt * bm;
    row_end = __builtin_amdgcn_readlane(w.s_end, slot);
}
// where a piece's accumulators go: workgroup g leaves at most two pieces, the end of the tile its
// share starts in (kb > 0) and the start of the tile its share ends in
__device__ __forceinline__ int piece_slot(int g, bool starts_inside) { return 2 * g + (starts_inside ? 0 : 1); }

// BR: weight rows per tile, 256 or 128 (SwiGLU: half of them rows of W1, half the same rows of W3).
// STAGES: LDS stages of one K tile each (token rows + weight rows), STAGES - 1 of them in flight.
// PERSIST: one workgroup per CU that takes whole tiles or, when they are few, an equal share of all
// tiles' K tiles; otherwise one workgroup per tile and surplus workgroups exit.
template <int EPI, int BM, int BR, int STAGES, bool KTAIL, bool PERSIST>
__global__ __launch_bounds__(64 * NW) void mid_gemm_bf16(const bf16_t* __restrict__ a, RowGather gather,
                                                     const int32_t* __restrict__ offsets,
                                                     const bf16_t* __restrict__ b0, const bf16_t* __restrict__ b1,
                                                     bf16_t* __restrict__ c, float* __restrict__ partials, int S, int N,
                                                     int K, int n_tiles, int XCDS) {
    constexpr int W_TILE = BR * ROW_BYTES;             // 32 or 16 KiB
    constexpr int X_TILE = BM * ROW_BYTES;             // 16 or 8 KiB
    constexpr int STAGE_BYTES = X_TILE + W_TILE;
    constexpr int WM = BM / 64, WN = NW / WM;          // wavefronts along the tokens (64 each) and along the weight rows
    constexpr int LX = BM / 8 / NW;                    // token load instructions per wavefront and K tile (4 or 2)
    constexpr int WB = BR / WN / 32;                   // 32-row weight blocks per wavefront (4 or 2)
    static_assert(BM == 128 || BM == 64, "two or one wavefront rows of 64 tokens");
    static_assert(EPI != kSwiglu || WB % 2 == 0, "a wavefront holds gate and up blocks of the same columns");
    constexpr int LW = BR / 8 / NW;                    // weight load instructions per wavefront and K tile
    constexpr int LPT = LX + LW;                       // loads per wavefront and K tile
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;  // output columns per tile
    constexpr int NB = EPI == kSwiglu ? WB / 2 : WB;   // output column blocks per wavefront
    static_assert((STAGES - 1) * LPT <= 63, "vmcnt counts 63 loads");
    static_assert(BM * BNO * 2 <= STAGES * STAGE_BYTES, "the output image reuses the stages");
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int G = gridDim.x;
    const Work work = make_work(offsets, S, n_tiles, K, lane, G, BM);
    // workgroup ids go round-robin over the XCDs: g numbers them XCD by XCD
    const int xcd = blockIdx.x % XCDS, idx = blockIdx.x / XCDS;
    const int g = xcd * (G / XCDS) + idx;
    // What this workgroup does, as a walk over tiles [L, L_end) in steps of L_step (whole tiles), or over
    // K-tile units [u, u_end) of the tile sequence (a share).
    const bool cut = PERSIST && work.sharers > 0;
    int L, L_end, L_step;
    long long u = 0, u_end = 0;
    if (!PERSIST) {  // one tile: XCD x holds tiles x * per_xcd .. in the order they are dispatched
        const int per_xcd = (work.tiles + XCDS - 1) / XCDS;
        L = xcd * per_xcd + idx;
        L_end = (idx < per_xcd && L < work.tiles) ? L + 1 : L;
        L_step = 1;
    } else if (!cut) {  // whole tiles: XCD x owns a contiguous range, its workgroups take it in turns
        L = (int)((long long)work.tiles * xcd / XCDS) + idx;
        L_end = (int)((long long)work.tiles * (xcd + 1) / XCDS);
        L_step = G / XCDS;
    } else {
        L = L_end = L_step = 0;
        u = share_begin(work, g);
        u_end = share_begin(work, g + 1);
    }
    const int rows_total = offsets[S];

    // ---- lane-constant parts of the addressing -------------------------------------------------------
    // Load instruction (w, i) of an operand fills tile rows (L? * w + i) * 8 .. +7; lane l lands in row
    // l >> 3 of those, chunk position l & 7, and therefore fetches global chunk (l & 7) ^ ((row >> 1) & 7).
    const int l_row = lane >> 3, l_pos = lane & 7;
    const uint32_t a_bytes = (uint32_t)(gather.perm != nullptr ? gather.rows : rows_total) * (uint32_t)K * 2u;
    const uint32_t b_bytes = (uint32_t)N * (uint32_t)K * 2u;
    int x_chunk[LX], w_chunk[LW];
#pragma unroll
    for (int i = 0; i < LX; ++i) x_chunk[i] = l_pos ^ ((((LX * wave + i) * 8 + l_row) >> 1) & 7);
#pragma unroll
    for (int i = 0; i < LW; ++i) w_chunk[i] = l_pos ^ ((((LW * wave + i) * 8 + l_row) >> 1) & 7);
    const bf16_t* wsel = (EPI == kSwiglu && wave >= NW / 2) ? b1 : b0;  // wavefronts 2, 3 load the W3 half
    const __amdgpu_buffer_rsrc_t a_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a), 0, (int)a_bytes, 0x00020000);
    // fragments: lane holds row lane % 32 and, in MFMA K-step kk, chunk 2 kk + lane / 32
    const int f_row = lane & 31;
    const int f_sw = (((lane >> 5) ^ ((f_row >> 1) & 7)) & 7) * 16;
    const int x_off = (wm * 64 + f_row) * ROW_BYTES + f_sw;  // + 32 rows per token block
    int w_off[WB];  // SwiGLU: the first half of the blocks are gate rows, the second half the matching up rows
#pragma unroll
    for (int i = 0; i < WB; ++i) {
        int rr;
        if (EPI == kSwiglu) rr = (i < WB / 2) ? wn * (BR / 2 / WN) + i * 32 : BR / 2 + wn * (BR / 2 / WN) + (i - WB / 2) * 32;
        else rr = wn * (BR / WN) + i * 32;
        w_off[i] = X_TILE + (rr + f_row) * ROW_BYTES + f_sw;
    }

    for (;;) {
        // ---- this trip: K tiles kb .. kb + cnt - 1 of output tile `tile` -----------------------------------
        int tile, kb, cnt;
        if (!cut) {
            if (L >= L_end) break;
            tile = L;
            kb = 0;
            cnt = work.kt;
            L += L_step;
        } else {
            if (u >= u_end) break;
            tile = (int)(u / work.kt);
            kb = (int)(u - (long long)tile * work.kt);
            cnt = (long long)(work.kt - kb) < u_end - u ? work.kt - kb : (int)(u_end - u);
            u += cnt;
        }
        int slot, row0, row_end, nt, slot_mtiles;
        decode_tile(work, S, lane, tile, BM, slot, row0, row_end, nt, slot_mtiles);
        const int n0 = nt * BNO;

        uint32_t x_voff[LX], w_voff[LW];
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            const int tr = (LX * wave + i) * 8 + l_row;
            int r = row0 + tr;
            const bool past = r >= row_end;
            r = past ? row_end - 1 : r;
            if (gather.perm != nullptr) r = gather.perm[r] / gather.k;  // the token's row of x, not a copy of it
            x_voff[i] = past ? a_bytes : ((uint32_t)r * (uint32_t)K + x_chunk[i] * 8) * 2u;
        }
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int tr = (LW * wave + i) * 8 + l_row;
            const int n = n0 + (EPI == kSwiglu ? tr % (BR / 2) : tr);  // SwiGLU: the second half = the same rows of W3
            w_voff[i] = n >= N ? b_bytes : ((uint32_t)n * (uint32_t)K + w_chunk[i] * 8) * 2u;
        }
        const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<bf16_t*>(wsel + (size_t)slot * N * K), 0, (int)b_bytes, 0x00020000);
        const int k_first = kb * BK, k_last = (kb + cnt - 1) * BK;
        // K tile number tk of this trip into stage st.  Past the trip's last tile the loads go on (no
        // branches in the loop) but out of range: zeros land in a stage that nobody reads any more.
        // The tiles of different slots start at different K tiles of their range and wrap around: started
        // together, all workgroups would read the same 128-byte column of rows a power of two apart at the
        // same time, which lands on few memory channels (second product of a layer with d_ff = 8192: 127
        // -> 100 us).  The tiles of one slot share the start: they stay in step, so their common token rows
        // and the weight panel common to its m-tiles are fetched once.  A start per n-tile as well costs up
        // to 15 % once the slot's token rows no longer stay in L2 beside the weight stream.
        const int k_rot = (int)(((unsigned)slot * kRotation) % (unsigned)cnt);
        // once: the weight panel of a slot of one m-tile is read by nobody else, and is loaded with the non-temporal hint
        auto issue_tile = [&](int st, int tk, auto once_tag) {
            constexpr int kWeightAux = decltype(once_tag)::value ? 2 : 0;
            int kk = tk + k_rot;
            kk = kk >= cnt ? kk - cnt : kk;
            int k0 = k_first + kk * BK;
            k0 = k0 < k_last ? k0 : k_last;
#pragma unroll
            for (int i = 0; i < LX; ++i) {
                uint32_t v = x_voff[i];
                if ((KTAIL && k0 + x_chunk[i] * 8 >= K) || tk >= cnt) v = a_bytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void*)(lds + st * STAGE_BYTES + (LX * wave + i) * 1024),
                                                         16, (int)v, k0 * 2, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < LW; ++i) {
                uint32_t v = w_voff[i];
                if ((KTAIL && k0 + w_chunk[i] * 8 >= K) || tk >= cnt) v = b_bytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    b_rsrc, (lds_void*)(lds + st * STAGE_BYTES + X_TILE + (LW * wave + i) * 1024), 16, (int)v, k0 * 2, 0, kWeightAux);
            }
        };

        floatx16 acc[WB][TB];
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < TB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

        bf16x8 xf[2][TB], wf[2][WB];
        auto load_frags = [&](int buf, int st, int kk) {
            const char* base = lds + st * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < TB; ++i)
                xf[buf][i] = *reinterpret_cast<const bf16x8*>(base + ((x_off + i * 32 * ROW_BYTES) ^ (kk * 32)));
#pragma unroll
            for (int i = 0; i < WB; ++i) wf[buf][i] = *reinterpret_cast<const bf16x8*>(base + (w_off[i] ^ (kk * 32)));
        };
        auto mfma_step = [&](int buf) {
#pragma unroll
            for (int ni = 0; ni < WB; ++ni)
#pragma unroll
                for (int mi = 0; mi < TB; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][ni], xf[buf][mi], acc[ni][mi], 0, 0, 0);
        };
        // a step's MFMAs with its fragment reads and (in the step after the barrier) the tile's
        // global->LDS loads slotted between them, so that no memory instruction queues up behind another
        auto interleave = [&](auto with_loads) {
            constexpr bool LOADS = decltype(with_loads)::value;
#pragma unroll
            for (int i = 0; i < TB * WB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                           // one MFMA
                if (i < TB + WB) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);          // one LDS read
                if (LOADS) __builtin_amdgcn_sched_group_barrier(0x010, (LPT + TB * WB - 1) / (TB * WB), 0);  // VMEM
            }
        };

        // ---- main loop -------------------------------------------------------------------------------------
        // Per K tile four MFMA steps of 16.  The barrier comes before the last step: by then every wavefront
        // holds its last fragments of tile t in registers, so the stage of tile t is free for the data of
        // tile t+STAGES, and tile t+1 has landed once only the loads of tiles t+2 .. t+STAGES-1 are pending.
        // The last step's MFMAs then cover the first fragment reads of tile t+1.
        // A wavefront whose 64 token rows all lie past the slot's end takes part in loads and barriers only.
        auto k_loop = [&](auto idle_tag, auto once_tag) {
            constexpr bool IDLE = decltype(idle_tag)::value;
            // prologue: the trip's K tiles 0 .. STAGES-1 on their way, tile 0 landed (every wavefront is past
            // the last barrier of the previous trip: nobody reads LDS any more)
#pragma unroll
            for (int p = 0; p < STAGES; ++p) issue_tile(p, p, once_tag);
            barrier_keep_loads<(STAGES - 1) * LPT>();
            if (!IDLE) load_frags(0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            int st = 0;
            for (int t = 0; t < cnt; ++t) {
                const int st1 = st + 1 == STAGES ? 0 : st + 1;
                if (!IDLE) {
                    load_frags(1, st, 1);
                    mfma_step(0);
                    interleave(std::false_type{});
                    __builtin_amdgcn_sched_barrier(0);
                    load_frags(0, st, 2);
                    mfma_step(1);
                    interleave(std::false_type{});
                    __builtin_amdgcn_sched_barrier(0);
                    load_frags(1, st, 3);
                    mfma_step(0);
                    interleave(std::false_type{});
                }
                __builtin_amdgcn_sched_barrier(0);
                barrier_keep_loads<(STAGES - 2) * LPT>();
                __builtin_amdgcn_sched_barrier(0);
                if (!IDLE) load_frags(0, st1, 0);
                issue_tile(st, t + STAGES, once_tag);
                if (!IDLE) {
                    mfma_step(1);
                    interleave(std::true_type{});
                }
                __builtin_amdgcn_sched_barrier(0);
                st = st1;
            }
        };
        // The weight panel of a slot of one m-tile is read by nobody else: non-temporal hint, so that the stream
        // does not push the token rows out of the caches (-5 to -12 % per product at 22-110 rows per slot).
        const bool once = slot_mtiles == 1;
        const bool idle = row0 + wm * 64 >= row_end;  // never with one row of wavefronts
        if (once) {
            if (BM == 128 && idle) k_loop(std::true_type{}, std::true_type{});
            else k_loop(std::false_type{}, std::true_type{});
        } else {
            if (BM == 128 && idle) k_loop(std::true_type{}, std::false_type{});
            else k_loop(std::false_type{}, std::false_type{});
        }
        // the surplus loads must have landed (as zeros) before the stages are written again
        barrier_keep_loads<0>();

        if (cut && cnt < work.kt) {
            // ---- a piece of a tile: raw accumulators to the workspace, [register][thread] --------------------
            float* dst = partials + (size_t)piece_slot(g, kb > 0) * (BM * BR) + tid;
#pragma unroll
            for (int i = 0; i < WB; ++i)
#pragma unroll
                for (int j = 0; j < TB; ++j) {
                    if (row0 + wm * 64 + j * 32 >= row_end) continue;  // a block without rows: the second kernel skips it too
#pragma unroll
                    for (int v = 0; v < 16; ++v) dst[((i * TB + j) * 16 + v) * (64 * NW)] = acc[i][j][v];
                }
            continue;
        }

        // ---- epilogue of a whole tile ------------------------------------------------------------------------
        // The MFMA layout gives a lane 4 consecutive columns of 32 different token rows; stored from
        // registers that is 8-byte scraps into 32 rows per instruction.  Instead the wavefronts put their
        // activated, rounded results into LDS as a [128 token rows][BNO columns] bf16 image (16-byte
        // chunk j of row r at chunk position j ^ (r & SWM)), and every wavefront then stores 32 rows, 16
        // bytes per lane, whole row segments of 2 BNO bytes.
        constexpr int ROWB = BNO * 2;   // bytes per image row
        constexpr int CPR = ROWB / 16;  // chunks per image row (8, 16 or 32)
        constexpr int SWM = CPR - 1 < 15 ? CPR - 1 : 15;
        if (row0 + wm * 64 < row_end) {
#pragma unroll
            for (int mi = 0; mi < TB; ++mi) {
                const int r = wm * 64 + mi * 32 + (lane & 31);
#pragma unroll
                for (int ni = 0; ni < NB; ++ni) {
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        floatx4 v;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float t = acc[ni][mi][4 * gq + q];
                            if (EPI == kSwiglu) t = t * __builtin_amdgcn_rcpf(1.0f + __expf(-t)) * acc[ni + NB][mi][4 * gq + q];
                            if (EPI == kRelu) t = fmaxf(t, 0.0f);
                            v[q] = t;
                        }
                        // columns wn*(BNO/WN) + ni*32 + 8 gq + 4*(lane/32) .. +3: chunk j, its lower or upper half
                        const int j = wn * (BNO / WN / 8) + ni * 4 + gq;
                        *reinterpret_cast<bf16x4*>(lds + r * ROWB + ((j ^ (r & SWM)) * 16) + (lane >> 5) * 8) =
                            __builtin_convertvector(v, bf16x4);
                    }
                }
            }
        }
        __syncthreads();
        constexpr int RPS = 64 / CPR;  // image rows per store instruction
        const int jc = lane % CPR;
        const int n = n0 + jc * 8;
#pragma unroll 4
        for (int it = 0; it < BM / NW / RPS; ++it) {
            const int r = wave * (BM / NW) + it * RPS + lane / CPR;
            const uint4 val = *reinterpret_cast<const uint4*>(lds + r * ROWB + ((jc ^ (r & SWM)) * 16));
            if (row0 + r < row_end && n < N) {
                // combine folded in (second product, one expert per token): the row goes to its token's row of the output
                const int dr = (EPI == kPlain && gather.out_perm != nullptr) ? gather.out_perm[row0 + r] : row0 + r;
                *reinterpret_cast<uint4*>(c + (size_t)dr * N + n) = val;
            }
        }
        __syncthreads();  // the image is read: the next trip's loads may overwrite it
    }
}

// Adds the pieces of each tile that the shares cut, in K order, and applies the epilogue.  A cut
// tile is found at a boundary between two shares; a launch covers every boundary, one workgroup each,
// which walks the 32 x 32 block positions of a wavefront's accumulators.
// Workgroup b - 1: boundary b = 1 .. G-1 lies between shares b-1 and b.  When the main kernel
// took whole tiles, which the host cannot know, every workgroup exits after reading slot_offsets.
template <int EPI, int BM, int BR>
__global__ __launch_bounds__(64 * NW) void mid_fixup(const int32_t* __restrict__ offsets, bf16_t* __restrict__ c,
                                                 const int32_t* __restrict__ out_perm,
                                                 const float* __restrict__ partials, int S, int N, int K,
                                                 int n_tiles, int G) {
    constexpr int WM = BM / 64, WN = NW / WM;  // as in the main kernel
    constexpr int WB = BR / WN / 32;
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    constexpr int NB = EPI == kSwiglu ? WB / 2 : WB;
    constexpr int UNITS = TB * NB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int b = blockIdx.x + 1;
    const Work work = make_work(offsets, S, n_tiles, K, lane, G, BM);
    if (b >= work.sharers) return;              // nothing was cut, or no share starts here
    const long long ub = share_begin(work, b);  // first unit of share b
    if (ub % work.kt == 0) return;              // the boundary falls between two tiles
    const int tile = (int)(ub / work.kt);
    const long long t_begin = (long long)tile * work.kt, t_end = t_begin + work.kt;
    const int g_first = share_of(work, t_begin), g_last = share_of(work, t_end - 1);
    if (g_first != b - 1) return;  // several boundaries inside one tile: the first of them does the work
    int slot, row0, row_end, nt, slot_mtiles;
    decode_tile(work, S, lane, tile, BM, slot, row0, row_end, nt, slot_mtiles);
    for (int unit = 0; unit < UNITS; ++unit) {
        const int mi = unit / NB, ni = unit % NB;
        if (row0 + wm * 64 + mi * 32 >= row_end) continue;  // this wavefront's block holds no rows: nothing was written
        floatx16 gate, up;
#pragma unroll
        for (int v = 0; v < 16; ++v) { gate[v] = 0.0f; up[v] = 0.0f; }
        for (int gg = g_first; gg <= g_last; ++gg) {
            // share g_first holds the start of the tile (its piece starts at K tile 0), the others start inside it
            const float* src = partials + (size_t)piece_slot(gg, gg != g_first) * (BM * BR) + tid;
            float ga[16], ua[16];  // all loads of a piece in flight together, then the adds
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                ga[v] = src[((ni * TB + mi) * 16 + v) * (64 * NW)];
                ua[v] = EPI == kSwiglu ? src[(((ni + NB) * TB + mi) * 16 + v) * (64 * NW)] : 0.0f;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                gate[v] += ga[v];
                up[v] += ua[v];
            }
        }
        // a lane holds token lane % 32 of its block and weight rows 8 gq + 4 (lane / 32) + 0..3
        const int r = row0 + wm * 64 + mi * 32 + (lane & 31);
        if (r >= row_end) continue;
        bf16_t* crow = c + (size_t)((EPI == kPlain && out_perm != nullptr) ? out_perm[r] : r) * N;
        const int col0 = nt * BNO + wn * (BNO / WN) + ni * 32 + (lane >> 5) * 4;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int n = col0 + 8 * gq;
            if (n >= N) continue;
            floatx4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float t = gate[4 * gq + q];
                if (EPI == kSwiglu) t = t * __builtin_amdgcn_rcpf(1.0f + __expf(-t)) * up[4 * gq + q];
                if (EPI == kRelu) t = fmaxf(t, 0.0f);
                v[q] = t;
            }
            *reinterpret_cast<bf16x4*>(crow + n) = __builtin_convertvector(v, bf16x4);
        }
    }
}

template <int EPI, int BM, int BR, int STAGES, bool KTAIL, bool PERSIST>
hipError_t launch_cfg(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1,
                      bf16_t* c, float* partials, long long m_tiles, int S, int N, int K, hipStream_t st) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    constexpr int kLds = STAGES * (BM * ROW_BYTES + BR * ROW_BYTES);
    static_assert(kLds <= 160 * 1024, "LDS of one CU");
    static_assert(!PERSIST || (size_t)2 * kGroups * BM * BR * sizeof(float) <= kMidPartialBytes,
                  "two pieces per workgroup fit the workspace");
    auto kern = mid_gemm_bf16<EPI, BM, BR, STAGES, KTAIL, PERSIST>;
    static std::atomic<bool> attr_set{false};  // set once per kernel; setting it twice from two threads is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int n_tiles = (N + BNO - 1) / BNO;
    DeviceShape shape;
    hipError_t es = device_shape(&shape);
    if (es != hipSuccess) return es;
    if (PERSIST) {
        kern<<<shape.groups, 64 * NW, kLds, st>>>(a, gather, offsets, b0, b1, c, partials, S, N, K, n_tiles, shape.xcds);
        if (shape.groups > 1)
            mid_fixup<EPI, BM, BR><<<shape.groups - 1, 64 * NW, 0, st>>>(offsets, c, gather.out_perm, partials, S, N, K, n_tiles,
                                                                        shape.groups);
    } else {
        const long long tiles = m_tiles * n_tiles;
        const unsigned blocks = (unsigned)((tiles + shape.xcds - 1) / shape.xcds * shape.xcds);
        kern<<<blocks, 64 * NW, kLds, st>>>(a, gather, offsets, b0, b1, c, partials, S, N, K, n_tiles, shape.xcds);
    }
    return hipGetLastError();
}

template <int EPI, int BM, int BR, int STAGES, bool PERSIST>
hipError_t launch_ktail(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1,
                        bf16_t* c, float* partials, long long m_tiles, int S, int N, int K, hipStream_t st) {
    if (K % BK == 0)
        return launch_cfg<EPI, BM, BR, STAGES, false, PERSIST>(a, gather, offsets, b0, b1, c, partials, m_tiles, S, N, K, st);
    return launch_cfg<EPI, BM, BR, STAGES, true, PERSIST>(a, gather, offsets, b0, b1, c, partials, m_tiles, S, N, K, st);
}

template <int EPI>
hipError_t launch_one(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1,
                      bf16_t* c, float* partials, long long A, int S, int N, int K, hipStream_t st) {
    DeviceShape shape;
    hipError_t es = device_shape(&shape);
    if (es != hipSuccess) return es;
    const int kCUs = shape.cus;
    // every slot adds at most one partial m-tile to the A / 128 whole ones
    const long long m_tiles = A / kTileRows + (S < A ? S : A);
    // Tiles of 256 weight rows, unless they would leave CUs without a tile (the second product of a
    // layer with a small d_model): then 128 weight rows and five stages, so that twice as many CUs
    // stream weights, each with as many bytes in flight; and if K is long, in a persistent launch
    // that cuts the tiles along K when even they are clearly fewer than the CUs (with a short K that
    // never pays, and the second kernel's launch is saved).
    constexpr int BNO = EPI == kSwiglu ? 128 : 256;
    // Few rows per slot: token tiles of 64 rows leave LDS for more stages, 96 (80 with 128 weight rows) KiB
    // of weights in flight per CU instead of 64.  (With SwiGLU and 128 weight rows a wavefront of the
    // 64-row arrangement would hold half a block of gate rows: that combination keeps 128 token rows.)
    const bool few_rows = A <= kRowsPerSlot64 * S;
    const long long m_tiles64 = A / 64 + (S < A ? S : A);
    const bool persist = (K + BK - 1) / BK >= kMinPersistK;
    if (m_tiles * ((N + BNO - 1) / BNO) <= kCUs) {
        if constexpr (EPI != kSwiglu) {
            if (few_rows && persist)
                return launch_ktail<EPI, 64, 128, 6, true>(a, gather, offsets, b0, b1, c, partials, m_tiles64, S, N, K, st);
            // a short K (no cutting) and so few 128-row tiles that they leave a quarter of the CUs idle even
            // if every slot has a partial tile: 64-row tiles, about twice as many
            const bool underfilled = !persist && m_tiles * ((N + 127) / 128) <= kCUs * 3 / 4;
            if (few_rows || underfilled)
                return launch_ktail<EPI, 64, 128, 6, false>(a, gather, offsets, b0, b1, c, partials, m_tiles64, S, N, K, st);
        }
        if (persist)
            return launch_ktail<EPI, 128, 128, 5, true>(a, gather, offsets, b0, b1, c, partials, m_tiles, S, N, K, st);
        return launch_ktail<EPI, 128, 128, 5, false>(a, gather, offsets, b0, b1, c, partials, m_tiles, S, N, K, st);
    }
    if (few_rows)
        return launch_ktail<EPI, 64, 256, 4, false>(a, gather, offsets, b0, b1, c, partials, m_tiles64, S, N, K, st);
    return launch_ktail<EPI, 128, 256, 3, false>(a, gather, offsets, b0, b1, c, partials, m_tiles, S, N, K, st);
}

}  // namespace

hipError_t launch_ffn_bf16_mid(const emoe_layer_desc& d, const void* x_perm, RowGather gather, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, void* y_perm, void* ws, int passes,
                               hipStream_t st) {
    const FfnWs lay = ffn_ws_layout(d);
    bf16_t* h = reinterpret_cast<bf16_t*>(static_cast<uint8_t*>(ws) + lay.h);
    float* partials = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + lay.partials);
    const bf16_t* xp = static_cast<const bf16_t*>(x_perm);
    const long long A = (long long)d.T * d.k;
    hipError_t e = hipSuccess;
    if (!(passes & 1)) {
    } else if (d.act == EMOE_ACT_SWIGLU)
        e = launch_one<kSwiglu>(xp, gather, offsets, static_cast<const bf16_t*>(w1), static_cast<const bf16_t*>(w3), h,
                                partials, A, d.S, d.d_ff, d.d_model, st);
    else
        e = launch_one<kRelu>(xp, gather, offsets, static_cast<const bf16_t*>(w1), nullptr, h, partials, A, d.S, d.d_ff,
                              d.d_model, st);
    if (e != hipSuccess || !(passes & 2)) return e;
    return launch_one<kPlain>(h, RowGather{nullptr, 1, 0, gather.out_perm}, offsets, static_cast<const bf16_t*>(w2), nullptr,
                              static_cast<bf16_t*>(y_perm), partials, A, d.S, d.d_model, d.d_ff, st);
}

}  // namespace emoe
