// Expert FFN for bf16 layers with many rows per slot: grouped GEMM on the gfx950 matrix cores
// (eMoE Section 1: the experts; Section 5.1: only resident, non-empty slots cost compute and
// memory reads).
//
//   pass 1: h[r, n]      = act(x_perm[r,:] . W1_s[n,:]) (* x_perm[r,:] . W3_s[n,:])   K = d_model
//   pass 2: y_perm[r, n] = h[r,:] . W2_s[n,:]                                         K = d_ff
//
// Tile: a workgroup of NW = 4 wavefronts (2 x 2, one per SIMD) owns 256 tokens x 256 weight rows;
// each wavefront accumulates 128 x 128 as 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 in fp32 (256
// accumulator registers).  Eight wavefronts (128 x 64 each) measured slower: more LDS reads per
// MFMA.  In the SwiGLU pass the 256 weight rows are 128 rows of W1 and the SAME 128 rows of
// W3, arranged so that a lane holds the gate and the up value of the same output element and the
// activation is applied in registers.  The weight rows go on the MFMA's row operand: a lane then
// owns four consecutive output columns of one token and stores them as one 8-byte write.
//
// Data movement: both operands are K-contiguous in memory.  K is walked in tiles of 64, so that a
// tile row is one whole 128-byte cache line (with 64-byte rows every line is requested twice, by
// consecutive K tiles; halving the requests to L2 was worth 8-15 % here, where the kernel runs at
// the chip's power limit).  An operand tile (256 rows x 128 bytes = 32 KiB) goes from global memory
// straight into LDS with buffer_load_dwordx4 ... lds (no staging registers, no LDS store
// instructions).  LDS is a ring of five operand tiles - token rows of K tile t in slot 2t mod 5,
// weight rows in slot 2t+1 mod 5 - so one and a half K tiles are in flight while one is multiplied.
// Each load instruction fills 1 KiB of LDS contiguously (8 rows x 128 bytes); the 16-byte chunk c
// of row r is stored at chunk position c ^ ((r >> 1) & 7), chosen by which global chunk a lane
// fetches, which makes the MFMA fragment reads (32 rows x one chunk per ds_read_b128) bank-conflict
// free without padding.  Buffer addressing gives a uniform (scalar) K offset plus a per-lane row
// offset, so the loop has no address arithmetic; in the K tail, chunks past K are fetched out of
// range and arrive as zeros.
//
// Schedule per K tile (four MFMA steps of 16 each): fragment reads for the next step and the loads
// of tile t+2 are slotted one by one between the MFMAs, so no memory instruction waits in a full
// queue while the matrix pipe idles.  One barrier per tile, before its last step.
//
// Epilogue: results go through LDS so that they leave as whole 256- or 512-byte row segments (see
// epilogue()); accumulators are read from their AGPRs one block at a time.
//
// Slots that do not fill their tiles: a slot's rows are spread evenly over its m-tiles in whole
// 32-row MFMA blocks (257 rows: tiles of 160 and 97 rows, not 256 and 1), a tile's blocks alternate
// between the two rows of wavefronts, and the K loop is compiled for 0 .. 4 blocks per wavefront, so
// that matrix work is done for blocks with rows only and both wavefront rows finish together.  A
// tile still costs a pass over its weight panel whatever it holds (8 slots of 257 rows at the Mixtral
// shape: 0.96 -> 0.88 ms; of 513 rows: 1.51 -> 1.41 ms; full tiles unchanged).
//
// Ragged groups: group sizes live on the device.  The launch is persistent (one workgroup per CU);
// every workgroup derives the list of (slot, m-tile, n-tile) tiles from slot_offsets and takes its
// share (see "work distribution" below).  Workgroup ids are dealt round-robin to the 8 XCDs, so
// ids are remapped: the workgroups of an XCD hold consecutive tiles of an order in which 32
// consecutive tiles form a block of 8 m-tiles x 4 n-tiles of one slot (see tile_in_slot), so that
// XCD's L2 supplies 12 operand panels for 32 tiles.
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

constexpr int BM = 256;                     // tokens per tile
constexpr int BR = 256;                     // weight rows per tile (SwiGLU: 128 of W1 + 128 of W3)
constexpr int BK = 64;                      // K elements per tile
constexpr int ROW_BYTES = BK * 2;           // 128: a tile row is one whole cache line
constexpr int TILE_BYTES = BM * ROW_BYTES;  // 32 KiB per operand
constexpr int SLOTS = 5;                    // LDS ring of operand tiles: x(t), w(t), x(t+1), w(t+1), x(t+2), ...
constexpr size_t LDS_BYTES = SLOTS * TILE_BYTES;  // 160 KiB, all of a CU's LDS
static_assert(BK / 16 == 4, "the K loop is written out for four MFMA K-steps per tile");
constexpr int kMaxSplits = 8;           // K pieces per leftover tile, at most
constexpr int kFixupGroups = (kMaxGroups - 1) * 16;  // workgroups of the fix-up launch: the most units there can be
constexpr int kPlanFloats = kTiledPlanBytes / 4;  // the plan sits ahead of the partial sums
constexpr unsigned kRotation = 21;  // K-tile rotation per slot
constexpr int NW = 4;            // wavefronts per workgroup, arranged 2 (tokens) x NW/2 (weight rows)
constexpr int WN = NW / 2;
constexpr int TB = 4;            // 32-token blocks per wavefront (128 tokens)
constexpr int WB = BR / WN / 32; // 32-row weight blocks per wavefront
constexpr int RPI = 1024 / ROW_BYTES;      // tile rows filled by one load instruction (8)
constexpr int LPW = BM / RPI / NW;         // load instructions per wavefront, per tile and operand (8)

enum Epilogue { kPlain = 0, kSwiglu = 1, kRelu = 2 };

// s_waitcnt immediate: vmcnt <= n and all LDS traffic done (vmcnt[3:0] | [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int wait_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0x0 << 8); }

// Workgroup barrier once at most `n` of this wavefront's global->LDS loads are still pending and
// all its LDS reads have returned.  __syncthreads() would drain every pending load (its release
// fence counts the LDS writes of the loads), which is exactly what the deep prefetch must avoid.
// The empty asm statements stop the compiler from moving LDS accesses across the barrier.
template <int N>
__device__ __forceinline__ void barrier_keep_loads() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(wait_imm(N));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// ---- work distribution ------------------------------------------------------------------------
// The launch is persistent: one workgroup per CU.  Output tiles are numbered in (slot, n-tile,
// m-tile) order of tile_in_slot.  The first `rounds * G` tiles are dealt out whole, `rounds` per
// workgroup, so that the 32 workgroups of an XCD hold 32 consecutive tiles at any time (one weight
// panel and the slot's token panels stay in that XCD's L2).  Round r covers tiles r*G .. (r+1)*G-1,
// 32 for each XCD: every XCD works its way through all slots, so slots whose tiles cost less (fewer
// rows than a tile holds) do not leave some XCDs idle while others still work (a contiguous range of
// tiles per XCD took 4-7 % longer at 250-500 rows per slot).  The `left` tiles that do not fill a
// round are split along K into `splits` pieces each, so that they too occupy (nearly) every CU: a
// piece writes its fp32 accumulators to the workspace and a small second kernel adds the pieces in
// order and applies the epilogue.  Everything is derived from slot_offsets on the device.
struct Plan {
    int tiles;   // output tiles in total
    int rounds;  // whole tiles per workgroup
    int left;    // tiles beyond rounds * G
    int splits;  // K pieces per leftover tile (1 = none)
};

__device__ __forceinline__ Plan make_plan(int tiles, int k_tiles, int G) {
    Plan p;
    p.tiles = tiles;
    p.rounds = p.tiles / G;
    p.left = p.tiles - p.rounds * G;
    int sp = p.left > 0 ? G / p.left : 1;
    const int by_k = k_tiles / 8;  // at least 8 K tiles (512 elements) per piece
    sp = sp < by_k ? sp : by_k;
    sp = sp > kMaxSplits ? kMaxSplits : sp;
    p.splits = sp < 1 ? 1 : sp;
    return p;
}

// Order of a slot's m_tiles x n_tiles output tiles.  The 32 workgroups of an XCD hold 32 consecutive
// tiles at any time and their L2 has to supply one operand panel per distinct m-tile and per
// distinct n-tile among them, so consecutive tiles should form compact blocks: the n-tiles are
// taken four at a time, and inside such a group of columns the m-tiles eight at a time, m fastest
// (12 panels for 32 tiles; m fastest over a whole tall slot would need up to 33).
// rem = number of the tile within the slot -> its m-tile and n-tile.
constexpr int kBlockM = 8, kBlockN = 4;
constexpr int kSkipBlocksUpToTiles = kBlockM;  // see the K loop's dispatch
__device__ __forceinline__ void tile_in_slot(int rem, int m_tiles, int n_tiles, int& mt, int& nt) {
    const int group = rem / (m_tiles * kBlockN);  // group of up to four n-tiles
    const int gn = n_tiles - group * kBlockN < kBlockN ? n_tiles - group * kBlockN : kBlockN;
    int r = rem - group * (m_tiles * kBlockN);
    const int full = m_tiles / kBlockM;           // whole blocks of eight m-tiles
    int mb = kBlockM, m0 = 0;
    if (r < full * kBlockM * gn) {
        m0 = (r / (kBlockM * gn)) * kBlockM;
        r %= kBlockM * gn;
    } else {
        r -= full * kBlockM * gn;
        m0 = full * kBlockM;
        mb = m_tiles - m0;
    }
    mt = m0 + r % mb;
    nt = group * kBlockN + r / mb;
}

// Rows per m-tile of a slot of `rows` rows cut into `tiles` tiles: the rows are spread evenly (in
// whole 32-row MFMA blocks), so that a slot of 257 rows becomes tiles of 160 and 97 rows instead of
// 256 and 1.  A tile costs a pass over its weight panel whatever it holds; what is saved is the
// matrix work of the blocks without rows, which both tiles then skip.
__device__ __forceinline__ int rows_per_tile(int rows, int tiles) {
    const int even = (rows + tiles - 1) / (tiles > 0 ? tiles : 1);
    return (even + 31) & ~31;  // <= BM, so tile number `tiles - 1` still starts inside the slot
}

// Which wavefronts multiply which of a tile's 32-row token blocks: the blocks alternate between
// the two wavefront rows, so that both finish together whatever the number of blocks that hold rows.
// -> tile block of block i of wavefront row wm, and the number of its blocks that hold rows.
__device__ __forceinline__ int tile_block(int wm, int i) { return 2 * i + wm; }
__device__ __forceinline__ int blocks_of_wavefront(int row0, int row_end, int wm) {
    return ((row_end - row0 + 31) / 32 - wm + 1) / 2;
}

// One 32 x 32 output block of a wavefront: token block mi, output-column block ni.  `gate` holds the
// accumulators (for SwiGLU the gate rows), `up` the matching up rows (unused otherwise).
// A lane holds token lane%32 and weight rows 8g + 4*(lane/32) + 0..3.
template <int EPI>
__device__ __forceinline__ void epilogue_block(const floatx16& gate, const floatx16& up, bf16_t* __restrict__ c,
                                               const int32_t* __restrict__ out_perm, int row0, int row_end, int n0, int N,
                                               int wm, int wn, int mi, int ni, int lane) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    const int r = row0 + tile_block(wm, mi) * 32 + (lane & 31);
    if (r >= row_end) return;
    bf16_t* crow = c + (size_t)((EPI == kPlain && out_perm != nullptr) ? out_perm[r] : r) * N;
    const int col0 = n0 + wn * (BNO / WN) + ni * 32 + (lane >> 5) * 4;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int n = col0 + 8 * g;
        if (n >= N) continue;
        floatx4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float t = gate[4 * g + q];
            if (EPI == kSwiglu) t = t / (1.0f + __expf(-t)) * up[4 * g + q];
            if (EPI == kRelu) t = fmaxf(t, 0.0f);
            v[q] = t;
        }
        bf16x4 o = __builtin_convertvector(v, bf16x4);
        *reinterpret_cast<bf16x4*>(crow + n) = o;
    }
}

// The slot table in registers: lane s of every wavefront holds slot s's row range and the number of
// the first output tile of that slot, so that finding a tile's slot is one ballot and three lane
// reads instead of a walk over slot_offsets in memory (a few thousand cycles per tile).
struct SlotTable {
    int begin, end;  // rows of slot `lane`
    int tiles;       // m-tiles of slot `lane`
    int first;       // number of the slot's first output tile (exclusive prefix of tiles * n_tiles)
    int total;       // all output tiles (uniform)
};

__device__ __forceinline__ SlotTable make_slot_table(const int32_t* __restrict__ offsets, int S, int n_tiles, int lane) {
    SlotTable t;
    t.begin = lane < S ? offsets[lane] : 0;
    t.end = lane < S ? offsets[lane + 1] : 0;
    t.tiles = (t.end - t.begin + BM - 1) / BM;
    const int span = t.tiles * n_tiles;
    int incl = span;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    t.first = incl - span;
    t.total = __builtin_amdgcn_readlane(incl, 63);
    return t;
}

__device__ __forceinline__ void decode_tile(const SlotTable& t, int S, int n_tiles, int lane, int L, int& slot,
                                            int& row0, int& row_end, int& nt, int& slot_tiles) {
    // slots are in tile order and an empty slot starts where its successor does: the last slot that
    // starts at or before L is the non-empty one that holds it
    const unsigned long long m = __ballot(lane < S && t.first <= L);
    slot = __popcll(m) - 1;
    const int rem = L - __builtin_amdgcn_readlane(t.first, slot);
    const int tiles = __builtin_amdgcn_readlane(t.tiles, slot);
    int mt;
    tile_in_slot(rem, tiles, n_tiles, mt, nt);
    const int b = __builtin_amdgcn_readlane(t.begin, slot), e = __builtin_amdgcn_readlane(t.end, slot);
    const int rpt = rows_per_tile(e - b, tiles);
    row0 = b + mt * rpt;
    row_end = row0 + rpt < e ? row0 + rpt : e;
    slot_tiles = tiles;
}

// Reads one accumulator where it lives (an AGPR).  Written out as an instruction so that the compiler
// moves accumulators to VALU registers one at a time, where they are used, instead of copying all
// 256 of them out at the end of the K loop (which needs every VGPR and spills the rest).
__device__ __forceinline__ float acc_read(float a) {
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// Epilogue of a whole tile.  The MFMA layout gives a lane 4 consecutive columns of 32 different
// token rows, so storing straight from registers writes 16-byte scraps into 32 rows per
// instruction.  Instead the wavefronts put their (activated, rounded) results into LDS as a
// [256 token rows][BNO columns] bf16 image, and after a barrier every wavefront stores 64 of its
// rows with 16 bytes per lane, 256 or 512 contiguous bytes per row.  In the image the 16-byte
// chunk j of row r sits at chunk position j ^ (r & 15), which keeps both the 8-byte writes and the
// 16-byte reads (nearly) free of bank conflicts.  All DMA loads have landed and all fragment reads
// are done when this runs; the barrier at the end keeps the next tile's loads off the image.
template <int EPI>
__device__ __forceinline__ void epilogue(floatx16 (&acc)[WB][TB], bf16_t* __restrict__ c,
                                         const int32_t* __restrict__ out_perm, char* lds, int row0,
                                         int row_end, int n0, int N, int wm, int wn, int wave, int lane) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    constexpr int NB = EPI == kSwiglu ? WB / 2 : WB;
    constexpr int ROWB = BNO * 2;      // bytes per image row
    constexpr int CPR = ROWB / 16;     // 16-byte chunks per image row
#pragma unroll
    for (int mi = 0; mi < TB; ++mi) {
        const int r = tile_block(wm, mi) * 32 + (lane & 31);  // token row of the tile
#pragma unroll
        for (int ni = 0; ni < NB; ++ni) {
            const floatx16& gate = acc[ni][mi];
            const floatx16& up = acc[EPI == kSwiglu ? ni + NB : ni][mi];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                floatx4 v;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float t = acc_read(gate[4 * g + q]);
                    if (EPI == kSwiglu) t = t * __builtin_amdgcn_rcpf(1.0f + __expf(-t)) * acc_read(up[4 * g + q]);
                    if (EPI == kRelu) t = fmaxf(t, 0.0f);
                    v[q] = t;
                }
                // columns wn*(BNO/2) + ni*32 + 8g + 4*(lane/32) .. +3: chunk j, its lower or upper half
                const int j = wn * (BNO / WN / 8) + ni * 4 + g;
                *reinterpret_cast<bf16x4*>(lds + r * ROWB + ((j ^ (r & 15)) * 16) + (lane >> 5) * 8) =
                    __builtin_convertvector(v, bf16x4);
            }
            __builtin_amdgcn_sched_barrier(0);  // one block at a time: the accumulators stay where they are until used
        }
    }
    __syncthreads();
    constexpr int RPS = 64 / CPR;  // image rows per store instruction (2 or 4)
    const int jc = lane % CPR;
    const int n = n0 + jc * 8;
#pragma unroll 4
    for (int it = 0; it < BM / NW / RPS; ++it) {
        const int r = wave * (BM / NW) + it * RPS + lane / CPR;
        const uint4 val = *reinterpret_cast<const uint4*>(lds + r * ROWB + ((jc ^ (r & 15)) * 16));
        if (row0 + r < row_end && n < N) {
            // combine folded in (second product, one expert per token): the row goes to its token's row of the output
            const int dr = (EPI == kPlain && out_perm != nullptr) ? out_perm[row0 + r] : row0 + r;
            *reinterpret_cast<uint4*>(c + (size_t)dr * N + n) = val;
        }
    }
    __syncthreads();
}

template <int EPI, bool KTAIL>
__global__ __launch_bounds__(64 * NW) void grouped_gemm_bf16(const bf16_t* __restrict__ a, RowGather gather,
                                                         const int32_t* __restrict__ offsets,
                                                         const bf16_t* __restrict__ b0,
                                                         const bf16_t* __restrict__ b1, bf16_t* __restrict__ c,
                                                         float* __restrict__ partials, int S, int N, int K,
                                                         int n_tiles, int XCDS) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;  // output columns per tile
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int k_tiles_all = (K + BK - 1) / BK;
    const int G = gridDim.x;
    const SlotTable table = make_slot_table(offsets, S, n_tiles, lane);
    const Plan plan = make_plan(table.total, k_tiles_all, G);
    if (blockIdx.x == 0 && tid == 0)  // for the fix-up kernel, which then need not derive it again
        *reinterpret_cast<int4*>(partials) = make_int4(plan.tiles, plan.rounds, plan.left, plan.splits);
    const int rows_total = offsets[S];
    const int xcd = blockIdx.x % XCDS, cu = blockIdx.x / XCDS, per_xcd = G / XCDS;
    const int sk_item = xcd * per_xcd + cu;  // this workgroup's piece of the leftover tiles

    // lane-constant parts of the addressing
    const int l_row = lane >> 3;  // row within a load instruction's eight rows
    const int l_pos = lane & 7;   // chunk position within the row, in LDS
    const uint32_t a_bytes = (uint32_t)(gather.perm != nullptr ? gather.rows : rows_total) * (uint32_t)K * 2u;
    const uint32_t b_bytes = (uint32_t)N * (uint32_t)K * 2u;
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(a, a_bytes);
    const bf16_t* wsel = (EPI == kSwiglu && wave >= NW / 2) ? b1 : b0;  // upper wavefronts load the W3 half
    const int f_row = lane & 31;
    const int f_sw = (((lane >> 5) ^ ((f_row >> 1) & 7)) & 7) * 16;
    const int x_off = (tile_block(wm, 0) * 32 + f_row) * ROW_BYTES + f_sw;  // token block 0 of this wavefront; block i: tile_block(wm, i)
    int w_off[WB];  // SwiGLU: weight blocks 0..WB/2-1 are gate rows, WB/2..WB-1 the matching up rows
#pragma unroll
    for (int i = 0; i < WB; ++i) {
        int rr;
        if (EPI == kSwiglu)
            rr = (i < WB / 2) ? wn * (BR / 2 / WN) + i * 32 : BR / 2 + wn * (BR / 2 / WN) + (i - WB / 2) * 32;
        else
            rr = wn * (BR / WN) + i * 32;
        w_off[i] = (rr + f_row) * ROW_BYTES + f_sw;
    }

    for (int item = 0; item <= plan.rounds; ++item) {
        // ---- what to do in this trip -------------------------------------------------------------
        int L, kb = 0, ke = k_tiles_all, piece = -1;
        if (item < plan.rounds) {
            L = item * G + xcd * per_xcd + cu;
        } else {
            if (sk_item >= plan.left * plan.splits) break;
            L = plan.rounds * G + sk_item / plan.splits;
            if (plan.splits > 1) {
                const int sp = sk_item % plan.splits;
                kb = (int)((long long)k_tiles_all * sp / plan.splits);
                ke = (int)((long long)k_tiles_all * (sp + 1) / plan.splits);
                piece = sk_item;
            }
        }
        int slot, row0, row_end, nt, slot_tiles;
        decode_tile(table, S, n_tiles, lane, L, slot, row0, row_end, nt, slot_tiles);
        const int n0 = nt * BNO;

        // ---- global -> LDS -------------------------------------------------------------------------
        // Wavefront w issues, per K tile and per operand, load instructions i = 0..LPW-1; instruction
        // (w, i) fills tile rows (LPW*w + i)*8 .. +7, 128 bytes each.  Lane l lands in row l>>3, chunk
        // position l&7 and therefore fetches global chunk (l&7) ^ ((row>>1)&7).
        uint32_t a_voff[LPW], b_voff[LPW];
        int chunk[LPW], a_row[LPW];
        // the rows of x come through perm: those loads go out first, the first weight tile is requested
        // while they are on their way (further down), and only then are the token addresses formed
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int tr = (LPW * wave + i) * RPI + l_row;  // row of the tile
            chunk[i] = l_pos ^ ((tr >> 1) & 7);
            int r = row0 + tr;
            r = r >= row_end ? row_end - 1 : r;
            a_row[i] = gather.perm != nullptr ? gather.perm[r] : r;  // the token's row of x (times k), not a copy of it
            int n = n0 + (EPI == kSwiglu ? tr % (BR / 2) : tr);  // SwiGLU: second half = same rows of W3
            n = n < N ? n : N - 1;
            b_voff[i] = ((uint32_t)n * (uint32_t)K + chunk[i] * 8) * 2u;
        }
        const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(wsel + (size_t)slot * N * K, b_bytes);
        const int k_tiles = ke - kb;
        const int k_first = kb * BK, k_last = (ke - 1) * BK;
        // one load instruction i of the token (tok) or weight tile of K tile number tk, into ring slot rs.
        // Near the end of K the loads go on (the loop body stays free of branches) but out of range:
        // zeros land in a slot that nobody reads any more.
        // The tiles of different slots start at different K tiles of their range (all workgroups on the
        // same 128-byte column of rows a power of two apart land on few memory channels); the tiles of a
        // slot share the start and so stay in step.  The order is a fixed function of the tile.
        const int k_rot = (int)(((unsigned)slot * kRotation) % (unsigned)k_tiles);
        auto k_of = [&](int tk) {
            int kk = tk + k_rot;
            kk = kk >= k_tiles ? kk - k_tiles : kk;
            const int k0 = k_first + kk * BK;
            return k0 < k_last ? k0 : k_last;
        };
        auto issue_load = [&](bool tok, int i, int rs, int tk) {
            const int k0 = k_of(tk);
            uint32_t voff = tok ? a_voff[i] : b_voff[i];
            // out of range (zeros arrive, memory is not touched): chunks past K, and the loads past the last tile
            if ((KTAIL && k0 + chunk[i] * 8 >= K) || tk >= k_tiles) voff = tok ? a_bytes : b_bytes;
            char* dst = lds + rs * TILE_BYTES + (LPW * wave + i) * 1024;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(tok ? a_rsrc : b_rsrc, (lds_void*)dst, 16, (int)voff, k0 * 2, 0, 0);
        };
        // the same for a weight tile whose bytes no other tile reads (a slot of one m-tile): non-temporal hint
        auto issue_weights_once = [&](int i, int rs, int tk) {
            const int k0 = k_of(tk);
            uint32_t voff = b_voff[i];
            if ((KTAIL && k0 + chunk[i] * 8 >= K) || tk >= k_tiles) voff = b_bytes;
            char* dst = lds + rs * TILE_BYTES + (LPW * wave + i) * 1024;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_void*)dst, 16, (int)voff, k0 * 2, 0, 2);
        };

        floatx16 acc[WB][TB];  // [weight block][token block]
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < TB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

        bf16x8 xf[2][TB], wf[2][WB];
        // Everything that touches the matrix cores is compiled for NB = 0 .. TB token blocks: the number
        // of this wavefront's 32-row blocks that hold rows of the tile (a ragged or evenly cut tile holds
        // fewer than 256 rows).  NB = TB is the full tile, NB = 0 a wavefront that only takes part in the
        // loads and barriers.
        // fragments of MFMA K-step kk of the tile whose token rows sit in ring slot sx and weight rows in sw
        auto load_frags = [&](auto nb_c, int buf, int sx, int sw, int kk) {
            constexpr int NB = decltype(nb_c)::value;
            if (NB == 0) return;
            const char* xb = lds + sx * TILE_BYTES;
            const char* wb = lds + sw * TILE_BYTES;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                xf[buf][i] = *reinterpret_cast<const bf16x8*>(xb + ((x_off + tile_block(0, i) * 32 * ROW_BYTES) ^ (kk * 32)));
#pragma unroll
            for (int i = 0; i < WB; ++i) wf[buf][i] = *reinterpret_cast<const bf16x8*>(wb + (w_off[i] ^ (kk * 32)));
        };
        auto mfma_step = [&](auto nb_c, int buf) {
            constexpr int NB = decltype(nb_c)::value;
#pragma unroll
            for (int ni = 0; ni < WB; ++ni)
#pragma unroll
                for (int m = 0; m < NB; ++m) {
                    const int mi = (ni & 1) ? NB - 1 - m : m;  // back and forth: only one operand changes between two MFMAs
                    acc[ni][mi] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][ni], xf[buf][mi], acc[ni][mi], 0, 0, 0);
                }
        };
        // the step's MFMAs with its LDS reads and LOADS global->LDS loads slotted in between, so that no
        // memory instruction waits in a full queue while the matrix pipe idles
        auto interleave = [&](auto nb_c, auto loads_c) {
            constexpr int NB = decltype(nb_c)::value;
            constexpr int LOADS = decltype(loads_c)::value;
            if constexpr (NB == TB) {
#pragma unroll
                for (int i = 0; i < TB * WB; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                           // one MFMA
                    if (i < TB + WB) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);          // one DS read
                    else if (i < TB + WB + LOADS) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // one VMEM
                }
            } else if constexpr (NB > 0) {  // fewer MFMAs than memory instructions: several of those per MFMA
                constexpr int MF = NB * WB;
                constexpr int DS_PER = (NB + WB + MF - 1) / MF, VM_PER = (LOADS + MF - 1) / MF;
#pragma unroll
                for (int i = 0; i < MF; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, DS_PER, 0);
                    if (VM_PER > 0) __builtin_amdgcn_sched_group_barrier(0x010, VM_PER, 0);
                }
            }
        };

        // ---- prologue: K tiles 0 and 1 of this piece on their way, the first landed ----------------
        // (every wavefront is past the last barrier of the previous trip, so nobody reads LDS any more)
        // Ring slots: token rows of K tile t in slot 2t mod 5, weight rows in slot 2t+1 mod 5.
#pragma unroll
        for (int i = 0; i < LPW; ++i) issue_load(false, i, 1, 0);
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int tr = (LPW * wave + i) * RPI + l_row;
            const bool past = row0 + tr >= row_end;  // rows past the slot's end: out of range, zeros without memory traffic
            const int r = gather.perm != nullptr ? a_row[i] / gather.k : a_row[i];
            a_voff[i] = past ? a_bytes : ((uint32_t)r * (uint32_t)K + chunk[i] * 8) * 2u;
        }
#pragma unroll
        for (int i = 0; i < LPW; ++i) issue_load(true, i, 0, 0);
#pragma unroll
        for (int i = 0; i < LPW; ++i) issue_load(true, i, 2, 1);
#pragma unroll
        for (int i = 0; i < LPW; ++i) issue_load(false, i, 3, 1);
        barrier_keep_loads<2 * LPW>();

        // ---- main loop -----------------------------------------------------------------------------
        // Per K tile: four MFMA steps of 16.  Token rows of tile t+2 are requested during steps 0 and 1
        // (into the slot that held the weight rows of tile t-1), weight rows of tile t+2 during step 3
        // (into the slot of this tile's token rows, dead after the barrier).  One barrier per tile,
        // before step 3: by then every wavefront has read its last fragments of tile t, and tile t+1
        // has landed once only the 8 newest loads (token rows of t+2) are pending.
        // A wavefront skips the fragment reads and MFMAs of its token blocks without rows: the kernel
        // runs at the chip's power limit, so work not done is speed for the others.
        auto k_loop = [&](auto nb_c, auto once_c) {
            constexpr bool IDLE = decltype(nb_c)::value == 0;
            load_frags(nb_c, 0, 0, 1, 0);
            __builtin_amdgcn_sched_barrier(0);
            int sx = 0;  // ring slot of tile t's token rows
            for (int t = 0; t < k_tiles; ++t) {
                const int sw = sx + 1 >= SLOTS ? sx + 1 - SLOTS : sx + 1;   // this tile's weight rows
                const int sx1 = sx + 2 >= SLOTS ? sx + 2 - SLOTS : sx + 2;  // next tile's token rows
                const int sw1 = sx + 3 >= SLOTS ? sx + 3 - SLOTS : sx + 3;  // next tile's weight rows
                const int sx2 = sx + 4 >= SLOTS ? sx + 4 - SLOTS : sx + 4;  // token rows of t+2 (held weights of t-1)
                load_frags(nb_c, 1, sx, sw, 1);
#pragma unroll
                for (int i = 0; i < LPW / 2; ++i) issue_load(true, i, sx2, t + 2);
                if (!IDLE) {
                    mfma_step(nb_c, 0);
                    interleave(nb_c, std::integral_constant<int, LPW / 2>{});
                }
                __builtin_amdgcn_sched_barrier(0);
                load_frags(nb_c, 0, sx, sw, 2);
#pragma unroll
                for (int i = LPW / 2; i < LPW; ++i) issue_load(true, i, sx2, t + 2);
                if (!IDLE) {
                    mfma_step(nb_c, 1);
                    interleave(nb_c, std::integral_constant<int, LPW / 2>{});
                }
                __builtin_amdgcn_sched_barrier(0);
                if (!IDLE) {
                    load_frags(nb_c, 1, sx, sw, 3);
                    mfma_step(nb_c, 0);
                    interleave(nb_c, std::integral_constant<int, 0>{});
                }
                __builtin_amdgcn_sched_barrier(0);
                barrier_keep_loads<LPW>();
                __builtin_amdgcn_sched_barrier(0);
                load_frags(nb_c, 0, sx1, sw1, 0);
#pragma unroll
                for (int i = 0; i < LPW; ++i) {  // weight rows of t+2 over this tile's token rows
                    if (decltype(once_c)::value) issue_weights_once(i, sx, t + 2);
                    else issue_load(false, i, sx, t + 2);
                }
                if (!IDLE) {
                    mfma_step(nb_c, 1);
                    interleave(nb_c, std::integral_constant<int, LPW>{});
                }
                __builtin_amdgcn_sched_barrier(0);
                sx = sx1;
            }
        };
        // Blocks without rows are skipped in slots of up to kBlockM tiles (one block of tile_in_slot), where a
        // tile's padding is a large share of the slot's matrix work.  In a taller slot the one ragged tile
        // multiplies its padding: the workgroups of an XCD share operand panels through L2 only while they
        // walk K in step, and a tile that finishes early falls out of step for good.  Skipping everywhere
        // fetches 5.4 instead of 3.15 GB from beyond L2 in the prefill layer's first product (Mixtral-8x22B
        // shape: 10.5 instead of 6.6 GB) and gains nothing: with the three policies (limit 4, 8, none) run
        // in turns inside one process, layer times differ by less than 1 % on every workload (prefill
        // 2.298 / 2.288 / 2.307 ms, fine-grained layer 0.845 / 0.842 / 0.836 ms).
        const int my_blocks = slot_tiles > kSkipBlocksUpToTiles ? TB : blocks_of_wavefront(row0, row_end, wm);
        static_assert(TB == 4, "written out for four token blocks per wavefront");
        // A slot of one m-tile: nobody else reads its weight panel, which is then loaded with the
        // non-temporal hint, so that the stream does not push the token rows out of the caches.
        if (slot_tiles == 1) {
            if (my_blocks >= 4) k_loop(std::integral_constant<int, 4>{}, std::true_type{});
            else if (my_blocks == 3) k_loop(std::integral_constant<int, 3>{}, std::true_type{});
            else if (my_blocks == 2) k_loop(std::integral_constant<int, 2>{}, std::true_type{});
            else if (my_blocks == 1) k_loop(std::integral_constant<int, 1>{}, std::true_type{});
            else k_loop(std::integral_constant<int, 0>{}, std::true_type{});
        } else {
            if (my_blocks >= 4) k_loop(std::integral_constant<int, 4>{}, std::false_type{});
            else if (my_blocks == 3) k_loop(std::integral_constant<int, 3>{}, std::false_type{});
            else if (my_blocks == 2) k_loop(std::integral_constant<int, 2>{}, std::false_type{});
            else if (my_blocks == 1) k_loop(std::integral_constant<int, 1>{}, std::false_type{});
            else k_loop(std::integral_constant<int, 0>{}, std::false_type{});
        }
        // surplus loads must not land in the next trip's tiles (or outlive the workgroup's LDS)
        barrier_keep_loads<0>();

        if (piece < 0) {
            epilogue<EPI>(acc, c, gather.out_perm, lds, row0, row_end, n0, N, wm, wn, wave, lane);
        } else {  // a K piece of a leftover tile: raw accumulators to the workspace, [register][thread]
            float* dst = partials + kPlanFloats + (size_t)piece * (BM * BR) + tid;
#pragma unroll
            for (int i = 0; i < WB; ++i)
#pragma unroll
                for (int j = 0; j < TB; ++j) {
                    if (row0 + tile_block(wm, j) * 32 >= row_end) continue;  // a block without rows: the fix-up skips it too
#pragma unroll
                    for (int v = 0; v < 16; ++v) dst[((i * TB + j) * 16 + v) * (64 * NW)] = acc_read(acc[i][j][v]);
                }
        }
    }
}

// Adds the K pieces of each leftover tile in piece order and applies the epilogue.  One unit of work
// per (leftover tile, 32 x 32 block position of the wavefronts), so the sum itself is spread over
// the chip.  The plan (how many leftover tiles, how many pieces)
// is read from the head of the workspace, where the main kernel left it: when nothing was split,
// which the host cannot know, every workgroup exits after one load.
constexpr int kFixupUnitsPerGroup = 4;  // units per workgroup of the fix-up launch, one per 64 * NW threads
template <int EPI>
__global__ __launch_bounds__(64 * NW * kFixupUnitsPerGroup) void splitk_fixup(const int32_t* __restrict__ offsets, bf16_t* __restrict__ c,
                                                        const int32_t* __restrict__ out_perm,
                                                        const int* __restrict__ hdr,
                                                        const float* __restrict__ partials, int S, int N, int K,
                                                        int n_tiles, int G) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    constexpr int NB = EPI == kSwiglu ? WB / 2 : WB;
    constexpr int UNITS = TB * NB;
    Plan plan;  // uniform address: scalar loads
    plan.tiles = hdr[0]; plan.rounds = hdr[1]; plan.left = hdr[2]; plan.splits = hdr[3];
    if (plan.splits <= 1) return;
    // a workgroup holds kFixupUnitsPerGroup independent units (there is no barrier in this kernel): when nothing was
    // cut, which is the common case, a quarter as many workgroups have to start only to find that out
    const int tid = threadIdx.x % (64 * NW), lane = tid & 63, wave = tid >> 6;
    const int u = blockIdx.x * kFixupUnitsPerGroup + threadIdx.x / (64 * NW);  // the launch covers the most units there can be
    if (u >= plan.left * UNITS) return;
    const int tile = u / UNITS, unit = u % UNITS;
    const int mi = unit / NB, ni = unit % NB;
    int slot, row0, row_end, nt, slot_tiles;
    // the slot table in registers, as in the main kernel: a walk over slot_offsets in memory is a chain of up to S
    // dependent loads, longer than everything else this kernel does
    const SlotTable table = make_slot_table(offsets, S, n_tiles, lane);
    decode_tile(table, S, n_tiles, lane, plan.rounds * G + tile, slot, row0, row_end, nt, slot_tiles);
    if (row0 + tile_block(wave / WN, mi) * 32 >= row_end) return;  // this wavefront's block holds no rows: nothing was written
    floatx16 gate, up;
#pragma unroll
    for (int v = 0; v < 16; ++v) { gate[v] = 0.0f; up[v] = 0.0f; }
    for (int sp = 0; sp < plan.splits; ++sp) {
        const float* src = partials + (size_t)(tile * plan.splits + sp) * (BM * BR) + tid;
        float g[16], w[16];  // all loads of a piece in flight together, then the adds
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            g[v] = src[((ni * TB + mi) * 16 + v) * (64 * NW)];
            w[v] = EPI == kSwiglu ? src[(((ni + NB) * TB + mi) * 16 + v) * (64 * NW)] : 0.0f;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            gate[v] += g[v];
            up[v] += w[v];
        }
    }
    epilogue_block<EPI>(gate, up, c, out_perm, row0, row_end, nt * BNO, N, wave / WN, wave % WN, mi, ni, lane);
}

template <int EPI, bool KTAIL>
hipError_t launch_cfg(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c,
                      float* partials, int S, int N, int K, int n_tiles, hipStream_t st) {
    auto kern = grouped_gemm_bf16<EPI, KTAIL>;
    static std::atomic<bool> attr_set{false};  // set once per kernel; setting it twice from two threads is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    DeviceShape shape;
    hipError_t es = device_shape(&shape);
    if (es != hipSuccess) return es;
    // persistent: one workgroup per CU (the partial sums of the tiles cut along K are sized for kMaxGroups)
    kern<<<shape.groups, 64 * NW, LDS_BYTES, st>>>(a, gather, offsets, b0, b1, c, partials, S, N, K, n_tiles, shape.xcds);
    splitk_fixup<EPI><<<kFixupGroups / kFixupUnitsPerGroup, 64 * NW * kFixupUnitsPerGroup, 0, st>>>(offsets, c, gather.out_perm, reinterpret_cast<const int*>(partials),
                                                        partials + kPlanFloats, S, N, K, n_tiles, shape.groups);
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_one(const bf16_t* a, RowGather gather, const int32_t* offsets, const bf16_t* b0, const bf16_t* b1, bf16_t* c,
                      float* partials, int S, int N, int K, hipStream_t st) {
    constexpr int BNO = EPI == kSwiglu ? BR / 2 : BR;
    const int n_tiles = (N + BNO - 1) / BNO;
    if (K % BK == 0) return launch_cfg<EPI, false>(a, gather, offsets, b0, b1, c, partials, S, N, K, n_tiles, st);
    return launch_cfg<EPI, true>(a, gather, offsets, b0, b1, c, partials, S, N, K, n_tiles, st);
}

}  // namespace

hipError_t launch_ffn_bf16_tiled(const emoe_layer_desc& d, const void* x_perm, RowGather gather,
                                 const int32_t* offsets,
                                 const void* w1, const void* w3, const void* w2, void* y_perm, void* ws,
                                 int passes, hipStream_t st) {
    const FfnWs lay = ffn_ws_layout(d);
    bf16_t* h = reinterpret_cast<bf16_t*>(static_cast<uint8_t*>(ws) + lay.h);
    float* partials = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + lay.partials);
    const bf16_t* xp = static_cast<const bf16_t*>(x_perm);
    hipError_t e = hipSuccess;
    if (!(passes & 1)) {
    } else if (d.act == EMOE_ACT_SWIGLU)
        e = launch_one<kSwiglu>(xp, gather, offsets, static_cast<const bf16_t*>(w1), static_cast<const bf16_t*>(w3), h,
                                partials, d.S, d.d_ff, d.d_model, st);
    else
        e = launch_one<kRelu>(xp, gather, offsets, static_cast<const bf16_t*>(w1), nullptr, h, partials, d.S, d.d_ff, d.d_model,
                              st);
    if (e != hipSuccess || !(passes & 2)) return e;
    return launch_one<kPlain>(h, RowGather{nullptr, 1, 0, gather.out_perm}, offsets, static_cast<const bf16_t*>(w2), nullptr, static_cast<bf16_t*>(y_perm),
                              partials, d.S, d.d_model, d.d_ff, st);
}

}  // namespace emoe
