// Stable counting sort of the A = T*k assignments by slot id and the row gather into slot-contiguous
// order.  The per-slot row counts are the per-expert "workload" of eMoE Section 3.2.2.
//
// Four launches (three up to 65 536 assignments: scan and place fused; two when all assignments fit
// one workgroup: count, scan and place fused), no atomics on global memory, so the result is the
// unique stable permutation:
//   1. count    : each workgroup histograms its chunk of kPermuteChunk assignments (LDS counters)
//   2. scan     : per slot, exclusive prefix over the workgroups; then prefix over the slots
//   3. place    : each workgroup ranks its assignments in order with wave ballots and writes
//                 perm / inv_perm
//   4. gather   : one wavefront per output row copies the token row, 16 bytes per lane (left out
//                 when the caller wants indices only)
// An assignment whose expert is not resident (only possible when the caller broke emoe_route's
// precondition) is left out: inv_perm = -1, and it appears in no slot.
#include <mutex>

#include "common.h"

namespace emoe {
namespace {

// Scratch of emoe_permute_static, the variant of emoe_permute for callers that cannot allocate: the
// per-workgroup slot counts live in this array instead of a caller workspace.  Every GPU the library
// runs on holds its own copy at its own address until the process ends.  In host code the array's
// name is only a stand-in for the symbol; its address on the current device comes from
// hipGetSymbolAddress (static_scratch() below) and that pointer is what kernels receive.
constexpr size_t kStaticScratchInts = 65536;  // int32 [ceil(A / 1024)][S]
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
int32_t* scratch_of_device[kMaxDevices] = {};

// The current device's copy of `scratch`, looked up once per device.
hipError_t static_scratch(int32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_of_device[dev] == nullptr) {
        int32_t* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        scratch_of_device[dev] = ptr;
    }
    *out = scratch_of_device[dev];
    return hipSuccess;
}

constexpr int kThreads = 256;
constexpr int kPasses = kPermuteChunk / kThreads;

__device__ __forceinline__ int key_of(const int32_t* __restrict__ topk_expert,
                                      const int32_t* __restrict__ slot_of_expert, int a, int A, int E, int S) {
    if (a >= A) return -1;
    int e = topk_expert[a];
    if (e < 0 || e >= E) return -1;
    int s = slot_of_expert[e];
    return (s >= 0 && s < S) ? s : -1;
}

__global__ __launch_bounds__(kThreads) void count_kernel(const int32_t* __restrict__ topk_expert,
                                                         const int32_t* __restrict__ slot_of_expert,
                                                         int32_t* __restrict__ block_counts, int A, int E, int S) {
    __shared__ int cnt[kMaxExperts];
    if (threadIdx.x < kMaxExperts) cnt[threadIdx.x] = 0;
    __syncthreads();
    const int base = blockIdx.x * kPermuteChunk;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        int key = key_of(topk_expert, slot_of_expert, base + p * kThreads + threadIdx.x, A, E, S);
        if (key >= 0) atomicAdd(&cnt[key], 1);
    }
    __syncthreads();
    if (threadIdx.x < S) block_counts[(size_t)blockIdx.x * S + threadIdx.x] = cnt[threadIdx.x];
}

// One workgroup of 1024 threads.  Wave w handles slots w, w+16, ...: its lanes stride over the
// workgroups of the count kernel and turn block_counts[b][s] into the exclusive prefix over b.
__global__ __launch_bounds__(1024) void scan_kernel(int32_t* __restrict__ block_counts, int n_blocks, int S,
                                                    int32_t* __restrict__ slot_counts,
                                                    int32_t* __restrict__ slot_offsets) {
    __shared__ int total[kMaxExperts];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    for (int s = wave; s < S; s += 16) {
        int carry = 0;
        for (int b0 = 0; b0 < n_blocks; b0 += 64) {
            const int b = b0 + lane;
            int c = b < n_blocks ? block_counts[(size_t)b * S + s] : 0;
            int incl = c;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                int up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            if (b < n_blocks) block_counts[(size_t)b * S + s] = carry + incl - c;
            carry += __shfl(incl, 63);
        }
        if (lane == 0) total[s] = carry;
    }
    __syncthreads();
    if (wave == 0) {
        int c = lane < S ? total[lane] : 0;
        int incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane < S) {
            slot_counts[lane] = c;
            slot_offsets[lane] = incl - c;
        }
        if (lane == S - 1) slot_offsets[S] = incl;
    }
}

__global__ __launch_bounds__(kThreads) void place_kernel(const int32_t* __restrict__ topk_expert,
                                                         const int32_t* __restrict__ slot_of_expert,
                                                         const int32_t* __restrict__ block_prefix,
                                                         const int32_t* __restrict__ slot_offsets,
                                                         int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                                         int A, int E, int S) {
    __shared__ int running[kMaxExperts];             // next free row of each slot for this workgroup
    __shared__ int wave_cnt[kThreads / 64][kMaxExperts];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if (threadIdx.x < S)
        running[threadIdx.x] = slot_offsets[threadIdx.x] + block_prefix[(size_t)blockIdx.x * S + threadIdx.x];
    const int base = blockIdx.x * kPermuteChunk;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int p = 0; p < kPasses; ++p) {
        const int a = base + p * kThreads + threadIdx.x;
        const int key = key_of(topk_expert, slot_of_expert, a, A, E, S);
        int rank = 0;
        int mine = 0;  // lane s ends up with this wave's count for slot s
        for (int s = 0; s < S; ++s) {
            unsigned long long m = __ballot(key == s);
            if (key == s) rank = __popcll(m & below);
            if (lane == s) mine = __popcll(m);
        }
        wave_cnt[wave][lane] = mine;
        __syncthreads();  // wave counts (and, first pass, running[]) visible
        if (key >= 0) {
            int r = running[key] + rank;
            for (int w = 0; w < wave; ++w) r += wave_cnt[w][key];
            perm[r] = a;
            inv_perm[a] = r;
        } else if (a < A) {
            inv_perm[a] = -1;
        }
        __syncthreads();  // everyone has read running[] and wave_cnt[]
        if (threadIdx.x < S) {
            int add = 0;
#pragma unroll
            for (int w = 0; w < kThreads / 64; ++w) add += wave_cnt[w][threadIdx.x];
            running[threadIdx.x] += add;
        }
        __syncthreads();  // running[] updated before the next pass reads it and rewrites wave_cnt[]
    }
}

// count + scan + place in one workgroup, for A <= kPermuteChunk (a decode step, a short prompt): two
// launches fewer.  One thread per assignment (16 wavefronts), one pass: every wavefront ranks its 64
// assignments per slot with ballots, wavefront 0 turns the 16 x S counts into the slots' offsets, and
// each assignment's row is its slot's offset + the counts of the wavefronts before its own + its rank.
constexpr int kSmallThreads = kPermuteChunk;
constexpr int kSmallWaves = kSmallThreads / 64;
__global__ __launch_bounds__(kSmallThreads) void sort_small_kernel(const int32_t* __restrict__ topk_expert,
                                                                   const int32_t* __restrict__ slot_of_expert,
                                                                   int32_t* __restrict__ slot_counts,
                                                                   int32_t* __restrict__ slot_offsets,
                                                                   int32_t* __restrict__ perm,
                                                                   int32_t* __restrict__ inv_perm, int A, int E, int S) {
    __shared__ int wave_cnt[kSmallWaves][kMaxExperts];  // [wavefront][slot]: count, then the first row of that wavefront's share
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int a = threadIdx.x;
    const int key = key_of(topk_expert, slot_of_expert, a, A, E, S);
    const unsigned long long below = (1ull << lane) - 1ull;
    int rank = 0, mine = 0;  // lane s ends up with this wavefront's count for slot s
    for (int s = 0; s < S; ++s) {
        const unsigned long long m = __ballot(key == s);
        if (key == s) rank = __popcll(m & below);
        if (lane == s) mine = __popcll(m);
    }
    wave_cnt[wave][lane] = mine;
    __syncthreads();
    if (wave == 0) {  // lane = slot: total, exclusive prefix over the slots, then the start of every wavefront's share
        int c = 0;
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) c += wave_cnt[w][lane];
        int incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane < S) {
            slot_counts[lane] = c;
            slot_offsets[lane] = incl - c;
        }
        if (lane == S - 1) slot_offsets[S] = incl;
        int run = incl - c;
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) {
            const int n = wave_cnt[w][lane];
            wave_cnt[w][lane] = run;
            run += n;
        }
    }
    __syncthreads();
    if (key >= 0) {
        const int r = wave_cnt[wave][key] + rank;
        perm[r] = a;
        inv_perm[a] = r;
    } else if (a < A) {
        inv_perm[a] = -1;
    }
}

// scan + place in one launch, for up to kScanPlaceBlocks chunks (65 536 assignments): every workgroup adds
// up the chunk counts of the count kernel itself - all of them for the slots' offsets, those of the
// chunks before its own for its first row in each slot - instead of waiting for a scan launch; with
// few chunks those are a few thousand cached integers.  One thread per assignment as in
// sort_small_kernel.  Workgroup 0 also writes slot_counts and slot_offsets.
constexpr int kScanPlaceBlocks = 64;
__global__ __launch_bounds__(kSmallThreads) void scan_place_kernel(const int32_t* __restrict__ topk_expert,
                                                                   const int32_t* __restrict__ slot_of_expert,
                                                                   const int32_t* __restrict__ block_counts, int n_blocks,
                                                                   int32_t* __restrict__ slot_counts,
                                                                   int32_t* __restrict__ slot_offsets,
                                                                   int32_t* __restrict__ perm,
                                                                   int32_t* __restrict__ inv_perm, int A, int E, int S) {
    __shared__ int wave_cnt[kSmallWaves][kMaxExperts];  // [wavefront][slot]: count, then the first row of that wavefront's share
    __shared__ int part_total[kSmallWaves][kMaxExperts], part_before[kSmallWaves][kMaxExperts];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int a = blockIdx.x * kSmallThreads + threadIdx.x;
    const int key = key_of(topk_expert, slot_of_expert, a, A, E, S);
    // wavefront w adds up chunks w, w + 16, ... for slot `lane`
    int total = 0, before = 0;
    if (lane < S) {
        for (int b = wave; b < n_blocks; b += kSmallWaves) {
            const int c = block_counts[(size_t)b * S + lane];
            total += c;
            if (b < (int)blockIdx.x) before += c;
        }
    }
    part_total[wave][lane] = total;
    part_before[wave][lane] = before;
    const unsigned long long below = (1ull << lane) - 1ull;
    int rank = 0, mine = 0;  // lane s ends up with this wavefront's count for slot s
    for (int s = 0; s < S; ++s) {
        const unsigned long long m = __ballot(key == s);
        if (key == s) rank = __popcll(m & below);
        if (lane == s) mine = __popcll(m);
    }
    wave_cnt[wave][lane] = mine;
    __syncthreads();
    if (wave == 0) {  // lane = slot
        int c = 0, b4 = 0;
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) {
            c += part_total[w][lane];
            b4 += part_before[w][lane];
        }
        int incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (blockIdx.x == 0) {
            if (lane < S) {
                slot_counts[lane] = c;
                slot_offsets[lane] = incl - c;
            }
            if (lane == S - 1) slot_offsets[S] = incl;
        }
        int run = incl - c + b4;
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) {
            const int n = wave_cnt[w][lane];
            wave_cnt[w][lane] = run;
            run += n;
        }
    }
    __syncthreads();
    if (key >= 0) {
        const int r = wave_cnt[wave][key] + rank;
        perm[r] = a;
        inv_perm[a] = r;
    } else if (a < A) {
        inv_perm[a] = -1;
    }
}

// One wavefront per grouped row: x_perm[r,:] = x[perm[r]/k,:].  Rows past the number of placed
// assignments (only when some were left out) are not written.
template <int kElemBytes>
__global__ __launch_bounds__(kThreads) void gather_kernel(const uint8_t* __restrict__ x,
                                                          const int32_t* __restrict__ perm,
                                                          const int32_t* __restrict__ slot_offsets,
                                                          uint8_t* __restrict__ x_perm, int A, int k, int d, int S) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= A || r >= slot_offsets[S]) return;
    const int t = perm[r] / k;
    const size_t row_bytes = (size_t)d * kElemBytes;
    const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * row_bytes);
    uint4* dst = reinterpret_cast<uint4*>(x_perm + (size_t)r * row_bytes);
    const int n16 = (int)(row_bytes / 16);
    for (int i = lane; i < n16; i += 64) dst[i] = src[i];
}

}  // namespace

hipError_t launch_permute(const emoe_layer_desc& d, const void* x, const int32_t* topk_expert,
                          const int32_t* slot_of_expert, int32_t* counts, int32_t* offsets, int32_t* perm,
                          int32_t* inv_perm, void* x_perm, void* ws, hipStream_t st) {
    const int A = d.T * d.k;
    const int n_blocks = (A + kPermuteChunk - 1) / kPermuteChunk;
    int32_t* block_counts = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(ws) + permute_ws_layout(d).block_counts);
    if (n_blocks == 1) {
        sort_small_kernel<<<1, kSmallThreads, 0, st>>>(topk_expert, slot_of_expert, counts, offsets, perm, inv_perm, A, d.E,
                                                  d.S);
    } else if (n_blocks <= kScanPlaceBlocks) {
        count_kernel<<<n_blocks, kThreads, 0, st>>>(topk_expert, slot_of_expert, block_counts, A, d.E, d.S);
        scan_place_kernel<<<n_blocks, kSmallThreads, 0, st>>>(topk_expert, slot_of_expert, block_counts, n_blocks, counts,
                                                              offsets, perm, inv_perm, A, d.E, d.S);
    } else {
        count_kernel<<<n_blocks, kThreads, 0, st>>>(topk_expert, slot_of_expert, block_counts, A, d.E, d.S);
        scan_kernel<<<1, 1024, 0, st>>>(block_counts, n_blocks, d.S, counts, offsets);
        place_kernel<<<n_blocks, kThreads, 0, st>>>(topk_expert, slot_of_expert, block_counts, offsets, perm,
                                                    inv_perm, A, d.E, d.S);
    }
    if (x_perm == nullptr) return hipGetLastError();  // indices only: the FFN reads x through perm
    const int rows_per_block = kThreads / 64;
    const int g = (A + rows_per_block - 1) / rows_per_block;
    if (d.dtype == EMOE_F32)
        gather_kernel<4><<<g, kThreads, 0, st>>>(static_cast<const uint8_t*>(x), perm, offsets,
                                                 static_cast<uint8_t*>(x_perm), A, d.k, d.d_model, d.S);
    else
        gather_kernel<2><<<g, kThreads, 0, st>>>(static_cast<const uint8_t*>(x), perm, offsets,
                                                 static_cast<uint8_t*>(x_perm), A, d.k, d.d_model, d.S);
    return hipGetLastError();
}

}  // namespace emoe

extern "C" int emoe_permute_static(const emoe_layer_desc* desc, const void* x, const int32_t* topk_expert,
                                   const int32_t* slot_of_expert, int32_t* slot_counts, int32_t* slot_offsets,
                                   int32_t* perm, int32_t* inv_perm, void* x_perm, void* stream) {
    using namespace emoe;
    int rc = validate_desc(desc);
    if (rc != EMOE_OK) return rc;
    if (!topk_expert || !slot_of_expert || !slot_counts || !slot_offsets || !perm || !inv_perm) return EMOE_ERR_NULL;
    if (x_perm && !x) return EMOE_ERR_NULL;
    const long long A = (long long)desc->T * desc->k;
    const long long n_blocks = (A + kPermuteChunk - 1) / kPermuteChunk;
    if (n_blocks * desc->S > (long long)kStaticScratchInts) return EMOE_ERR_WORKSPACE;  // beyond the static scratch
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (desc->T == 0) {
        hipError_t z1 = launch_fill_i32(slot_counts, desc->S, 0, st);
        hipError_t z2 = launch_fill_i32(slot_offsets, desc->S + 1, 0, st);
        return (z1 == hipSuccess && z2 == hipSuccess) ? EMOE_OK : EMOE_ERR_DEVICE;
    }
    int32_t* ptr = nullptr;
    if (static_scratch(&ptr) != hipSuccess) return EMOE_ERR_DEVICE;
    // Nothing in the scratch has to start at zero: the count kernel writes every entry that the scan
    // and place kernels read, so what the previous call left there is overwritten before it is read.
    hipError_t e = launch_permute(*desc, x, topk_expert, slot_of_expert, slot_counts, slot_offsets, perm, inv_perm, x_perm,
                                  ptr, st);
    return e == hipSuccess ? EMOE_OK : EMOE_ERR_DEVICE;
}
