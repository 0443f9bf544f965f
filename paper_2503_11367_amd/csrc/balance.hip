// mmattn_balance: Alg. 1 of the paper (section 3.2.1) in its LPT reading --
// blocks visited by (W descending, index ascending), each given to the rank
// with (load ascending, rank ascending).  Integer-only; one workgroup, because
// the greedy loop is inherently serial and the inputs are at most a few
// thousand blocks.
//
//   phase 1  every thread ranks its blocks by counting the blocks that precede
//            them in the visiting order (a total order, so ranks are a
//            permutation); the workloads are staged in LDS when they fit;
//   phase 2  wavefront 0 runs the greedy loop.  Up to 64 ranks (SLOTS == 1): the
//            lanes hold the ranks sorted by (load, rank), the block goes to lane
//            0's rank and one ballot re-inserts its grown key.  More ranks: lane
//            l keeps the loads of ranks l, l+64, ... in registers (SLOTS of
//            them, a template parameter chosen from P) and its own local
//            minimum; a wave-level lexicographic min picks the receiving rank;
//   phase 3  per-rank CSR lists in ascending block index by counting, for each
//            block, the earlier blocks of the same rank.
#include "common.h"

namespace mm {

constexpr int kBalThreads = 1024;
constexpr int kBalSlots = MMATTN_MAX_RANKS / kWave;   // most ranks per lane
constexpr int kBalLdsW = 8192;                        // workloads staged in LDS up to this many blocks

struct MinKey { uint64_t load; uint32_t rank; };

__device__ __forceinline__ bool key_less(const MinKey& a, const MinKey& b) {
    return a.load < b.load || (a.load == b.load && a.rank < b.rank);
}

// minimum of v over the 64 lanes, returned wave-uniform: prefix minima inside each
// row of 16 lanes (row_shr 1,2,4,8), then lane 15 of a row into the next row
// (row_bcast:15) and lane 31 into the upper half (row_bcast:31); lane 63 ends up
// with the minimum.  Lanes without a source keep the identity.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    constexpr int kId = -1;                 // 0xFFFFFFFF, identity of the unsigned minimum
#define MM_MIN_DPP(ctrl, rows)                                                                  \
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp(kId, (int)v, ctrl, rows, 0xf, false))
    MM_MIN_DPP(0x111, 0xf);                 // row_shr:1
    MM_MIN_DPP(0x112, 0xf);                 // row_shr:2
    MM_MIN_DPP(0x114, 0xf);                 // row_shr:4
    MM_MIN_DPP(0x118, 0xf);                 // row_shr:8
    MM_MIN_DPP(0x142, 0xa);                 // row_bcast:15 into rows 1 and 3
    MM_MIN_DPP(0x143, 0xc);                 // row_bcast:31 into rows 2 and 3
#undef MM_MIN_DPP
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// lexicographic minimum of (load, rank) over the wavefront: three 32-bit minima,
// each restricted to the lanes that tie on the more significant parts
__device__ __forceinline__ MinKey wave_min(MinKey k) {
    const uint32_t hi = (uint32_t)(k.load >> 32), lo = (uint32_t)k.load;
    const uint32_t hi_min = wave_min_u32(hi);
    const uint32_t lo_min = wave_min_u32(hi == hi_min ? lo : 0xFFFFFFFFu);
    const bool tie = hi == hi_min && lo == lo_min;
    MinKey r;
    r.load = ((uint64_t)hi_min << 32) | lo_min;
    r.rank = wave_min_u32(tie ? k.rank : 0xFFFFFFFFu);
    return r;
}

// the value held by the next higher lane (wavefront shift left by one; lane 63 keeps
// its own, which the caller never uses)
__device__ __forceinline__ uint32_t lane_above(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x130 /* wave_shl:1 */, 0xf, 0xf, false);
}

template <int SLOTS>
__global__ void __launch_bounds__(kBalThreads)
balance_kernel(const uint64_t* __restrict__ W, int32_t nB, int32_t P,
               int32_t* __restrict__ rank_of_block, uint64_t* __restrict__ load,
               int32_t* __restrict__ rank_off, int32_t* __restrict__ rank_blocks) {
    __shared__ __attribute__((aligned(16))) uint16_t rob[MMATTN_MAX_BLOCKS];
    __shared__ int32_t count[MMATTN_MAX_RANKS + 1];
    __shared__ __attribute__((aligned(16))) uint64_t w_lds[kBalLdsW];
    const int tid = threadIdx.x;

    // phase 1: visiting order, kept in rank_blocks until phase 3 overwrites it
    int32_t* order = rank_blocks;
    const bool staged = nB <= kBalLdsW;                // workgroup-uniform
    if (staged) {
        for (int b = tid; b < nB; b += kBalThreads) w_lds[b] = W[b];
        __syncthreads();
    }
    const uint64_t* Wp = staged ? w_lds : W;           // phase 2 reads the workloads through this
    for (int b = tid; b < nB; b += kBalThreads) {
        int pos = 0;
        if (staged) {
            const uint64_t wb = w_lds[b];
            typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
            const u64x2* w2 = (const u64x2*)w_lds;     // two workloads per LDS read
            const int pairs = nB >> 1;
#pragma unroll 4
            for (int c2 = 0; c2 < pairs; ++c2) {
                const u64x2 wc = w2[c2];
                pos += (wc.x > wb || (wc.x == wb && 2 * c2 < b)) ? 1 : 0;
                pos += (wc.y > wb || (wc.y == wb && 2 * c2 + 1 < b)) ? 1 : 0;
            }
            if (nB & 1) {
                const uint64_t wc = w_lds[nB - 1];
                pos += (wc > wb || (wc == wb && nB - 1 < b)) ? 1 : 0;
            }
        } else {
            const uint64_t wb = W[b];
            for (int c = 0; c < nB; ++c) {
                const uint64_t wc = W[c];
                pos += (wc > wb || (wc == wb && c < b)) ? 1 : 0;
            }
        }
        order[pos] = b;
    }
    for (int g = tid; g <= P; g += kBalThreads) count[g] = 0;
    __syncthreads();

    // phase 2: greedy assignment by wavefront 0
    if (SLOTS == 1 && P == 1 && tid < kWave) {
        // a single rank receives every block
        uint64_t sum = 0;
        for (int b = tid; b < nB; b += kWave) {
            rank_of_block[b] = 0;
            rob[b] = 0;
            sum += Wp[b];
        }
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
        if (tid == 0) load[0] = sum;
    } else if (SLOTS == 1 && tid < kWave) {
        // At most one rank per lane: the lanes hold the ranks SORTED by (load, rank), lane 0
        // the least loaded.  A block goes to lane 0's rank; its new key is re-inserted at
        // the position given by how many other keys are smaller (one ballot), the keys
        // before that position move down one lane.  All per-block decisions are scalar.
        const int lane = tid;
        uint32_t lo = lane < P ? 0u : 0xFFFFFFFFu, hi = lo;          // load; lanes >= P: +inf
        uint32_t rk = lane < P ? (uint32_t)lane : 0xFFFFFFFFu;
        for (int t0 = 0; t0 < nB; t0 += kWave) {
            const int t = t0 + lane;
            const int32_t my_b = t < nB ? order[t] : 0;
            const uint64_t my_w = t < nB ? Wp[my_b] : 0;
            const int n = min(kWave, nB - t0);
            for (int u = 0; u < n; ++u) {
                const int32_t b = __builtin_amdgcn_readlane(my_b, u);
                const uint64_t w = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(my_w >> 32), u) << 32) |
                                   (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)my_w, u);
                const uint32_t g = (uint32_t)__builtin_amdgcn_readlane((int)rk, 0);
                const uint64_t grown = (((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, 0) << 32) |
                                        (uint32_t)__builtin_amdgcn_readlane((int)lo, 0)) + w;
                const uint64_t mine = ((uint64_t)hi << 32) | lo;
                const bool less = lane > 0 && (mine < grown || (mine == grown && rk < g));
                const int at = __popcll(__ballot(less));              // new lane of rank g
                // lanes below `at` take their upper neighbour's key, lane `at` the grown one
                const uint32_t lo_up = lane_above(lo), hi_up = lane_above(hi), rk_up = lane_above(rk);
                if (lane < at) { lo = lo_up; hi = hi_up; rk = rk_up; }
                else if (lane == at) { lo = (uint32_t)grown; hi = (uint32_t)(grown >> 32); rk = g; }
                if (lane == 0) {
                    rank_of_block[b] = (int32_t)g;
                    rob[b] = (uint16_t)g;
                }
            }
        }
        if (lane < P) load[rk] = ((uint64_t)hi << 32) | lo;
    } else if (tid < kWave) {
        const int lane = tid;
        uint64_t mine[SLOTS];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) mine[s] = 0;
        MinKey local;                       // this lane's least-loaded rank
        local.load = lane < P ? 0 : ~0ull;
        local.rank = lane < P ? (uint32_t)lane : 0xFFFFFFFFu;
        for (int t0 = 0; t0 < nB; t0 += kWave) {
            const int t = t0 + lane;
            const int32_t my_b = t < nB ? order[t] : 0;
            const uint64_t my_w = t < nB ? Wp[my_b] : 0;
            const int n = min(kWave, nB - t0);
            for (int u = 0; u < n; ++u) {
                const int32_t b = __builtin_amdgcn_readlane(my_b, u);
                const uint32_t wlo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)my_w, u);
                const uint32_t whi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(my_w >> 32), u);
                const uint64_t w = ((uint64_t)whi << 32) | wlo;
                const uint32_t g = wave_min(local).rank;
                if ((int)(g & (kWave - 1)) == lane) {
                    const int slot = g / kWave;
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s)
                        if (s == slot) mine[s] += w;
                    // recompute the lane's local minimum over its ranks
                    local.load = ~0ull;
                    local.rank = 0xFFFFFFFFu;
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s) {
                        const uint32_t r = (uint32_t)(lane + s * kWave);
                        if ((int)r < P) {
                            MinKey cand{mine[s], r};
                            if (key_less(cand, local)) local = cand;
                        }
                    }
                    rank_of_block[b] = (int32_t)g;
                    rob[b] = (uint16_t)g;
                }
            }
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int r = lane + s * kWave;
            if (r < P) load[r] = mine[s];
        }
    }
    __syncthreads();

    // phase 3: CSR lists, ascending block index inside each rank
    for (int b = tid; b < nB; b += kBalThreads) atomicAdd(&count[rob[b] + 1], 1);
    __syncthreads();
    if (tid == 0)
        for (int g = 0; g < P; ++g) count[g + 1] += count[g];
    __syncthreads();
    for (int g = tid; g <= P; g += kBalThreads) rank_off[g] = count[g];
    for (int b = tid; b < nB; b += kBalThreads) {
        const uint16_t g = rob[b];
        int before = 0;
        typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
        const u16x8* rob8 = (const u16x8*)rob;         // eight ranks per LDS read
        const int octets = b >> 3;
#pragma unroll 2
        for (int c8 = 0; c8 < octets; ++c8) {
            const u16x8 r = rob8[c8];
#pragma unroll
            for (int u = 0; u < 8; ++u) before += r[u] == g ? 1 : 0;
        }
        for (int c = octets << 3; c < b; ++c) before += rob[c] == g ? 1 : 0;
        rank_blocks[count[g] + before] = b;
    }
}

int launch_balance(const uint64_t* d_W, int32_t nB, int32_t P, int32_t* d_rank_of_block,
                   uint64_t* d_load, int32_t* d_rank_off, int32_t* d_rank_blocks, hipStream_t st) {
    // registers per lane for the rank loads: the smallest instantiation that holds P ranks
    if (P <= kWave)
        hipLaunchKernelGGL(balance_kernel<1>, dim3(1), dim3(kBalThreads), 0, st, d_W, nB, P,
                           d_rank_of_block, d_load, d_rank_off, d_rank_blocks);
    else if (P <= 4 * kWave)
        hipLaunchKernelGGL(balance_kernel<4>, dim3(1), dim3(kBalThreads), 0, st, d_W, nB, P,
                           d_rank_of_block, d_load, d_rank_off, d_rank_blocks);
    else
        hipLaunchKernelGGL(balance_kernel<kBalSlots>, dim3(1), dim3(kBalThreads), 0, st, d_W, nB, P,
                           d_rank_of_block, d_load, d_rank_off, d_rank_blocks);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
