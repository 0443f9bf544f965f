// Preparation kernels for the attention passes: block-list sanitising,
// permuted transposes of operand tensors, and compaction of the tile classes
// into per-tile work lists (so that fully masked tiles are never visited --
// the block skipping of paper section 3.2.1) ordered longest first (the
// intra-GPU balance concern of section 3.2.2: long query blocks start early so
// that the tail of the launch is short).
#include "attn_common.h"

namespace mm {

// ---- block list ------------------------------------------------------------
// One workgroup: clears the error flag and the plan tickets that follow it (the
// flag block is kFlagInts int32 wide), then copies the block list, replacing
// out-of-range entries by 0 and raising the flag.
__global__ void __launch_bounds__(256)
validate_blocks_kernel(const int32_t* __restrict__ blocks, int32_t n_blocks, int64_t n_seq_blocks,
                       int32_t* __restrict__ clean, int32_t* __restrict__ err) {
    int bad = 0;
    for (int i = threadIdx.x; i < n_blocks; i += 256) {
        int32_t b = blocks[i];
        if (b < 0 || b >= n_seq_blocks) {
            bad = 1;
            b = 0;
        }
        clean[i] = b;
    }
    bad = __syncthreads_or(bad);
    if (threadIdx.x < kFlagInts) err[threadIdx.x] = threadIdx.x == 0 ? bad : 0;
}

int launch_validate_blocks(const int32_t* blocks, int32_t n_blocks, int64_t n_seq_blocks,
                           int32_t* clean, int32_t* err, hipStream_t st) {
    hipLaunchKernelGGL(validate_blocks_kernel, dim3(1), dim3(256), 0, st, blocks, n_blocks,
                       n_seq_blocks, clean, err);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

// ---- work lists ---------------------------------------------------------------
// One wavefront per line (a q-tile's row of classes, or a k-tile's column) compacts
// the line's non-empty tiles.  The wavefront that finishes last (a ticket counter,
// zeroed by validate_blocks_kernel) then ranks the lines: order[rank] = line, by
// (count descending, line ascending), so that heavy lines are scheduled first.
constexpr int kCompactChunk = 2048;
__global__ void __launch_bounds__(64)
compact_kernel(const uint8_t* __restrict__ cls, int32_t n_lines, int32_t n_items,
               int64_t line_stride, int64_t item_stride, int32_t* __restrict__ count,
               uint32_t* __restrict__ list, int32_t* __restrict__ order,
               int32_t* __restrict__ ticket, int32_t* __restrict__ csz_out, int32_t groups) {
    const int line = blockIdx.x;
    const int lane = threadIdx.x;
    int base = 0;
    for (int j0 = 0; j0 < n_items; j0 += kWave) {
        const int j = j0 + lane;
        uint8_t c = MMATTN_TILE_EMPTY;
        if (j < n_items) c = cls[line * line_stride + j * item_stride];
        const bool act = c != MMATTN_TILE_EMPTY;
        const uint64_t m = __ballot(act);
        if (act) {
            const int pos = base + __popcll(m & ((1ull << lane) - 1));
            list[(int64_t)line * n_items + pos] =
                (uint32_t)j | (c == MMATTN_TILE_PARTIAL ? kPartialFlag : 0u);
        }
        base += __popcll(m);
    }
    int last = 0;
    if (lane == 0) {
        __hip_atomic_store(&count[line], base, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();                   // the count is visible before the ticket is taken
        last = atomicAdd(ticket, 1) == n_lines - 1;
    }
    if (!__shfl(last, 0)) return;
    __threadfence();
    // the counts go through LDS in chunks, so that the quadratic comparison reads
    // (all lanes the same address: a broadcast) never go back to memory
    __shared__ int32_t cnt_s[kCompactChunk];
    if (csz_out) {                             // suggested slice length for cutting the lists
        int64_t total = 0;
        int longest = 0, lists = 0;
        for (int a = lane; a < n_lines; a += kWave) {
            const int c = __hip_atomic_load(&count[a], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            total += c;
            longest = max(longest, c);
            lists += c > 0 ? 1 : 0;
        }
        for (int off = 32; off > 0; off >>= 1) {
            total += __shfl_xor(total, off);
            longest = max(longest, __shfl_xor(longest, off));
            lists += __shfl_xor(lists, off);
        }
        if (lane == 0) *csz_out = slice_length(total, longest, lists, groups, n_items);
    }
    for (int a0 = 0; a0 < n_lines; a0 += kWave) {
        const int a = a0 + lane;
        const int ca = a < n_lines
                           ? __hip_atomic_load(&count[a], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
        int pos = 0;
        for (int b0 = 0; b0 < n_lines; b0 += kCompactChunk) {
            const int nb = min(kCompactChunk, n_lines - b0);
            __syncthreads();                 // single-wave workgroup: orders the LDS accesses
            for (int b = lane; b < nb; b += kWave)
                cnt_s[b] = __hip_atomic_load(&count[b0 + b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            for (int b = 0; b < nb; ++b) {
                const int cb = cnt_s[b];
                pos += (cb > ca || (cb == ca && b0 + b < a)) ? 1 : 0;
            }
        }
        if (a < n_lines) order[pos] = a;
    }
}

// zero fill of two equally sized buffers (a kernel rather than a memset node, so
// that the call can sit inside a captured graph)
__global__ void __launch_bounds__(256)
zero_pair_kernel(u32x4* __restrict__ a, u32x4* __restrict__ b, size_t n16) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        a[i] = z;
        b[i] = z;
    }
}

int launch_zero_kv(void* dk, void* dv, size_t bytes_each, hipStream_t st) {
    const size_t n16 = bytes_each / 16;           // S*Hkv*D*2 with D in {64,128}: a multiple of 16
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 4096);
    hipLaunchKernelGGL(zero_pair_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)dk, (u32x4*)dv, n16);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

int launch_compact_rows(const TilePlan& p, hipStream_t st) {
    hipLaunchKernelGGL(compact_kernel, dim3(p.nq), dim3(64), 0, st, p.cls, p.nq, p.nk,
                       (int64_t)p.nk, (int64_t)1, p.kcount, p.klist, p.qorder, p.ticket, p.csz, p.groups);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

int launch_compact_cols(const TilePlanT& p, hipStream_t st) {
    hipLaunchKernelGGL(compact_kernel, dim3(p.nk), dim3(64), 0, st, p.cls, p.nk, p.nq,
                       (int64_t)1, (int64_t)p.nk, p.qcount, p.qlist, p.korder, p.ticket, (int32_t*)nullptr, 1);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
