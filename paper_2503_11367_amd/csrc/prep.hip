// Preparation kernels for the attention passes: block-list sanitising and
// compaction of the tile classes into per-tile work lists (so that fully masked tiles are never visited --
// the block skipping of paper section 3.2.1) ordered longest first (the
// intra-GPU balance concern of section 3.2.2: long query blocks start early so
// that the tail of the launch is short).
#include "attn_common.h"

namespace mm {

// ---- block list ------------------------------------------------------------
// One workgroup: clears the error flag (the flag block is kFlagInts int32 wide),
// then copies the block list, replacing
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
// the line's non-empty tiles.
__global__ void __launch_bounds__(64)
compact_kernel(const uint8_t* __restrict__ cls, int32_t n_lines, int32_t n_items,
               int64_t line_stride, int64_t item_stride, int32_t* __restrict__ count,
               uint32_t* __restrict__ list) {
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
    if (lane == 0) count[line] = base;
}

// Ranks the lines: order[rank] = line, by (count descending, line ascending), so that
// heavy lines are scheduled first.  One thread per line; every thread counts the lines
// that precede its own, reading the counts through LDS in chunks (all lanes the same
// address: a broadcast).  Workgroup 0 also derives the slice length for cutting the
// lists (csz_out, may be null) from the total, the longest and the non-empty lists.
constexpr int kRankThreads = 256;
constexpr int kRankChunk = 2048;
__global__ void __launch_bounds__(kRankThreads)
rank_lines_kernel(const int32_t* __restrict__ count, int32_t n_lines, int32_t n_items,
                  int32_t* __restrict__ order, int32_t* __restrict__ csz_out, int32_t groups) {
    __shared__ __attribute__((aligned(16))) int32_t cnt_s[kRankChunk];
    const int tid = threadIdx.x;
    const int a = blockIdx.x * kRankThreads + tid;
    const int ca = a < n_lines ? count[a] : 0;
    int pos = 0;
    for (int b0 = 0; b0 < n_lines; b0 += kRankChunk) {
        const int nb = min(kRankChunk, n_lines - b0);
        __syncthreads();
        for (int b = tid; b < ((nb + 3) & ~3); b += kRankThreads) cnt_s[b] = b < nb ? count[b0 + b] : -1;
        __syncthreads();
        // four counts per LDS read; the tail of the last quad is padded with -1 (never ahead)
        for (int b = 0; b < nb; b += 4) {
            const int4 cb = *(const int4*)&cnt_s[b];
            pos += (cb.x > ca || (cb.x == ca && b0 + b < a)) ? 1 : 0;
            pos += (cb.y > ca || (cb.y == ca && b0 + b + 1 < a)) ? 1 : 0;
            pos += (cb.z > ca || (cb.z == ca && b0 + b + 2 < a)) ? 1 : 0;
            pos += (cb.w > ca || (cb.w == ca && b0 + b + 3 < a)) ? 1 : 0;
        }
    }
    if (a < n_lines) order[pos] = a;

    if (csz_out && blockIdx.x == 0) {          // workgroup-uniform
        __shared__ int64_t tot_s[kRankThreads];
        __shared__ int32_t max_s[kRankThreads], num_s[kRankThreads];
        int64_t total = 0;
        int longest = 0, lists = 0;
        for (int b = tid; b < n_lines; b += kRankThreads) {
            const int c = count[b];
            total += c;
            longest = max(longest, c);
            lists += c > 0 ? 1 : 0;
        }
        tot_s[tid] = total; max_s[tid] = longest; num_s[tid] = lists;
        __syncthreads();
        for (int off = kRankThreads / 2; off > 0; off >>= 1) {
            if (tid < off) {
                tot_s[tid] += tot_s[tid + off];
                max_s[tid] = max(max_s[tid], max_s[tid + off]);
                num_s[tid] += num_s[tid + off];
            }
            __syncthreads();
        }
        if (tid == 0) *csz_out = slice_length(tot_s[0], max_s[0], num_s[0], groups, n_items);
    }
}

static int launch_lists(const uint8_t* cls, int32_t n_lines, int32_t n_items, int64_t line_stride,
                        int64_t item_stride, int32_t* count, uint32_t* list, int32_t* order,
                        int32_t* csz_out, int32_t groups, hipStream_t st) {
    hipLaunchKernelGGL(compact_kernel, dim3(n_lines), dim3(64), 0, st, cls, n_lines, n_items,
                       line_stride, item_stride, count, list);
    hipLaunchKernelGGL(rank_lines_kernel, dim3((n_lines + kRankThreads - 1) / kRankThreads),
                       dim3(kRankThreads), 0, st, (const int32_t*)count, n_lines, n_items, order,
                       csz_out, groups);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
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
    return launch_lists(p.cls, p.nq, p.nk, (int64_t)p.nk, (int64_t)1, p.kcount, p.klist, p.qorder,
                        p.csz, p.groups, st);
}

int launch_compact_cols(const TilePlanT& p, hipStream_t st) {
    return launch_lists(p.cls, p.nk, p.nq, (int64_t)1, (int64_t)p.nk, p.qcount, p.qlist, p.korder,
                        nullptr, 1, st);
}

}  // namespace mm
