// Preparation kernels for the attention passes: block-list sanitising,
// permuted transposes of operand tensors, and compaction of the tile classes
// into per-tile work lists (so that fully masked tiles are never visited --
// the block skipping of paper section 3.2.1) ordered longest first (the
// intra-GPU balance concern of section 3.2.2: long query blocks start early so
// that the tail of the launch is short).
#include "attn_common.h"

namespace mm {

// ---- block list ------------------------------------------------------------
__global__ void sanitize_blocks_kernel(const int32_t* __restrict__ blocks, int32_t n_blocks,
                                       int64_t n_seq_blocks, int32_t* __restrict__ clean,
                                       int32_t* __restrict__ err) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_blocks) return;
    int32_t b = blocks[i];
    if (b < 0 || b >= n_seq_blocks) {
        atomicOr(err, 1);
        b = 0;
    }
    clean[i] = b;
}

__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

int launch_validate_blocks(const int32_t* blocks, int32_t n_blocks, int64_t n_seq_blocks,
                           int32_t* clean, int32_t* err, hipStream_t st) {
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, st, err);
    hipLaunchKernelGGL(sanitize_blocks_kernel, dim3((n_blocks + 255) / 256), dim3(256), 0, st,
                       blocks, n_blocks, n_seq_blocks, clean, err);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

// ---- permuted transpose  X[n][H][D] -> XT[H][D][n_pad] -----------------------
// Inside every group of 16 consecutive tokens the stored order is
// [0..3, 8..11, 4..7, 12..15]; tokens >= n read as zero.
__global__ void __launch_bounds__(256)
transpose_perm_kernel(const ushort_t* __restrict__ x, ushort_t* __restrict__ xt, int64_t n,
                      int64_t n_pad, int32_t H, int32_t D) {
    __shared__ ushort_t tile[64][64 + 2];
    const int64_t n0 = (int64_t)blockIdx.x * 64;
    const int d0 = blockIdx.y * 64;
    const int h = blockIdx.z;
    const int tid = threadIdx.x;
    for (int i = 0; i < 2; ++i) {
        const int tok = tid / 8 + 32 * i;
        const int dc = (tid % 8) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (n0 + tok < n)
            v = *(const uint4*)(x + ((n0 + tok) * H + h) * (int64_t)D + d0 + dc);
        const ushort_t* e = (const ushort_t*)&v;
        for (int u = 0; u < 8; ++u) tile[tok][dc + u] = e[u];
    }
    __syncthreads();
    for (int i = 0; i < 2; ++i) {
        const int d = tid / 8 + 32 * i;
        const int p0 = (tid % 8) * 8;
        uint4 v;
        ushort_t* e = (ushort_t*)&v;
        for (int u = 0; u < 8; ++u) {
            const int pos = p0 + u;
            const int tok = (pos & ~15) + perm16_index_of_pos(pos & 15);
            e[u] = tile[tok][d];
        }
        *(uint4*)(xt + ((int64_t)h * D + d0 + d) * n_pad + n0 + p0) = v;
    }
}

int launch_transpose_perm(const void* x, void* xt, int64_t n, int64_t n_pad, int32_t H, int32_t D,
                          hipStream_t st) {
    dim3 grid((unsigned)(n_pad / 64), (unsigned)(D / 64), (unsigned)H);
    hipLaunchKernelGGL(transpose_perm_kernel, grid, dim3(256), 0, st, (const ushort_t*)x,
                       (ushort_t*)xt, n, n_pad, H, D);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

// ---- work lists ---------------------------------------------------------------
// One wavefront per line (a q-tile's row of classes, or a k-tile's column).
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

// order[rank] = line, ranks by (count descending, line ascending)
__global__ void __launch_bounds__(1024)
order_kernel(const int32_t* __restrict__ count, int32_t n, int32_t* __restrict__ order) {
    for (int a = threadIdx.x; a < n; a += 1024) {
        const int ca = count[a];
        int pos = 0;
        for (int b = 0; b < n; ++b) {
            const int cb = count[b];
            pos += (cb > ca || (cb == ca && b < a)) ? 1 : 0;
        }
        order[pos] = a;
    }
}

int launch_compact_rows(const TilePlan& p, hipStream_t st) {
    hipLaunchKernelGGL(compact_kernel, dim3(p.nq), dim3(64), 0, st, p.cls, p.nq, p.nk,
                       (int64_t)p.nk, (int64_t)1, p.kcount, p.klist);
    hipLaunchKernelGGL(order_kernel, dim3(1), dim3(1024), 0, st, p.kcount, p.nq, p.qorder);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

int launch_compact_cols(const TilePlanT& p, hipStream_t st) {
    hipLaunchKernelGGL(compact_kernel, dim3(p.nk), dim3(64), 0, st, p.cls, p.nk, p.nq,
                       (int64_t)1, (int64_t)p.nk, p.qcount, p.qlist);
    hipLaunchKernelGGL(order_kernel, dim3(1), dim3(1024), 0, st, p.qcount, p.nk, p.korder);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
