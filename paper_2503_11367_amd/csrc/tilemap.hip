// Tile map (paper section 3.2.1): for every (q-tile, k-tile) the number of
// unmasked (query,key) pairs and the class EMPTY / FULL / PARTIAL; a tile whose
// mask block is all zeros is the one the attention kernels skip.  Row sums give
// the per-block workloads W_b that Alg. 1 balances.
//
// Integer ALU work.  One wavefront per tile pair, four k-tiles per workgroup
// sharing the q-tile's words in LDS.  A k-tile is a handful of "runs" (maximal
// stretches of keys with the same sample/span/modality fields: a text run, a
// modality span); for one query row and one run the number of visible keys has
// a closed form -- the whole run if it is the row's own span, the keys up to
// the row's position (and inside its look-back window, if it has one for that
// modality) if the row looks back at that modality in its sample, else none --
// so every lane takes a few rows and walks the runs.  Exact for
// any layout; a tile whose keys all differ degenerates to one run per key.
//
// The same device code serves the attention kernels' private maps: there the q rows
// are a rank's local rows (positions looked up through its block list) and the
// last q-tile may be ragged.
#include "tilemap_body.h"

namespace mm {

__global__ void __launch_bounds__(kTmThreads)
tile_map_kernel(const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
                int64_t n_seq_blocks, int64_t n_rows, const TileMapJobs jobs) {
    tile_map_body(blockIdx.x, bits, blocks, block, n_seq_blocks, n_rows, jobs);
}

__global__ void __launch_bounds__(256)
row_pairs_kernel(const uint32_t* __restrict__ cnt, int32_t nk, uint64_t* __restrict__ rowpairs) {
    __shared__ uint64_t part[256];
    const int64_t i = blockIdx.x;
    uint64_t s = 0;
    for (int j = threadIdx.x; j < nk; j += 256) s += cnt[i * nk + j];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) rowpairs[i] = part[0];
}

int launch_tile_map(const uint64_t* d_bits, int64_t S, const int32_t* d_blocks, int32_t block,
                    int64_t n_rows, int32_t tq, int32_t tk, uint8_t* d_cls, uint32_t* d_cnt,
                    uint64_t* d_rowpairs, hipStream_t st) {
    if (n_rows <= 0) return MMATTN_OK;
    TileMapJobs jobs;
    jobs.j[0] = jobs.j[1] = tile_map_job(S, n_rows, tq, tk, d_cls, d_cnt);
    hipLaunchKernelGGL(tile_map_kernel, dim3(jobs.j[0].gx * jobs.j[0].gy), dim3(kTmThreads), 0, st, d_bits,
                       d_blocks, block, d_blocks ? S / block : (int64_t)0, n_rows, jobs);
    MM_LAUNCH_CHECK();
    if (d_rowpairs) {
        hipLaunchKernelGGL(row_pairs_kernel, dim3(jobs.j[0].gy), dim3(256), 0, st, d_cnt, jobs.j[0].nk,
                           d_rowpairs);
        MM_LAUNCH_CHECK();
    }
    return MMATTN_OK;
}

}  // namespace mm
