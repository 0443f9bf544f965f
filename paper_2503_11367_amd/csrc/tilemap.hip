// Tile map (paper section 3.2.1): for every (q-tile, k-tile) the number of
// unmasked (query,key) pairs and the class EMPTY / FULL / PARTIAL; a tile whose
// mask block is all zeros is the one the attention kernels skip.  Row sums give
// the per-block workloads W_b that Alg. 1 balances.
//
// Integer ALU work.  One wavefront per tile pair, four k-tiles per workgroup
// sharing the q-tile's words in LDS.  When both the q-tile and the k-tile are
// "uniform" (every token carries the same sample/span/modality/attend fields -- the
// common case inside a text run or a modality span) the count has a closed
// form in the tile coordinates; otherwise the wave evaluates the predicate for
// every pair.  Both paths are exact.
//
// The same kernel serves the attention kernels' private maps: there the q rows
// are a rank's local rows (positions looked up through its block list) and the
// last q-tile may be ragged.
#include "common.h"

namespace mm {

constexpr int kTmThreads = 256;
constexpr int kTmWaves = kTmThreads / kWave;
constexpr int kTmQChunk = 256;     // q rows staged in LDS at a time

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__global__ void __launch_bounds__(kTmThreads)
tile_map_kernel(const uint64_t* __restrict__ bits, int64_t S,
                const int32_t* __restrict__ blocks, int32_t block, int64_t n_rows,
                int32_t tq, int32_t tk, int32_t nk,
                uint8_t* __restrict__ cls, uint32_t* __restrict__ cnt) {
    __shared__ uint32_t q_ss[kTmQChunk];
    __shared__ uint32_t q_att[kTmQChunk];
    __shared__ int64_t q_pos[kTmQChunk];
    __shared__ int s_flags[4];      // [0] q uniform, [1] q positions contiguous

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t i = blockIdx.y;
    const int64_t j = (int64_t)blockIdx.x * kTmWaves + wave;
    const int64_t r0 = i * tq;
    const int64_t rows = min((int64_t)tq, n_rows - r0);      // ragged last q-tile
    const bool wave_active = j < nk;
    const int64_t k0 = j * tk;

    // key-side words of this wave's k-tile, tk/64 per lane, and their uniformity
    uint32_t k_first = 0, k_mod_first = 0;
    bool k_uniform = true;
    if (wave_active) {
        k_first = word_ss(bits[k0]);
        k_mod_first = word_mod(bits[k0]);
        bool same = true;
        for (int64_t k = k0 + lane; k < k0 + tk; k += kWave) {
            const uint64_t w = bits[k];
            same &= word_ss(w) == k_first && word_mod(w) == k_mod_first;
        }
        k_uniform = __all(same);
    }

    uint32_t total = 0;
    for (int64_t c0 = 0; c0 < rows; c0 += kTmQChunk) {
        const int n = (int)min((int64_t)kTmQChunk, rows - c0);
        __syncthreads();
        if ((int)threadIdx.x < n) {
            int64_t p = row_pos(blocks, block, r0 + c0 + threadIdx.x);
            uint64_t w = bits[p];
            q_pos[threadIdx.x] = p;
            q_ss[threadIdx.x] = word_ss(w);
            q_att[threadIdx.x] = word_att(w);
        }
        __syncthreads();
        // chunk-level uniformity of the q side (fields equal, positions contiguous)
        bool ok = true;
        if ((int)threadIdx.x < n)
            ok = q_ss[threadIdx.x] == q_ss[0] && q_att[threadIdx.x] == q_att[0] &&
                 q_pos[threadIdx.x] == q_pos[0] + threadIdx.x;
        const bool q_uniform = __syncthreads_and(ok);
        if (!wave_active) continue;

        if (q_uniform && k_uniform) {
            const uint32_t ss_q = q_ss[0], at_q = q_att[0];
            const bool same_span = (ss_q & 0xFFFFu) != 0 && ss_q == k_first;
            const bool back = (ss_q >> 16) == (k_first >> 16) && ((at_q >> k_mod_first) & 1u);
            if (same_span) {
                total += (uint32_t)n * (uint32_t)tk;
            } else if (back) {
                // pairs with k <= q:  sum_q clamp(q - k0 + 1, 0, tk)
                uint32_t part = 0;
                for (int r = lane; r < n; r += kWave) {
                    int64_t v = q_pos[0] + r - k0 + 1;
                    part += (uint32_t)max((int64_t)0, min(v, (int64_t)tk));
                }
                total += wave_sum(part);
            }
        } else {
            uint32_t part = 0;
            for (int64_t k = k0 + lane; k < k0 + tk; k += kWave) {
                const uint64_t wk = bits[k];
                const uint32_t ss_k = word_ss(wk), mod_k = word_mod(wk);
                for (int r = 0; r < n; ++r)
                    part += visible(q_ss[r], q_att[r], q_pos[r], ss_k, mod_k, k) ? 1u : 0u;
            }
            total += wave_sum(part);
        }
    }
    if (wave_active && lane == 0) {
        const uint32_t full = (uint32_t)rows * (uint32_t)tk;
        if (cnt) cnt[i * nk + j] = total;
        if (cls)
            cls[i * nk + j] = total == 0 ? MMATTN_TILE_EMPTY
                              : (total == full ? MMATTN_TILE_FULL : MMATTN_TILE_PARTIAL);
    }
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
    const int64_t nq = (n_rows + tq - 1) / tq;
    const int32_t nk = (int32_t)(S / tk);
    if (nq == 0) return MMATTN_OK;
    dim3 grid((unsigned)((nk + kTmWaves - 1) / kTmWaves), (unsigned)nq);
    hipLaunchKernelGGL(tile_map_kernel, grid, dim3(kTmThreads), 0, st, d_bits, S, d_blocks, block,
                       n_rows, tq, tk, nk, d_cls, d_cnt);
    MM_LAUNCH_CHECK();
    if (d_rowpairs) {
        hipLaunchKernelGGL(row_pairs_kernel, dim3((unsigned)nq), dim3(256), 0, st, d_cnt, nk,
                           d_rowpairs);
        MM_LAUNCH_CHECK();
    }
    return MMATTN_OK;
}

}  // namespace mm
