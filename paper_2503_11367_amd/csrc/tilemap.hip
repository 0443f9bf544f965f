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

// One launch serves up to two maps of the same rows (the second map's workgroups follow
// the first's in the one-dimensional grid).
// kpw: k-tiles per wavefront (each wavefront walks kpw consecutive k-tiles, so that on
// large maps the q-tile's words are staged once for 4*kpw tile pairs)
struct TileMapJob {
    int32_t tq, tk, nk, kpw;
    uint32_t gx, gy;                     // workgroups this map needs
    uint8_t* cls;
    uint32_t* cnt;
};
struct TileMapJobs { TileMapJob j[2]; };

__global__ void __launch_bounds__(kTmThreads)
tile_map_kernel(const uint64_t* __restrict__ bits, int64_t S,
                const int32_t* __restrict__ blocks, int32_t block, int64_t n_rows,
                const TileMapJobs jobs) {
    const uint32_t n_first = jobs.j[0].gx * jobs.j[0].gy;
    const bool second = blockIdx.x >= n_first;               // workgroup-uniform
    const TileMapJob& J = jobs.j[second ? 1 : 0];
    const uint32_t wg = blockIdx.x - (second ? n_first : 0u);
    const uint32_t wg_x = wg % J.gx, wg_y = wg / J.gx;       // k-tile group, q-tile
    const int32_t tq = J.tq, tk = J.tk, nk = J.nk, kpw = J.kpw;
    uint8_t* __restrict__ cls = J.cls;
    uint32_t* __restrict__ cnt = J.cnt;
    __shared__ uint32_t q_ss[kTmQChunk];
    __shared__ uint32_t q_att[kTmQChunk];
    __shared__ int64_t q_pos[kTmQChunk];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t i = wg_y;
    const int64_t r0 = i * tq;
    const int64_t rows = min((int64_t)tq, n_rows - r0);      // ragged last q-tile
    // words of the q rows c0 .. c0+n-1 of the tile into LDS (all threads; two barriers)
    auto stage_rows = [&](int64_t c0, int n) {
        __syncthreads();
        if ((int)threadIdx.x < n) {
            int64_t p = row_pos(blocks, block, r0 + c0 + threadIdx.x);
            uint64_t w = bits[p];
            q_pos[threadIdx.x] = p;
            q_ss[threadIdx.x] = word_ss(w);
            q_att[threadIdx.x] = word_att(w);
        }
        __syncthreads();
    };
    const bool single = rows <= kTmQChunk;                   // workgroup-uniform
    if (single) stage_rows(0, (int)rows);

    for (int jj = 0; jj < kpw; ++jj) {
        const int64_t j = ((int64_t)wg_x * kTmWaves + wave) * kpw + jj;
        const bool wave_active = j < nk;
        const int64_t k0 = j * tk;
        uint32_t part = 0;
        for (int64_t c0 = 0; c0 < rows; c0 += kTmQChunk) {
            const int n = (int)min((int64_t)kTmQChunk, rows - c0);
            if (!single) stage_rows(c0, n);
            if (!wave_active) continue;

            for (int kc = 0; kc < tk; kc += kWave) {
                // run starts among this chunk's keys: a key whose fields differ from its
                // predecessor's (the first key of the chunk always starts one)
                const int n_keys = min(kWave, tk - kc);
                const uint64_t wk = lane < n_keys ? bits[k0 + kc + lane] : 0;
                const uint32_t ss_k = word_ss(wk), mod_k = word_mod(wk);
                const uint32_t ss_p = __shfl_up(ss_k, 1), mod_p = __shfl_up(mod_k, 1);
                const bool starts = lane < n_keys && (lane == 0 || ss_k != ss_p || mod_k != mod_p);
                uint64_t m = __ballot(starts);
                while (m) {
                    const int a = __ffsll((unsigned long long)m) - 1;
                    m &= m - 1;
                    const int b = m ? __ffsll((unsigned long long)m) - 1 : n_keys;   // the run is keys a..b-1
                    const uint32_t ss_r = __shfl(ss_k, a), mod_r = __shfl(mod_k, a);
                    const int64_t first = k0 + kc + a;
                    const int64_t len = b - a;
                    for (int r = lane; r < n; r += kWave) {
                        const uint32_t ss_q = q_ss[r], att = q_att[r];
                        const bool same_span = (ss_q & 0xFFFFu) != 0 && ss_q == ss_r;
                        const bool back = (ss_q >> 16) == (ss_r >> 16) && ((att >> mod_r) & 1u);
                        // keys of the run at or before the row's position ...
                        const int64_t upto = max((int64_t)0, min(q_pos[r] - first + 1, len));
                        // ... minus those a look-back window over the row's own modality cuts off
                        const uint32_t win = att_window(att);
                        const bool windowed = win != 0 && mod_r == att_modality(att);
                        const int64_t cut = windowed ? max((int64_t)0, min(q_pos[r] - win + 1 - first, len)) : 0;
                        part += (uint32_t)(same_span ? len : (back ? upto - cut : 0));
                    }
                }
            }
        }
        const uint32_t total = wave_sum(part);
        if (wave_active && lane == 0) {
            const uint32_t full = (uint32_t)rows * (uint32_t)tk;
            if (cnt) cnt[i * nk + j] = total;
            if (cls)
                cls[i * nk + j] = total == 0 ? MMATTN_TILE_EMPTY
                                  : (total == full ? MMATTN_TILE_FULL : MMATTN_TILE_PARTIAL);
        }
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

static TileMapJob tile_map_job(int64_t S, int64_t n_rows, int32_t tq, int32_t tk, uint8_t* d_cls,
                               uint32_t* d_cnt) {
    const int64_t nq = (n_rows + tq - 1) / tq;
    const int32_t nk = (int32_t)(S / tk);
    // k-tiles per wavefront: one while the map has few tile pairs, up to 8 once there are
    // enough pairs for a thousand workgroups anyway
    const int64_t kpw64 = nq * nk / (kTmWaves * 1024);
    const int32_t kpw = (int32_t)std::max<int64_t>(1, std::min<int64_t>(8, kpw64));
    const int32_t per_wg = kTmWaves * kpw;
    return TileMapJob{tq, tk, nk, kpw, (uint32_t)((nk + per_wg - 1) / per_wg), (uint32_t)nq, d_cls, d_cnt};
}

int launch_tile_map(const uint64_t* d_bits, int64_t S, const int32_t* d_blocks, int32_t block,
                    int64_t n_rows, int32_t tq, int32_t tk, uint8_t* d_cls, uint32_t* d_cnt,
                    uint64_t* d_rowpairs, hipStream_t st) {
    if (n_rows <= 0) return MMATTN_OK;
    TileMapJobs jobs;
    jobs.j[0] = jobs.j[1] = tile_map_job(S, n_rows, tq, tk, d_cls, d_cnt);
    hipLaunchKernelGGL(tile_map_kernel, dim3(jobs.j[0].gx * jobs.j[0].gy), dim3(kTmThreads), 0, st, d_bits, S,
                       d_blocks, block, n_rows, jobs);
    MM_LAUNCH_CHECK();
    if (d_rowpairs) {
        hipLaunchKernelGGL(row_pairs_kernel, dim3(jobs.j[0].gy), dim3(256), 0, st, d_cnt, jobs.j[0].nk,
                           d_rowpairs);
        MM_LAUNCH_CHECK();
    }
    return MMATTN_OK;
}

// two class maps of the same rows (different tile shapes) in one launch
int launch_tile_maps(const uint64_t* d_bits, int64_t S, const int32_t* d_blocks, int32_t block,
                     int64_t n_rows, int32_t tq_a, int32_t tk_a, uint8_t* d_cls_a, int32_t tq_b,
                     int32_t tk_b, uint8_t* d_cls_b, hipStream_t st) {
    if (n_rows <= 0) return MMATTN_OK;
    TileMapJobs jobs;
    jobs.j[0] = tile_map_job(S, n_rows, tq_a, tk_a, d_cls_a, nullptr);
    jobs.j[1] = tile_map_job(S, n_rows, tq_b, tk_b, d_cls_b, nullptr);
    hipLaunchKernelGGL(tile_map_kernel, dim3(jobs.j[0].gx * jobs.j[0].gy + jobs.j[1].gx * jobs.j[1].gy),
                       dim3(kTmThreads), 0, st, d_bits, S, d_blocks, block, n_rows, jobs);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
