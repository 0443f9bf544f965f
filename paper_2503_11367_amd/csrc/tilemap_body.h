// Device bodies of the tile map (paper section 3.2.1) and of the block-list check, shared
// by the public tile-map kernel and by the first launch of the attention passes, where
// they run side by side with that pass's other independent preparation work.
#pragma once
#include <algorithm>
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

// Workgroup `wg_index` (of tile_map_workgroups(jobs)) of the map(s); kTmThreads threads.
// `blocks` may be a caller's unchecked list: an entry outside [0, n_seq_blocks) counts
// as block 0, exactly as validate_blocks_body rewrites it.
__device__ __forceinline__ void
tile_map_body(uint32_t wg_index, const uint64_t* __restrict__ bits,
              const int32_t* __restrict__ blocks, int32_t block, int64_t n_seq_blocks, int64_t n_rows,
              const TileMapJobs& jobs) {
    const uint32_t n_first = jobs.j[0].gx * jobs.j[0].gy;
    const bool second = wg_index >= n_first;                 // workgroup-uniform
    const TileMapJob& J = jobs.j[second ? 1 : 0];
    const uint32_t wg = wg_index - (second ? n_first : 0u);
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
            int64_t p = row_pos_checked(blocks, block, n_seq_blocks, r0 + c0 + threadIdx.x);
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

// ---- block list ------------------------------------------------------------
// One workgroup of 256 threads: clears the error flag block (kFlagInts int32 words), then
// copies the block list, replacing out-of-range entries by 0 and raising the flag.
constexpr int kFlagInts = 4;
__device__ __forceinline__ void
validate_blocks_body(const int32_t* __restrict__ blocks, int32_t n_blocks, int64_t n_seq_blocks,
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

inline TileMapJob tile_map_job(int64_t S, int64_t n_rows, int32_t tq, int32_t tk, uint8_t* d_cls,
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

inline uint32_t tile_map_workgroups(const TileMapJobs& jobs, int n_maps) {
    uint32_t n = jobs.j[0].gx * jobs.j[0].gy;
    if (n_maps > 1) n += jobs.j[1].gx * jobs.j[1].gy;
    return n;
}

}  // namespace mm
