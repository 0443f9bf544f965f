// mmattn_fwd: multimodal-masked attention forward for one rank's query blocks
// against all keys/values (paper section 4.3: row-wise attention for local
// queries over the gathered K/V; section 4.2: mask evaluated from the per-token
// bitfield; section 3.2.1: all-zero mask blocks are skipped).
//
// Work item = (q-tile of 128 local rows, HPW query heads of one KV head); each
// head gets 4 wavefronts of 32 query rows, and all heads of the workgroup share
// the K/V tiles in LDS (grouped-query heads read the same keys under the same
// mask, so packing them halves the K/V traffic per flop).  For every active
// k-tile of 64 keys:
//   S^T = K Q^T   (MFMA 32x32x16 bf16; A = K fragment from LDS, B = Q
//                  fragment held in registers) -- computing the transpose puts
//                  one query per lane column, so the online-softmax row max /
//                  row sum are in-lane reductions plus one lane^32 exchange;
//   P^T -> bf16, fed straight back as the B operand of
//   O^T += V^T P^T (A = V fragment read from the row-major V tile with the LDS
//                  transpose read ds_read_b64_tr_b16).
// K/V tiles go HBM/L2 -> LDS directly (global_load_lds_dwordx4, no registers)
// through a ring of NST stages: the transfers of the next tiles overlap the
// math of the current one and there is one workgroup barrier per tile.
// The loop is a software pipeline over half tiles (32 keys): while the
// probabilities of one half tile are exponentiated and multiplied into O, the
// scores of the next one are already being formed.  Registers (about 230 per
// lane) and LDS (the ring) allow one workgroup of 8 wavefronts per CU, two
// wavefronts per SIMD, so latencies are covered inside the wave: operand
// fragments are requested four MFMAs ahead and the instruction order is pinned
// slot by slot (see `step`).
// FULL tiles skip the predicate; PARTIAL tiles evaluate it per element from the
// 64-bit words (query word in registers, key words from LDS).
#include <mutex>
#include <type_traits>
#include "attn_common.h"
#include "tilemap_body.h"

namespace mm {

constexpr int kFwdBM = 128;     // query rows per q-tile
constexpr int kFwdBN = 64;      // keys per k-tile
// how far (in powers of two) the running row maximum may drift from the shift that
// the probabilities are taken relative to before the shift follows it; inside
// this band probabilities stay within 2^+-kShiftSlack, harmless in fp32/bf16
constexpr float kShiftSlack = 64.0f;

// A bound on the scores of a wavefront's rows: |s| <= |q| |k| scale log2(e) (Cauchy-Schwarz)
// with the largest key norm of the KV head.  When it stays below kScoreBound for all 32
// rows, the probabilities 2^s are within 2^+-kScoreBound of 1 with the shift at 0, nothing
// can overflow or vanish, and the wavefront runs without tracking the running maximum at
// all (the results are those of the tracked path whenever that one would not have moved
// its shift).  2^kScoreBound times 2^30 keys still fits fp32.
constexpr float kScoreBound = 90.0f;
constexpr int kNormChunks = 64;     // partial maxima of the squared key norms per KV head

// Largest squared key norm of every KV head, as kNormChunks partial maxima per head (no
// atomics: the attention kernel takes the maximum of its head's partials).  One workgroup
// of 256 threads per (chunk, head of the launch); a chunk is S / kNormChunks consecutive keys.
template <int D>
__device__ __forceinline__ void
key_norm_body(int chunk, int g, const ushort_t* __restrict__ K, int64_t S, int32_t Hkv_s,
              float* __restrict__ knorm) {
    constexpr int TPK = D / 8;                            // threads per key, 8 elements each
    constexpr int KPP = 256 / TPK;                        // keys per pass
    __shared__ float wmax[4];
    const int64_t per = S / kNormChunks, k0 = chunk * per;
    const int sub = threadIdx.x % TPK, kk = threadIdx.x / TPK;
    float best = 0.f;
    for (int64_t k = kk; k < per; k += KPP) {
        const bf16x8 x = __builtin_bit_cast(bf16x8, *(const u32x4*)(K + ((k0 + k) * Hkv_s + g) * (int64_t)D + sub * 8));
        float a = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) a += (float)x[u] * (float)x[u];
#pragma unroll
        for (int off = TPK / 2; off > 0; off >>= 1) a += __shfl_xor(a, off);
        best = fmaxf(best, a);                            // a NaN norm is dropped here and caught by the row bound
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) best = fmaxf(best, __shfl_xor(best, off));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0)
        knorm[(int64_t)g * kNormChunks + chunk] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
}

// grid (kNormChunks, heads of the launch): the key norms alone, for a call whose plan is
// already in the workspace
template <int D>
__global__ void __launch_bounds__(256)
key_norm_kernel(const ushort_t* __restrict__ K, int64_t S, int32_t Hkv_s, float* __restrict__ knorm) {
    key_norm_body<D>((int)blockIdx.x, (int)blockIdx.y, K, S, Hkv_s, knorm);
}

// Everything the forward prepares that depends on nothing but the caller's inputs, in one
// launch: the workgroups of the tile map first, then one that checks the block list, then
// those of the key norms.  The tile map reads the caller's list with the same rule for bad
// entries as the check applies, so neither waits for the other.
struct FwdPrologue {
    TileMapJobs maps;
    uint32_t n_map_wgs;
    const uint64_t* bits;
    const int32_t* blocks;
    int32_t n_blocks, block;
    int64_t n_seq_blocks, n_rows;
    int32_t* clean;
    int32_t* err;
    const ushort_t* K;
    int64_t S;
    int32_t Hkv_s;
    float* knorm;
};
template <int D>
__global__ void __launch_bounds__(256)
fwd_prologue_kernel(const FwdPrologue p) {
    static_assert(kTmThreads == 256, "one workgroup shape for all three jobs");
    if (blockIdx.x < p.n_map_wgs) {
        tile_map_body(blockIdx.x, p.bits, p.blocks, p.block, p.n_seq_blocks, p.n_rows, p.maps);
    } else if (blockIdx.x == p.n_map_wgs) {
        validate_blocks_body(p.blocks, p.n_blocks, p.n_seq_blocks, p.clean, p.err);
    } else {
        const uint32_t w = blockIdx.x - p.n_map_wgs - 1u;
        key_norm_body<D>((int)(w % kNormChunks), (int)(w / kNormChunks), p.K, p.S, p.Hkv_s, p.knorm);
    }
}

template <int D, int NST>
struct FwdSmem {
    alignas(1024) unsigned char k[NST][kFwdBN * D * 2];   // rotated tiles, see SwzTile
    alignas(1024) unsigned char v[NST][kFwdBN * D * 2];
    alignas(256) uint64_t kw[NST][kFwdBN];                // mask words of a PARTIAL tile's keys, by ring stage
};

// HPW query heads per workgroup (4 wavefronts each), NST LDS stages; one workgroup per
// CU at D = 128 (LDS), so HPW wavefronts per SIMD.
template <int D, int HPW, int NST>
__global__ void __launch_bounds__(256 * HPW, HPW)
fwd_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
           const ushort_t* __restrict__ V, const uint64_t* __restrict__ bits,
           const int32_t* __restrict__ blocks, int32_t block, int64_t n_loc, int64_t S,
           int32_t Hq, int32_t Hkv, int32_t Hq_s, int32_t Hkv_s, float scale_log2, TilePlan plan,
           FwdSplit split, const int32_t* __restrict__ err, const float* __restrict__ knorm,
           ushort_t* __restrict__ O, float* __restrict__ LSE, float* __restrict__ Opart,
           float* __restrict__ MLpart) {
    // Hq, Hkv: heads this launch runs (a window of KV heads and their query heads, the
    // tensor pointers already advanced to its first head); Hq_s, Hkv_s: heads per token
    // in memory
    constexpr int NDS = D / 16;           // contraction steps over head_dim
    constexpr int NDB = D / 32;           // 32-wide output blocks over head_dim
    constexpr int NW = 4 * HPW;           // wavefronts per workgroup
    using KT = SwzTile<D, 1>;             // K: 16-byte row fragments
    using VT = SwzTile<D, 4>;             // V: transpose reads
    constexpr int RB = D * 2;
    constexpr int kStageBytes = kFwdBN * RB;
    constexpr int NI = kStageBytes / 1024 / NW;      // 1 KiB transfers per wave per tensor
    static_assert(NI >= 1, "tile too small for this many wavefronts");
    __shared__ FwdSmem<D, NST> sm;
    // The loads that find the work item form a chain (error flag, q-tile of this rank,
    // its list length, the list, the tiles); the independent ones are issued together and
    // the early exits are taken after the row's own loads have been issued, so that a
    // work item starts after three round trips instead of six.
    const int err_flag = *err;
    const int csz_dev = *plan.csz;

    // ---- work decode: KV heads are pinned to XCDs (workgroups are dealt
    // round-robin to the 8 XCDs) so that one head's K/V stays in one L2 --------
    const int rep = Hq / Hkv;
    int tile_rank, h0;                    // h0: first of the HPW heads of this workgroup
    const int items = gridDim.x / split.cmax;
    const int chunk = blockIdx.x / items; // which slice of the q-tile's k-tile list (0 when not split)
    {
        const int bid = blockIdx.x - chunk * items;
        if (Hkv % 8 == 0) {
            const int x = bid & 7, slot = bid >> 3, hx = Hq / 8 / HPW;
            tile_rank = slot / hx;
            const int e = (slot - tile_rank * hx) * HPW;
            h0 = (x + 8 * (e / rep)) * rep + e % rep;
        } else {
            const int hp = Hq / HPW;
            tile_rank = bid / hp;
            h0 = (bid - tile_rank * hp) * HPW;
        }
    }
    const int g = h0 / rep;
    const int qt = plan.qorder[tile_rank];
    if (err_flag) return;
    // this workgroup's slice of the active list: csz entries from chunk * csz on; the
    // length is the list builder's suggestion, but never below what the grid provides for
    const int kc_total = plan.kcount[qt];
    const int csz = max(csz_dev, split.csz);
    const uint32_t* klist = plan.klist + (int64_t)qt * plan.nk + chunk * csz;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = h0 + wave / 4, w4 = wave & 3;
    const int li = lane & 31, hh = lane >> 5;

    // ---- this lane's query: row, position, mask fields, Q fragments ------------
    const int64_t row = (int64_t)qt * kFwdBM + w4 * 32 + li;
    const bool row_ok = row < n_loc;
    int64_t q_pos = 0;
    uint32_t q_ss = 0, q_causal = 0;     // q_causal: the attend-set if the causal bit is set, else 0
    bf16x8 qf[NDS];
    if (row_ok) {
        q_pos = row_pos(blocks, block, row);
        const uint64_t w = bits[q_pos];
        q_ss = word_ss(w);
        q_causal = word_att(w);
        const ushort_t* qp = Q + (row * Hq_s + h) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
            qf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qp + ds * 16));
    } else {
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) qf[ds] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
    }

    // the k-tile list is fetched 64 entries at a time, one per lane, and read back
    // with readlane: no vector load inside the steady-state loop besides the tiles.
    // (Fetched before the list length is known: entries past it, inside the q-tile's row
    // of the list array, are read but never used.)
    uint32_t list_chunk = chunk * csz + lane < plan.nk ? klist[lane] : 0u;
    // this lane's partial maximum of the head's squared key norms (see kScoreBound)
    static_assert(kNormChunks == 64, "one partial maximum per lane");
    float kn2 = knorm[(int64_t)g * kNormChunks + lane];

    const int nchunk = max(1, (kc_total + csz - 1) / csz);
    if (chunk >= nchunk) return;          // workgroup-uniform
    const int n_active = max(0, min(kc_total - chunk * csz, csz));

    floatx16 o[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_run = 0.f, m_true = -INFINITY, l_run = 0.f;   // shift, running maximum (log2 units), row sum

    // ---- tile transfers: which global chunk lands at this lane's LDS slot --------
    uint32_t gk[NI], gv[NI];              // byte offsets inside a tile of K / V
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int R = 4 * (wave * NI + i) + (lane >> 4), p = lane & 15;
        int r, c;
        KT::src_of(R, p, r, c);
        gk[i] = (uint32_t)(((r * Hkv_s + g) * D + c * 8) * 2);
        VT::src_of(R, p, r, c);
        gv[i] = (uint32_t)(((r * Hkv_s + g) * D + c * 8) * 2);
    }
    const uint32_t lds_k = lds_addr_of(sm.k[0]) + (wave * NI) * 1024;
    const uint32_t lds_v = lds_addr_of(sm.v[0]) + (wave * NI) * 1024;
    const uint32_t lds_kw = lds_addr_of(sm.kw[0]);
    auto issue_tile = [&](uint32_t entry, int stage) {
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kFwdBN;
        const ushort_t* kt = K + k0 * Hkv_s * D;       // wave-uniform tile bases
        const ushort_t* vt = V + k0 * Hkv_s * D;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            dma16(kt, gk[i], lds_k + stage * kStageBytes + i * 1024);
            dma16(vt, gv[i], lds_v + stage * kStageBytes + i * 1024);
        }
        // the mask words of a PARTIAL tile's 64 keys travel with the tile (two 256-byte pieces,
        // the workgroup's first two wavefronts): no load that the workgroup has to wait for
        if ((entry & kPartialFlag) && wave < 2)
            dma4(bits + k0, (uint32_t)(wave * 256 + lane * 4), lds_kw + stage * (8 * kFwdBN) + wave * 256);
    };

    // ---- LDS read offsets (bytes) ---------------------------------------------------
    // (LDS byte addresses inside stage 0; stage, half tile and key-row offsets are
    // compile-time constants that end up in the instructions' offset fields)
    uint32_t kaddr[NDS];                   // K fragment of row li, contraction step ds
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds) kaddr[ds] = lds_addr_of(sm.k[0]) + KT::byte_of(li, 2 * ds + hh);
    // transpose read: inside a 16-lane group lane s fetches 4 elements of row
    // (s/4), columns 4*(s%4)..; the group ends up holding column (s) x 4 rows.
    const int s16 = lane & 15, grp = lane >> 4;
    uint32_t vaddr[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
        vaddr[db] = lds_addr_of(sm.v[0]) + VT::byte_of(4 * hh + s16 / 4, 4 * db + 2 * (grp & 1) + ((s16 & 3) >> 1)) +
                   8 * (s16 & 1);

    auto entry_at = [&](int it) -> uint32_t {
        return __builtin_amdgcn_readlane(list_chunk, it & 63);
    };

    // Every ordinary vector load issued so far (Q fragments, mask word, list chunk)
    // is awaited here, once: the compiler then has nothing pending when the loop
    // starts and inserts no waits of its own inside it (such a wait would also
    // drain the tile transfers, which it cannot see).
    wait_vmcnt<0>();

    // does this wavefront need the running maximum at all?
    bool tracked;
    {
        float qn2 = 0.f;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
#pragma unroll
            for (int u = 0; u < 8; ++u) qn2 += (float)qf[ds][u] * (float)qf[ds][u];
        qn2 += __shfl_xor(qn2, 32);                       // the row's other 64 head-dim values
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) kn2 = fmaxf(kn2, __shfl_xor(kn2, off));
        const float bound = __builtin_sqrtf(qn2 * kn2) * scale_log2 * 1.01f;
        tracked = !__all(bound <= kScoreBound);           // NaN or infinite norms take the tracked path
    }

    // ---- software pipeline over half tiles (32 keys) ---------------------------------
    // While the probabilities of one half tile are exponentiated and multiplied into
    // O, the scores of the next half tile are already being formed, so the matrix
    // and the vector pipes of a wave overlap.  Tiles j and j+1 are resident, up to
    // NST-2 more are in flight.  With two wavefronts per SIMD the LDS latency has to
    // be covered inside the wave: every operand fragment is requested NKF matrix
    // instructions before its use, and the order below is pinned slot by slot
    // (one MFMA, one fragment request, one slice of vector work per slot).
    static_assert(NST >= 3, "the pipeline needs two resident tiles and one in flight");
    constexpr int NKF = NDS / 2;           // fragments in flight; equals NDB
    static_assert(NKF == NDB, "slot plan assumes head_dim/32 fragments in flight");
    constexpr int EPS = 16 / NDS;          // probabilities formed per S slot
#define MM_SLOT_END() __builtin_amdgcn_sched_barrier(0)
    // `off`: byte offset of the half tile from stage 0 of its ring (compile-time once unrolled)
    auto read_k = [&](int off, int ds) __attribute__((always_inline)) -> bf16x8 {
        return __builtin_bit_cast(bf16x8, *(lds_u4)(uintptr_t)(kaddr[ds] + (uint32_t)off));
    };
    auto read_v = [&](int off, int ks, int db) __attribute__((always_inline)) -> bf16x8 {
        const uint32_t p0 = vaddr[db] + (uint32_t)(off + ks * 16 * RB);
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)p0);
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(p0 + 8 * RB));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // max over the two half-waves (lanes l and l^32 hold the same query)
    auto pair_max = [&](float x) __attribute__((always_inline)) -> float {
        // both copies go in equal; the swap leaves the lower half-wave's values in
        // one register and the upper half-wave's in the other, in all 64 lanes
        float a = x, b = x;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
        return fmaxf(a, b);
    };
    // raw scores of keys 32*kb .. +31 of the tile in `stage` (prologue only)
    auto scores = [&](int off, floatx16& s) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) s = mfma32(read_k(off, ds), qf[ds], s);
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] *= scale_log2;
    };
    // (the query-side parts of the predicate, window included, are per-lane constants here)
    // `kw_off`: byte offset of the tile's mask words in sm.kw (its ring stage)
    typedef const uint64_t __attribute__((address_space(3))) * lds_u8;
    auto mask_scores = [&](uint32_t entry, int kw_off, int kb, floatx16& s) __attribute__((always_inline)) {
        if (__builtin_expect((entry & kPartialFlag) != 0u, 0)) {   // workgroup-uniform; FULL tiles fall through
            const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kFwdBN;
            // Usually the 32 keys of the half tile are one run of equal mask fields: then every
            // row sees one contiguous range of them, found once per row, and an element costs a
            // subtraction and a comparison; wavefronts whose rows see all 32 keys do nothing.
            const uint64_t wk = *(lds_u8)(uintptr_t)(lds_kw + (uint32_t)(kw_off + (kb * 32 + li) * 8));
            const uint32_t ss_k = word_ss(wk), mod_k = word_mod(wk);
            const uint32_t ss0 = __builtin_amdgcn_readfirstlane(ss_k), mod0 = __builtin_amdgcn_readfirstlane(mod_k);
            if (__all(ss_k == ss0 && mod_k == mod0)) {       // wave-uniform
                const KeyRange r = visible_range(q_ss, q_causal, (int32_t)q_pos, ss0, mod0,
                                                 (int32_t)k0 + kb * 32, 32);
                if (!__all(r.all_of(32))) {
                    const uint32_t first = 4u * hh;          // key index of this lane's element (q4, j) = (0, 0)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (!r.sees(first + (uint32_t)(8 * q4 + j))) s[q4 * 4 + j] = -INFINITY;
                }
                return;
            }
            // element by element: the words of keys 8*q4 + 4*hh + 0..3 of the half tile, 32 bytes
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const uint32_t a = lds_kw + (uint32_t)(kw_off + (kb * 32 + 8 * q4 + 4 * hh) * 8);
                const u32x4 w01 = *(lds_u4)(uintptr_t)a, w23 = *(lds_u4)(uintptr_t)(a + 16);
                const uint64_t w4[4] = {w01[0] | ((uint64_t)w01[1] << 32), w01[2] | ((uint64_t)w01[3] << 32),
                                        w23[0] | ((uint64_t)w23[1] << 32), w23[2] | ((uint64_t)w23[3] << 32)};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int kl = kb * 32 + 8 * q4 + 4 * hh + j;
                    if (!visible(q_ss, q_causal, q_pos, word_ss(w4[j]), word_mod(w4[j]), k0 + kl)) s[q4 * 4 + j] = -INFINITY;
                }
                // four elements at a time: the comparison results live in scalar registers
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // Softmax is invariant under a per-query shift of the scores, so the shift m_run only
    // has to keep 2^(s - m_run) inside the fp32/bf16 exponent range.  It starts at 0 and
    // follows the true running maximum m_true only when the two drift more than
    // kShiftSlack apart: for ordinary score magnitudes it stays 0 and the probabilities
    // are plain exp2 of the scaled scores, with no per-element subtraction.
    // The scores of the half tile leave this function already shifted.
    auto new_max = [&](float m_loc, floatx16& s) __attribute__((always_inline)) {
        m_true = fmaxf(m_true, m_loc);
        // an all-masked prefix (m_true = -inf) keeps the shift
        const bool move = m_true != -INFINITY && fabsf(m_true - m_run) > kShiftSlack;
        if (__any(move)) {
            const float m_new = move ? m_true : m_run;
            // lowering by more than the exponent range only happens while O and l are still 0
            const float alpha = __builtin_amdgcn_exp2f(fminf(m_run - m_new, 126.f));
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
            m_run = m_new;
        }
        if (__any(m_run != 0.f)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] -= m_run;
        }
    };
    // One pipeline step.  kf[] holds the first NKF K fragments of the NEXT half tile
    // (at kn) on entry and those of the half tile after it (at kp) on exit.  The
    // step is a sequence of NDS + 2*NDB slots, each one MFMA, one fragment request
    // and an even share of the vector work: a wave cannot issue for some cycles after
    // an MFMA and the matrix pipe is busy for 32, so about four plain vector
    // instructions per slot are free and more stretch the slot.
    auto step = [&](auto TRACK_, int kn, floatx16& s_next, const floatx16& s_cur, int vb, int kp, bf16x8 (&kf)[NKF],
                    uint32_t e_next, int kw_next, int kb_next, bool live_next) __attribute__((always_inline)) {
        constexpr bool TRACK = decltype(TRACK_)::value;    // follow the running maximum (else the shift stays 0)
        constexpr int PPS = EPS / 2;       // probability pairs exponentiated per S slot
        constexpr int MPS = 16 / NDB;      // scores scaled per early / folded into the maximum per late PV slot
        constexpr int DPS = 8 / NDB;       // row-sum updates per late PV slot
        bf16x8 vf[NKF], pf0, pf1;
        float ef[16];                      // exp2 of the current scores
        uint32_t pw[8];                    // the same as bf16 pairs, in score-register order
        float m_loc = -INFINITY;
        // The empty asm statements tie each slice of vector work to its slot: without
        // them the compiler gathers the slices where their results are consumed.
        MM_SLOT_END();
#pragma unroll
        for (int t = 0; t < NDS + 2 * NDB; ++t) {
            // ---- matrix instruction and the fragment request that refills its operand ----
            if (t < NDS) {
                if (t == 0) {
                    floatx16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.f;
                    s_next = mfma32(kf[0], qf[0], z);
                } else {
                    s_next = mfma32(kf[t % NKF], qf[t], s_next);
                }
                if (t < NKF) kf[t] = read_k(kn, NKF + t);
                else vf[t - NKF] = read_v(vb, 0, t - NKF);
            } else if (t < NDS + NDB) {        // keys 0..15 of the half tile
                if (t == NDS) pf0 = __builtin_bit_cast(bf16x8, u32x4{pw[0], pw[1], pw[2], pw[3]});
                o[t - NDS] = mfma32(vf[t - NDS], pf0, o[t - NDS]);
                vf[t - NDS] = read_v(vb, 1, t - NDS);
            } else {                           // keys 16..31; next step's K fragments
                if (t == NDS + NDB) pf1 = __builtin_bit_cast(bf16x8, u32x4{pw[4], pw[5], pw[6], pw[7]});
                o[t - NDS - NDB] = mfma32(vf[t - NDS - NDB], pf1, o[t - NDS - NDB]);
                kf[t - NDS - NDB] = read_k(kp, t - NDS - NDB);
            }
            // ---- vector work ----
            if (t >= 1 && t <= NDS) {          // round the previous slot's exponentials to bf16
#pragma unroll
                for (int u = 0; u < PPS; ++u) {
                    const int pr = (t - 1) * PPS + u;
                    const bf16x2 pb = {(__bf16)ef[2 * pr], (__bf16)ef[2 * pr + 1]};
                    pw[pr] = __builtin_bit_cast(uint32_t, pb);
                    asm volatile("" : "+v"(pw[pr]));
                }
            }
            if (t < NDS) {
#pragma unroll
                for (int u = 0; u < EPS; ++u) {
                    const int r = t * EPS + u;
                    ef[r] = __builtin_amdgcn_exp2f(s_cur[r]);
                    asm volatile("" : "+v"(ef[r]));
                }
            } else if (t < NDS + NDB) {
                // the finished scores become exponents of 2
#pragma unroll
                for (int u = 0; u < MPS; ++u) {
                    const int r = (t - NDS) * MPS + u;
                    s_next[r] *= scale_log2;
                    asm volatile("" : "+v"(s_next[r]));
                }
            } else {
                // row sums of the bf16-rounded probabilities (what the PV product sees)
#pragma unroll
                for (int u = 0; u < DPS; ++u) {
                    const int pr = (t - NDS - NDB) * DPS + u;
                    l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[pr]),
                                                            bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l_run, false);
                }
                if (TRACK) {
#pragma unroll
                    for (int u = 0; u < MPS; ++u) m_loc = fmaxf(m_loc, s_next[(t - NDS - NDB) * MPS + u]);
                    asm volatile("" : "+v"(m_loc));
                }
                asm volatile("" : "+v"(l_run));
            }
            MM_SLOT_END();
            if (t == NDS + NDB - 1) mask_scores(e_next, kw_next, kb_next, s_next);
        }
        if (TRACK && live_next) new_max(pair_max(m_loc), s_next);   // past the last tile the scores are stale data
    };
    auto wait_landed = [&](int younger) __attribute__((always_inline)) {
        if (younger >= 2) wait_vmcnt<4 * NI>();
        else if (younger == 1) wait_vmcnt<2 * NI>();
        else wait_vmcnt<0>();
    };

    // the whole walk over the active tiles, once with and once without maximum tracking
    auto walk = [&](auto TRACK_) __attribute__((always_inline)) {
        constexpr bool TRACK = decltype(TRACK_)::value;
        uint32_t pend[NST - 1];                // list entries of tiles j .. j+NST-2
#pragma unroll
        for (int j = 0; j < NST - 1; ++j) {
            pend[j] = 0u;
            if (j < n_active) {
                pend[j] = entry_at(j);
                issue_tile(pend[j], j);
            }
        }
        floatx16 s_a, s_b;                     // scores of the current / next half tile, alternating
        bf16x8 kf[NKF];                        // leading K fragments of the next half tile
        if (n_active > 0) {
            wait_landed(min(NST - 2, n_active - 1));
            __syncthreads();
            scores(0, s_a);
            mask_scores(pend[0], 0, 0, s_a);
            if (TRACK) {
                float m_loc = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) m_loc = fmaxf(m_loc, s_a[r]);
                new_max(pair_max(m_loc), s_a);
            }
#pragma unroll
            for (int i = 0; i < NKF; ++i) kf[i] = read_k(32 * RB, i);
        }
        // The ring position of tile j is j mod NST; the loops are unrolled NST-fold so that
        // every stage index below is a compile-time constant.  STEADY: the tile NST-1 ahead
        // exists (so does tile j+1), and the number of transfers in flight is known.
        auto tile = [&](auto STEADY_, int j, int st) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(STEADY_)::value;
            constexpr int kHalf = 32 * RB;
            const int st1 = (st + 1) % NST, sn = (st + NST - 1) % NST;
            const bool more = STEADY || j + 1 < n_active;
            const bool ahead = STEADY || j + NST - 1 < n_active;
            // tile j+1 has landed once at most the transfers of the tiles after it remain
            if (STEADY) wait_landed(NST - 3);
            else wait_landed(max(0, min(NST - 3, n_active - 2 - j)));
            __syncthreads();               // everyone's share landed; stage of tile j-1 is free
            uint32_t fresh = 0u;
            if (ahead) {
                if (((j + NST - 1) & 63) == 0) {
                    // next 64 list entries (this vector load also drains the transfers in flight)
                    const int i = j + NST - 1 + lane;
                    list_chunk = i < n_active ? klist[i] : 0u;
                    wait_vmcnt<0>();       // awaited here so that no wait is needed after the branch
                }
                fresh = entry_at(j + NST - 1);
                // the two heads' wavefronts share the SIMDs pairwise and leave the barrier together:
                // the first head's issue their transfers now, the second head's after the first half
                // tile, so that each SIMD's matrix pipe is fed by one of the two meanwhile
                if (HPW == 1 || wave < 4) issue_tile(fresh, sn);
            }
            const uint32_t e_cur = pend[0], e_next = pend[1];
#pragma unroll
            for (int i = 0; i + 1 < NST - 1; ++i) pend[i] = pend[i + 1];
            pend[NST - 2] = fresh;
            // first half of tile j (scores in s_a) while the second half's scores form in s_b
            step(TRACK_, st * kStageBytes + kHalf, s_b, s_a, st * kStageBytes, st1 * kStageBytes, kf, e_cur, st * (8 * kFwdBN),
                 1, true);
            if (HPW > 1 && wave >= 4 && ahead) issue_tile(fresh, sn);
            // second half of tile j while the first half of tile j+1 forms in s_a (stale but
            // harmless data past the last tile)
            step(TRACK_, st1 * kStageBytes, s_a, s_b, st * kStageBytes + kHalf, st1 * kStageBytes + kHalf, kf,
                 more ? e_next : 0u, st1 * (8 * kFwdBN), 0, more);
        };
        int j0 = 0;
        for (; j0 + 2 * NST - 1 <= n_active; j0 += NST) {
#pragma unroll
            for (int st = 0; st < NST; ++st) tile(std::true_type{}, j0 + st, st);
        }
        for (; j0 < n_active; j0 += NST) {
#pragma unroll
            for (int st = 0; st < NST; ++st) {
                if (j0 + st >= n_active) break;
                tile(std::false_type{}, j0 + st, st);
            }
        }
    };
    if (tracked) walk(std::true_type{});
    else walk(std::false_type{});
#undef MM_SLOT_END
    // ---- epilogue -----------------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!row_ok) return;
    if (nchunk > 1) {
        // partial result of this slice: unnormalised O^T, the shift and the row sum
        const int64_t rows = (int64_t)plan.nq * kFwdBM;
        const int64_t pr = ((int64_t)chunk * rows + row) * Hq + h;
        float* op = Opart + pr * D + 4 * hh;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                floatx4 out;
#pragma unroll
                for (int u = 0; u < 4; ++u) out[u] = o[db][c * 4 + u];
                *(floatx4*)(op + db * 32 + c * 8) = out;
            }
        if (hh == 0) {
            MLpart[pr * 2] = m_run;
            MLpart[pr * 2 + 1] = l_tot;
        }
        return;
    }
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    ushort_t* op = O + (row * Hq_s + h) * (int64_t)D + 4 * hh;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            bf16x4 out;
#pragma unroll
            for (int u = 0; u < 4; ++u) out[u] = (__bf16)(o[db][c * 4 + u] * inv);
            *(u32x2*)(op + db * 32 + c * 8) = __builtin_bit_cast(u32x2, out);
        }
    if (hh == 0)
        LSE[(int64_t)h * n_loc + row] =
            l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
}

// Aggregation of the slices of split q-tiles (paper section 3.2.2: partial results of
// the sub-blocks are combined by one more kernel): with shift m_c, row sum l_c and
// unnormalised output o_c per slice, O = sum_c o_c 2^(m_c - m) / sum_c l_c 2^(m_c - m)
// for m = max m_c.  One thread per (row, head, 4 head-dim values).
__global__ void __launch_bounds__(256)
fwd_combine_kernel(TilePlan plan, FwdSplit split, int64_t n_loc, int32_t Hq, int32_t Hq_s, int32_t D,
                   const int32_t* __restrict__ err, const float* __restrict__ Opart,
                   const float* __restrict__ MLpart, ushort_t* __restrict__ O,
                   float* __restrict__ LSE) {
    if (*err) return;
    const int dq4 = D / 4;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t rh = gid / dq4;
    const int d0 = (int)(gid % dq4) * 4;
    const int64_t row = rh / Hq;
    const int h = (int)(rh % Hq);
    if (row >= n_loc) return;
    const int kc_total = plan.kcount[row / kFwdBM];
    const int csz = max(*plan.csz, split.csz);
    const int nchunk = max(1, (kc_total + csz - 1) / csz);
    if (nchunk == 1) return;              // written by the attention kernel itself
    const int64_t rows = (int64_t)plan.nq * kFwdBM;
    float m = -INFINITY;
    for (int c = 0; c < nchunk; ++c) {
        const float* ml = MLpart + (((int64_t)c * rows + row) * Hq + h) * 2;
        if (ml[1] > 0.f) m = fmaxf(m, ml[0]);
    }
    floatx4 num = {0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    for (int c = 0; c < nchunk; ++c) {
        const int64_t pr = ((int64_t)c * rows + row) * Hq + h;
        const float lc = MLpart[pr * 2 + 1];
        if (!(lc > 0.f)) continue;
        const float w = __builtin_amdgcn_exp2f(MLpart[pr * 2] - m);
        const floatx4 oc = *(const floatx4*)(Opart + pr * D + d0);
        num += oc * w;
        den += lc * w;
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
    bf16x4 out;
#pragma unroll
    for (int u = 0; u < 4; ++u) out[u] = (__bf16)(num[u] * inv);
    *(u32x2*)(O + (row * Hq_s + h) * (int64_t)D + d0) = __builtin_bit_cast(u32x2, out);
    if (d0 == 0)
        LSE[(int64_t)h * n_loc + row] = den > 0.f ? (m + __builtin_amdgcn_logf(den)) * kLn2 : -INFINITY;
}

// ---- host side ---------------------------------------------------------------------
// Workspace: the plan (independent of which heads run) first, then the partial
// results of split q-tile lists for `Hkv_run` KV heads run in one launch.
struct FwdLayout {
    size_t err, clean_blocks, cls, kcount, klist, qorder, knorm, opart, mlpart, total;
    int32_t nq, nk;
    FwdSplit split;
};

static FwdLayout fwd_layout(int64_t S, int64_t n_loc, int32_t n_blocks, int32_t Hq, int32_t Hkv,
                            int32_t D, int32_t Hkv_run) {
    FwdLayout L;
    const int32_t Hq_run = Hq / Hkv * Hkv_run;
    L.nq = (int32_t)((n_loc + kFwdBM - 1) / kFwdBM);
    L.nk = (int32_t)(S / kFwdBN);
    L.split = list_split(L.nq, L.nk, Hq_run / ((Hq / Hkv) % 2 == 0 ? 2 : 1));
    size_t off = 0;
    L.err = off;          off += 256;
    L.clean_blocks = off; off += align_up((size_t)n_blocks * 4, 256);
    L.cls = off;          off += align_up((size_t)L.nq * L.nk, 256);
    L.kcount = off;       off += align_up((size_t)L.nq * 4, 256);
    L.klist = off;        off += align_up((size_t)L.nq * L.nk * 4, 256);
    L.qorder = off;       off += align_up((size_t)L.nq * 4, 256);
    L.knorm = off;        off += align_up((size_t)Hkv * kNormChunks * 4, 256);
    const size_t prow = L.split.cmax > 1 ? (size_t)L.split.cmax * L.nq * kFwdBM * Hq_run : 0;
    L.opart = off;        off += align_up(prow * D * 4, 256);
    L.mlpart = off;       off += align_up(prow * 8, 256);
    L.total = off;
    return L;
}

size_t fwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D) {
    // n_blocks is not known here; n_loc/16 bounds it (block >= 16)
    return fwd_layout(S, n_loc, (int32_t)(n_loc / 16 + 1), Hq, Hkv, D, Hkv).total;
}

size_t fwd_heads_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D) {
    // any window of KV heads: fewer heads per launch split the lists further
    size_t most = 0;
    for (int32_t c = 1; c <= Hkv; ++c)
        most = std::max(most, fwd_layout(S, n_loc, (int32_t)(n_loc / 16 + 1), Hq, Hkv, D, c).total);
    return most;
}

template <int D, int HPW, int NST>
static void launch_fwd_kernel(const AttnArgs& a, int64_t n_loc, int32_t nq, float scale_log2,
                              const int32_t* clean, const TilePlan& plan, const FwdSplit& split,
                              const int32_t* err, const float* knorm, void* o, float* lse, float* opart,
                              float* mlpart, hipStream_t st) {
    const int32_t rep = a.Hq / a.Hkv, Hq_run = rep * a.kv_count;
    const int64_t qo = (int64_t)a.kv_begin * rep * a.D, ko = (int64_t)a.kv_begin * a.D;
    const unsigned grid = (unsigned)((int64_t)nq * Hq_run / HPW * split.cmax);
    hipLaunchKernelGGL((fwd_kernel<D, HPW, NST>), dim3(grid), dim3(256 * HPW), 0, st,
                       (const ushort_t*)a.q + qo, (const ushort_t*)a.k + ko, (const ushort_t*)a.v + ko,
                       a.bits, clean, a.block, n_loc, a.S, Hq_run, a.kv_count, a.Hq, a.Hkv, scale_log2,
                       plan, split, err, knorm, (ushort_t*)o + qo, lse + (int64_t)a.kv_begin * rep * n_loc,
                       opart, mlpart);
}

// ---- forward without a caller workspace ---------------------------------------------
// The scratch of mmattn_fwd_static: one array per GPU, part of the loaded code object, so
// that callers that may not allocate (graph capture, tight serving loops) need no workspace
// of their own.  In host code the array's name stands for the symbol only, not for device
// memory: its device address is looked up once per device and that pointer is what the
// kernels get.
static __device__ __align__(256) unsigned char scratch[MMATTN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

int launch_fwd_static(const AttnArgs& a, void* o, float* lse, hipStream_t st) {
    int dev = -1;
    MM_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MMATTN_ERR_UNSUPPORTED;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            MM_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) return MMATTN_ERR_HIP;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    // nothing in the scratch has to start at zero: every call rebuilds the status word, the
    // block list and the plan before reading them, and reads back only the partial results
    // its own workgroups wrote
    return launch_fwd(a, o, lse, ptr, st);
}

int launch_fwd(const AttnArgs& a, void* o, float* lse, void* ws, hipStream_t st) {
    const int64_t n_loc = (int64_t)a.n_blocks * a.block;
    const FwdLayout L = fwd_layout(a.S, n_loc, (int32_t)(n_loc / 16 + 1), a.Hq, a.Hkv, a.D, a.kv_count);
    float* opart = (float*)((char*)ws + L.opart);
    float* mlpart = (float*)((char*)ws + L.mlpart);
    char* base = (char*)ws;
    int32_t* err = (int32_t*)(base + L.err);
    int32_t* clean = (int32_t*)(base + L.clean_blocks);
    TilePlan plan;
    plan.nq = L.nq; plan.nk = L.nk; plan.tq = kFwdBM; plan.tk = kFwdBN;
    plan.cls = (uint8_t*)(base + L.cls);
    plan.kcount = (int32_t*)(base + L.kcount);
    plan.klist = (uint32_t*)(base + L.klist);
    plan.qorder = (int32_t*)(base + L.qorder);
    plan.csz = err + kFlagInts;
    plan.groups = a.Hq / a.Hkv * a.kv_count / (a.Hq / a.Hkv % 2 == 0 ? 2 : 1);

    const float scale_log2 = a.scale * kLog2e;
    const int32_t rep = a.Hq / a.Hkv;
    const bool pair = rep % 2 == 0;                // two heads of a KV group per workgroup
    // largest key norms of the window's heads (data, not plan: every call)
    float* knorm = (float*)(base + L.knorm) + (int64_t)a.kv_begin * kNormChunks;
    const ushort_t* kw = (const ushort_t*)a.k + (int64_t)a.kv_begin * a.D;
    if (!a.plan_ready) {
        FwdPrologue p;
        p.maps.j[0] = p.maps.j[1] = tile_map_job(a.S, n_loc, kFwdBM, kFwdBN, plan.cls, nullptr);
        p.n_map_wgs = tile_map_workgroups(p.maps, 1);
        p.bits = a.bits; p.blocks = a.blocks; p.n_blocks = a.n_blocks; p.block = a.block;
        p.n_seq_blocks = a.S / a.block; p.n_rows = n_loc;
        p.clean = clean; p.err = err;
        p.K = kw; p.S = a.S; p.Hkv_s = a.Hkv; p.knorm = knorm;
        const unsigned grid = p.n_map_wgs + 1u + (unsigned)(kNormChunks * a.kv_count);
        if (a.D == 128) hipLaunchKernelGGL(fwd_prologue_kernel<128>, dim3(grid), dim3(256), 0, st, p);
        else            hipLaunchKernelGGL(fwd_prologue_kernel<64>, dim3(grid), dim3(256), 0, st, p);
        MM_LAUNCH_CHECK();
        const int rc = launch_compact_rows(plan, st);
        if (rc) return rc;
    } else {
        if (a.D == 128)
            hipLaunchKernelGGL(key_norm_kernel<128>, dim3(kNormChunks, (unsigned)a.kv_count), dim3(256), 0, st, kw,
                               a.S, a.Hkv, knorm);
        else
            hipLaunchKernelGGL(key_norm_kernel<64>, dim3(kNormChunks, (unsigned)a.kv_count), dim3(256), 0, st, kw,
                               a.S, a.Hkv, knorm);
    }
    stage_begin(MMATTN_STAGE_FWD, st);
    if (a.D == 128) {
        if (pair) launch_fwd_kernel<128, 2, 4>(a, n_loc, L.nq, scale_log2, clean, plan, L.split, err, knorm, o, lse, opart, mlpart, st);
        else      launch_fwd_kernel<128, 1, 3>(a, n_loc, L.nq, scale_log2, clean, plan, L.split, err, knorm, o, lse, opart, mlpart, st);
    } else {
        if (pair) launch_fwd_kernel<64, 2, 4>(a, n_loc, L.nq, scale_log2, clean, plan, L.split, err, knorm, o, lse, opart, mlpart, st);
        else      launch_fwd_kernel<64, 1, 3>(a, n_loc, L.nq, scale_log2, clean, plan, L.split, err, knorm, o, lse, opart, mlpart, st);
    }
    if (L.split.cmax > 1) {
        const int32_t Hq_run = rep * a.kv_count;
        const int64_t threads = n_loc * Hq_run * (a.D / 4);
        hipLaunchKernelGGL(fwd_combine_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           plan, L.split, n_loc, Hq_run, a.Hq, a.D, err, opart, mlpart,
                           (ushort_t*)o + (int64_t)a.kv_begin * rep * a.D,
                           lse + (int64_t)a.kv_begin * rep * n_loc);
    }
    stage_end(MMATTN_STAGE_FWD, st);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
