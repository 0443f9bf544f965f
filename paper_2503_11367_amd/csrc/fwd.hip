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
// through a ring of NST stages: the transfers of the next NST-1 tiles overlap the
// math of the current one and there is one workgroup barrier per tile.
// FULL tiles skip the predicate; PARTIAL tiles evaluate it per element from the
// 64-bit words (query word in registers, key words from LDS).
#include "attn_common.h"

namespace mm {

constexpr int kFwdBM = 128;     // query rows per q-tile
constexpr int kFwdBN = 64;      // keys per k-tile
// the running row max is only raised when it would grow by more than this many
// powers of two; until then probabilities are taken relative to the stale max
// (they stay below 2^kRescaleThreshold, harmless in fp32/bf16) and the
// accumulator rescale is skipped
constexpr float kRescaleThreshold = 8.0f;

template <int D, int NST>
struct FwdSmem {
    alignas(1024) unsigned char k[NST][kFwdBN * D * 2];   // rotated tiles, see SwzTile
    alignas(1024) unsigned char v[NST][kFwdBN * D * 2];
    uint32_t kss[kFwdBN];                                 // sample/span fields of a PARTIAL tile's keys
};

// HPW query heads per workgroup (4 wavefronts each), NST LDS stages.
template <int D, int HPW, int NST>
__global__ void __launch_bounds__(256 * HPW, 2)
fwd_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
           const ushort_t* __restrict__ V, const uint64_t* __restrict__ bits,
           const int32_t* __restrict__ blocks, int32_t block, int64_t n_loc, int64_t S,
           int32_t Hq, int32_t Hkv, float scale_log2, TilePlan plan,
           const int32_t* __restrict__ err, ushort_t* __restrict__ O, float* __restrict__ LSE) {
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
    if (*err) return;

    // ---- work decode: KV heads are pinned to XCDs (workgroups are dealt
    // round-robin to the 8 XCDs) so that one head's K/V stays in one L2 --------
    const int rep = Hq / Hkv;
    int tile_rank, h0;                    // h0: first of the HPW heads of this workgroup
    {
        const int bid = blockIdx.x;
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
    const int n_active = plan.kcount[qt];
    const uint32_t* klist = plan.klist + (int64_t)qt * plan.nk;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = h0 + wave / 4, w4 = wave & 3;
    const int li = lane & 31, hh = lane >> 5;

    // ---- this lane's query: row, position, mask fields, Q fragments ------------
    const int64_t row = (int64_t)qt * kFwdBM + w4 * 32 + li;
    const bool row_ok = row < n_loc;
    int64_t q_pos = 0;
    uint32_t q_ss = 0, q_causal = 0;
    bf16x8 qf[NDS];
    if (row_ok) {
        q_pos = row_pos(blocks, block, row);
        const uint64_t w = bits[q_pos];
        q_ss = word_ss(w);
        q_causal = word_causal(w);
        const ushort_t* qp = Q + (row * Hq + h) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
            qf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qp + ds * 16));
    } else {
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) qf[ds] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
    }

    floatx16 o[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // ---- tile transfers: which global chunk lands at this lane's LDS slot --------
    uint32_t gk[NI], gv[NI];              // byte offsets inside a tile of K / V
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int R = 4 * (wave * NI + i) + (lane >> 4), p = lane & 15;
        int r, c;
        KT::src_of(R, p, r, c);
        gk[i] = (uint32_t)(((r * Hkv + g) * D + c * 8) * 2);
        VT::src_of(R, p, r, c);
        gv[i] = (uint32_t)(((r * Hkv + g) * D + c * 8) * 2);
    }
    const uint32_t lds_k = lds_addr_of(sm.k[0]) + (wave * NI) * 1024;
    const uint32_t lds_v = lds_addr_of(sm.v[0]) + (wave * NI) * 1024;
    auto issue_tile = [&](uint32_t entry, int stage) {
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kFwdBN;
        const ushort_t* kt = K + k0 * Hkv * D;         // wave-uniform tile bases
        const ushort_t* vt = V + k0 * Hkv * D;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            dma16(kt, gk[i], lds_k + stage * kStageBytes + i * 1024);
            dma16(vt, gv[i], lds_v + stage * kStageBytes + i * 1024);
        }
    };

    // ---- LDS read offsets (bytes) ---------------------------------------------------
    int koff[NDS];                         // K fragment of row li, contraction step ds
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds) koff[ds] = KT::byte_of(li, 2 * ds + hh);
    // transpose read: inside a 16-lane group lane s fetches 4 elements of row
    // (s/4), columns 4*(s%4)..; the group ends up holding column (s) x 4 rows.
    const int s16 = lane & 15, grp = lane >> 4;
    int voff[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
        voff[db] = VT::byte_of(4 * hh + s16 / 4, 4 * db + 2 * (grp & 1) + ((s16 & 3) >> 1)) +
                   8 * (s16 & 1);

    // the k-tile list is fetched 64 entries at a time, one per lane, and read back
    // with readlane: no vector load inside the steady-state loop besides the tiles
    uint32_t list_chunk = lane < n_active ? klist[lane] : 0u;
    auto entry_at = [&](int it) -> uint32_t {
        return __builtin_amdgcn_readlane(list_chunk, it & 63);
    };

    // Every ordinary vector load issued so far (Q fragments, mask word, list chunk)
    // is awaited here, once: the compiler then has nothing pending when the loop
    // starts and inserts no waits of its own inside it (such a wait would also
    // drain the tile transfers, which it cannot see).
    wait_vmcnt<0>();

    // prologue: tiles 0 .. NST-2 in flight; pend[] holds their list entries
    uint32_t pend[NST - 1];
#pragma unroll
    for (int j = 0; j < NST - 1; ++j) {
        pend[j] = 0u;
        if (j < n_active) {
            pend[j] = entry_at(j);
            issue_tile(pend[j], j);
        }
    }

    int st = 0;                            // stage of tile `it`
    for (int it = 0; it < n_active; ++it) {
        const uint32_t entry = pend[0];
        const bool partial = (entry & kPartialFlag) != 0;
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kFwdBN;
        // tile `it` has landed once at most the transfers of the younger tiles remain
        const int younger = min(NST - 2, n_active - 1 - it);
        if (younger >= 2) wait_vmcnt<(NST > 3 ? 4 * NI : 0)>();
        else if (younger == 1) wait_vmcnt<(NST > 2 ? 2 * NI : 0)>();
        else wait_vmcnt<0>();
        __syncthreads();                   // everyone's share landed; stage of tile it-1 is free
        uint32_t fresh = 0u;
        if (it + NST - 1 < n_active) {
            if (((it + NST - 1) & 63) == 0) {
                // next 64 list entries (this vector load also drains the transfers in flight)
                const int j = it + NST - 1 + lane;
                list_chunk = j < n_active ? klist[j] : 0u;
                wait_vmcnt<0>();           // awaited here so that no wait is needed after the branch
            }
            fresh = entry_at(it + NST - 1);
            int sn = st + NST - 1;
            if (sn >= NST) sn -= NST;
            issue_tile(fresh, sn);
        }
#pragma unroll
        for (int j = 0; j + 1 < NST - 1; ++j) pend[j] = pend[j + 1];
        pend[NST - 2] = fresh;
        if (partial && tid < kFwdBN) sm.kss[tid] = word_ss(bits[k0 + tid]);
        const unsigned char* kb_base = sm.k[st];
        const unsigned char* vb_base = sm.v[st];

        // ---- S^T = K Q^T --------------------------------------------------------
        floatx16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *(const u32x4*)(kb_base + kb * 32 * RB + koff[ds]));
                s[kb] = mfma32(a, qf[ds], s[kb]);
            }
        }
        // ---- mask ----------------------------------------------------------------
        if (partial) {
            __syncthreads();               // key words of this tile are in LDS (workgroup-uniform branch)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kl = kb * 32 + c_row(r, hh);
                    if (!visible(q_ss, q_causal, q_pos, sm.kss[kl], k0 + kl)) s[kb][r] = -INFINITY;
                }
        }
        // ---- online softmax (base 2) ---------------------------------------------
        float m_loc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) m_loc = fmaxf(m_loc, s[kb][r]);
        m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32));
        const float m_cand = fmaxf(m_run, m_loc * scale_log2);
        // (-inf) - (-inf) is NaN and compares false: an all-masked prefix keeps -inf
        const float m_new = (m_cand - m_run > kRescaleThreshold) ? m_cand : m_run;
        if (__any(m_new != m_run)) {
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
            m_run = m_new;
        }
        const float m_use = m_run == -INFINITY ? 0.f : m_run;
        bf16x8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(s[kb][r] * scale_log2 - m_use);
                pf[kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
            }
        // row sums of the bf16-rounded probabilities (what the PV product sees)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bf16x2 pr = {pf[ks][2 * u], pf[ks][2 * u + 1]};
                l_run = __builtin_amdgcn_fdot2_f32_bf16(pr, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l_run, false);
            }
        // ---- O^T += V^T P^T --------------------------------------------------------
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                typedef short shortx4 __attribute__((ext_vector_type(4)));
                typedef shortx4 __attribute__((address_space(3))) * lds_s4;
                const unsigned char* p0 = vb_base + ks * 16 * RB + voff[db];
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)p0);
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(p0 + 8 * RB));
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                o[db] = mfma32(a, pf[ks], o[db]);
            }
        }
        if (++st == NST) st = 0;
    }

    // ---- epilogue -----------------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (row_ok) {
        ushort_t* op = O + (row * Hq + h) * (int64_t)D + 4 * hh;
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
}

// ---- host side ---------------------------------------------------------------------
struct FwdLayout {
    size_t err, clean_blocks, cls, kcount, klist, qorder, total;
    int32_t nq, nk;
};

static FwdLayout fwd_layout(int64_t S, int64_t n_loc, int32_t n_blocks) {
    FwdLayout L;
    L.nq = (int32_t)((n_loc + kFwdBM - 1) / kFwdBM);
    L.nk = (int32_t)(S / kFwdBN);
    size_t off = 0;
    L.err = off;          off += 256;
    L.clean_blocks = off; off += align_up((size_t)n_blocks * 4, 256);
    L.cls = off;          off += align_up((size_t)L.nq * L.nk, 256);
    L.kcount = off;       off += align_up((size_t)L.nq * 4, 256);
    L.klist = off;        off += align_up((size_t)L.nq * L.nk * 4, 256);
    L.qorder = off;       off += align_up((size_t)L.nq * 4, 256);
    L.total = off;
    return L;
}

size_t fwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D) {
    (void)Hq; (void)Hkv; (void)D;
    // n_blocks is not known here; n_loc/16 bounds it (block >= 16)
    return fwd_layout(S, n_loc, (int32_t)(n_loc / 16 + 1)).total;
}

template <int D, int HPW, int NST>
static void launch_fwd_kernel(const AttnArgs& a, int64_t n_loc, int32_t nq, float scale_log2,
                              const int32_t* clean, const TilePlan& plan, const int32_t* err, void* o,
                              float* lse, hipStream_t st) {
    const unsigned grid = (unsigned)((int64_t)nq * a.Hq / HPW);
    hipLaunchKernelGGL((fwd_kernel<D, HPW, NST>), dim3(grid), dim3(256 * HPW), 0, st,
                       (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v, a.bits, clean,
                       a.block, n_loc, a.S, a.Hq, a.Hkv, scale_log2, plan, err, (ushort_t*)o, lse);
}

int launch_fwd(const AttnArgs& a, void* o, float* lse, void* ws, hipStream_t st) {
    const int64_t n_loc = (int64_t)a.n_blocks * a.block;
    const FwdLayout L = fwd_layout(a.S, n_loc, (int32_t)(n_loc / 16 + 1));
    char* base = (char*)ws;
    int32_t* err = (int32_t*)(base + L.err);
    int32_t* clean = (int32_t*)(base + L.clean_blocks);
    TilePlan plan;
    plan.nq = L.nq; plan.nk = L.nk; plan.tq = kFwdBM; plan.tk = kFwdBN;
    plan.cls = (uint8_t*)(base + L.cls);
    plan.kcount = (int32_t*)(base + L.kcount);
    plan.klist = (uint32_t*)(base + L.klist);
    plan.qorder = (int32_t*)(base + L.qorder);

    int rc = launch_validate_blocks(a.blocks, a.n_blocks, a.S / a.block, clean, err, st);
    if (rc) return rc;
    rc = launch_tile_map(a.bits, a.S, clean, a.block, n_loc, kFwdBM, kFwdBN, plan.cls, nullptr,
                         nullptr, st);
    if (rc) return rc;
    rc = launch_compact_rows(plan, st);
    if (rc) return rc;

    const float scale_log2 = a.scale * kLog2e;
    const bool pair = (a.Hq / a.Hkv) % 2 == 0;     // two heads of a KV group per workgroup
    stage_begin(MMATTN_STAGE_FWD, st);
    if (a.D == 128) {
        if (pair) launch_fwd_kernel<128, 2, 3>(a, n_loc, L.nq, scale_log2, clean, plan, err, o, lse, st);
        else      launch_fwd_kernel<128, 1, 2>(a, n_loc, L.nq, scale_log2, clean, plan, err, o, lse, st);
    } else {
        if (pair) launch_fwd_kernel<64, 2, 3>(a, n_loc, L.nq, scale_log2, clean, plan, err, o, lse, st);
        else      launch_fwd_kernel<64, 1, 2>(a, n_loc, L.nq, scale_log2, clean, plan, err, o, lse, st);
    }
    stage_end(MMATTN_STAGE_FWD, st);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
