// mmattn_fwd: multimodal-masked attention forward for one rank's query blocks
// against all keys/values (paper section 4.3: row-wise attention for local
// queries over the gathered K/V; section 4.2: mask evaluated from the per-token
// bitfield; section 3.2.1: all-zero mask blocks are skipped).
//
// Work item = (q-tile of 128 local rows, Q head); 4 wavefronts, each owning 32
// query rows.  For every active k-tile of 64 keys:
//   S^T = K Q^T   (MFMA 32x32x16 bf16; A = K fragment from LDS, B = Q
//                  fragment held in registers) -- computing the transpose puts
//                  one query per lane column, so the online-softmax row max /
//                  row sum are in-lane reductions plus one lane^32 exchange;
//   P^T -> bf16, fed straight back as the B operand of
//   O^T += V^T P^T (A = V fragment read from the row-major V tile with the LDS
//                  transpose read ds_read_b64_tr_b16).
// FULL tiles skip the predicate; PARTIAL tiles evaluate it per element from the
// 64-bit words (query word in registers, key words from LDS).
#include "attn_common.h"

namespace mm {

constexpr int kFwdBM = 128;     // query rows per workgroup
constexpr int kFwdBN = 64;      // keys per k-tile
constexpr int kFwdThreads = 256;

template <int D>
struct FwdSmem {
    static constexpr int KP = D + 8;      // K row pitch (elements): 16-lane b128 reads conflict-free
    static constexpr int VP = D + 32;     // V row pitch: 4 rows x 64 B of a transpose read hit distinct banks
    ushort_t k[kFwdBN * KP];
    ushort_t v[kFwdBN * VP];
    uint32_t kss[kFwdBN];                 // sample/span fields of the tile's keys
};

template <int D>
__global__ void __launch_bounds__(kFwdThreads, 2)
fwd_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
           const ushort_t* __restrict__ V, const uint64_t* __restrict__ bits,
           const int32_t* __restrict__ blocks, int32_t block, int64_t n_loc, int64_t S,
           int32_t Hq, int32_t Hkv, float scale_log2, TilePlan plan,
           const int32_t* __restrict__ err, ushort_t* __restrict__ O, float* __restrict__ LSE) {
    constexpr int NDS = D / 16;           // contraction steps over head_dim
    constexpr int NDB = D / 32;           // 32-wide output blocks over head_dim
    constexpr int KP = FwdSmem<D>::KP, VP = FwdSmem<D>::VP;
    __shared__ FwdSmem<D> sm;
    if (*err) return;

    // ---- work decode: KV heads are pinned to XCDs (workgroups are dealt
    // round-robin to the 8 XCDs) so that one head's K/V stays in one L2 --------
    const int rep = Hq / Hkv;
    int tile_rank, h;
    {
        const int bid = blockIdx.x;
        if (Hkv % 8 == 0) {
            const int x = bid & 7, slot = bid >> 3, hx = Hq / 8;
            tile_rank = slot / hx;
            const int e = slot - tile_rank * hx;
            const int kvh = x + 8 * (e / rep);
            h = kvh * rep + e % rep;
        } else {
            tile_rank = bid / Hq;
            h = bid - tile_rank * Hq;
        }
    }
    const int g = h / rep;
    const int qt = plan.qorder[tile_rank];
    const int n_active = plan.kcount[qt];
    const uint32_t* klist = plan.klist + (int64_t)qt * plan.nk;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, hh = lane >> 5;

    // ---- this lane's query: row, position, mask fields, Q fragments ------------
    const int64_t row = (int64_t)qt * kFwdBM + wave * 32 + li;
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

    // ---- global -> register staging of one K/V tile -----------------------------
    constexpr int CH = D / 8;                          // 16-byte chunks per row
    constexpr int NLD = kFwdBN * CH / kFwdThreads;     // chunks per thread per tensor
    u32x4 kreg[NLD], vreg[NLD];
    uint32_t kssreg = 0;
    auto load_tile = [&](int it) {
        const int64_t k0 = (int64_t)(klist[it] & ~kPartialFlag) * kFwdBN;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * kFwdThreads, r = c / CH, cc = c % CH;
            const int64_t off = ((k0 + r) * Hkv + g) * (int64_t)D + cc * 8;
            kreg[i] = *(const u32x4*)(K + off);
            vreg[i] = *(const u32x4*)(V + off);
        }
        if (tid < kFwdBN) kssreg = word_ss(bits[k0 + tid]);
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * kFwdThreads, r = c / CH, cc = c % CH;
            *(u32x4*)(sm.k + r * KP + cc * 8) = kreg[i];
            *(u32x4*)(sm.v + r * VP + cc * 8) = vreg[i];
        }
        if (tid < kFwdBN) sm.kss[tid] = kssreg;
    };

    // LDS read offsets (elements)
    const int k_off = li * KP + hh * 8;
    // transpose read: inside a 16-lane group lane s fetches 4 elements of row
    // (s/4), columns 4*(s%4)..; the group ends up holding column (s) x 4 rows.
    const int s16 = lane & 15, grp = lane >> 4;
    const int v_off = (4 * hh + s16 / 4) * VP + 16 * (grp & 1) + 4 * (s16 & 3);

    if (n_active > 0) load_tile(0);
    for (int it = 0; it < n_active; ++it) {
        const uint32_t entry = klist[it];
        const bool partial = (entry & kPartialFlag) != 0;
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kFwdBN;
        __syncthreads();
        store_tile();
        __syncthreads();
        if (it + 1 < n_active) load_tile(it + 1);

        // ---- S^T = K Q^T --------------------------------------------------------
        floatx16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *(const u32x4*)(sm.k + kb * 32 * KP + k_off + ds * 16));
                s[kb] = mfma32(a, qf[ds], s[kb]);
            }
        }
        // ---- mask ----------------------------------------------------------------
        if (partial) {
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
        const float m_new = fmaxf(m_run, m_loc * scale_log2);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        float l_add = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(s[kb][r] * scale_log2 - m_use);
                l_add += p;
                pf[kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
            }
        l_run = l_run * alpha + l_add;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        // ---- O^T += V^T P^T --------------------------------------------------------
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                typedef short shortx4 __attribute__((ext_vector_type(4)));
                typedef shortx4 __attribute__((address_space(3))) * lds_s4;
                const ushort_t* p0 = sm.v + v_off + (ks * 16) * VP + db * 32;
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)p0);
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(p0 + 8 * VP));
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                o[db] = mfma32(a, pf[ks], o[db]);
            }
        }
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
    const unsigned grid = (unsigned)((int64_t)L.nq * a.Hq);
    stage_begin(MMATTN_STAGE_FWD, st);
    if (a.D == 128)
        hipLaunchKernelGGL(fwd_kernel<128>, dim3(grid), dim3(kFwdThreads), 0, st,
                           (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v, a.bits,
                           clean, a.block, n_loc, a.S, a.Hq, a.Hkv, scale_log2, plan, err,
                           (ushort_t*)o, lse);
    else
        hipLaunchKernelGGL(fwd_kernel<64>, dim3(grid), dim3(kFwdThreads), 0, st,
                           (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v, a.bits,
                           clean, a.block, n_loc, a.S, a.Hq, a.Hkv, scale_log2, plan, err,
                           (ushort_t*)o, lse);
    stage_end(MMATTN_STAGE_FWD, st);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
