// mmattn_bwd: backward of the multimodal-masked attention for one rank's query
// blocks (training needs it: the paper's iteration is one forward and one
// backward pass; the attention definition is the one section 3.2.2 / 4.3 rely
// on).  With P = exp(S - LSE), Delta = rowsum(dO o O), dS = P o (dP - Delta):
//   dV = P^T dO,  dK = scale dS^T Q   (sums over this rank's rows and over the
//                                      Hq/Hkv query heads of the KV head)
//   dQ = scale dS K
// Launches:
//   delta_kernel   Delta and LSE in base-2 units, padded to whole q-tiles;
//   dkv_kernel     key-outer: a workgroup owns 128 keys of one KV head (32 per
//                  wavefront), keeps dK^T/dV^T accumulators and its K fragments
//                  in registers, its V tile in LDS, and streams the active
//                  32-row query tiles of every head of the group through an LDS
//                  ring.  When there are too few (k-tile, KV head) units to fill
//                  the chip, a unit's step list is cut into chunks that run as
//                  separate workgroups (the intra-GPU balancing idea of paper
//                  section 3.2.2 applied to the key-outer pass); chunks of one
//                  unit add their fp32 partial sums atomically and a small
//                  kernel converts them to bf16;
//   dq_kernel      query-outer, same shape as the forward kernel.
// All contractions are 32x32x16 bf16 MFMAs.  Tiles go global -> LDS directly
// (no registers) into rotation-swizzled layouts; a tile that is needed both as
// row fragments and transposed is stored once (SwzTile MODE 0) and read with
// ds_read_b128 / ds_read_b64_tr_b16.
#include <type_traits>
#include "attn_common.h"

namespace mm {

// ---------------------------------------------------------------- delta ------
// One thread per 8 elements; D/8 consecutive lanes reduce one (row, head).
// Output ld[Hq][n_pad][2] = (LSE in base-2 units, Delta); rows n_loc .. n_pad-1 are
// padding: LSE = +inf (probability 0), Delta = 0.
template <int D>
__global__ void __launch_bounds__(256)
delta_kernel(const ushort_t* __restrict__ O, const ushort_t* __restrict__ dO,
             const float* __restrict__ lse, int64_t n_loc, int64_t n_pad, int32_t Hq,
             float* __restrict__ ld) {
    constexpr int TPR = D / 8;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t rh = gid / TPR;                       // row*Hq + h over padded rows
    const int c = (int)(gid % TPR);
    const int64_t row = rh / Hq;
    const int h = (int)(rh % Hq);
    float acc = 0.f;
    const bool in_pad = row < n_pad;
    const bool ok = row < n_loc;
    if (ok) {
        const int64_t e = (row * Hq + h) * (int64_t)D + c * 8;
        const bf16x8 x = __builtin_bit_cast(bf16x8, *(const u32x4*)(O + e));
        const bf16x8 y = __builtin_bit_cast(bf16x8, *(const u32x4*)(dO + e));
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (float)x[u] * (float)y[u];
    }
#pragma unroll
    for (int off = TPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (in_pad && c == 0) {           // ld[h][row] = (base-2 LSE, Delta)
        float* out = ld + ((int64_t)h * n_pad + row) * 2;
        out[0] = ok ? lse[(int64_t)h * n_loc + row] * kLog2e : INFINITY;
        out[1] = ok ? acc : 0.f;
    }
}

// 4-byte-per-lane variant of dma16 (lane l's dword lands at lds_addr + 4*l)
__device__ __forceinline__ void dma4(const void* base_uniform, uint32_t off, uint32_t lds_addr) {
    const uint64_t b = (uint64_t)base_uniform;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const uint64_t sb = ((uint64_t)hi << 32) | lo;
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(off), "s"(sb), "s"(lds_addr)
                 : "memory");
}

// ---------------------------------------------------------------- dK / dV ----
constexpr int kKvBN = 128;      // keys per workgroup
constexpr int kKvBM = 32;       // query rows per step
constexpr int kKvThreads = 256;
constexpr int kKvNST = 2;       // LDS ring stages for the Q/dO tiles
#ifndef MM_KV_OCC
#define MM_KV_OCC 2
#endif

template <int D>
struct KvSmem {
    alignas(1024) unsigned char v[kKvBN * D * 2];               // this workgroup's V rows (MODE 1)
    alignas(1024) unsigned char q[kKvNST][kKvBM * D * 2];       // MODE 0: rows and transpose
    alignas(1024) unsigned char d[kKvNST][kKvBM * D * 2];
    alignas(256) float ld[kKvNST][4][64];                       // per wave: (lse2, delta) of 32 rows
    uint32_t q_ss[kKvBM];                                       // mask fields of a PARTIAL step's rows
    uint32_t q_causal[kKvBM];
    int32_t q_pos[kKvBM];
};

struct KvChunking {
    int32_t cmax;        // chunks per (k-tile, KV head) unit at most
    int32_t len;         // steps per chunk
};

template <int D>
__global__ void __launch_bounds__(kKvThreads, MM_KV_OCC)
dkv_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
           const ushort_t* __restrict__ V, const ushort_t* __restrict__ dO,
           const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
           int64_t n_loc, int64_t n_pad, int64_t S, int32_t Hq, int32_t Hkv, float scale,
           float scale_log2, const float* __restrict__ ld_g,
           TilePlanT plan, KvChunking ch, const int32_t* __restrict__ err,
           ushort_t* __restrict__ dK, ushort_t* __restrict__ dV, float* __restrict__ accK,
           float* __restrict__ accV) {
    constexpr int NDS = D / 16, NDB = D / 32;
    constexpr int RB = D * 2;
    using QT = SwzTile<D, 0>;
    using VT = SwzTile<D, 1>;
    constexpr int NI = kKvBM * RB / 1024 / 4;          // 1 KiB transfers per wave per tensor per step
    constexpr int NIV = kKvBN * RB / 1024 / 4;         // same for the V tile
    constexpr int kStage = kKvBM * RB;
    __shared__ KvSmem<D> sm;
    if (*err) return;

    // ---- work decode: chunk index slowest, then k-tile rank (longest first), KV
    // heads pinned to XCDs ------------------------------------------------------
    const int rep = Hq / Hkv;
    int chunk, tile_rank, g;
    {
        const int units = plan.nk * Hkv;
        const int bid = blockIdx.x;
        chunk = bid / units;
        const int u = bid - chunk * units;
        if (Hkv % 8 == 0) {
            const int x = u & 7, slot = u >> 3, gx = Hkv / 8;
            tile_rank = slot / gx;
            g = x + 8 * (slot - tile_rank * gx);
        } else {
            tile_rank = u / Hkv;
            g = u - tile_rank * Hkv;
        }
    }
    const int kt = plan.korder[tile_rank];
    const int n_q = plan.qcount[kt];
    const int n_steps_all = n_q * rep;
    const int step0 = chunk * ch.len;
    if (step0 >= n_steps_all && chunk > 0) return;             // nothing for this chunk
    const int n_steps = max(0, min(ch.len, n_steps_all - step0));   // 0: chunk 0 writes zeros
    const bool shared_unit = n_steps_all > ch.len;             // several chunks: accumulate atomically
    const uint32_t* qlist = plan.qlist + (int64_t)kt * plan.nq;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, hh = lane >> 5;

    // this lane's key: position, mask fields, K fragments (B operand of S = Q K^T)
    const int64_t key = (int64_t)kt * kKvBN + wave * 32 + li;
    const uint32_t k_ss = word_ss(bits[key]);
    bf16x8 kf[NDS];
    {
        const int64_t off = (key * Hkv + g) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
            kf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(K + off + ds * 16));
    }
    floatx16 dk[NDB], dv[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk[db][r] = 0.f; dv[db][r] = 0.f; }

    // ---- transfers -------------------------------------------------------------------
    // V tile of the workgroup's 128 keys (once)
    {
        const ushort_t* vt = V + ((int64_t)kt * kKvBN * Hkv) * D;
#pragma unroll
        for (int i = 0; i < NIV; ++i) {
            const int R = 4 * (wave * NIV + i) + (lane >> 4), p = lane & 15;
            int r, c;
            VT::src_of(R, p, r, c);
            dma16(vt, (uint32_t)(((r * Hkv + g) * D + c * 8) * 2),
                  lds_addr_of(sm.v) + (wave * NIV + i) * 1024);
        }
    }
    // Q/dO tile of one step: (row, chunk) this lane fetches for each of its transfers
    int tr_row[NI], tr_chunk[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int R = 4 * (wave * NI + i) + (lane >> 4), p = lane & 15;
        QT::src_of(R, p, tr_row[i], tr_chunk[i]);
    }
    const uint32_t lds_q = lds_addr_of(sm.q[0]) + (wave * NI) * 1024;
    const uint32_t lds_d = lds_addr_of(sm.d[0]) + (wave * NI) * 1024;
    const uint32_t lds_ld = lds_addr_of(sm.ld[0][0]) + wave * 256;
    const int64_t row_stride = (int64_t)Hq * D;        // elements between consecutive local rows
    auto issue_step = [&](uint32_t entry, int hq, int stage) {
        const int64_t r0 = (int64_t)(entry & ~kPartialFlag) * kKvBM;
        const int64_t last = n_loc - 1 - r0;           // rows past the end re-read the last row
        const ushort_t* qb = Q + (r0 * Hq + hq) * (int64_t)D;
        const ushort_t* db_ = dO + (r0 * Hq + hq) * (int64_t)D;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int64_t rr = min((int64_t)tr_row[i], last);
            const uint32_t off = (uint32_t)((rr * row_stride + tr_chunk[i] * 8) * 2);
            dma16(qb, off, lds_q + stage * kStage + i * 1024);
            dma16(db_, off, lds_d + stage * kStage + i * 1024);
        }
        // (lse2, delta) pairs of the 32 rows: 256 contiguous bytes of the padded array
        dma4(ld_g + ((int64_t)hq * n_pad + r0) * 2, (uint32_t)(lane * 4), lds_ld + stage * (4 * 256));
    };

    // the step list is fetched 64 entries at a time, one per lane, and read back with
    // readlane; (head, list index) of the next step advance incrementally
    auto fetch_chunk = [&](int first_step) -> uint32_t {
        const int gs = step0 + first_step + lane;
        return gs < n_steps_all ? qlist[gs % n_q] : 0u;
    };
    uint32_t list_chunk = n_steps > 0 ? fetch_chunk(0) : 0u;
    int hq_next = g * rep + (n_q > 0 ? step0 / n_q : 0);       // head of the step to issue next
    int qi_next = n_q > 0 ? step0 % n_q : 0;                   // its index in the q list
    uint32_t entry = 0u;
    RowFragAddr<QT, D> qrow;      // Q and dO tiles share layout and lane pattern
    TrFragAddr<QT, D> qtr;
    RowFragAddr<VT, D> vrow;
    qrow.init(lane);
    qtr.init(lane);
    vrow.init(lane);
    const unsigned char* v_mine = sm.v + wave * 32 * RB;   // my 32 keys' rows (a multiple of the period)
    if (n_steps > 0) {
        entry = __builtin_amdgcn_readlane(list_chunk, 0);
        issue_step(entry, hq_next, 0);
        if (++qi_next == n_q) { qi_next = 0; ++hq_next; }
    }
    int st = 0;
    for (int step = 0; step < n_steps; ++step) {
        const bool partial = (entry & kPartialFlag) != 0;
        wait_vmcnt<0>();                    // this step's tiles (and, first time, V) have landed
        __syncthreads();
        uint32_t entry_next = 0u;
        if (step + 1 < n_steps) {
            if (((step + 1) & 63) == 0) list_chunk = fetch_chunk(step + 1);
            entry_next = __builtin_amdgcn_readlane(list_chunk, (step + 1) & 63);
            issue_step(entry_next, hq_next, st ^ 1);
            if (++qi_next == n_q) { qi_next = 0; ++hq_next; }
        }
        if (partial) {
            if (tid < kKvBM) {
                const int64_t r = min((int64_t)(entry & ~kPartialFlag) * kKvBM + tid, n_loc - 1);
                const int64_t p = row_pos(blocks, block, r);
                const uint64_t w = bits[p];
                sm.q_ss[tid] = word_ss(w);
                sm.q_causal[tid] = word_causal(w);
                sm.q_pos[tid] = (int32_t)p;
            }
            __syncthreads();
        }
        const unsigned char* qt = sm.q[st];
        const unsigned char* dt = sm.d[st];
        const float* ld = sm.ld[st][wave];

        // S = Q K^T and dP = dO V^T : rows = the step's 32 queries, columns = my 32 keys
        floatx16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
            s = mfma32(qrow.read(qt, 0, ds), kf[ds], s);
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
            dp = mfma32(qrow.read(dt, 0, ds), vrow.read(v_mine, 0, ds), dp);
        bf16x8 pf[2], dsf[2];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // rows 8c+4hh .. +3: (lse2, delta) pairs
            const floatx4 a4 = *(const floatx4*)(ld + 2 * (8 * c + 4 * hh));
            const floatx4 b4 = *(const floatx4*)(ld + 2 * (8 * c + 4 * hh) + 4);
            const float l_[4] = {a4[0], a4[2], b4[0], b4[2]};
            const float d_[4] = {a4[1], a4[3], b4[1], b4[3]};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = 4 * c + u;
                const int qr = 8 * c + 4 * hh + u;
                float p = __builtin_amdgcn_exp2f(s[r] * scale_log2 - l_[u]);
                if (partial && !visible(sm.q_ss[qr], sm.q_causal[qr], sm.q_pos[qr], k_ss, key)) p = 0.f;
                pf[r >> 3][r & 7] = (__bf16)p;
                dsf[r >> 3][r & 7] = (__bf16)(p * (dp[r] - d_[u]));
            }
        }
        // dV^T += dO^T P ;  dK^T += Q^T dS
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                dv[db] = mfma32(qtr.read(dt, ks, db), pf[ks], dv[db]);
                dk[db] = mfma32(qtr.read(qt, ks, db), dsf[ks], dk[db]);
            }
        st ^= 1;
        entry = entry_next;
    }
    wait_vmcnt<0>();                        // (no steps: the V transfer must still finish)

    // ---- epilogue: lane holds key `key`, 4 consecutive d per register quad ------------
    const int64_t obase = (key * Hkv + g) * (int64_t)D + 4 * hh;
    if (shared_unit) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t e = obase + db * 32 + (r >> 2) * 8 + (r & 3);
                unsafeAtomicAdd(accK + e, dk[db][r] * scale);
                unsafeAtomicAdd(accV + e, dv[db][r]);
            }
    } else {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                bf16x4 ok, ov;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    ok[u] = (__bf16)(dk[db][c * 4 + u] * scale);
                    ov[u] = (__bf16)dv[db][c * 4 + u];
                }
                *(u32x2*)(dK + obase + db * 32 + c * 8) = __builtin_bit_cast(u32x2, ok);
                *(u32x2*)(dV + obase + db * 32 + c * 8) = __builtin_bit_cast(u32x2, ov);
            }
    }
}

// zero (before) / convert to bf16 (after) the fp32 accumulators of the units whose
// step list was cut into several chunks; one workgroup per (k-tile, KV head)
template <bool FINISH>
__global__ void __launch_bounds__(256)
dkv_shared_units_kernel(TilePlanT plan, KvChunking ch, int32_t rep, int32_t Hkv, int32_t D,
                        const int32_t* __restrict__ err, float* __restrict__ accK,
                        float* __restrict__ accV, ushort_t* __restrict__ dK,
                        ushort_t* __restrict__ dV) {
    if (*err) return;
    const int kt = blockIdx.x, g = blockIdx.y;
    if (plan.qcount[kt] * rep <= ch.len) return;
    const int per_row = D / 4;                           // float4 per key row
    for (int i = threadIdx.x; i < kKvBN * per_row; i += 256) {
        const int r = i / per_row, c = i - r * per_row;
        const int64_t e = (((int64_t)kt * kKvBN + r) * Hkv + g) * (int64_t)D + c * 4;
        if (!FINISH) {
            *(floatx4*)(accK + e) = floatx4{0.f, 0.f, 0.f, 0.f};
            *(floatx4*)(accV + e) = floatx4{0.f, 0.f, 0.f, 0.f};
        } else {
            const floatx4 a = *(const floatx4*)(accK + e), b = *(const floatx4*)(accV + e);
            bf16x4 oa, ob;
#pragma unroll
            for (int u = 0; u < 4; ++u) { oa[u] = (__bf16)a[u]; ob[u] = (__bf16)b[u]; }
            *(u32x2*)(dK + e) = __builtin_bit_cast(u32x2, oa);
            *(u32x2*)(dV + e) = __builtin_bit_cast(u32x2, ob);
        }
    }
}

// ---------------------------------------------------------------- dQ ---------
constexpr int kDqBM = 128, kDqBN = 64;

template <int D, int NST>
struct DqSmem {
    alignas(1024) unsigned char k[NST][kDqBN * D * 2];    // MODE 0: rows (S^T) and transpose (dQ^T)
    alignas(1024) unsigned char v[NST][kDqBN * D * 2];    // same layout: rows (dP^T)
    uint32_t kss[kDqBN];
};

template <int D, int HPW, int NST>
__global__ void __launch_bounds__(256 * HPW, 2)
dq_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
          const ushort_t* __restrict__ V, const ushort_t* __restrict__ dO,
          const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
          int64_t n_loc, int64_t n_pad, int64_t S, int32_t Hq, int32_t Hkv, float scale,
          float scale_log2, const float* __restrict__ ld_g,
          TilePlan plan, const int32_t* __restrict__ err, ushort_t* __restrict__ dQ) {
    constexpr int NDS = D / 16, NDB = D / 32;
    constexpr int NW = 4 * HPW;
    constexpr int RB = D * 2;
    using KT = SwzTile<D, 0>;
    using VT = KT;                        // same layout: one set of row-fragment offsets serves both
    constexpr int kStageBytes = kDqBN * RB;
    constexpr int NI = kStageBytes / 1024 / NW;
    static_assert(NI >= 1, "tile too small for this many wavefronts");
    __shared__ DqSmem<D, NST> sm;
    if (*err) return;

    const int rep = Hq / Hkv;
    int tile_rank, h0;
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

    const int64_t row = (int64_t)qt * kDqBM + w4 * 32 + li;     // < n_pad
    const bool row_ok = row < n_loc;
    int64_t q_pos = 0;
    uint32_t q_ss = 0, q_causal = 0;
    const float my_lse2 = ld_g[((int64_t)h * n_pad + row) * 2];         // +inf on padding rows
    const float my_delta = ld_g[((int64_t)h * n_pad + row) * 2 + 1];
    bf16x8 qf[NDS], dof[NDS];
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds) {
        qf[ds] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
        dof[ds] = qf[ds];
    }
    if (row_ok) {
        q_pos = row_pos(blocks, block, row);
        const uint64_t w = bits[q_pos];
        q_ss = word_ss(w);
        q_causal = word_causal(w);
        const int64_t off = (row * Hq + h) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            qf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(Q + off + ds * 16));
            dof[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(dO + off + ds * 16));
        }
    }
    floatx16 dq[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.f;

    uint32_t gk[NI], gv[NI];
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
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kDqBN;
        const ushort_t* kt_ = K + k0 * Hkv * D;
        const ushort_t* vt_ = V + k0 * Hkv * D;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            dma16(kt_, gk[i], lds_k + stage * kStageBytes + i * 1024);
            dma16(vt_, gv[i], lds_v + stage * kStageBytes + i * 1024);
        }
    };

    RowFragAddr<KT, D> krow;
    TrFragAddr<KT, D> ktr;
    krow.init(lane);
    ktr.init(lane);

    uint32_t list_chunk = lane < n_active ? klist[lane] : 0u;
    auto entry_at = [&](int it) -> uint32_t {
        return __builtin_amdgcn_readlane(list_chunk, it & 63);
    };
    uint32_t pend[NST - 1];
#pragma unroll
    for (int j = 0; j < NST - 1; ++j) {
        pend[j] = 0u;
        if (j < n_active) {
            pend[j] = entry_at(j);
            issue_tile(pend[j], j);
        }
    }

    int st = 0;
    for (int it = 0; it < n_active; ++it) {
        const uint32_t entry = pend[0];
        const bool partial = (entry & kPartialFlag) != 0;
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kDqBN;
        const int younger = min(NST - 2, n_active - 1 - it);
        if (younger >= 2) wait_vmcnt<(NST > 3 ? 4 * NI : 0)>();
        else if (younger == 1) wait_vmcnt<(NST > 2 ? 2 * NI : 0)>();
        else wait_vmcnt<0>();
        __syncthreads();
        uint32_t fresh = 0u;
        if (it + NST - 1 < n_active) {
            if (((it + NST - 1) & 63) == 0) {
                const int j = it + NST - 1 + lane;
                list_chunk = j < n_active ? klist[j] : 0u;
            }
            fresh = entry_at(it + NST - 1);
            int sn = st + NST - 1;
            if (sn >= NST) sn -= NST;
            issue_tile(fresh, sn);
        }
#pragma unroll
        for (int j = 0; j + 1 < NST - 1; ++j) pend[j] = pend[j + 1];
        pend[NST - 2] = fresh;
        if (partial) {
            if (tid < kDqBN) sm.kss[tid] = word_ss(bits[k0 + tid]);
            __syncthreads();
        }
        const unsigned char* kb_base = sm.k[st];
        const unsigned char* vb_base = sm.v[st];

        bf16x8 dsf[4];
        auto half = [&](auto KB) __attribute__((always_inline)) {
            constexpr int kb = decltype(KB)::value;
            floatx16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds)
                s = mfma32(krow.read(kb_base, kb, ds), qf[ds], s);
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds)
                dp = mfma32(krow.read(vb_base, kb, ds), dof[ds], dp);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kl = kb * 32 + c_row(r, hh);
                float p = __builtin_amdgcn_exp2f(s[r] * scale_log2 - my_lse2);
                if (partial && !visible(q_ss, q_causal, q_pos, sm.kss[kl], k0 + kl)) p = 0.f;
                dsf[kb * 2 + (r >> 3)][r & 7] = (__bf16)(p * (dp[r] - my_delta));
            }
        };
        half(std::integral_constant<int, 0>{});
        half(std::integral_constant<int, 1>{});
        // dQ^T += K^T dS^T
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                dq[db] = mfma32(ktr.read(kb_base, ks, db), dsf[ks], dq[db]);
        if (++st == NST) st = 0;
    }

    if (row_ok) {
        ushort_t* op = dQ + (row * Hq + h) * (int64_t)D + 4 * hh;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                bf16x4 out;
#pragma unroll
                for (int u = 0; u < 4; ++u) out[u] = (__bf16)(dq[db][c * 4 + u] * scale);
                *(u32x2*)(op + db * 32 + c * 8) = __builtin_bit_cast(u32x2, out);
            }
    }
}

// ---------------------------------------------------------------- host -------
struct BwdLayout {
    size_t err, clean_blocks, ld, cls_a, kcount, klist, qorder, cls_b, qcount, qlist,
        korder, acc_k, acc_v, total;
    int32_t nq_a, nk_a, nq_b, nk_b;
    int64_t n_pad;
    KvChunking ch;
};

// Cut the step lists only when the (k-tile, KV head) units alone cannot fill the
// chip a few times over (512 resident workgroups).
static KvChunking kv_chunking(int32_t nk_b, int32_t nq_b, int32_t Hq, int32_t Hkv) {
    const int64_t units = (int64_t)nk_b * Hkv;
    const int64_t max_steps = (int64_t)nq_b * (Hq / Hkv);
    int64_t cmax = (2048 + units - 1) / units;
    if (cmax > 8) cmax = 8;
    if (cmax < 1) cmax = 1;
    int64_t len = (max_steps + cmax - 1) / cmax;
    if (len < 32) len = 32;
    cmax = (max_steps + len - 1) / len;
    if (cmax < 1) cmax = 1;
    return KvChunking{(int32_t)cmax, (int32_t)len};
}

static BwdLayout bwd_layout(int64_t S, int64_t n_loc, int32_t n_blocks, int32_t Hq, int32_t Hkv,
                            int32_t D) {
    BwdLayout L;
    L.nq_a = (int32_t)((n_loc + kDqBM - 1) / kDqBM);
    L.nk_a = (int32_t)(S / kDqBN);
    L.nq_b = (int32_t)((n_loc + kKvBM - 1) / kKvBM);
    L.nk_b = (int32_t)(S / kKvBN);
    L.n_pad = (int64_t)L.nq_a * kDqBM;
    L.ch = kv_chunking(L.nk_b, L.nq_b, Hq, Hkv);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    L.err = take(256);
    L.clean_blocks = take((size_t)n_blocks * 4);
    L.ld = take((size_t)Hq * L.n_pad * 8);
    L.cls_a = take((size_t)L.nq_a * L.nk_a);
    L.kcount = take((size_t)L.nq_a * 4);
    L.klist = take((size_t)L.nq_a * L.nk_a * 4);
    L.qorder = take((size_t)L.nq_a * 4);
    L.cls_b = take((size_t)L.nq_b * L.nk_b);
    L.qcount = take((size_t)L.nk_b * 4);
    L.qlist = take((size_t)L.nq_b * L.nk_b * 4);
    L.korder = take((size_t)L.nk_b * 4);
    const size_t acc = L.ch.cmax > 1 ? (size_t)S * Hkv * D * 4 : 0;
    L.acc_k = take(acc);
    L.acc_v = take(acc);
    L.total = off;
    return L;
}

size_t bwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D) {
    return bwd_layout(S, n_loc, (int32_t)(n_loc / 16 + 1), Hq, Hkv, D).total;
}

template <int D, int HPW, int NST>
static void launch_dq_kernel(const AttnArgs& a, const void* d_o, int64_t n_loc, const BwdLayout& L,
                             float scale_log2, const int32_t* clean, const float* ld,
                             const TilePlan& pa, const int32_t* err, void* dq,
                             hipStream_t st) {
    const unsigned grid = (unsigned)((int64_t)L.nq_a * a.Hq / HPW);
    hipLaunchKernelGGL((dq_kernel<D, HPW, NST>), dim3(grid), dim3(256 * HPW), 0, st,
                       (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v,
                       (const ushort_t*)d_o, a.bits, clean, a.block, n_loc, L.n_pad, a.S, a.Hq, a.Hkv,
                       a.scale, scale_log2, ld, pa, err, (ushort_t*)dq);
}

template <int D>
static int launch_bwd_d(const AttnArgs& a, const void* o, const float* lse, const void* d_o,
                        void* dq, void* dk, void* dv, void* ws, hipStream_t st) {
    const int64_t n_loc = (int64_t)a.n_blocks * a.block;
    const BwdLayout L = bwd_layout(a.S, n_loc, (int32_t)(n_loc / 16 + 1), a.Hq, a.Hkv, D);
    char* base = (char*)ws;
    int32_t* err = (int32_t*)(base + L.err);
    int32_t* clean = (int32_t*)(base + L.clean_blocks);
    float* ld = (float*)(base + L.ld);
    float* acc_k = (float*)(base + L.acc_k);
    float* acc_v = (float*)(base + L.acc_v);
    TilePlan pa;
    pa.nq = L.nq_a; pa.nk = L.nk_a; pa.tq = kDqBM; pa.tk = kDqBN;
    pa.cls = (uint8_t*)(base + L.cls_a);
    pa.kcount = (int32_t*)(base + L.kcount);
    pa.klist = (uint32_t*)(base + L.klist);
    pa.qorder = (int32_t*)(base + L.qorder);
    TilePlanT pb;
    pb.nq = L.nq_b; pb.nk = L.nk_b; pb.tq = kKvBM; pb.tk = kKvBN;
    pb.cls = (uint8_t*)(base + L.cls_b);
    pb.qcount = (int32_t*)(base + L.qcount);
    pb.qlist = (uint32_t*)(base + L.qlist);
    pb.korder = (int32_t*)(base + L.korder);

    int rc = launch_validate_blocks(a.blocks, a.n_blocks, a.S / a.block, clean, err, st);
    if (rc) return rc;
    rc = launch_tile_map(a.bits, a.S, clean, a.block, n_loc, kDqBM, kDqBN, pa.cls, nullptr, nullptr, st);
    if (rc) return rc;
    rc = launch_compact_rows(pa, st);
    if (rc) return rc;
    rc = launch_tile_map(a.bits, a.S, clean, a.block, n_loc, kKvBM, kKvBN, pb.cls, nullptr, nullptr, st);
    if (rc) return rc;
    rc = launch_compact_cols(pb, st);
    if (rc) return rc;

    const float scale_log2 = a.scale * kLog2e;
    {
        const int64_t threads = L.n_pad * a.Hq * (D / 8);
        hipLaunchKernelGGL(delta_kernel<D>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           (const ushort_t*)o, (const ushort_t*)d_o, lse, n_loc, L.n_pad, a.Hq, ld);
    }
    const int rep = a.Hq / a.Hkv;
    if (L.ch.cmax > 1)
        hipLaunchKernelGGL(dkv_shared_units_kernel<false>, dim3(L.nk_b, a.Hkv), dim3(256), 0, st, pb,
                           L.ch, rep, a.Hkv, D, err, acc_k, acc_v, (ushort_t*)dk, (ushort_t*)dv);
    stage_begin(MMATTN_STAGE_DKV, st);
    hipLaunchKernelGGL(dkv_kernel<D>, dim3((unsigned)((int64_t)L.nk_b * a.Hkv * L.ch.cmax)),
                       dim3(kKvThreads), 0, st, (const ushort_t*)a.q, (const ushort_t*)a.k,
                       (const ushort_t*)a.v, (const ushort_t*)d_o, a.bits, clean, a.block, n_loc,
                       L.n_pad, a.S, a.Hq, a.Hkv, a.scale, scale_log2, ld, pb, L.ch, err,
                       (ushort_t*)dk, (ushort_t*)dv, acc_k, acc_v);
    stage_end(MMATTN_STAGE_DKV, st);
    if (L.ch.cmax > 1)
        hipLaunchKernelGGL(dkv_shared_units_kernel<true>, dim3(L.nk_b, a.Hkv), dim3(256), 0, st, pb,
                           L.ch, rep, a.Hkv, D, err, acc_k, acc_v, (ushort_t*)dk, (ushort_t*)dv);
    const bool pair = rep % 2 == 0;
    stage_begin(MMATTN_STAGE_DQ, st);
    if (pair) launch_dq_kernel<D, 2, 3>(a, d_o, n_loc, L, scale_log2, clean, ld, pa, err, dq, st);
    else      launch_dq_kernel<D, 1, 2>(a, d_o, n_loc, L, scale_log2, clean, ld, pa, err, dq, st);
    stage_end(MMATTN_STAGE_DQ, st);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

int launch_bwd(const AttnArgs& a, const void* o, const float* lse, const void* d_o, void* dq,
               void* dk, void* dv, void* ws, hipStream_t st) {
    if (a.D == 128) return launch_bwd_d<128>(a, o, lse, d_o, dq, dk, dv, ws, st);
    return launch_bwd_d<64>(a, o, lse, d_o, dq, dk, dv, ws, st);
}

}  // namespace mm
