// mmattn_bwd: backward of the multimodal-masked attention for one rank's query
// blocks (training needs it: the paper's iteration is one forward and one
// backward pass; the attention definition is the one section 3.2.2 / 4.3 rely
// on).  With P = exp(S - LSE), Delta = rowsum(dO o O), dS = P o (dP - Delta):
//   dV = P^T dO,  dK = scale dS^T Q   (sums over this rank's rows and over the
//                                      Hq/Hkv query heads of the KV head)
//   dQ = scale dS K
// Launches:
//   bwd_prologue_kernel  the two tile maps and the check of the block list; for large
//                  shares also the inputs of the key-outer pass (see below);
//   dq_kernel      query-outer: a workgroup of four wavefronts owns 128 query rows of one
//                  head and walks the active 64-key tiles (two-stage K/V ring).  It forms
//                  Delta from the O and dO rows it holds.  On small shares it runs first and
//                  leaves the key-outer pass its inputs: head-major copies of Q and dO padded
//                  to whole q-tiles, -LSE/scale and -Delta per row, every row's mask inputs;
//                  on large shares it runs last;
//   dkv_kernel     key-outer: a workgroup owns 128 keys of one KV head and streams
//                  the active 64-row query tiles of its share of the group's heads
//                  through LDS rings; per 32-key block one wavefront forms P and
//                  accumulates dV^T, its partner takes P one step later and
//                  accumulates dK^T.  When there are too few (k-tile, KV head) units
//                  to fill the chip, a unit's heads are split over several workgroups
//                  (the intra-GPU balancing idea of paper section 3.2.2 applied to
//                  the key-outer pass: split the work of a block, write partial
//                  results, aggregate in one more launch), and a k-tile whose list of
//                  query tiles is far longer than the others' (keys that nearly every
//                  row attends) is cut into list slices, each a workgroup of its own;
//                  the partials are fp32, live in a pool of per-k-tile slots and are
//                  summed in a fixed order by dkv_reduce_kernel.
// All contractions are 32x32x16 bf16 MFMAs.  Tiles go global -> LDS directly
// (no registers) into rotation-swizzled layouts; a tile that is needed both as
// row fragments and transposed is stored once (SwzTile MODE 0) and read with
// ds_read_b128 / ds_read_b64_tr_b16.
#include <type_traits>
#include "attn_common.h"
#include "tilemap_body.h"
#include <hip/hip_ext.h>

namespace mm {

// ---------------------------------------------------------------- prep -------
// What the key-outer pass reads per row:
//   ldk[Hq][2][n_pad] = -LSE/scale, then -Delta with Delta = rowsum(dO o O) (padding rows
//                      n_loc .. n_pad-1: -inf, 0): the pass starts its S and dP accumulators
//                      from these
//   info[3][n_pad]     uint32: every local row's sample/span field, attend-set (0 without
//                      the causal bit) and sequence position (the mask inputs of the pass)
//   ld[Hq][2][n_pad]   (only when a preparation of its own writes all this) LSE in base-2
//                      units, then Delta, for the query-outer pass (padding rows: +inf, 0)
//   qh, doh [Hq][n_pad][D]  head-major copies of Q and dO (padding rows zero): there a tile
//                      is 64 consecutive rows of ONE head, which in the token-major layout
//                      are Hq*D*2 bytes apart -- a power-of-two stride that lands a whole
//                      tile stream on a few L2 sets (measured: half of all tile requests
//                      missed).
// Written by the query-outer pass on its way when that pass runs first (small shares, see
// launch_bwd_d), else by the workgroups below: one thread per 8 elements; D/8 consecutive
// lanes reduce one (row, head).  `blocks` is the caller's unchecked list (an entry outside
// [0, n_seq_blocks) counts as block 0, as in the checked copy the later kernels use).
struct BwdPrepArgs {
    const ushort_t *Q, *O, *dO;
    const float* lse;
    const uint64_t* bits;
    const int32_t* blocks;
    int32_t block, Hq;
    int64_t n_seq_blocks, n_loc, n_pad;
    float inv_scale;
    float *ld, *ldk;
    uint32_t* info;
    ushort_t *qh, *doh;
};
template <int D>
__device__ __forceinline__ void bwd_prep_body(int64_t wg, const BwdPrepArgs& p) {
    const ushort_t* __restrict__ Q = p.Q;
    const ushort_t* __restrict__ O = p.O;
    const ushort_t* __restrict__ dO = p.dO;
    const int64_t n_loc = p.n_loc, n_pad = p.n_pad;
    const int32_t Hq = p.Hq;
    ushort_t* __restrict__ qh = p.qh;
    ushort_t* __restrict__ doh = p.doh;
    constexpr int TPR = D / 8;
    const int64_t gid = wg * 256 + threadIdx.x;
    // head-major thread order: a workgroup writes 16 consecutive rows of one head's copies
    // (4 KiB contiguous) and reads 256-byte pieces of the token-major inputs; measured 7 us
    // faster on the 8k workload than contiguous reads with the writes scattered over the heads
    const int64_t rh = gid / TPR;                       // h*n_pad + row over padded rows
    const int c = (int)(gid % TPR);
    const int64_t row = rh % n_pad;
    const int h = (int)(rh / n_pad);
    float acc = 0.f;
    const bool in_pad = h < Hq;
    const bool ok = row < n_loc;
    u32x4 qv = {0u, 0u, 0u, 0u}, dv = {0u, 0u, 0u, 0u};
    if (ok) {
        const int64_t e = (row * Hq + h) * (int64_t)D + c * 8;
        qv = *(const u32x4*)(Q + e);
        dv = *(const u32x4*)(dO + e);
        const bf16x8 x = __builtin_bit_cast(bf16x8, *(const u32x4*)(O + e));
        const bf16x8 y = __builtin_bit_cast(bf16x8, dv);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (float)x[u] * (float)y[u];
    }
#pragma unroll
    for (int off = TPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (in_pad) {
        const int64_t e = ((int64_t)h * n_pad + row) * D + c * 8;
        *(u32x4*)(qh + e) = qv;
        *(u32x4*)(doh + e) = dv;
        if (c == 0) {
            const float l = ok ? p.lse[(int64_t)h * n_loc + row] : INFINITY;
            float* out = p.ld + (int64_t)h * 2 * n_pad + row;
            out[0] = l * kLog2e;
            out[n_pad] = ok ? acc : 0.f;
            float* outk = p.ldk + (int64_t)h * 2 * n_pad + row;
            outk[0] = -l * p.inv_scale;
            outk[n_pad] = ok ? -acc : 0.f;
            if (h == 0) {
                uint32_t ss = 0u, ca = 0u;
                int64_t pos = 0;
                if (ok) {
                    pos = row_pos_checked(p.blocks, p.block, p.n_seq_blocks, row);
                    const uint64_t w = p.bits[pos];
                    ss = word_ss(w);
                    ca = word_att(w);
                }
                p.info[row] = ss;
                p.info[n_pad + row] = ca;
                p.info[2 * n_pad + row] = (uint32_t)pos;
            }
        }
    }
}

// ---------------------------------------------------------------- prologue ---
// Everything the backward prepares that depends on nothing but the caller's inputs, in one
// launch: the workgroups of the two tile maps (query-outer for dQ, key-outer for dK/dV),
// then one that checks the block list, then (large shares only) those of the preparation
// above.  The tile maps read the caller's list with the same rule for bad entries as the
// check applies, so nothing in the launch waits for anything else.
struct BwdPrologue {
    TileMapJobs maps;
    uint32_t n_map_wgs;
    int32_t n_blocks;
    int32_t* clean;
    int32_t* err;
    BwdPrepArgs prep;
};
template <int D>
__global__ void __launch_bounds__(256)
bwd_prologue_kernel(const BwdPrologue p) {
    static_assert(kTmThreads == 256, "one workgroup shape for all three jobs");
    if (blockIdx.x < p.n_map_wgs) {
        tile_map_body(blockIdx.x, p.prep.bits, p.prep.blocks, p.prep.block, p.prep.n_seq_blocks,
                      p.prep.n_loc, p.maps);
    } else if (blockIdx.x == p.n_map_wgs) {
        validate_blocks_body(p.prep.blocks, p.n_blocks, p.prep.n_seq_blocks, p.clean, p.err);
    } else {
        bwd_prep_body<D>((int64_t)(blockIdx.x - p.n_map_wgs - 1u), p.prep);
    }
}

// ---------------------------------------------------------------- dK / dV ----
// Key-outer pass with role-specialised wavefronts.  A workgroup owns 128 keys of
// one KV head; for each 32-key block there is a "V wave" and a "K wave" (8
// wavefronts, the two of a block share a SIMD).  A step is 64 query rows of one
// head, handled as two units of 32 rows:
//   V wave, unit u:    S = Q K^T -> P = exp2(S - LSE) (masked) -> bf16;
//                      dV^T += dO^T P;   P goes to LDS for its partner;
//   K wave, one step later:  dP = dO V^T;  dS = P o (dP - Delta);  dK^T += Q^T dS.
// The K wave runs one step behind, so one workgroup barrier per step orders the
// P hand-over, and neither role needs both accumulators.  Inside a wave the units
// form a software pipeline like the forward kernel's: while the element-wise work
// of unit u runs, the first product of unit u+1 (S or dP) is already being formed,
// then the second product of unit u follows; operand fragments are requested a
// few MFMAs ahead and the instruction order is pinned slot by slot.
// Rings: Q tiles of steps i-1 (K wave), i, i+1 (V wave) are resident while
// i+2 lands: 4 stages, unrolled so that their LDS offsets are immediates; dO
// tiles of steps i-1, i are resident while i+1 lands: 3 stages, addressed
// through per-iteration base registers.
constexpr int kKvBN = 128;      // keys per workgroup
constexpr int kKvBM = 64;       // query rows per step
constexpr int kKvThreads = 512;
constexpr int kKvQst = 4;       // Q ring stages
constexpr int kKvDst = 3;       // dO ring stages

template <int D>
struct KvSmem {
    alignas(1024) unsigned char q[kKvQst][kKvBM * D * 2];       // MODE 0: rows and transpose
    alignas(1024) unsigned char d[kKvDst][kKvBM * D * 2];
    alignas(1024) unsigned char p[2][4][2 * 2 * 64 * 16];       // P hand-over: [step parity][key block][unit][half][lane] 16 B
    alignas(256) float ld[kKvQst][2][kKvBM];                    // lse2 and delta of a step's rows
    alignas(256) uint32_t info[kKvQst][3][kKvBM];               // sample/span field, causal flag, position of a step's rows
};

// A (k-tile, KV head) unit is processed by `cmax` workgroups, each taking `hpc`
// of the group's query heads (cmax * hpc = Hq/Hkv).
struct KvChunking {
    int32_t cmax;
    int32_t hpc;
};

template <int D>
__global__ void __launch_bounds__(kKvThreads, 2)
dkv_kernel(const ushort_t* __restrict__ Qh, const ushort_t* __restrict__ K,
           const ushort_t* __restrict__ V, const ushort_t* __restrict__ dOh,
           const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
           int64_t n_loc, int64_t n_pad, int64_t S, int32_t Hq, int32_t Hkv, float scale,
           float scale_log2, const uint32_t* __restrict__ info_g, const float* __restrict__ ldk_g,
           TilePlanT plan, KvChunking ch, const int32_t* __restrict__ err,
           ushort_t* __restrict__ dK, ushort_t* __restrict__ dV, float* __restrict__ pool) {
    constexpr int NDS = D / 16, NDB = D / 32;
    constexpr int RB = D * 2;
    using QT = SwzTile<D, 0>;
    constexpr int NI = kKvBM * RB / 1024 / 8;          // 1 KiB transfers per wave per tensor per step
    constexpr int kStage = kKvBM * RB;
    constexpr int kUnit = 32 * RB;                     // bytes of a unit's 32 rows
    static_assert(NI >= 1, "head_dim");
    constexpr int NKF = NDS / 2;                       // fragments in flight; equals NDB
    static_assert(NKF == NDB, "slot plan assumes head_dim/32 fragments in flight");
    constexpr int NS = NDS + 2 * NDB;                  // slots (MFMAs) per unit
    constexpr int SLV = NDS + NDB - 1;                 // slots that carry element-wise work
    constexpr int PER = 16 * QT::RPS, NV = PER / 8;    // transpose-read address period
    __shared__ KvSmem<D> sm;
    if (*err) return;

    // ---- work decode: chunk index slowest, then work item (longest first: the first
    // slices of the sliced lists, the other slices, the unsliced lists; then the unused
    // slice entries, which exit), KV heads pinned to XCDs ---------------------------
    const int rep = Hq / Hkv;
    int chunk, tile_rank, g;
    {
        const int units = (plan.nk + plan.n_extra) * Hkv;
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
    int kt, slice = 0;
    {
        const int sliced = plan.slicing[kSlicedTiles], used = plan.slicing[kExtraUsed];
        if (tile_rank < sliced) {
            kt = plan.korder[tile_rank];
        } else if (tile_rank < sliced + used) {
            kt = plan.extra[2 * (tile_rank - sliced)];
            slice = plan.extra[2 * (tile_rank - sliced) + 1];
        } else if (tile_rank < plan.nk + used) {
            kt = plan.korder[tile_rank - used];
        } else {
            return;                                    // workgroup-uniform
        }
    }
    const int slice_len = plan.slicing[kSliceLen];
    const int first = slice * slice_len;               // this workgroup's part of the k-tile's list
    const int n_q = max(0, min(slice_len, plan.qcount[kt] - first));
    const int slot0 = plan.pbase[kt];
    const bool shared_unit = slot0 >= 0;               // several workgroups per unit: fp32 partials, summed later
    const int n_steps = n_q * ch.hpc;                  // 0 (no query sees these keys): writes zeros
    const int head0 = g * rep + chunk * ch.hpc;        // first query head of this workgroup
    const uint32_t* qlist = plan.qlist + (int64_t)kt * plan.nq + first;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool k_role = wave >= 4;                     // waves 0-3: V role, 4-7: K role
    const int kblk = wave & 3;                         // 32-key block of this wave
    const int li = lane & 31, hh = lane >> 5;

    // this lane's key; the role's resident operand (B operand, 8 head-dim values per step):
    // V role keeps K (for S = Q K^T), K role keeps V (for dP = dO V^T)
    const int64_t key = (int64_t)kt * kKvBN + kblk * 32 + li;
    const uint32_t k_ss = word_ss(bits[key]), k_mod = word_mod(bits[key]);
    bf16x8 res[NDS];
    {
        const ushort_t* src = k_role ? V : K;
        const int64_t off = (key * Hkv + g) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
            res[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(src + off + ds * 16));
    }
    floatx16 acc[NDB];                                 // dV^T (V role) or dK^T (K role)
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    // ---- transfers (all 8 wavefronts share every tile) ------------------------------
    uint32_t tr_off[NI];                               // byte offset inside a (head-major) tile this lane fetches
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        int r, c;
        QT::src_of(4 * (wave * NI + i) + (lane >> 4), lane & 15, r, c);
        tr_off[i] = (uint32_t)((r * D + c * 8) * 2);
    }
    const uint32_t lds_q = lds_addr_of(sm.q[0]) + (wave * NI) * 1024;
    const uint32_t lds_d = lds_addr_of(sm.d[0]) + (wave * NI) * 1024;
    const uint32_t lds_ld = lds_addr_of(sm.ld[0][0]);
    const uint32_t lds_info = lds_addr_of(sm.info[0][0]);
    // Tile addresses are kept as running pointers (the head's base advances by one head
    // stride when the walk reaches the next head), so that issuing a step's transfers costs
    // a shift and an add per tensor: a wave issues one instruction every four cycles, and
    // what it spends on address arithmetic here the matrix pipe of its SIMD spends idle.
    const int64_t head_stride = n_pad * D;                      // elements per head of Qh / dOh
    const ushort_t* qh_next = Qh + (int64_t)head0 * head_stride;     // head of the next Q tile to issue
    const ushort_t* doh_next = dOh + (int64_t)head0 * head_stride;
    // the rows' constants and mask inputs travel with the Q tile, one 256-byte piece per wave:
    // wave 0: -LSE rows, wave 1: -Delta rows (per head), waves 2-4: the rows' mask inputs
    const float* row_next = wave < 2 ? ldk_g + ((int64_t)head0 * 2 + wave) * n_pad
                                     : (const float*)(info_g + (int64_t)(wave - 2) * n_pad);
    const int64_t row_stride = wave < 2 ? 2 * n_pad : 0;
    const uint32_t row_lds = wave < 2 ? lds_ld + wave * (4 * kKvBM) : lds_info + (wave - 2) * (4 * kKvBM);
    const uint32_t row_lds_stage = wave < 2 ? 8 * kKvBM : 12 * kKvBM;
    auto issue_q = [&](uint32_t entry, int stage) {             // Q tile and the rows' constants / mask inputs
        const int64_t r0 = (int64_t)(entry & ~kPartialFlag) * kKvBM;   // 64 consecutive rows, padded with zeros
        const ushort_t* tile = qh_next + r0 * D;
#pragma unroll
        for (int i = 0; i < NI; ++i) dma16(tile, tr_off[i], lds_q + stage * kStage + i * 1024);
        if (wave < 5) dma4(row_next + r0, (uint32_t)(lane * 4), row_lds + stage * row_lds_stage);
    };
    auto next_head = [&]() {
        qh_next += head_stride;
        doh_next += head_stride;
        row_next += row_stride;
    };
    auto issue_d = [&](uint32_t entry, const ushort_t* head_base, int stage) {
        const ushort_t* tile = head_base + (int64_t)(entry & ~kPartialFlag) * (kKvBM * D);
#pragma unroll
        for (int i = 0; i < NI; ++i) dma16(tile, tr_off[i], lds_d + stage * kStage + i * 1024);
    };

    // Step s is query tile qlist[n_q-1 - s%n_q] of head head0 + s/n_q: every k-tile
    // of a head walks the query tiles from the last one down, so the workgroups
    // that are resident together read the same Q/dO tiles at about the same time
    // and share them in L2.  The list is fetched 64 entries at a time, one per lane,
    // and read back with readlane.
    auto fetch_chunk = [&](int first_step) -> uint32_t {
        const int s_ = first_step + lane;
        return s_ < n_steps ? qlist[n_q - 1 - s_ % n_q] : 0u;
    };
    uint32_t list_chunk = n_steps > 0 ? fetch_chunk(0) : 0u;
    int qi_next = 0;                                   // position in the walk of the step whose Q tile is issued next

    // ---- fragment addresses (LDS byte addresses at ring stage 0) ---------------------
    // row fragments feed the first product (V role: Q ring, K role: dO ring), transpose
    // fragments the second (V role: dO ring, K role: Q ring)
    uint32_t row_addr[NDS], tr_addr[NDB][NV];
    {
        RowFragAddr<QT, D> fr;
        TrFragAddr<QT, D> ft;
        fr.init(lane);
        ft.init(lane);
        const uint32_t rbase = lds_addr_of(k_role ? sm.d[0] : sm.q[0]);
        const uint32_t tbase = lds_addr_of(k_role ? sm.q[0] : sm.d[0]);
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) row_addr[ds] = rbase + (uint32_t)fr.off[ds];
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < NV; ++v) tr_addr[db][v] = tbase + (uint32_t)ft.off[db][v];
    }
    // P hand-over slot of this lane, and the row constants (4 consecutive rows per 16-byte
    // read: lse2 for the V role, delta for the K role)
    const uint32_t p_addr = lds_addr_of(sm.p[0][kblk]) + lane * 16;
    const uint32_t rc_addr = lds_ld + (k_role ? 4 * kKvBM : 0) + hh * 16;

    auto read_row = [&](uint32_t a, int imm) __attribute__((always_inline)) -> bf16x8 {
        return __builtin_bit_cast(bf16x8, *(lds_u4)(uintptr_t)(a + (uint32_t)imm));
    };
    // transpose fragment of rows ks*16.. (ks counted inside the 64-row tile), columns db*32..
    auto read_tr = [&](const uint32_t (&a)[NDB][NV], int imm, int ks, int db) __attribute__((always_inline)) -> bf16x8 {
        const int r_lo = ks * 16, r_hi = ks * 16 + 8;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(
            a[db][(r_lo % PER) / 8] + (uint32_t)(imm + (r_lo / PER) * PER * RB)));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(
            a[db][(r_hi % PER) / 8] + (uint32_t)(imm + (r_hi / PER) * PER * RB)));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // Every ordinary vector load issued so far (resident fragments, mask word, list
    // chunk) is awaited here, once: the compiler then has nothing pending when the
    // loop starts and inserts no waits of its own inside it (such a wait would also
    // drain the tile transfers, which it cannot see).
    wait_vmcnt<0>();

    // prologue: Q tiles of steps 0 and 1 and the dO tile of step 0; ent[] holds the
    // list entries of steps i, i+1, i+2 and hq_d the head of the next dO tile
    uint32_t ent[3] = {0u, 0u, 0u};
    const ushort_t *doh_d = doh_next, *doh_d1 = doh_next;     // dO heads of steps i+1 and i+2 (dO is issued one step after Q)
    if (n_steps > 0) {
        ent[0] = __builtin_amdgcn_readlane(list_chunk, 0);
        issue_q(ent[0], 0);
        issue_d(ent[0], doh_next, 0);
        if (++qi_next == n_q) { qi_next = 0; next_head(); }
        doh_d = doh_next;
        if (n_steps > 1) {
            ent[1] = __builtin_amdgcn_readlane(list_chunk, 1);
            issue_q(ent[1], 1);
            if (++qi_next == n_q) { qi_next = 0; next_head(); }
        }
        doh_d1 = doh_next;
    }

#define MM_SLOT_END() __builtin_amdgcn_sched_barrier(0)
    floatx16 xa, xb;                       // S (V role) / dP (K role) of the current and the next unit, alternating
    bf16x8 rf[NKF];                        // leading row fragments of the next first product
    floatx4 cin[4];                        // start values of the next first product: the row constants of ITS rows
    u32x4 pin[2];                          // K role: P of the current unit

    // first product without overlap (start-up only)
    // the accumulator of a first product starts from its rows' constants (-LSE/scale for S,
    // -Delta for dP, staged with the Q tile): 16 element rows = four 16-byte reads
    auto start_values = [&](uint32_t base, int imm, floatx4 (&c)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            c[q4] = *(const floatx4 __attribute__((address_space(3)))*)(uintptr_t)(base + (uint32_t)(imm + q4 * 32));
    };
    auto as_acc = [&](const floatx4 (&c)[4]) __attribute__((always_inline)) -> floatx16 {
        floatx16 x;
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = c[r >> 2][r & 3];
        return x;
    };
    auto first_plain = [&](floatx16& x, const uint32_t (&a)[NDS], int imm, uint32_t rcb, int rc_imm) __attribute__((always_inline)) {
        floatx4 c0[4];
        start_values(rcb, rc_imm, c0);
        x = as_acc(c0);
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) x = mfma32(read_row(a[ds], imm), res[ds], x);
    };
    // PARTIAL steps: rows 8*q4 + 4*hh + 0..3 (+32 per unit) of the step's mask inputs, 16 bytes per read
    const uint32_t info_addr = lds_info + hh * 16;
    auto mask_elements = [&](floatx16& x, int imm) __attribute__((always_inline)) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const u32x4 ss = *(lds_u4)(uintptr_t)(info_addr + (uint32_t)(imm + q4 * 32));
            const u32x4 ca = *(lds_u4)(uintptr_t)(info_addr + (uint32_t)(imm + q4 * 32 + 4 * kKvBM));
            const u32x4 ps = *(lds_u4)(uintptr_t)(info_addr + (uint32_t)(imm + q4 * 32 + 8 * kKvBM));
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (!visible(ss[j], ca[j], (int64_t)ps[j], k_ss, k_mod, key))
                    x[q4 * 4 + j] = -INFINITY;
        }
    };
    auto mask_unit = [&](floatx16& x, int imm) __attribute__((always_inline)) {
        // Usually the unit's 32 rows are one run: equal mask fields, consecutive positions.
        // Then the rows that see this lane's key are one contiguous range, found once, an
        // element costs a subtraction and a comparison, and a wavefront all of whose keys are
        // seen by all 32 rows does nothing.
        const uint32_t ra = lds_info + (uint32_t)imm + (uint32_t)li * 4u;
        const uint32_t ss_r = *(lds_u1)(uintptr_t)ra, ca_r = *(lds_u1)(uintptr_t)(ra + 4 * kKvBM);
        const uint32_t ps_r = *(lds_u1)(uintptr_t)(ra + 8 * kKvBM);
        const uint32_t ss0 = __builtin_amdgcn_readfirstlane(ss_r), ca0 = __builtin_amdgcn_readfirstlane(ca_r);
        const uint32_t ps0 = __builtin_amdgcn_readfirstlane(ps_r);
        if (__all(ss_r == ss0 && ca_r == ca0 && ps_r == ps0 + (uint32_t)li)) {      // wave-uniform
            const KeyRange r = visible_rows(ss0, ca0, (int32_t)ps0, k_ss, k_mod, (int32_t)key, 32);
            if (!__all(r.all_of(32))) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (!r.sees(4u * hh + (uint32_t)(8 * q4 + j))) x[q4 * 4 + j] = -INFINITY;
            }
            return;
        }
        mask_elements(x, imm);
    };
    // One unit: NS slots, each one MFMA, one fragment request and a share of the
    // element-wise work (see the forward kernel).  KR: std::true_type for the K role.
    //   x_next <- first product of the NEXT unit: fragments 0..NKF-1 are in rf[],
    //             the others are read at a1_hi[..] + off1 (run-time, uniform) + imm1
    //   x_cur  -> P or dS of this unit (bf16), second product from the transpose
    //             fragments at a2 + imm2, row groups ks0 and ks0+1
    //   rf[]   <- fragments 0..NKF-1 of the first product after that: a1n_lo[..] + imm1n
    //   cin[]  holds the start values of x_next on entry (the row constants of the next
    //             unit's rows); after the first slot it is refilled from rcb + rc_imm with
    //             those of the unit after next
    //   hook() runs after the second slot (scalar work hidden behind the matrix pipe)
    //   V role: this unit's P is stored at pb + p_imm;  K role: it is read from there (the
    //             first half is in pin[0] on entry) and pin[0] <- the next unit's, at
    //             pb + p_imm_n (-1 when that P is not published yet)
    auto unit = [&](auto KR_, floatx16& x_next, const floatx16& x_cur, const uint32_t* a1_hi, int off1,
                    int imm1, const uint32_t* a1n_lo, int imm1n, const uint32_t (&a2)[NDB][NV], int imm2,
                    int ks0, uint32_t rcb, int rc_imm, uint32_t pb,
                    int p_imm, int p_imm_n, auto&& hook) __attribute__((always_inline)) {
        constexpr bool KR = decltype(KR_)::value;
        bf16x8 tf[NKF], pf0, pf1;
        float ev[16];
        uint32_t pw[8];
        auto slot_of = [](int e) { return e * SLV / 16; };
        auto read_rc = [&](uint32_t base, int imm, int q4) __attribute__((always_inline)) -> floatx4 {
            return *(const floatx4 __attribute__((address_space(3)))*)(uintptr_t)(base + (uint32_t)(imm + q4 * 32));
        };
        auto read_p = [&](int imm) __attribute__((always_inline)) -> u32x4 {
            return *(const u32x4 __attribute__((address_space(3)))*)(uintptr_t)(pb + (uint32_t)imm);
        };
        MM_SLOT_END();
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            // ---- matrix instruction and the request that refills its operand ----
            if (t < NDS) {
                if (t == 0) {
                    x_next = mfma32(rf[0], res[0], as_acc(cin));
                } else {
                    x_next = mfma32(rf[t % NKF], res[t], x_next);
                }
                if (t < NKF) rf[t] = read_row(a1_hi[t] + (uint32_t)off1, imm1);
                else tf[t - NKF] = read_tr(a2, imm2, ks0, t - NKF);
            } else if (t < NDS + NDB) {
                if (t == NDS) pf0 = __builtin_bit_cast(bf16x8, u32x4{pw[0], pw[1], pw[2], pw[3]});
                acc[t - NDS] = mfma32(tf[t - NDS], pf0, acc[t - NDS]);
                tf[t - NDS] = read_tr(a2, imm2, ks0 + 1, t - NDS);
            } else {
                if (t == NDS + NDB) pf1 = __builtin_bit_cast(bf16x8, u32x4{pw[4], pw[5], pw[6], pw[7]});
                acc[t - NDS - NDB] = mfma32(tf[t - NDS - NDB], pf1, acc[t - NDS - NDB]);
                rf[t - NDS - NDB] = read_row(a1n_lo[t - NDS - NDB], imm1n);
            }
            // ---- element-wise work ----
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (slot_of(2 * k + 1) + 1 == t) {              // round a finished pair to bf16
                    const bf16x2 pb2 = {(__bf16)ev[2 * k], (__bf16)ev[2 * k + 1]};
                    pw[k] = __builtin_bit_cast(uint32_t, pb2);
                    asm volatile("" : "+v"(pw[k]));
                }
            // V role: publish the unit's probabilities for the partner wave, in the unit's last
            // two slots (the partner reads them after the next barrier; LDS operations complete
            // in order, so a store in the middle of the unit delays the fragment reads queued
            // behind it, which the coming MFMAs wait for: 2.5 % of the kernel's time)
            if (!KR && t >= NS - 2) {
                const int k4 = t - (NS - 2);
                const u32x4 o4 = {pw[4 * k4], pw[4 * k4 + 1], pw[4 * k4 + 2], pw[4 * k4 + 3]};
                *(u32x4 __attribute__((address_space(3)))*)(uintptr_t)(pb + (uint32_t)(p_imm + k4 * 1024)) = o4;
            }
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (slot_of(e) == t) {
                    if (!KR) {
                        // x_cur is S - LSE/scale; masked entries are -inf: exp2 gives 0 (padding
                        // rows have LSE = +inf)
                        ev[e] = __builtin_amdgcn_exp2f(x_cur[e] * scale_log2);
                    } else {
                        // x_cur is dP - Delta
                        const uint32_t w = pin[e >> 3][(e & 7) >> 1];
                        const float pv = __builtin_bit_cast(float, (e & 1) ? (w & 0xffff0000u) : (w << 16));
                        ev[e] = pv * x_cur[e];
                    }
                    asm volatile("" : "+v"(ev[e]));
                }
            // start values of the first product formed in the NEXT unit: four rows per read,
            // spread over the unit (cin[] was consumed by the first slot's MFMA)
            if (t == 1) cin[0] = read_rc(rcb, rc_imm, 0);
            if (t == 2) cin[1] = read_rc(rcb, rc_imm, 1);
            if (t == SLV + 1) {
                cin[2] = read_rc(rcb, rc_imm, 2);
                cin[3] = read_rc(rcb, rc_imm, 3);
            }
            // K role: P of this unit's last 8 element rows, then of the next unit's first 8
            if (KR && t == (slot_of(8) > 4 ? slot_of(8) - 4 : 0)) pin[1] = read_p(p_imm + 1024);
            if (KR && t == SLV + 2 && p_imm_n >= 0) pin[0] = read_p(p_imm_n);
            MM_SLOT_END();
            // the two roles of a key block share a SIMD and leave the barrier together: the K
            // role issues its transfers half a unit after the V role, so that the SIMD's matrix
            // pipe always has one of the two feeding it
            if (t == (KR ? NS / 2 + 1 : 1)) hook();
        }
    };

    // top of iteration i, common to both roles: everything issued one iteration ago has
    // landed (Q and row constants of step i+1, dO of step i); after the barrier step i-1's
    // P is published and the stages of step i-2 are free, so the next transfers start.
    // Returns whether step i is PARTIAL.
    int dst = 0;                           // dO ring stage of step i
    auto top = [&](int i, auto&& after_barrier) __attribute__((always_inline)) -> bool {
        wait_vmcnt<0>();
        __syncthreads();
        after_barrier();                   // LDS reads that should start right away
        return i < n_steps && (ent[0] & kPartialFlag) != 0;
    };
    // the transfers of iteration i: Q tile (+ row data) of step i+2, dO tile of step i+1.
    // Called from inside the iteration's first unit so that the scalar bookkeeping runs
    // in the shadow of its matrix instructions.
    auto issue = [&](int i) __attribute__((always_inline)) {
        if (i + 2 < n_steps) {
            if (((i + 2) & 63) == 0) {
                list_chunk = fetch_chunk(i + 2);
                wait_vmcnt<0>();           // nothing else is in flight here
            }
            ent[2] = __builtin_amdgcn_readlane(list_chunk, (i + 2) & 63);
            issue_q(ent[2], (i + 2) & (kKvQst - 1));
            if (++qi_next == n_q) { qi_next = 0; next_head(); }
        }
        if (i + 1 < n_steps) {
            int dn = dst + 1;
            if (dn == kKvDst) dn = 0;
            issue_d(ent[1], doh_d, dn);
        }
        doh_d = doh_d1;
        doh_d1 = doh_next;
        ent[0] = ent[1];
        ent[1] = ent[2];
    };
    constexpr int kLdStage = 8 * kKvBM;    // bytes of a stage of row constants
    // byte step from dO stage `dst` to the next one
    auto d_step = [&]() -> int { return dst + 1 == kKvDst ? -(kKvDst - 1) * kStage : kStage; };

    if (!k_role) {
        // ---- V role: step i (units 2i, 2i+1).  Unrolled over the Q ring so that the
        // stage offsets are immediates; the dO tile of step i is addressed through dtr[].
        uint32_t dtr[NDB][NV];
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < NV; ++v) dtr[db][v] = tr_addr[db][v];
        for (int i0 = 0; i0 <= n_steps; i0 += kKvQst) {
#pragma unroll
            for (int u = 0; u < kKvQst; ++u) {
                const int i = i0 + u;
                if (i > n_steps) break;
                const int qs0 = u, qs1 = (u + 1) % kKvQst;
                const bool partial = top(i, [] {});
                if (i == 0 && n_steps > 0) {
                    first_plain(xa, row_addr, 0, rc_addr, 0);
#pragma unroll
                    for (int j = 0; j < NKF; ++j) rf[j] = read_row(row_addr[j], kUnit);
                    start_values(rc_addr, 128, cin);
                }
                if (i < n_steps) {
                    if (partial) mask_unit(xa, qs0 * (12 * kKvBM));
                    unit(std::false_type{}, xb, xa, &row_addr[NKF], 0, qs0 * kStage + kUnit, &row_addr[0],
                         qs1 * kStage, dtr, 0, 0, rc_addr, qs1 * kLdStage,
                         p_addr, (u & 1) * 16384, -1, [&] { issue(i); });
                    if (partial) mask_unit(xb, qs0 * (12 * kKvBM) + 128);
                    unit(std::false_type{}, xa, xb, &row_addr[NKF], 0, qs1 * kStage, &row_addr[0],
                         qs1 * kStage + kUnit, dtr, 0, 2, rc_addr, qs1 * kLdStage + 128,
                         p_addr, (u & 1) * 16384 + 2048, -1, [] {});
                } else {
                    issue(i);
                }
                const int delta = d_step();
                if (++dst == kKvDst) dst = 0;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int v = 0; v < NV; ++v) dtr[db][v] += (uint32_t)delta;
            }
        }
    } else {
        // ---- K role: step i-1 (units 2i-2, 2i-1) and the first product of step i.  All
        // ring positions are run-time here: drow[] is the dO tile of step i (the one of
        // step i-1 lies dprev bytes from it), qtr[] the Q tile of step i-1, rcc
        // the row constants of step i, pp the P buffer of step i-1.
        uint32_t drow[NDS], qtr[NDB][NV];
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) drow[ds] = row_addr[ds];
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < NV; ++v) qtr[db][v] = tr_addr[db][v] + (uint32_t)((kKvQst - 1) * kStage);
        int dprev = 0, qpos = kKvQst - 1;
        uint32_t rcc = rc_addr;
        uint32_t pp = p_addr + 16384u;
        for (int i = 0; i <= n_steps; ++i) {
            top(i, [&] {
                if (i >= 1) pin[0] = *(const u32x4 __attribute__((address_space(3)))*)(uintptr_t)(pp);
            });
            if (i == 0 && n_steps > 0) {
                first_plain(xa, drow, 0, rc_addr, 0);
#pragma unroll
                for (int j = 0; j < NKF; ++j) rf[j] = read_row(drow[j], kUnit);
                start_values(rc_addr, 128, cin);
            }
            if (i >= 1) {
                unit(std::true_type{}, xb, xa, &drow[NKF], dprev, kUnit, &drow[0], 0, qtr, 0, 0, rcc, 0,
                     pp, 0, 2048, [&] { issue(i); });
                unit(std::true_type{}, xa, xb, &drow[NKF], 0, 0, &drow[0], kUnit, qtr, 0, 2, rcc, 128,
                     pp, 2048, -1, [] {});
            } else {
                issue(i);
            }
            // advance: dO ring, Q ring position of step i, row constants, P parity
            const int delta = d_step();
            if (++dst == kKvDst) dst = 0;
            dprev = -delta;
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds) drow[ds] += (uint32_t)delta;
            const int qdelta = qpos + 1 == kKvQst ? -(kKvQst - 1) : 1;
            qpos += qdelta;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int v = 0; v < NV; ++v) qtr[db][v] += (uint32_t)(qdelta * kStage);
            rcc = rc_addr + (uint32_t)(((i + 1) & (kKvQst - 1)) * kLdStage);
            pp = p_addr + (uint32_t)((i & 1) * 16384);
        }
    }
#undef MM_SLOT_END

    // ---- epilogue: lane holds key `key`, 4 consecutive d per register quad ------------
    const int64_t obase = (key * Hkv + g) * (int64_t)D + 4 * hh;
    const float osc = k_role ? scale : 1.0f;
    if (shared_unit) {
        // this workgroup's partial sums, fp32, in its own slot: dK [128][Hkv][D], then dV
        const int64_t tile_elems = (int64_t)kKvBN * Hkv * D;
        float* dst = pool + ((int64_t)(slot0 + slice * ch.cmax + chunk) * 2 + (k_role ? 0 : 1)) * tile_elems +
                     ((int64_t)(kblk * 32 + li) * Hkv + g) * D + 4 * hh;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                floatx4 out;
#pragma unroll
                for (int u = 0; u < 4; ++u) out[u] = acc[db][c * 4 + u] * osc;
                *(floatx4*)(dst + db * 32 + c * 8) = out;
            }
    } else {
        ushort_t* dst = k_role ? dK : dV;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                bf16x4 out;
#pragma unroll
                for (int u = 0; u < 4; ++u) out[u] = (__bf16)(acc[db][c * 4 + u] * osc);
                *(u32x2*)(dst + obase + db * 32 + c * 8) = __builtin_bit_cast(u32x2, out);
            }
    }
}

// sum the fp32 partials of every k-tile that several workgroups worked on (slices of
// its list, chunks of a KV group's query heads) in a fixed order and write bf16.
// grid (k-tile, part of the tile); kRedIt x 4 elements per thread
constexpr int kRedIt = 1;
constexpr int kRedPerWg = 256 * 4 * kRedIt;
__global__ void __launch_bounds__(256)
dkv_reduce_kernel(TilePlanT plan, int32_t Hkv, int32_t D, const int32_t* __restrict__ err,
                  const float* __restrict__ pool, ushort_t* __restrict__ dK, ushort_t* __restrict__ dV) {
    if (*err) return;
    const int kt = blockIdx.x;
    const int slot0 = plan.pbase[kt];
    if (slot0 < 0) return;                             // written directly by its one workgroup
    const int c = plan.slicing[kSliceLen];
    const int slots = max(1, (plan.qcount[kt] + c - 1) / c) * plan.hc;
    const int64_t tile_elems = (int64_t)kKvBN * Hkv * D;
    const float* src = pool + (int64_t)slot0 * 2 * tile_elems;
    // tile_elems = 128 * Hkv * D is a multiple of kRedPerWg (D >= 64), so no bounds test
    floatx4 a[kRedIt], b[kRedIt];
#pragma unroll
    for (int it = 0; it < kRedIt; ++it) {
        const int64_t e = (int64_t)blockIdx.y * kRedPerWg + (it * 256 + threadIdx.x) * 4;
        a[it] = *(const floatx4*)(src + e) + *(const floatx4*)(src + 2 * tile_elems + e);
        b[it] = *(const floatx4*)(src + tile_elems + e) + *(const floatx4*)(src + 3 * tile_elems + e);
    }
    for (int s = 2; s < slots; ++s)
#pragma unroll
        for (int it = 0; it < kRedIt; ++it) {
            const int64_t e = (int64_t)blockIdx.y * kRedPerWg + (it * 256 + threadIdx.x) * 4;
            a[it] += *(const floatx4*)(src + (int64_t)s * 2 * tile_elems + e);
            b[it] += *(const floatx4*)(src + ((int64_t)s * 2 + 1) * tile_elems + e);
        }
#pragma unroll
    for (int it = 0; it < kRedIt; ++it) {
        const int64_t e = (int64_t)blockIdx.y * kRedPerWg + (it * 256 + threadIdx.x) * 4;
        bf16x4 oa, ob;
#pragma unroll
        for (int u = 0; u < 4; ++u) { oa[u] = (__bf16)a[it][u]; ob[u] = (__bf16)b[it][u]; }
        const int64_t o = (int64_t)kt * tile_elems + e;
        *(u32x2*)(dK + o) = __builtin_bit_cast(u32x2, oa);
        *(u32x2*)(dV + o) = __builtin_bit_cast(u32x2, ob);
    }
}

// ---------------------------------------------------------------- dQ ---------
constexpr int kDqBM = 128, kDqBN = 64;

template <int D, int NST>
struct DqSmem {
    alignas(1024) unsigned char k[NST][kDqBN * D * 2];    // MODE 0: rows (S^T) and transpose (dQ^T)
    alignas(1024) unsigned char v[NST][kDqBN * D * 2];    // same layout: rows (dP^T)
    alignas(256) uint64_t kw[NST][kDqBN];                 // mask words of a PARTIAL tile's keys, by ring stage
    alignas(16) float park[4][3][64][4];                  // per wavefront: twelve registers parked while a tile is masked
};

template <int D, int HPW, int NST>
__global__ void __launch_bounds__(256 * HPW, 2)
dq_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
          const ushort_t* __restrict__ V, const ushort_t* __restrict__ dO,
          const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
          int64_t n_loc, int64_t n_pad, int64_t S, int32_t Hq, int32_t Hkv, float scale,
          float scale_log2, const ushort_t* __restrict__ O, const float* __restrict__ lse,
          const float* __restrict__ ld_g, TilePlan plan, FwdSplit split, const int32_t* __restrict__ err,
          ushort_t* __restrict__ dQ, float* __restrict__ dQpart,
          ushort_t* __restrict__ qh, ushort_t* __restrict__ doh, float* __restrict__ ldk,
          uint32_t* __restrict__ info) {
    constexpr int NDS = D / 16, NDB = D / 32;
    constexpr int NW = 4 * HPW;
    constexpr int RB = D * 2;
    using KT = SwzTile<D, 0>;
    using VT = KT;                        // same layout: one set of row-fragment offsets serves both
    constexpr int kStageBytes = kDqBN * RB;
    constexpr int NI = kStageBytes / 1024 / NW;
    static_assert(NI >= 1, "tile too small for this many wavefronts");
    __shared__ DqSmem<D, NST> sm;
    // independent loads of the work-item lookup are issued together and the early exits are
    // taken after the row's own loads (see the forward kernel)
    const int err_flag = *err;
    const int csz_dev = *plan.csz;

    const int rep = Hq / Hkv;
    int tile_rank, h0;
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
    const int kc_total = plan.kcount[qt];
    const int csz = max(csz_dev, split.csz);
    const uint32_t* klist = plan.klist + (int64_t)qt * plan.nk + chunk * csz;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = h0 + wave / 4, w4 = wave & 3;
    const int li = lane & 31, hh = lane >> 5;

    const int64_t row = (int64_t)qt * kDqBM + w4 * 32 + li;     // < n_pad
    const bool row_ok = row < n_loc;
    int64_t q_pos = 0;
    uint32_t q_ss = 0, q_causal = 0;
    // LSE in base-2 units: +inf on padding rows; a row that sees no key has LSE = -inf and all
    // its scores masked (-inf): taking +inf for it as well makes every probability 0 instead
    // of exp2(-inf + inf).  Delta = rowsum(dO o O) comes from the preparation (ld_g given) or
    // is formed here from the row's O and dO (this lane's 64 head-dim values, then the other
    // half-wave's).
    const bool own_delta = ld_g == nullptr;             // kernel argument: uniform
    float my_lse2 = INFINITY, my_delta = 0.f;
    if (!own_delta) {
        const float l2 = ld_g[(int64_t)h * 2 * n_pad + row];
        my_lse2 = l2 == -INFINITY ? INFINITY : l2;
        my_delta = ld_g[((int64_t)h * 2 + 1) * n_pad + row];
    }
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
        q_causal = word_att(w);
        const int64_t off = (row * Hq + h) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            qf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(Q + off + ds * 16));
            dof[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(dO + off + ds * 16));
        }
        if (own_delta) {
            const float l2 = lse[(int64_t)h * n_loc + row] * kLog2e;
            my_lse2 = l2 == -INFINITY ? INFINITY : l2;
            bf16x8 of[NDS];
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds)
                of[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(O + off + ds * 16));
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds)
#pragma unroll
                for (int u = 0; u < 8; ++u) my_delta += (float)of[ds][u] * (float)dof[ds][u];
        }
    }
    if (own_delta) my_delta += __shfl_xor(my_delta, 32);
    // entries past the list's length, inside the q-tile's row of the list array, are read
    // but never used
    uint32_t list_chunk = chunk * csz + lane < plan.nk ? klist[lane] : 0u;

    const int nchunk = max(1, (kc_total + csz - 1) / csz);
    if (chunk >= nchunk) return;          // workgroup-uniform
    const int n_active = max(0, min(kc_total - chunk * csz, csz));

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
    const uint32_t lds_kw = lds_addr_of(sm.kw[0]);
    auto issue_tile = [&](uint32_t entry, int stage) {
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kDqBN;
        const ushort_t* kt_ = K + k0 * Hkv * D;
        const ushort_t* vt_ = V + k0 * Hkv * D;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            dma16(kt_, gk[i], lds_k + stage * kStageBytes + i * 1024);
            dma16(vt_, gv[i], lds_v + stage * kStageBytes + i * 1024);
        }
        // the mask words of a PARTIAL tile's 64 keys travel with the tile (see the forward kernel)
        if ((entry & kPartialFlag) && wave < 2)
            dma4(bits + k0, (uint32_t)(wave * 256 + lane * 4), lds_kw + stage * (8 * kDqBN) + wave * 256);
    };

    // fragment addresses (LDS byte addresses at ring stage 0): K and V rows share the lane
    // pattern (same tile layout) but live in different rings; K is also read transposed
    constexpr int PER = 16 * KT::RPS, NV = PER / 8;
    // The V ring follows the K ring in LDS; with a short ring every V offset still fits
    // the 16-bit offset field, so the K row addresses serve both.
    constexpr int kVOff = NST * kStageBytes;
    static_assert(2 * NST * kStageBytes <= 65536, "V ring out of reach of the offset field");
    uint32_t krow_a[NDS], ktr_a[NDB][NV];
    {
        RowFragAddr<KT, D> fr;
        TrFragAddr<KT, D> ft;
        fr.init(lane);
        ft.init(lane);
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            krow_a[ds] = lds_addr_of(sm.k[0]) + (uint32_t)fr.off[ds];
        }
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < NV; ++v) ktr_a[db][v] = lds_addr_of(sm.k[0]) + (uint32_t)ft.off[db][v];
    }
    auto read_row = [&](uint32_t a, int imm) __attribute__((always_inline)) -> bf16x8 {
        return __builtin_bit_cast(bf16x8, *(lds_u4)(uintptr_t)(a + (uint32_t)imm));
    };
    auto read_tr = [&](int imm, int ks, int db) __attribute__((always_inline)) -> bf16x8 {
        const int r_lo = ks * 16, r_hi = ks * 16 + 8;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(
            ktr_a[db][(r_lo % PER) / 8] + (uint32_t)(imm + (r_lo / PER) * PER * RB)));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(
            ktr_a[db][(r_hi % PER) / 8] + (uint32_t)(imm + (r_hi / PER) * PER * RB)));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    auto entry_at = [&](int it) -> uint32_t {
        return __builtin_amdgcn_readlane(list_chunk, it & 63);
    };
    // all ordinary vector loads so far are awaited once, before the transfers start
    // (see the note in the forward kernel)
    wait_vmcnt<0>();

    // A tile is two phases: S and dP of its 64 keys (32 MFMAs, hardly any vector work), then
    // the element-wise work and the dQ products (16 MFMAs under about 180 vector
    // instructions); the compiler schedules inside each.
    constexpr int PD = NST - 1;            // tiles it .. it+PD-1 are resident or in flight
    uint32_t pend[PD];
#pragma unroll
    for (int j = 0; j < PD; ++j) {
        pend[j] = 0u;
        if (j < n_active) {
            pend[j] = entry_at(j);
            issue_tile(pend[j], j);
        }
    }

    constexpr int kHalf = 32 * RB;
    floatx16 sv[2], dpv[2];                // scores and dP of the tile's two halves, between the phases
    // phase 1 of the tile at LDS offset `tile`
    auto phase_sdp = [&](int tile, int kw_off, bool partial, int64_t k0) __attribute__((always_inline)) {
        // Two independent accumulation chains, alternated; their K and V row fragments are
        // requested two pairs of MFMAs ahead (the compiler on its own requests them one
        // ahead and waits before almost every MFMA), across the two halves of the tile.
        constexpr int NP = 2 * NDS;        // MFMA pairs of the tile
        bf16x8 kfr[2], vfr[2];
        // this phase is almost only matrix instructions: it runs at the lower priority, the
        // element-wise phase at the higher one, so that of the two workgroups on a CU the one
        // with vector work to do gets the issue slots first (measured: -2.3 %)
        __builtin_amdgcn_s_setprio(0);
        auto fetch = [&](int i) __attribute__((always_inline)) {
            const int off = tile + (i / NDS) * kHalf;
            kfr[i & 1] = read_row(krow_a[i % NDS], off);
            vfr[i & 1] = read_row(krow_a[i % NDS], kVOff + off);
        };
        fetch(0);
        fetch(1);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) { sv[kb][r] = 0.f; dpv[kb][r] = 0.f; }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int kb = i / NDS, ds = i % NDS;
            sv[kb] = mfma32(kfr[i & 1], qf[ds], sv[kb]);
            dpv[kb] = mfma32(vfr[i & 1], dof[ds], dpv[kb]);
            if (i + 2 < NP) fetch(i + 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (partial) {
            // the query-side fields are per-lane constants; passed through an empty asm so that
            // what the predicate derives from them is computed here and not kept in registers
            // across the whole loop
            uint32_t qs = q_ss, qa = q_causal, qp = (uint32_t)q_pos;
            asm volatile("" : "+v"(qs), "+v"(qa), "+v"(qp));
            // The kernel has no register to spare, so twelve accumulator registers are parked in
            // LDS while a PARTIAL tile is masked (rare) and fetched back afterwards: the masking
            // code gets room without costing the main loop anything.
            uint32_t zero = 0u;
            asm volatile("" : "+v"(zero));                   // lane index taken afresh, see below
            const uint32_t ln = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, zero));
            const uint32_t park_a = lds_addr_of(sm.park) + (uint32_t)(wave & 3) * 3072u + ln * 16u;
            typedef floatx4 __attribute__((address_space(3))) * lds_f4;
            *(lds_f4)(uintptr_t)park_a = floatx4{dq[NDB - 1][0], dq[NDB - 1][1], dq[NDB - 1][2], dq[NDB - 1][3]};
            *(lds_f4)(uintptr_t)(park_a + 1024u) = floatx4{dq[NDB - 1][4], dq[NDB - 1][5], dq[NDB - 1][6], dq[NDB - 1][7]};
            *(lds_f4)(uintptr_t)(park_a + 2048u) = floatx4{dq[NDB - 1][8], dq[NDB - 1][9], dq[NDB - 1][10], dq[NDB - 1][11]};
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                // usually the 32 keys of the half tile are one run of equal mask fields: every row
                // then sees one contiguous range of them (see the forward kernel)
                typedef const uint64_t __attribute__((address_space(3))) * lds_u8;
                const uint64_t wk = *(lds_u8)(uintptr_t)(lds_kw + (uint32_t)(kw_off + kb * 256) + (ln & 31u) * 8u);
                const uint32_t ss_k = word_ss(wk), mod_k = word_mod(wk);
                const uint32_t ss0 = __builtin_amdgcn_readfirstlane(ss_k), mod0 = __builtin_amdgcn_readfirstlane(mod_k);
                if (__all(ss_k == ss0 && mod_k == mod0)) {       // wave-uniform
                    const KeyRange r = visible_range(qs, qa, (int32_t)qp, ss0, mod0, (int32_t)k0 + kb * 32, 32);
                    if (!__all(r.all_of(32))) {
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (!r.sees((ln >> 5) * 4u + (uint32_t)(8 * q4 + j))) sv[kb][q4 * 4 + j] = -INFINITY;
                    }
                    continue;
                }
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    // the words of keys 8*q4 + 4*hh + 0..3 of the half tile, one pair at a time
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int kl = kb * 32 + 8 * q4 + 4 * hh + j;
                        const uint64_t w1 = *(lds_u8)(uintptr_t)(lds_kw + (uint32_t)(kw_off + kb * 256 + (8 * q4 + j) * 8) + (ln >> 5) * 32u);
                        if (!visible(qs, qa, (int64_t)qp, word_ss(w1), word_mod(w1), k0 + kl)) sv[kb][q4 * 4 + j] = -INFINITY;
                        // one element at a time: no register is free for a second one's temporaries
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            {
                const floatx4 p0 = *(lds_f4)(uintptr_t)park_a, p1 = *(lds_f4)(uintptr_t)(park_a + 1024u);
                const floatx4 p2 = *(lds_f4)(uintptr_t)(park_a + 2048u);
#pragma unroll
                for (int u = 0; u < 4; ++u) { dq[NDB - 1][u] = p0[u]; dq[NDB - 1][4 + u] = p1[u]; dq[NDB - 1][8 + u] = p2[u]; }
            }
        }
    };
    // phase 2: dS = P o (dP - Delta) as bf16, then dQ^T += K^T dS^T
    auto phase_dq = [&](int tile) __attribute__((always_inline)) {
        bf16x8 dsf[4];
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // masked entries are -inf: exp2 gives 0 (padding rows have LSE = +inf)
                const float p = __builtin_amdgcn_exp2f(sv[kb][r] * scale_log2 - my_lse2);
                dsf[kb * 2 + (r >> 3)][r & 7] = (__bf16)(p * (dpv[kb][r] - my_delta));
            }
        // K^T fragments requested two MFMAs ahead
        constexpr int NM = 4 * NDB;
        bf16x8 tf[2];
        tf[0] = read_tr(tile, 0, 0);
        tf[1] = read_tr(tile, 1 / NDB, 1 % NDB);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            dq[m % NDB] = mfma32(tf[m & 1], dsf[m / NDB], dq[m % NDB]);
            if (m + 2 < NM) tf[m & 1] = read_tr(tile, (m + 2) / NDB, (m + 2) % NDB);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The ring position of tile `it` is it mod NST; the loop is unrolled NST-fold so that
    // every LDS offset is an immediate.
    auto tiles = [&](auto&& body) __attribute__((always_inline)) {
        for (int it0 = 0; it0 < n_active; it0 += NST) {
#pragma unroll
            for (int st = 0; st < NST; ++st) {
                const int it = it0 + st;
                if (it >= n_active) break;
                const int sn = (st + PD) % NST;          // stage of tile it-1, free after the barrier
                const uint32_t entry = pend[0];
                const bool partial = (entry & kPartialFlag) != 0;
                const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kDqBN;
                const int younger = min(PD - 1, n_active - 1 - it);
                if (younger >= 2) wait_vmcnt<(PD > 2 ? 4 * NI : 0)>();
                else if (younger == 1) wait_vmcnt<(PD > 1 ? 2 * NI : 0)>();
                else wait_vmcnt<0>();
                __syncthreads();
                uint32_t fresh = 0u;
                if (it + PD < n_active) {
                    if (((it + PD) & 63) == 0) {
                        const int j = it + PD + lane;
                        list_chunk = j < n_active ? klist[j] : 0u;
                        wait_vmcnt<0>();       // awaited here so that no wait is needed after the branch
                    }
                    fresh = entry_at(it + PD);
                    issue_tile(fresh, sn);
                }
#pragma unroll
                for (int j = 0; j + 1 < PD; ++j) pend[j] = pend[j + 1];
                pend[PD - 1] = fresh;
                body(it, st, partial, k0);
            }
        }
    };
    tiles([&](int it, int st, bool partial, int64_t k0) __attribute__((always_inline)) {
        phase_sdp(st * kStageBytes, st * (8 * kDqBN), partial, k0);
        phase_dq(st * kStageBytes);
    });

    // When this pass runs ahead of the key-outer pass (qh given), the workgroup that holds a
    // row's Q and dO anyway (the first slice of a split list) leaves that pass its inputs: the
    // head-major copies, the start values of its accumulators and, once per row, the mask
    // inputs (see bwd_prep_body).  All rows below n_pad are written (padding rows: zeros).
    if (qh != nullptr && chunk == 0) {
        ushort_t* qd = qh + ((int64_t)h * n_pad + row) * D + hh * 8;
        ushort_t* dd = doh + ((int64_t)h * n_pad + row) * D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            *(u32x4*)(qd + ds * 16) = __builtin_bit_cast(u32x4, qf[ds]);
            *(u32x4*)(dd + ds * 16) = __builtin_bit_cast(u32x4, dof[ds]);
        }
        if (hh == 0) {
            const float l = row_ok ? lse[(int64_t)h * n_loc + row] : INFINITY;
            ldk[(int64_t)h * 2 * n_pad + row] = -l * (1.0f / scale);
            ldk[((int64_t)h * 2 + 1) * n_pad + row] = -my_delta;
            if (h == 0) {
                info[row] = q_ss;
                info[n_pad + row] = q_causal;
                info[2 * n_pad + row] = (uint32_t)q_pos;
            }
        }
    }
    if (!row_ok) return;
    if (nchunk > 1) {
        // this slice's partial sum, fp32, summed over the slices by dq_combine_kernel
        float* op = dQpart + (((int64_t)chunk * n_pad + row) * Hq + h) * D + 4 * hh;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                floatx4 out;
#pragma unroll
                for (int u = 0; u < 4; ++u) out[u] = dq[db][c * 4 + u] * scale;
                *(floatx4*)(op + db * 32 + c * 8) = out;
            }
        return;
    }
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

// sums the slices of split q-tiles in a fixed order; one thread per 4 elements
__global__ void __launch_bounds__(256)
dq_combine_kernel(TilePlan plan, FwdSplit split, int64_t n_loc, int64_t n_pad, int32_t Hq, int32_t D,
                  const int32_t* __restrict__ err, const float* __restrict__ dQpart,
                  ushort_t* __restrict__ dQ) {
    if (*err) return;
    const int dq4 = D / 4;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t rh = gid / dq4;
    const int d0 = (int)(gid % dq4) * 4;
    const int64_t row = rh / Hq;
    const int h = (int)(rh % Hq);
    if (row >= n_loc) return;
    const int kc_total = plan.kcount[row / kDqBM];
    const int csz = max(*plan.csz, split.csz);
    const int nchunk = max(1, (kc_total + csz - 1) / csz);
    if (nchunk == 1) return;              // written by dq_kernel itself
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < nchunk; ++c)
        acc += *(const floatx4*)(dQpart + (((int64_t)c * n_pad + row) * Hq + h) * D + d0);
    bf16x4 out;
#pragma unroll
    for (int u = 0; u < 4; ++u) out[u] = (__bf16)acc[u];
    *(u32x2*)(dQ + (row * Hq + h) * (int64_t)D + d0) = __builtin_bit_cast(u32x2, out);
}

// ---------------------------------------------------------------- host -------
struct BwdLayout {
    size_t err, clean_blocks, ld, info, ldk, qh, doh, cls_a, kcount, klist, qorder, cls_b, qcount, qlist,
        korder, slicing, pbase, extra, pool, dq_part, total;
    int32_t nq_a, nk_a, nq_b, nk_b, n_extra;
    int64_t n_pad;
    KvChunking ch;
    FwdSplit split;                   // list slices of the query-outer (dQ) pass
};

// Split the query heads of a (k-tile, KV head) unit over several workgroups only
// when the units alone cannot fill the chip a few times over (256 resident
// workgroups).
static KvChunking kv_chunking(int32_t nk_b, int32_t Hq, int32_t Hkv) {
    const int64_t units = (int64_t)nk_b * Hkv;
    const int32_t rep = Hq / Hkv;
    int32_t cmax = 1;                  // smallest divisor of rep that yields >= 1024 workgroups, else rep
    for (int32_t c = 1; c <= rep; ++c) {
        if (rep % c) continue;
        cmax = c;
        if (units * c >= 1024) break;
    }
    return KvChunking{cmax, rep / cmax};
}

static BwdLayout bwd_layout(int64_t S, int64_t n_loc, int32_t n_blocks, int32_t Hq, int32_t Hkv,
                            int32_t D) {
    BwdLayout L;
    L.nq_a = (int32_t)((n_loc + kDqBM - 1) / kDqBM);
    L.nk_a = (int32_t)(S / kDqBN);
    L.nq_b = (int32_t)((n_loc + kKvBM - 1) / kKvBM);
    L.nk_b = (int32_t)(S / kKvBN);
    L.n_pad = (int64_t)L.nq_a * kDqBM;
    L.ch = kv_chunking(L.nk_b, Hq, Hkv);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    L.err = take(256);
    L.clean_blocks = take((size_t)n_blocks * 4);
    L.ld = take((size_t)Hq * 2 * L.n_pad * 4);
    L.info = take((size_t)3 * L.n_pad * 4);
    L.ldk = take((size_t)Hq * 2 * L.n_pad * 4);
    L.qh = take((size_t)Hq * L.n_pad * D * 2);
    L.doh = take((size_t)Hq * L.n_pad * D * 2);
    L.cls_a = take((size_t)L.nq_a * L.nk_a);
    L.kcount = take((size_t)L.nq_a * 4);
    L.klist = take((size_t)L.nq_a * L.nk_a * 4);
    L.qorder = take((size_t)L.nq_a * 4);
    L.cls_b = take((size_t)L.nq_b * L.nk_b);
    L.qcount = take((size_t)L.nk_b * 4);
    L.qlist = take((size_t)L.nq_b * L.nk_b * 4);
    L.korder = take((size_t)L.nk_b * 4);
    // list slices of the key-outer pass: none for short lists; else as many extra slices as
    // bring the launch to about 2048 workgroups, at most 256
    L.n_extra = L.nq_b >= 16 ? std::min(256, 2048 / (Hkv * L.ch.cmax)) : 0;
    L.slicing = take(kSliceInts * 4);
    L.pbase = take((size_t)L.nk_b * 4);
    L.extra = take((size_t)std::max(L.n_extra, 1) * 8);
    // partial-sum slots: every k-tile's workgroups when the heads are chunked, else the sliced
    // k-tiles' first slices (at most one per extra slice); plus the extra slices
    const size_t slots = (L.ch.cmax > 1 ? (size_t)L.nk_b * L.ch.cmax : (size_t)std::min(L.nk_b, L.n_extra)) +
                         (size_t)L.n_extra * L.ch.cmax;
    L.pool = take(slots * 2 * kKvBN * Hkv * D * 4);
    L.split = list_split(L.nq_a, L.nk_a, Hq);          // dq_kernel: one workgroup per (q-tile, head)
    L.dq_part = take(L.split.cmax > 1 ? (size_t)L.split.cmax * L.n_pad * Hq * D * 4 : 0);
    L.total = off;
    return L;
}

size_t bwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D) {
    return bwd_layout(S, n_loc, (int32_t)(n_loc / 16 + 1), Hq, Hkv, D).total;
}

// qh == nullptr: the preparation has run (ld holds the rows' LSE and Delta); else this pass
// forms Delta itself and writes the key-outer pass's inputs
template <int D, int HPW, int NST>
static void launch_dq_kernel(const AttnArgs& a, const void* o, const float* lse, const void* d_o,
                             int64_t n_loc, const BwdLayout& L, float scale_log2, const int32_t* clean,
                             const float* ld, const TilePlan& pa, const int32_t* err, void* dq,
                             float* dq_part, ushort_t* qh, ushort_t* doh, float* ldk, uint32_t* info,
                             hipStream_t st) {
    const unsigned grid = (unsigned)((int64_t)L.nq_a * a.Hq / HPW * L.split.cmax);
    hipLaunchKernelGGL((dq_kernel<D, HPW, NST>), dim3(grid), dim3(256 * HPW), 0, st,
                       (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v,
                       (const ushort_t*)d_o, a.bits, clean, a.block, n_loc, L.n_pad, a.S, a.Hq, a.Hkv,
                       a.scale, scale_log2, (const ushort_t*)o, lse, ld, pa, L.split, err, (ushort_t*)dq,
                       dq_part, qh, doh, ldk, info);
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
    uint32_t* info = (uint32_t*)(base + L.info);
    float* ldk = (float*)(base + L.ldk);
    ushort_t* qh = (ushort_t*)(base + L.qh);
    ushort_t* doh = (ushort_t*)(base + L.doh);
    float* pool = (float*)(base + L.pool);
    TilePlan pa;
    pa.nq = L.nq_a; pa.nk = L.nk_a; pa.tq = kDqBM; pa.tk = kDqBN;
    pa.cls = (uint8_t*)(base + L.cls_a);
    pa.kcount = (int32_t*)(base + L.kcount);
    pa.klist = (uint32_t*)(base + L.klist);
    pa.qorder = (int32_t*)(base + L.qorder);
    pa.csz = err + kFlagInts;
    pa.groups = a.Hq;
    TilePlanT pb;
    pb.nq = L.nq_b; pb.nk = L.nk_b; pb.tq = kKvBM; pb.tk = kKvBN;
    pb.cls = (uint8_t*)(base + L.cls_b);
    pb.qcount = (int32_t*)(base + L.qcount);
    pb.qlist = (uint32_t*)(base + L.qlist);
    pb.korder = (int32_t*)(base + L.korder);
    pb.n_extra = L.n_extra; pb.hc = L.ch.cmax; pb.hpc = L.ch.hpc; pb.groups = a.Hkv * L.ch.cmax;
    pb.slicing = (int32_t*)(base + L.slicing);
    pb.pbase = (int32_t*)(base + L.pbase);
    pb.extra = (int32_t*)(base + L.extra);

    // The key-outer pass needs head-major copies of Q and dO, its rows' constants and mask
    // inputs.  The query-outer pass holds every row's Q and dO in registers and can leave them
    // on its way at little cost, which saves a pass over Q, O and dO -- but then it has to run
    // first, and the copies are as old as that pass is long when the key-outer pass reads
    // them.  Measured (same box, alternating): whole steps -1.0 % at 8k and -0.3 % at 32k
    // (copies of 128 MiB), +0.4 % at 128k and +1.0 % on the packed 64k share (256 MiB, the
    // size of the last-level cache): there the copies come from a preparation of their own,
    // right before the key-outer pass, and the query-outer pass runs last.
    const bool dq_first = (size_t)2 * a.Hq * L.n_pad * D * 2 <= ((size_t)128 << 20);
    const float scale_log2 = a.scale * kLog2e;
    {
        BwdPrologue p;
        p.maps.j[0] = tile_map_job(a.S, n_loc, kDqBM, kDqBN, pa.cls, nullptr);
        p.maps.j[1] = tile_map_job(a.S, n_loc, kKvBM, kKvBN, pb.cls, nullptr);
        p.n_map_wgs = tile_map_workgroups(p.maps, 2);
        p.n_blocks = a.n_blocks;
        p.clean = clean; p.err = err;
        p.prep = BwdPrepArgs{(const ushort_t*)a.q, (const ushort_t*)o, (const ushort_t*)d_o, lse, a.bits,
                             a.blocks, a.block, a.Hq, a.S / a.block, n_loc, L.n_pad, 1.0f / a.scale,
                             ld, ldk, info, qh, doh};
        const int64_t threads = dq_first ? 0 : L.n_pad * a.Hq * (D / 8);
        const unsigned grid = p.n_map_wgs + 1u + (unsigned)((threads + 255) / 256);
        hipLaunchKernelGGL(bwd_prologue_kernel<D>, dim3(grid), dim3(256), 0, st, p);
        MM_LAUNCH_CHECK();
    }
    int rc = launch_compact_both(pa, pb, st);
    if (rc) return rc;
    // One query head per workgroup of four wavefronts and a two-stage ring: two such
    // workgroups share a CU with independent barriers.  Measured against a workgroup of
    // two heads (eight wavefronts sharing the K/V tiles, three or four stages, also with
    // the two heads' phases half a tile out of step): equal at 128k, 1 % to 4 % faster
    // elsewhere.
    auto run_dq = [&]() {
        stage_begin(MMATTN_STAGE_DQ, st);
        float* dq_part = (float*)(base + L.dq_part);
        if (dq_first)
            launch_dq_kernel<D, 1, 2>(a, o, lse, d_o, n_loc, L, scale_log2, clean, nullptr, pa, err, dq,
                                      dq_part, qh, doh, ldk, info, st);
        else
            launch_dq_kernel<D, 1, 2>(a, o, lse, d_o, n_loc, L, scale_log2, clean, ld, pa, err, dq,
                                      dq_part, nullptr, nullptr, nullptr, nullptr, st);
        if (L.split.cmax > 1) {
            const int64_t threads = n_loc * a.Hq * (D / 4);
            hipLaunchKernelGGL(dq_combine_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                               pa, L.split, n_loc, L.n_pad, a.Hq, D, err, dq_part, (ushort_t*)dq);
        }
        stage_end(MMATTN_STAGE_DQ, st);
    };
    if (dq_first) run_dq();
    {
        const dim3 grid((unsigned)((int64_t)(L.nk_b + L.n_extra) * a.Hkv * L.ch.cmax));
        const StageEvents& ev = g_stage_events[MMATTN_STAGE_DKV];
        if (ev.start && ev.stop) {
            // the dominant kernel's own begin and end times, when a caller asked for them: the
            // pair of events rides on the dispatch itself, with no extra packets on the stream
            // around the kernel (measured: 12 us per call less than two event records)
            hipExtLaunchKernelGGL(dkv_kernel<D>, grid, dim3(kKvThreads), 0, st, ev.start, ev.stop, 0,
                                  (const ushort_t*)qh, (const ushort_t*)a.k, (const ushort_t*)a.v,
                                  (const ushort_t*)doh, a.bits, clean, a.block, n_loc, L.n_pad, a.S, a.Hq,
                                  a.Hkv, a.scale, scale_log2, info, ldk, pb, L.ch, err, (ushort_t*)dk,
                                  (ushort_t*)dv, pool);
        } else {
            stage_begin(MMATTN_STAGE_DKV, st);
            hipLaunchKernelGGL(dkv_kernel<D>, grid, dim3(kKvThreads), 0, st, (const ushort_t*)qh,
                               (const ushort_t*)a.k, (const ushort_t*)a.v, (const ushort_t*)doh, a.bits, clean,
                               a.block, n_loc, L.n_pad, a.S, a.Hq, a.Hkv, a.scale, scale_log2, info, ldk, pb,
                               L.ch, err, (ushort_t*)dk, (ushort_t*)dv, pool);
            stage_end(MMATTN_STAGE_DKV, st);
        }
    }
    if (L.ch.cmax > 1 || L.n_extra > 0) {
        const int64_t tile_elems = (int64_t)kKvBN * a.Hkv * D;
        stage_begin(MMATTN_STAGE_DKV_REDUCE, st);
        hipLaunchKernelGGL(dkv_reduce_kernel, dim3((unsigned)L.nk_b, (unsigned)(tile_elems / kRedPerWg)),
                           dim3(256), 0, st, pb, a.Hkv, D, err, (const float*)pool, (ushort_t*)dk, (ushort_t*)dv);
        stage_end(MMATTN_STAGE_DKV_REDUCE, st);
    }
    if (!dq_first) run_dq();
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

int launch_bwd(const AttnArgs& a, const void* o, const float* lse, const void* d_o, void* dq,
               void* dk, void* dv, void* ws, hipStream_t st) {
    if (a.D == 128) return launch_bwd_d<128>(a, o, lse, d_o, dq, dk, dv, ws, st);
    return launch_bwd_d<64>(a, o, lse, d_o, dq, dk, dv, ws, st);
}

}  // namespace mm
