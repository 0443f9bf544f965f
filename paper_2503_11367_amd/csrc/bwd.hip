// mmattn_bwd: backward of the multimodal-masked attention for one rank's query
// blocks (training needs it: the paper's iteration is one forward and one
// backward pass; the attention definition is the one section 3.2.2 / 4.3 rely
// on).  With P = exp(S - LSE), Delta = rowsum(dO o O), dS = P o (dP - Delta):
//   dV = P^T dO,  dK = scale dS^T Q   (sums over this rank's rows and over the
//                                      Hq/Hkv query heads of the KV head)
//   dQ = scale dS K
// Three launches, deterministic (no atomics):
//   delta_kernel   Delta and LSE in base-2 units;
//   dkv_kernel     key-outer: a workgroup owns 128 keys of one KV head (32 per
//                  wavefront), keeps dK^T/dV^T accumulators and its K/V
//                  fragments in registers and streams the active 32-row query
//                  tiles of every head of the group through LDS;
//   dq_kernel      query-outer, same shape as the forward kernel.
// All contractions are 32x32x16 bf16 MFMAs; tiles that need a transposed
// operand are read with ds_read_b64_tr_b16 from a row-major copy whose pitch
// suits that access pattern.
#include <type_traits>
#include "attn_common.h"

namespace mm {

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef shortx4 __attribute__((address_space(3))) * lds_s4;

// A-operand fragment (32 rows of the transposed tile x 16 contraction indices)
// read from a row-major [contraction index][row] tile: two transpose reads.
__device__ __forceinline__ bf16x8 read_tr_frag(const ushort_t* p, int pitch) {
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)p);
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(p + 8 * pitch));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// ---------------------------------------------------------------- delta ------
// One thread per 8 elements; D/8 consecutive lanes reduce one (row, head).
template <int D>
__global__ void __launch_bounds__(256)
delta_kernel(const ushort_t* __restrict__ O, const ushort_t* __restrict__ dO,
             const float* __restrict__ lse, int64_t n_loc, int32_t Hq,
             float* __restrict__ delta, float* __restrict__ lse2) {
    constexpr int TPR = D / 8;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t rh = gid / TPR;                       // row*Hq + h
    const int c = (int)(gid % TPR);
    float acc = 0.f;
    const bool ok = rh < n_loc * Hq;
    if (ok) {
        const u32x4 a = *(const u32x4*)(O + rh * D + c * 8);
        const u32x4 b = *(const u32x4*)(dO + rh * D + c * 8);
        const bf16x8 x = __builtin_bit_cast(bf16x8, a), y = __builtin_bit_cast(bf16x8, b);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (float)x[u] * (float)y[u];
    }
#pragma unroll
    for (int off = TPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (ok && c == 0) {
        const int64_t row = rh / Hq;
        const int h = (int)(rh % Hq);
        delta[(int64_t)h * n_loc + row] = acc;
        lse2[(int64_t)h * n_loc + row] = lse[(int64_t)h * n_loc + row] * kLog2e;
    }
}

// ---------------------------------------------------------------- dK / dV ----
constexpr int kKvBN = 128;      // keys per workgroup
constexpr int kKvBM = 32;       // query rows per step
constexpr int kKvThreads = 256;

template <int D>
struct KvSmem {
    static constexpr int NP = D + 8;      // pitch for row-fragment reads
    static constexpr int TP = D + 32;     // pitch for transpose reads
    ushort_t q[kKvBM * NP];
    ushort_t qt[kKvBM * TP];
    ushort_t d[kKvBM * NP];
    ushort_t dt[kKvBM * TP];
    float lse2[kKvBM];
    float delta[kKvBM];
    uint32_t q_ss[kKvBM];
    uint32_t q_causal[kKvBM];
    int32_t q_pos[kKvBM];
};

template <int D>
__global__ void __launch_bounds__(kKvThreads, 2)
dkv_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
           const ushort_t* __restrict__ V, const ushort_t* __restrict__ dO,
           const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
           int64_t n_loc, int64_t S, int32_t Hq, int32_t Hkv, float scale, float scale_log2,
           const float* __restrict__ lse2, const float* __restrict__ delta, TilePlanT plan,
           const int32_t* __restrict__ err, ushort_t* __restrict__ dK, ushort_t* __restrict__ dV) {
    constexpr int NDS = D / 16, NDB = D / 32;
    constexpr int NP = KvSmem<D>::NP, TP = KvSmem<D>::TP;
    __shared__ KvSmem<D> sm;
    if (*err) return;

    const int rep = Hq / Hkv;
    int tile_rank, g;
    {
        const int bid = blockIdx.x;
        if (Hkv % 8 == 0) {
            const int x = bid & 7, slot = bid >> 3, gx = Hkv / 8;
            tile_rank = slot / gx;
            g = x + 8 * (slot - tile_rank * gx);
        } else {
            tile_rank = bid / Hkv;
            g = bid - tile_rank * Hkv;
        }
    }
    const int kt = plan.korder[tile_rank];
    const int n_q = plan.qcount[kt];
    const uint32_t* qlist = plan.qlist + (int64_t)kt * plan.nq;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, hh = lane >> 5;

    // this lane's key: position, mask fields, K and V fragments (B operands)
    const int64_t key = (int64_t)kt * kKvBN + wave * 32 + li;
    const uint32_t k_ss = word_ss(bits[key]);
    bf16x8 kf[NDS], vf[NDS];
    {
        const int64_t off = (key * Hkv + g) * (int64_t)D + hh * 8;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            kf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(K + off + ds * 16));
            vf[ds] = __builtin_bit_cast(bf16x8, *(const u32x4*)(V + off + ds * 16));
        }
    }
    floatx16 dk[NDB], dv[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk[db][r] = 0.f; dv[db][r] = 0.f; }

    // staging: 32 rows x D of Q and dO -> 2 * 32 * D/8 chunks of 16 B
    constexpr int CH = D / 8;
    constexpr int NLD = (kKvBM * CH + kKvThreads - 1) / kKvThreads;   // per tensor per thread
    u32x4 qreg[NLD], dreg[NLD];
    float lreg = 0.f, dlreg = 0.f;
    uint32_t ssreg = 0, careg = 0;
    int32_t posreg = 0;
    const int n_steps = n_q * rep;

    auto load_step = [&](int step) {
        const int hq = g * rep + step / n_q;
        const int64_t r0 = (int64_t)(qlist[step % n_q] & ~kPartialFlag) * kKvBM;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * kKvThreads;
            const int r = c / CH, cc = c % CH;
            qreg[i] = u32x4{0u, 0u, 0u, 0u};
            dreg[i] = u32x4{0u, 0u, 0u, 0u};
            if (c < kKvBM * CH && r0 + r < n_loc) {
                const int64_t off = ((r0 + r) * Hq + hq) * (int64_t)D + cc * 8;
                qreg[i] = *(const u32x4*)(Q + off);
                dreg[i] = *(const u32x4*)(dO + off);
            }
        }
        if (tid < kKvBM) {
            const int64_t r = r0 + tid;
            if (r < n_loc) {
                lreg = lse2[(int64_t)hq * n_loc + r];
                dlreg = delta[(int64_t)hq * n_loc + r];
                const int64_t p = row_pos(blocks, block, r);
                const uint64_t w = bits[p];
                ssreg = word_ss(w);
                careg = word_causal(w);
                posreg = (int32_t)p;
            } else {
                lreg = INFINITY;        // exp2(s - inf) = 0: padded rows contribute nothing
                dlreg = 0.f;
                ssreg = 0xFFFFFFFFu; careg = 0; posreg = -1;
            }
        }
    };
    auto store_step = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * kKvThreads;
            const int r = c / CH, cc = c % CH;
            if (c < kKvBM * CH) {
                *(u32x4*)(sm.q + r * NP + cc * 8) = qreg[i];
                *(u32x4*)(sm.qt + r * TP + cc * 8) = qreg[i];
                *(u32x4*)(sm.d + r * NP + cc * 8) = dreg[i];
                *(u32x4*)(sm.dt + r * TP + cc * 8) = dreg[i];
            }
        }
        if (tid < kKvBM) {
            sm.lse2[tid] = lreg; sm.delta[tid] = dlreg;
            sm.q_ss[tid] = ssreg; sm.q_causal[tid] = careg; sm.q_pos[tid] = posreg;
        }
    };

    const int a_off = li * NP + hh * 8;                       // row-fragment reads
    const int s16 = lane & 15, grp = lane >> 4;
    const int t_off = (4 * hh + s16 / 4) * TP + 16 * (grp & 1) + 4 * (s16 & 3);

    if (n_steps > 0) load_step(0);
    for (int step = 0; step < n_steps; ++step) {
        const bool partial = (qlist[step % n_q] & kPartialFlag) != 0;
        __syncthreads();
        store_step();
        __syncthreads();
        if (step + 1 < n_steps) load_step(step + 1);

        // S = Q K^T and dP = dO V^T : rows = the step's 32 queries, columns = my 32 keys
        floatx16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            const bf16x8 aq = __builtin_bit_cast(bf16x8, *(const u32x4*)(sm.q + a_off + ds * 16));
            s = mfma32(aq, kf[ds], s);
        }
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            const bf16x8 ad = __builtin_bit_cast(bf16x8, *(const u32x4*)(sm.d + a_off + ds * 16));
            dp = mfma32(ad, vf[ds], dp);
        }
        bf16x8 pf[2], dsf[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int qr = c_row(r, hh);
            float p = __builtin_amdgcn_exp2f(s[r] * scale_log2 - sm.lse2[qr]);
            if (partial && !visible(sm.q_ss[qr], sm.q_causal[qr], sm.q_pos[qr], k_ss, key)) p = 0.f;
            const float dsv = p * (dp[r] - sm.delta[qr]);
            pf[r >> 3][r & 7] = (__bf16)p;
            dsf[r >> 3][r & 7] = (__bf16)dsv;
        }
        // dV^T += dO^T P ;  dK^T += Q^T dS
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const bf16x8 ad = read_tr_frag(sm.dt + t_off + ks * 16 * TP + db * 32, TP);
                dv[db] = mfma32(ad, pf[ks], dv[db]);
                const bf16x8 aq = read_tr_frag(sm.qt + t_off + ks * 16 * TP + db * 32, TP);
                dk[db] = mfma32(aq, dsf[ks], dk[db]);
            }
    }

    // epilogue: lane holds key `key`, 4 consecutive d per register quad
    ushort_t* kp = dK + (key * Hkv + g) * (int64_t)D + 4 * hh;
    ushort_t* vp = dV + (key * Hkv + g) * (int64_t)D + 4 * hh;
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
            *(u32x2*)(kp + db * 32 + c * 8) = __builtin_bit_cast(u32x2, ok);
            *(u32x2*)(vp + db * 32 + c * 8) = __builtin_bit_cast(u32x2, ov);
        }
}

// ---------------------------------------------------------------- dQ ---------
constexpr int kDqBM = 128, kDqBN = 64, kDqThreads = 256;

template <int D>
struct DqSmem {
    static constexpr int NP = D + 8, TP = D + 32;
    ushort_t k[kDqBN * NP];
    ushort_t kt[kDqBN * TP];
    ushort_t v[kDqBN * NP];
    uint32_t kss[kDqBN];
};

template <int D>
__global__ void __launch_bounds__(kDqThreads, 2)
dq_kernel(const ushort_t* __restrict__ Q, const ushort_t* __restrict__ K,
          const ushort_t* __restrict__ V, const ushort_t* __restrict__ dO,
          const uint64_t* __restrict__ bits, const int32_t* __restrict__ blocks, int32_t block,
          int64_t n_loc, int64_t S, int32_t Hq, int32_t Hkv, float scale, float scale_log2,
          const float* __restrict__ lse2, const float* __restrict__ delta, TilePlan plan,
          const int32_t* __restrict__ err, ushort_t* __restrict__ dQ) {
    constexpr int NDS = D / 16, NDB = D / 32;
    constexpr int NP = DqSmem<D>::NP, TP = DqSmem<D>::TP;
    __shared__ DqSmem<D> sm;
    if (*err) return;

    const int rep = Hq / Hkv;
    int tile_rank, h;
    {
        const int bid = blockIdx.x;
        if (Hkv % 8 == 0) {
            const int x = bid & 7, slot = bid >> 3, hx = Hq / 8;
            tile_rank = slot / hx;
            const int e = slot - tile_rank * hx;
            h = (x + 8 * (e / rep)) * rep + e % rep;
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

    const int64_t row = (int64_t)qt * kDqBM + wave * 32 + li;
    const bool row_ok = row < n_loc;
    int64_t q_pos = 0;
    uint32_t q_ss = 0, q_causal = 0;
    float my_lse2 = INFINITY, my_delta = 0.f;
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
        my_lse2 = lse2[(int64_t)h * n_loc + row];
        my_delta = delta[(int64_t)h * n_loc + row];
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

    constexpr int CH = D / 8;
    constexpr int NLD = kDqBN * CH / kDqThreads;
    u32x4 kreg[NLD], vreg[NLD];
    uint32_t kssreg = 0;
    auto load_tile = [&](int it) {
        const int64_t k0 = (int64_t)(klist[it] & ~kPartialFlag) * kDqBN;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * kDqThreads, r = c / CH, cc = c % CH;
            const int64_t off = ((k0 + r) * Hkv + g) * (int64_t)D + cc * 8;
            kreg[i] = *(const u32x4*)(K + off);
            vreg[i] = *(const u32x4*)(V + off);
        }
        if (tid < kDqBN) kssreg = word_ss(bits[k0 + tid]);
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * kDqThreads, r = c / CH, cc = c % CH;
            *(u32x4*)(sm.k + r * NP + cc * 8) = kreg[i];
            *(u32x4*)(sm.kt + r * TP + cc * 8) = kreg[i];
            *(u32x4*)(sm.v + r * NP + cc * 8) = vreg[i];
        }
        if (tid < kDqBN) sm.kss[tid] = kssreg;
    };

    const int a_off = li * NP + hh * 8;
    const int s16 = lane & 15, grp = lane >> 4;
    const int t_off = (4 * hh + s16 / 4) * TP + 16 * (grp & 1) + 4 * (s16 & 3);

    if (n_active > 0) load_tile(0);
    for (int it = 0; it < n_active; ++it) {
        const uint32_t entry = klist[it];
        const bool partial = (entry & kPartialFlag) != 0;
        const int64_t k0 = (int64_t)(entry & ~kPartialFlag) * kDqBN;
        __syncthreads();
        store_tile();
        __syncthreads();
        if (it + 1 < n_active) load_tile(it + 1);

        bf16x8 dsf[4];
        auto half = [&](auto KB) __attribute__((always_inline)) {
            constexpr int kb = decltype(KB)::value;
            floatx16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds) {
                const bf16x8 ak = __builtin_bit_cast(
                    bf16x8, *(const u32x4*)(sm.k + kb * 32 * NP + a_off + ds * 16));
                s = mfma32(ak, qf[ds], s);
            }
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds) {
                const bf16x8 av = __builtin_bit_cast(
                    bf16x8, *(const u32x4*)(sm.v + kb * 32 * NP + a_off + ds * 16));
                dp = mfma32(av, dof[ds], dp);
            }
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
            for (int db = 0; db < NDB; ++db) {
                const bf16x8 a = read_tr_frag(sm.kt + t_off + ks * 16 * TP + db * 32, TP);
                dq[db] = mfma32(a, dsf[ks], dq[db]);
            }
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
    size_t err, clean_blocks, delta, lse2, cls_a, kcount, klist, qorder, cls_b, qcount, qlist,
        korder, total;
    int32_t nq_a, nk_a, nq_b, nk_b;
};

static BwdLayout bwd_layout(int64_t S, int64_t n_loc, int32_t n_blocks, int32_t Hq) {
    BwdLayout L;
    L.nq_a = (int32_t)((n_loc + kDqBM - 1) / kDqBM);
    L.nk_a = (int32_t)(S / kDqBN);
    L.nq_b = (int32_t)((n_loc + kKvBM - 1) / kKvBM);
    L.nk_b = (int32_t)(S / kKvBN);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    L.err = take(256);
    L.clean_blocks = take((size_t)n_blocks * 4);
    L.delta = take((size_t)Hq * n_loc * 4);
    L.lse2 = take((size_t)Hq * n_loc * 4);
    L.cls_a = take((size_t)L.nq_a * L.nk_a);
    L.kcount = take((size_t)L.nq_a * 4);
    L.klist = take((size_t)L.nq_a * L.nk_a * 4);
    L.qorder = take((size_t)L.nq_a * 4);
    L.cls_b = take((size_t)L.nq_b * L.nk_b);
    L.qcount = take((size_t)L.nk_b * 4);
    L.qlist = take((size_t)L.nq_b * L.nk_b * 4);
    L.korder = take((size_t)L.nk_b * 4);
    L.total = off;
    return L;
}

size_t bwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D) {
    (void)Hkv; (void)D;
    return bwd_layout(S, n_loc, (int32_t)(n_loc / 16 + 1), Hq).total;
}

template <int D>
static int launch_bwd_d(const AttnArgs& a, const void* o, const float* lse, const void* d_o,
                        void* dq, void* dk, void* dv, void* ws, hipStream_t st) {
    const int64_t n_loc = (int64_t)a.n_blocks * a.block;
    const BwdLayout L = bwd_layout(a.S, n_loc, (int32_t)(n_loc / 16 + 1), a.Hq);
    char* base = (char*)ws;
    int32_t* err = (int32_t*)(base + L.err);
    int32_t* clean = (int32_t*)(base + L.clean_blocks);
    float* delta = (float*)(base + L.delta);
    float* lse2 = (float*)(base + L.lse2);
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
        const int64_t threads = n_loc * a.Hq * (D / 8);
        hipLaunchKernelGGL(delta_kernel<D>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           (const ushort_t*)o, (const ushort_t*)d_o, lse, n_loc, a.Hq, delta, lse2);
    }
    stage_begin(MMATTN_STAGE_DKV, st);
    hipLaunchKernelGGL(dkv_kernel<D>, dim3((unsigned)((int64_t)L.nk_b * a.Hkv)), dim3(kKvThreads), 0,
                       st, (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v,
                       (const ushort_t*)d_o, a.bits, clean, a.block, n_loc, a.S, a.Hq, a.Hkv, a.scale,
                       scale_log2, lse2, delta, pb, err, (ushort_t*)dk, (ushort_t*)dv);
    stage_end(MMATTN_STAGE_DKV, st);
    stage_begin(MMATTN_STAGE_DQ, st);
    hipLaunchKernelGGL(dq_kernel<D>, dim3((unsigned)((int64_t)L.nq_a * a.Hq)), dim3(kDqThreads), 0, st,
                       (const ushort_t*)a.q, (const ushort_t*)a.k, (const ushort_t*)a.v,
                       (const ushort_t*)d_o, a.bits, clean, a.block, n_loc, a.S, a.Hq, a.Hkv, a.scale,
                       scale_log2, lse2, delta, pa, err, (ushort_t*)dq);
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
