// Device-side building blocks shared by the forward and backward attention
// kernels: MFMA fragment types for gfx950, the tile-plan structures the prep
// kernels write into the workspace, and the layout conventions.
//
// MFMA used: v_mfma_f32_32x32x16_bf16 (C[32x32] += A[32x16] * B[16x32]).
//   lane l, half hh = l/32, i = l%32
//   A operand: row i,    k = 8*hh .. 8*hh+7        (8 bf16 per lane)
//   B operand: column i, k = 8*hh .. 8*hh+7
//   C/D:       column i, rows 8*(r/4) + 4*hh + r%4  for r = 0..15
// A contraction index may be permuted freely as long as A and B agree; the
// kernels feed a C tile straight back as a B operand, which fixes the
// permutation  slot s of half hh  <->  index 4*hh + s (s<4), 8 + 4*hh + s-4.
// Operands read from "transposed" tiles therefore store each group of 16
// contraction indices in the order [0..3, 8..11, 4..7, 12..15] (kPerm16), so a
// lane's 8 values are 16 contiguous bytes.
#pragma once
#include "common.h"

namespace mm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned short ushort_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// row of a 32x32 C tile held in register r by a lane of half hh
__device__ __forceinline__ int c_row(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

// ---- LDS tiles filled by direct global->LDS loads ------------------------------
// global_load_lds_dwordx4 writes lane l's 16 bytes at (wave-uniform base) + 16*l,
// so a tile cannot be padded; instead every 256-byte "super-row" R (one row for
// D=128, two rows for D=64) is rotated: its 16-byte chunk c' sits at position
// (c' + rot(R)) & 15.  Measured on gfx950 (LDS conflict counters): 16-byte
// row-fragment reads are conflict free when 16 consecutive rows get 16 distinct
// rotations; transpose reads (4 rows x 64 B per pass) when 4 consecutive rows
// are a quarter of the banks apart.
//   MODE 1: rot = R        row fragments only            (like a 272-byte pitch)
//   MODE 4: rot = 4R       transpose reads only          (like a 320-byte pitch)
//   MODE 0: rot = ((R&3)<<2) | ((R>>2)&3)   both access patterns
template <int D, int MODE>
struct SwzTile {
    static constexpr int RB = D * 2;          // bytes per row
    static constexpr int CPR = RB / 16;       // 16-byte chunks per row
    static constexpr int RPS = 256 / RB;      // rows per super-row
    __device__ static __forceinline__ int rot(int R) {
        return MODE == 1 ? R : (MODE == 4 ? 4 * R : (((R & 3) << 2) | ((R >> 2) & 3)));
    }
    // byte offset of chunk c of row r
    __device__ static __forceinline__ int byte_of(int r, int c) {
        const int R = r / RPS, cp = (r % RPS) * CPR + c;
        return R * 256 + (((cp + rot(R)) & 15) << 4);
    }
    // (row, chunk) stored at position p of super-row R
    __device__ static __forceinline__ void src_of(int R, int p, int& r, int& c) {
        const int cp = (p - rot(R)) & 15;
        r = R * RPS + cp / CPR;
        c = cp % CPR;
    }
};

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef shortx4 __attribute__((address_space(3))) * lds_s4;
typedef const u32x4 __attribute__((address_space(3))) * lds_u4;
typedef const uint32_t __attribute__((address_space(3))) * lds_u1;

// Per-lane LDS byte offsets of MFMA operand fragments inside a SwzTile, computed
// once.  The rotation repeats every 16 super-rows, so row offsets that are
// multiples of PER = 16*RPS rows are plain address increments (immediates).
//
// Row fragments: operand row `li` (+ a multiple of 32 rows), elements
// 16*ds + 8*hh .. +7.
template <class Tile, int D>
struct RowFragAddr {
    static constexpr int NDS = D / 16;
    int off[NDS];
    __device__ __forceinline__ void init(int lane) {
        const int li = lane & 31, hh = lane >> 5;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) off[ds] = Tile::byte_of(li, 2 * ds + hh);
    }
    // rows32: which block of 32 rows (compile-time constant after unrolling)
    __device__ __forceinline__ bf16x8 read(const unsigned char* tile, int rows32, int ds) const {
        return __builtin_bit_cast(bf16x8, *(const u32x4*)(tile + rows32 * 32 * Tile::RB + off[ds]));
    }
};

// Fragments of the TRANSPOSE of a row-major tile (A operand whose contraction
// index runs over the tile's rows): 32 columns db*32.. x 16 rows ks*16.., rows in
// the permutation that matches a C tile fed back as B operand.  Two transpose
// reads (rows +0 and +8).
template <class Tile, int D>
struct TrFragAddr {
    static constexpr int NDB = D / 32;
    static constexpr int PER = 16 * Tile::RPS;      // rows after which the rotation repeats
    static constexpr int NV = PER / 8;              // distinct 8-row offsets inside a period
    int off[NDB][NV];
    __device__ __forceinline__ void init(int lane) {
        const int hh = lane >> 5, s16 = lane & 15, grp = (lane >> 4) & 1;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int row = v * 8 + 4 * hh + (s16 >> 2);
                const int col = db * 32 + 16 * grp + 4 * (s16 & 3);
                off[db][v] = Tile::byte_of(row, col >> 3) + (col & 7) * 2;
            }
    }
    __device__ __forceinline__ bf16x8 read(const unsigned char* tile, int ks, int db) const {
        const int r_lo = ks * 16, r_hi = ks * 16 + 8;            // compile-time after unrolling
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s4)(tile + (r_lo / PER) * PER * Tile::RB + off[db][(r_lo % PER) / 8]));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s4)(tile + (r_hi / PER) * PER * Tile::RB + off[db][(r_hi % PER) / 8]));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
};

// One wave-wide 1 KiB transfer: lane l's 16 bytes at base + off land in LDS at
// lds_addr + 16*l (base and lds_addr wave-uniform; lds_addr goes through M0).
// Issued as inline asm so the compiler's wait-count pass does not treat every
// later LDS read as dependent on it; completion is awaited explicitly with
// wait_vmcnt<N>() before the barrier that publishes the tile.  Vector loads
// retire in order, so "at most N outstanding" means everything issued before
// the last N has landed; waits the compiler inserts for its own vector loads can
// only be stricter than needed.
__device__ __forceinline__ void dma16(const void* base_uniform, uint32_t off, uint32_t lds_addr) {
    const uint64_t b = (uint64_t)base_uniform;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const uint64_t sb = ((uint64_t)hi << 32) | lo;
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(off), "s"(sb), "s"(lds_addr)
                 : "memory", "m0");
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
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// wait until at most N of this wave's vector-memory loads (incl. LDS transfers) are outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Tile plan of one rank share, built by the prep kernels.
//   q-tiles of tq local rows (last one ragged), k-tiles of tk keys
//   cls[nq][nk]              MMATTN_TILE_*
//   klist[nq][nk], kcount[nq]  active k-tiles of each q-tile, ascending;
//                            entry = k-tile index | (PARTIAL ? kPartialFlag : 0)
//   qorder[nq]               q-tiles by kcount descending (longest first)
//   csz[1]                   slice length the list builder suggests for cutting the
//                            lists into slices (see list_split), from the actual lengths
constexpr uint32_t kPartialFlag = 0x80000000u;

struct TilePlan {
    int32_t nq, nk, tq, tk;
    uint8_t* cls;
    int32_t* kcount;
    uint32_t* klist;
    int32_t* qorder;
    int32_t* csz;
    int32_t groups;      // workgroups per q-tile (head groups) of the launch the plan is built for
};

// slices of a q-tile's active k-tile list: the launch provides cmax slices per q-tile,
// so a slice has at least csz list entries; cmax == 1 means the lists are not split
struct FwdSplit {
    int32_t cmax, csz;
};
// Intra-GPU balancing (paper section 3.2.2) for the query-outer kernels: when a share
// has too few (q-tile, head group) work items to fill the chip, every q-tile's active
// k-tile list is cut into slices that run as separate workgroups and write partial
// results, aggregated by one more launch.  The host fixes how many slices a q-tile may
// have (grid size, partial buffers): two to four times (short / long sequences; unused
// slices are workgroups that exit at once, about 4 us per thousand) what lists of full
// length would need for about 1024 workgroups.  The slice length itself is chosen on the device from the
// actual list lengths (slice_length below) and is never shorter than csz.
// `groups`: workgroups per q-tile (head groups).
inline FwdSplit list_split(int32_t nq, int32_t nk, int32_t groups) {
    const int64_t items = (int64_t)nq * groups;
    int64_t cmax = 1;
    if (items < 512) {
        cmax = (nk >= 512 ? 4 : 2) * ((1024 + items - 1) / items);
        const int64_t most = nk / 2 > 1 ? nk / 2 : 1;         // at least two tiles per slice
        if (cmax > most) cmax = most;
        if (cmax > 64) cmax = 64;
    }
    FwdSplit sp;
    sp.csz = (int32_t)((nk + cmax - 1) / cmax);
    sp.cmax = (nk + sp.csz - 1) / sp.csz;                     // no empty trailing slices
    return sp;
}
// Slice length from the lists themselves (total entries, longest list, non-empty
// lists; `groups` workgroups walk every list).
//   Lists of about equal length: a quarter of one CU's share of all entries, i.e. about
//   1024 equal slices, which the 256 CUs finish in whole rounds.
//   Uneven lists: the slices that finish last cost about one slice of time, while every
//   slice costs a fixed amount of bandwidth for its partial result (worth about 1/32 of
//   a tile's time across the chip); c + W/(32 c) is smallest at c = sqrt(W/32).
// At least 8 tiles, at most the whole list.
__host__ __device__ inline int32_t slice_length(int64_t total, int32_t longest, int32_t lists,
                                                int32_t groups, int32_t nk) {
    const int64_t work = total * groups;
    int64_t c;
    if ((int64_t)longest * lists * 4 <= total * 5) {          // longest <= 1.25 x mean
        c = (work + 1023) / 1024;
    } else {
        c = (int64_t)__builtin_sqrtf((float)work / 32.0f) + 1;
    }
    if (c < 8) c = 8;
    if (c > nk) c = nk;
    return (int32_t)c;
}

// transposed plan for key-outer kernels: for each k-tile the active q-tiles
struct TilePlanT {
    int32_t nq, nk, tq, tk;
    uint8_t* cls;
    int32_t* qcount;     // [nk]
    uint32_t* qlist;     // [nk][nq]
    int32_t* korder;     // [nk] by qcount descending
    // list slices (intra-GPU balancing, paper section 3.2.2, for the key-outer pass): a
    // k-tile whose list is much longer than a CU's share of all the work is cut into
    // slices of `slicing[kSliceLen]` entries that run as separate workgroups and write
    // partial sums.  Chosen on the device (by the list builder) from the lists themselves.
    int32_t n_extra;     // host: most slices beyond the first, over all k-tiles (grid, table size)
    int32_t hc, hpc;     // host: workgroups per (k-tile, KV head, slice) and query heads of each
    int32_t groups;      // host: workgroups that walk every list (KV heads x hc)
    int32_t* slicing;    // [kSliceInts]: slice length, sliced k-tiles, extra slices in use
    int32_t* pbase;      // [nk] first partial-sum slot of the k-tile, -1: written directly
    int32_t* extra;      // [n_extra][2] (k-tile, slice index >= 1) by k-tile, then slice
};
constexpr int kSliceLen = 0, kSlicedTiles = 1, kExtraUsed = 2, kSliceInts = 4;

// The kFlagInts int32 words at `err` (cleared by validate_blocks_body) are the error flag and
// spare words; the word after them holds the slice length chosen by the list builder.
int launch_compact_rows(const TilePlan& p, hipStream_t st);
int launch_compact_cols(const TilePlanT& p, hipStream_t st);
int launch_compact_both(const TilePlan& pa, const TilePlanT& pb, hipStream_t st);

}  // namespace mm
