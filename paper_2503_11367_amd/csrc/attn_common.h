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

// position p (0..15) inside a stored group of 16  ->  logical index
__host__ __device__ inline int perm16_index_of_pos(int p) {
    return p < 4 ? p : (p < 8 ? p + 4 : (p < 12 ? p - 4 : p));
}

// row of a 32x32 C tile held in register r by a lane of half hh
__device__ __forceinline__ int c_row(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

// ---- LDS tiles filled by direct global->LDS loads ------------------------------
// global_load_lds_dwordx4 writes lane l's 16 bytes at (wave-uniform base) + 16*l,
// so a tile cannot be padded; instead every 256-byte "super-row" R (one row for
// D=128, two rows for D=64) is rotated: its 16-byte chunk c' sits at position
// (c' + ROT*R) & 15.  The bank of every element is then the same as in a padded
// layout of pitch 256+16*ROT bytes: ROT=1 makes 16-byte row-fragment reads
// conflict free, ROT=4 the transpose reads (LDS: 64 banks of 4 B for these widths).
template <int D, int ROT>
struct SwzTile {
    static constexpr int RB = D * 2;          // bytes per row
    static constexpr int CPR = RB / 16;       // 16-byte chunks per row
    static constexpr int RPS = 256 / RB;      // rows per super-row
    // byte offset of chunk c of row r
    __device__ static __forceinline__ int byte_of(int r, int c) {
        const int R = r / RPS, cp = (r % RPS) * CPR + c;
        return R * 256 + (((cp + ROT * R) & 15) << 4);
    }
    // (row, chunk) stored at position p of super-row R
    __device__ static __forceinline__ void src_of(int R, int p, int& r, int& c) {
        const int cp = (p - ROT * R) & 15;
        r = R * RPS + cp / CPR;
        c = cp % CPR;
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
                 : "memory");
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
constexpr uint32_t kPartialFlag = 0x80000000u;

struct TilePlan {
    int32_t nq, nk, tq, tk;
    uint8_t* cls;
    int32_t* kcount;
    uint32_t* klist;
    int32_t* qorder;
};

// transposed plan for key-outer kernels: for each k-tile the active q-tiles
struct TilePlanT {
    int32_t nq, nk, tq, tk;
    uint8_t* cls;
    int32_t* qcount;     // [nk]
    uint32_t* qlist;     // [nk][nq]
    int32_t* korder;     // [nk] by qcount descending
};

int launch_transpose_perm(const void* x, void* xt, int64_t n, int64_t n_pad, int32_t H, int32_t D,
                          hipStream_t st);
int launch_compact_rows(const TilePlan& p, hipStream_t st);
int launch_compact_cols(const TilePlanT& p, hipStream_t st);
int launch_validate_blocks(const int32_t* blocks, int32_t n_blocks, int64_t n_seq_blocks,
                           int32_t* clean, int32_t* err, hipStream_t st);

}  // namespace mm
