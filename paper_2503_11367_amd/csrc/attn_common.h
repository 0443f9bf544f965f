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
