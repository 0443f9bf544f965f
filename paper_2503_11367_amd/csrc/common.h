// Internal helpers shared by the HIP translation units of libmmattn.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "mmattn.h"

#define MM_HIP_TRY(expr)                                        \
    do {                                                        \
        hipError_t e_ = (expr);                                 \
        if (e_ != hipSuccess) return MMATTN_ERR_HIP;            \
    } while (0)

#define MM_LAUNCH_CHECK()                                       \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return MMATTN_ERR_HIP; \
    } while (0)

namespace mm {

constexpr int kWave = 64;

// Mask word fields (paper section 4.2 layout as fixed in mmattn.h).
constexpr int kSpanShift = 12;
constexpr int kSampleShift = 28;
constexpr int kWindowShift = 44;
constexpr int kCausalBit = 63;

// Compact views used by the kernels.  `ss`: low 16 bits span id, next 16 bits
// sample id; equal `ss` words mean same sample AND same span.  Key side `mod`:
// the token's own modality (bits 8-11 of the word); values above 7 have no attend
// bit and count as 8.  Query side `att`: 0 without the causal bit, else the
// attend-set (bits 0-7; bits 8-11 stay zero, so modality 8 is never attended), the
// own modality (bits 12-15) and the look-back window (bits 16-31).
__host__ __device__ inline uint32_t word_ss(uint64_t w) { return (uint32_t)(w >> kSpanShift); }
__host__ __device__ inline uint32_t word_mod(uint64_t w) {
    const uint32_t m = (uint32_t)(w >> 8) & 0xFu;
    return m < 8u ? m : 8u;
}
__host__ __device__ inline uint32_t word_att(uint64_t w) {
    if (!(w >> kCausalBit)) return 0u;
    return (uint32_t)(w & 0xFFu) | (word_mod(w) << 12) | ((uint32_t)(w >> kWindowShift) << 16);
}
__host__ __device__ inline uint32_t att_window(uint32_t att) { return att >> 16; }
__host__ __device__ inline uint32_t att_modality(uint32_t att) { return (att >> 12) & 0xFu; }

// vis(q,k) = same_sample && ((causal(q) && k<=q && attend(q)[modality(k)] &&
//                             (window(q)==0 || modality(k)!=modality(q) || q-k<window(q))) ||
//                            (span(q)!=0 && span(q)==span(k)))
__device__ __forceinline__ bool visible(uint32_t ss_q, uint32_t att_q, int64_t q,
                                        uint32_t ss_k, uint32_t mod_k, int64_t k) {
    const bool same_sample = (ss_q >> 16) == (ss_k >> 16);
    const bool same_span = (ss_q & 0xFFFFu) != 0 && ss_q == ss_k;
    const bool attends = (att_q >> mod_k) & 1u;
    // positions are below 2^31, so 32-bit arithmetic serves: k <= q  <=>  the 32-bit
    // difference is below 2^31.  Farthest visible look-back: window - 1 for keys of the own
    // modality (no window: 0 - 1 wraps to the maximum), unlimited otherwise
    const uint32_t back = (uint32_t)q - (uint32_t)k;
    const uint32_t reach = mod_k == att_modality(att_q) ? att_window(att_q) - 1u : 0x7FFFFFFFu;
    return same_span || (same_sample && attends && back <= min(reach, 0x7FFFFFFFu));
}

// A stretch of n consecutive keys, the first at position k_first, that all carry the
// fields (ss_k, mod_k): the keys a query sees among them are one contiguous range (the whole
// stretch for its own span; else the keys up to its position, from the start of its
// look-back window on, if it looks back at that modality in its sample).  Key index idx in
// 0..n-1 is visible iff (uint32_t)(idx - lo) <= last; an empty range has lo far past n.
struct KeyRange {
    uint32_t lo, last;
    __device__ __forceinline__ bool sees(uint32_t idx) const { return idx - lo <= last; }
    __device__ __forceinline__ bool all_of(int n) const { return lo == 0u && last == (uint32_t)(n - 1); }
};
__device__ __forceinline__ KeyRange visible_range(uint32_t ss_q, uint32_t att_q, int32_t q, uint32_t ss_k,
                                                  uint32_t mod_k, int32_t k_first, int32_t n) {
    const bool same_sample = (ss_q >> 16) == (ss_k >> 16);
    const bool same_span = (ss_q & 0xFFFFu) != 0 && ss_q == ss_k;
    const bool attends = (att_q >> mod_k) & 1u;
    const int32_t rel = q - k_first;                       // index of the last key at or before the query
    const int32_t win = (int32_t)att_window(att_q);
    const bool windowed = win != 0 && mod_k == att_modality(att_q);
    int32_t hi = same_sample && attends ? min(rel, n - 1) : -1;
    int32_t lo = windowed ? max(rel - win + 1, 0) : 0;
    if (same_span) { lo = 0; hi = n - 1; }
    const bool empty = hi < lo;
    return KeyRange{empty ? 0x40000000u : (uint32_t)lo, empty ? 0u : (uint32_t)(hi - lo)};
}

// The transposed case: n query rows at consecutive positions q_first, q_first + 1, ... that
// all carry the fields (ss_q, att_q), seen from one key: the rows that see the key are one
// contiguous range (all of them for the key's own span; else the rows from the key's
// position on, as far as their look-back window reaches).
__device__ __forceinline__ KeyRange visible_rows(uint32_t ss_q, uint32_t att_q, int32_t q_first, uint32_t ss_k,
                                                 uint32_t mod_k, int32_t k, int32_t n) {
    const bool same_sample = (ss_q >> 16) == (ss_k >> 16);
    const bool same_span = (ss_q & 0xFFFFu) != 0 && ss_q == ss_k;
    const bool attends = (att_q >> mod_k) & 1u;
    const int32_t rel = k - q_first;                       // index of the first row at or after the key
    const int32_t win = (int32_t)att_window(att_q);
    const bool windowed = win != 0 && mod_k == att_modality(att_q);
    int32_t lo = same_sample && attends ? max(rel, 0) : n;
    int32_t hi = windowed ? min(rel + win - 1, n - 1) : n - 1;
    if (same_span) { lo = 0; hi = n - 1; }
    const bool empty = hi < lo;
    return KeyRange{empty ? 0x40000000u : (uint32_t)lo, empty ? 0u : (uint32_t)(hi - lo)};
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Global token position of local row r of a rank share (blocks == nullptr:
// identity, the whole sequence).
__device__ __forceinline__ int64_t row_pos(const int32_t* blocks, int32_t block, int64_t r) {
    if (!blocks) return r;
    int64_t b = r / block;
    return (int64_t)blocks[b] * block + (r - b * block);
}

// The same for a block list nobody has checked yet: an entry outside [0, n_seq_blocks)
// counts as block 0.
__device__ __forceinline__ int64_t row_pos_checked(const int32_t* blocks, int32_t block,
                                                   int64_t n_seq_blocks, int64_t r) {
    if (!blocks) return r;
    const int64_t b = r / block;
    int64_t g = blocks[b];
    if (g < 0 || g >= n_seq_blocks) g = 0;
    return g * block + (r - b * block);
}

// ---- entry points implemented per translation unit (host side) -------------
int launch_mfma_ceiling(int32_t iters, int32_t random_operands, float* sink, double* flops,
                        hipStream_t st);
int launch_encode(const mmattn_span* spans, int32_t n_spans, const int64_t* sample_off,
                  int32_t n_samples, int64_t S, uint64_t* d_bits, void* ws, hipStream_t st);
int launch_tile_map(const uint64_t* d_bits, int64_t S, const int32_t* d_blocks, int32_t block,
                    int64_t n_rows, int32_t tq, int32_t tk, uint8_t* d_cls, uint32_t* d_cnt,
                    uint64_t* d_rowpairs, hipStream_t st);
int launch_balance(const uint64_t* d_W, int32_t nB, int32_t P, int32_t* d_rank_of_block,
                   uint64_t* d_load, int32_t* d_rank_off, int32_t* d_rank_blocks, hipStream_t st);

// optional per-stage event pairs (measurement aid, see mmattn_stage_events)
struct StageEvents { hipEvent_t start, stop; };
extern StageEvents g_stage_events[MMATTN_STAGE_COUNT];
inline void stage_begin(int stage, hipStream_t st) {
    if (g_stage_events[stage].start) (void)hipEventRecord(g_stage_events[stage].start, st);
}
inline void stage_end(int stage, hipStream_t st) {
    if (g_stage_events[stage].stop) (void)hipEventRecord(g_stage_events[stage].stop, st);
}

struct AttnArgs {
    const void *q, *k, *v;
    const uint64_t* bits;
    const int32_t* blocks;
    int32_t n_blocks, block;
    int64_t S;
    int32_t Hq, Hkv, D;
    float scale;
    // forward only: the window of KV heads to run (with their query heads), and whether
    // the plan in the workspace is the one an earlier call built for the same share
    int32_t kv_begin, kv_count, plan_ready;
};
size_t fwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D);
size_t fwd_heads_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D);
size_t bwd_workspace(int64_t S, int64_t n_loc, int32_t Hq, int32_t Hkv, int32_t D);
int launch_fwd(const AttnArgs& a, void* o, float* lse, void* ws, hipStream_t st);
int launch_fwd_static(const AttnArgs& a, void* o, float* lse, hipStream_t st);
int launch_zero_kv(void* dk, void* dv, size_t bytes_each, hipStream_t st);
int launch_bwd(const AttnArgs& a, const void* o, const float* lse, const void* d_o,
               void* dq, void* dk, void* dv, void* ws, hipStream_t st);

}  // namespace mm
