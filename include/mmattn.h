/* mmattn -- multimodal-masked attention for workload-balanced context
 * parallelism on AMD MI355X (gfx950).  C ABI; all pointers are plain device
 * or host pointers as stated per argument; no C++ or framework types.
 *
 * The five calls follow the paper's statement of the problem:
 *   section 4.2  (bitfield attention mask: one 64-bit word per token)
 *   section 3.2.1 (blocks whose mask block is all zeros are skipped; per-block
 *                  workload counted row-wise; Alg. 1 LPT assignment)
 *   section 4.3  (each rank computes row-wise attention for its local queries
 *                  against all gathered keys and values)
 *
 * Conventions
 *   S        sequence length (tokens), K/V cover all S tokens
 *   block    balancer block size N_B (tokens); a rank owns a list of blocks
 *   local row r of a rank  <->  global token blocks[r / block]*block + r % block
 *   Hq, Hkv  query / key-value heads, Hq % Hkv == 0, Q head h uses KV head
 *            h / (Hq/Hkv)
 *   layouts  q_loc, o_loc, do_loc, dq_loc : [n_loc, Hq, D]   bf16, D contiguous
 *            k, v, dk, dv                 : [S, Hkv, D]      bf16
 *            lse                          : [Hq, n_loc]      fp32, natural log
 *            bits                         : [S]              uint64
 *
 * Mask word (LSB first): bits 0-7 attend-set (bit m = may attend modality m),
 * bits 8-11 own modality, bits 12-27 span id (0 = not in a bidirectional
 * span), bits 28-43 sample id, bits 44-59 look-back window W over keys of the
 * own modality (0 = unlimited), bit 63 causal bit.  Visibility of key k to
 * query q:
 *   sample(q)==sample(k) && ( (causal(q) && k<=q && attend(q)[modality(k)] &&
 *                              (W(q)==0 || modality(k)!=modality(q) || q-k<W(q))) ||
 *                             (span(q)!=0 && span(q)==span(k)) )
 * Text tokens attend every modality; a span's attend-set is all ones minus its
 * deny mask, so with no deny masks the backward term is plain causal
 * visibility.  The attend-set has 8 bits: modalities are 0 (text) .. 7.
 *
 * Ownership: the caller owns every buffer and the stream.  The library
 * allocates no device memory, never synchronises the stream and keeps no
 * state between calls (the one exception, the optional timing events of
 * mmattn_stage_events, is stated there; mmattn_fwd_staged creates and destroys
 * HIP events inside the call); scratch comes in through `ws` (size
 * from mmattn_workspace_size, 256-byte aligned) and may be reused by the next
 * call on the same stream.  Host pointers are read before the call returns.
 * Results are deterministic: no atomics on floating-point data, every sum is
 * taken in a fixed order.
 *
 * Errors: every call returns MMATTN_OK (0) or a negative mmattn_status.  All
 * argument checks run on the host before any GPU work is enqueued; nothing is
 * launched when a check fails.  Launch/runtime failures give MMATTN_ERR_HIP.
 */
#ifndef MMATTN_H
#define MMATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MMATTN_OK = 0,
    MMATTN_ERR_NULL = -1,        /* a required pointer is null */
    MMATTN_ERR_SHAPE = -2,       /* sizes inconsistent (divisibility, ranges) */
    MMATTN_ERR_UNSUPPORTED = -3, /* valid but not built (head_dim, dtype, limits) */
    MMATTN_ERR_WORKSPACE = -4,   /* ws null/misaligned/too small */
    MMATTN_ERR_LAYOUT = -5,      /* span/sample list malformed */
    MMATTN_ERR_HIP = -6          /* HIP runtime reported an error */
} mmattn_status;

typedef enum { MMATTN_BF16 = 0 } mmattn_dtype;

typedef enum {
    MMATTN_OP_ENCODE = 0, MMATTN_OP_TILE_MAP = 1, MMATTN_OP_BALANCE = 2,
    MMATTN_OP_FWD = 3, MMATTN_OP_BWD = 4, MMATTN_OP_FWD_HEADS = 5
} mmattn_op;

enum { MMATTN_TILE_EMPTY = 0, MMATTN_TILE_FULL = 1, MMATTN_TILE_PARTIAL = 2 };

/* A bidirectional (image/audio/...) span.  Tokens outside every span are
 * causal text.  flags bit 0 (MMATTN_SPAN_NONCAUSAL) clears the causal bit of
 * the span's tokens: they then see only their own span (section 4.2's
 * encoder tokens "without the causal bit").  flags bits 8-15: mask of
 * modalities (bit m = modality m, m in 0..7) that the span's tokens do not
 * attend among the earlier tokens; their own span stays visible.  flags bit 1
 * (MMATTN_SPAN_NOBIDIR): the span's tokens keep span id 0, so they see only
 * earlier tokens of the modalities they attend (an answer of section 5.5's
 * shared-question pattern: attends text and its own modality); such a span
 * must keep the causal bit and must attend its own modality, so that every
 * token sees at least itself (else MMATTN_ERR_LAYOUT).  flags bits 16-31: a
 * look-back window W in tokens (0 = none): among the earlier keys of the
 * span's own modality its tokens see only those less than W positions back;
 * other modalities and the own-span term are not limited.  Attention sinks
 * plus a sliding window (section 5.5's "lambda" pattern) are two NOBIDIR spans
 * per sample: the sinks with one modality, the rest with another and the
 * window.  The paper does not say how its bitfield holds this pattern; the
 * window field is an extension of the section 4.2 word. */
typedef struct { int64_t start, len; int32_t modality, flags; } mmattn_span;
#define MMATTN_SPAN_NONCAUSAL 1
#define MMATTN_SPAN_NOBIDIR   2
#define MMATTN_SPAN_DENY_SHIFT 8   /* flags bits 8-15: modalities the span's tokens do NOT attend */
#define MMATTN_SPAN_WINDOW_SHIFT 16 /* flags bits 16-31: look-back window over the own modality, tokens */
#define MMATTN_MAX_SPANS   65535
#define MMATTN_MAX_SAMPLES 65535
#define MMATTN_MAX_BLOCKS  16384   /* nB accepted by mmattn_balance */
#define MMATTN_MAX_RANKS   1024    /* P accepted by mmattn_balance */

/* Bytes of scratch the given call needs for these sizes (0 if none).  For
 * ENCODE pass n_blocks = n_spans and block = n_samples; for TILE_MAP and
 * BALANCE the result is 0.  Returns 0 for invalid sizes as well; the call
 * itself reports the error. */
size_t mmattn_workspace_size(int op, int64_t S, int32_t n_blocks, int32_t block,
                             int32_t Hq, int32_t Hkv, int32_t D);

/* Section 4.2: build the per-token 64-bit mask words.
 *   spans      host, n_spans entries sorted by start, disjoint, inside one
 *              sample each, modality in 1..7; span id = index+1
 *   sample_off host, n_samples+1 increasing offsets, [0]=0, [n_samples]=S
 *   d_bits     device, S words, overwritten
 *   ws         device scratch (staging of the two lists when there are more than
 *              64 spans or samples; both lists travel as kernel arguments, so
 *              the host arrays are read before the call returns and may be
 *              freed or changed right after it, whatever memory they are in)
 * MMATTN_ERR_LAYOUT for unsorted/overlapping/out-of-range spans, a span that
 * crosses a sample boundary, or bad offsets. */
int mmattn_mask_encode(const mmattn_span* spans, int32_t n_spans,
                       const int64_t* sample_off, int32_t n_samples,
                       int64_t S, uint64_t* d_bits,
                       void* ws, size_t ws_bytes, void* stream);

/* Section 3.2.1: classify every (q-tile, k-tile) of the S x S mask and count
 * its unmasked pairs; a tile whose mask block is all zeros is EMPTY (skipped
 * by the attention kernels).
 *   d_bits     device, S words
 *   tq, tk     tile shape in tokens; S % tq == 0, S % tk == 0,
 *              tq*tk <= 2^31
 *   d_cls      device uint8  [S/tq][S/tk]  MMATTN_TILE_*           (may be null)
 *   d_cnt      device uint32 [S/tq][S/tk]  unmasked pairs per tile
 *   d_rowpairs device uint64 [S/tq]        W_b = pairs of q-tile b (may be null)
 */
int mmattn_tile_map(const uint64_t* d_bits, int64_t S, int32_t tq, int32_t tk,
                    uint8_t* d_cls, uint32_t* d_cnt, uint64_t* d_rowpairs,
                    void* stream);

/* Alg. 1 (section 3.2.1), LPT: visit blocks by (W descending, index
 * ascending); give each to the rank with (load ascending, rank ascending).
 * Integer-only and deterministic.
 *   d_W            device uint64 [nB] workloads
 *   d_rank_of_block device int32 [nB]
 *   d_load         device uint64 [P]   sum of W per rank
 *   d_rank_off     device int32 [P+1]  CSR offsets into d_rank_blocks
 *   d_rank_blocks  device int32 [nB]   each rank's blocks, ascending index
 * 1 <= nB <= MMATTN_MAX_BLOCKS, 1 <= P <= MMATTN_MAX_RANKS. */
int mmattn_balance(const uint64_t* d_W, int32_t nB, int32_t P,
                   int32_t* d_rank_of_block, uint64_t* d_load,
                   int32_t* d_rank_off, int32_t* d_rank_blocks, void* stream);

/* Section 4.3 / 4.2: attention forward for one rank's query blocks against
 * all S keys/values under the bitfield mask; fully masked tiles are skipped.
 *   q_loc,k,v,bits,blocks  device inputs (layouts above); blocks[n_blocks]
 *                          int32 block indices in [0, S/block), distinct
 *   o_loc, lse             device outputs, overwritten; a row with no visible
 *                          key gets O = 0 and LSE = -inf
 *   scale                  softmax scale (1/sqrt(D) usually), > 0
 * Requires S % 128 == 0, block % 16 == 0, S % block == 0, D in {64,128},
 * 16-byte aligned tensors, S <= 2^30, Hq <= 4096, n_blocks * block <=
 * 65535 * 64 (else MMATTN_ERR_UNSUPPORTED).  n_blocks may be 0 (Alg. 1 leaves a rank empty when
 * there are more ranks than blocks): nothing is read or written, and q_loc,
 * blocks, o_loc, lse may be null.
 * Block indices live on the device, so their range is checked there: the first
 * int32 of `ws` is the call's status word, 0 after a good call and non-zero when
 * some blocks[i] lay outside [0, S/block).  In that case the attention kernels
 * return at once and the outputs keep whatever they held before the call; the
 * call itself still returns MMATTN_OK (the host never waits for the device).
 * The same holds for mmattn_fwd_heads, mmattn_fwd_staged and mmattn_bwd (there
 * dq_loc, dk, dv are the outputs left untouched).  Repeated block indices are
 * not detected: the rows are then simply computed twice, and in the backward
 * they contribute twice to dk, dv. */
int mmattn_fwd(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
               const int32_t* blocks, int32_t n_blocks, int32_t block,
               int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale, int dtype,
               void* o_loc, float* lse, void* ws, size_t ws_bytes, void* stream);

/* mmattn_fwd for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and checks as mmattn_fwd without
 * `ws`: the scratch is an array of MMATTN_STATIC_SCRATCH_BYTES that is part of
 * the library's code object (every GPU the library runs on holds its own copy
 * until the process ends).  The call allocates and frees nothing.
 *   - the device that `stream` belongs to must be the current device;
 *   - shares needing more scratch than that (mmattn_workspace_size(
 *     MMATTN_OP_FWD, ...) says how much) give MMATTN_ERR_WORKSPACE; nothing is
 *     launched then.  Shares with at least 512 (128-row tile, head pair) work
 *     items need about 5 bytes per (128-row tile, 64-key tile) pair, 1.3 MiB at
 *     131072 keys x 16384 rows; smaller shares are cut into list slices whose
 *     fp32 partial results can take far more (up to 64 x the size of O in fp32);
 *   - all calls on one GPU share the one array: calls that overlap on a GPU
 *     (different streams, different threads) race and must be ordered by the
 *     caller.  The status word of the block-index check lives in that array and
 *     is not visible to the caller: out-of-range indices leave the outputs
 *     untouched, as in mmattn_fwd. */
#define MMATTN_STATIC_SCRATCH_BYTES (32u << 20)
int mmattn_fwd_static(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
                      const int32_t* blocks, int32_t n_blocks, int32_t block,
                      int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale, int dtype,
                      void* o_loc, float* lse, void* stream);

/* Section 4.3 (keys and values are gathered head by head and the attention of
 * the heads already gathered overlaps the transfers of the next ones):
 * mmattn_fwd restricted to the KV heads [kv_head_begin, kv_head_begin +
 * kv_head_count) and their Hq/Hkv query heads each.  Tensors and layouts are
 * those of mmattn_fwd (full Hq / Hkv strides); only the window's heads of k, v
 * are read and only the window's heads of o_loc, lse are written, so the
 * caller may still be filling the other heads of k, v on another stream.
 *   plan_ready  0: build the share's tile plan in `ws` first (as mmattn_fwd
 *               does); nonzero: reuse the plan left in `ws` by an earlier call
 *               of this function with the same bits, blocks, block, S, Hq,
 *               Hkv, D that has completed or precedes this call on `stream`
 *   ws          mmattn_workspace_size(MMATTN_OP_FWD_HEADS, ...) bytes, valid
 *               for every window
 * Calls sharing one `ws` must be ordered (one stream, or events).
 * MMATTN_ERR_SHAPE for a window outside [0, Hkv). */
int mmattn_fwd_heads(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
                     const int32_t* blocks, int32_t n_blocks, int32_t block,
                     int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale, int dtype,
                     int32_t kv_head_begin, int32_t kv_head_count, int32_t plan_ready,
                     void* o_loc, float* lse, void* ws, size_t ws_bytes, void* stream);

/* Section 4.3 on one GPU: the forward with K/V arriving head by head.  For
 * each window of `heads_per_stage` KV heads, in order, the window's heads of
 * k_src, v_src are copied into k_stage, v_stage on `copy_stream` (a stand-in
 * for the arrival of the gathered heads) and `stream` waits for that window
 * only before running mmattn_fwd_heads on it, so the transfers of the later
 * windows overlap the attention of the earlier ones.
 *   k_src, v_src      device [S,Hkv,D], read on copy_stream once everything
 *                     enqueued on `stream` before this call has completed
 *   k_stage, v_stage  device [S,Hkv,D], overwritten with k_src, v_src (may be the
 *                     same buffers as k_src, v_src: then nothing is copied)
 *   copy_stream       a HIP stream other than `stream`, default priority
 *   ws                mmattn_workspace_size(MMATTN_OP_FWD_HEADS, ...) bytes
 * When the call returns, all work has been enqueued; `stream` has been made to
 * wait for every copy, so later work on `stream` may reuse all buffers.
 * Creates and destroys up to Hkv/heads_per_stage + 1 HIP events (no device
 * memory).  Hkv % heads_per_stage == 0, at most MMATTN_MAX_STAGES windows. */
#define MMATTN_MAX_STAGES 64
int mmattn_fwd_staged(const void* q_loc, const void* k_src, const void* v_src,
                      void* k_stage, void* v_stage, const uint64_t* bits,
                      const int32_t* blocks, int32_t n_blocks, int32_t block,
                      int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale, int dtype,
                      int32_t heads_per_stage, void* o_loc, float* lse,
                      void* ws, size_t ws_bytes, void* copy_stream, void* stream);

/* Backward of mmattn_fwd for the same rank share.
 *   o_loc, lse   what mmattn_fwd wrote;  do_loc upstream gradient
 *   dq_loc       [n_loc,Hq,D] overwritten
 *   dk, dv       [S,Hkv,D] overwritten with THIS rank's partial sums over its
 *                rows and over the Hq/Hkv query heads of each KV head (rows
 *                of keys no query of the rank sees become 0)
 * With P = exp(S - LSE), Delta = rowsum(dO o O), dS = P o (dP - Delta):
 * dV = P^T dO, dK = scale dS^T Q, dQ = scale dS K.  When there are few key
 * tiles the query heads of a KV head are summed in two stages (fp32 partials
 * in `ws`, fixed order).  Same shape requirements as mmattn_fwd.  With
 * n_blocks == 0 dk and dv are overwritten with zeros and the per-row
 * arguments may be null. */
int mmattn_bwd(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
               const int32_t* blocks, int32_t n_blocks, int32_t block,
               int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale, int dtype,
               const void* o_loc, const float* lse, const void* do_loc,
               void* dq_loc, void* dk, void* dv, void* ws, size_t ws_bytes, void* stream);

/* Measurement aid (not part of the method): while a pair of HIP events is set
 * for a stage, every later mmattn_fwd / mmattn_bwd call records ev_start just
 * before and ev_stop just after that stage's main kernel on the call's stream,
 * so a harness can time one kernel inside a multi-launch call (FWD and DQ
 * include the aggregation launch when lists are split; DKV_REDUCE is the
 * partial-sum launch after the dK/dV kernel, recorded only when it runs; a
 * complete pair for DKV travels with the kernel's dispatch instead and carries
 * the kernel's own begin and end times).  Pass
 * nulls to clear.  stage: MMATTN_STAGE_*.  The only process-wide state in the library;
 * not thread-safe.  Returns MMATTN_ERR_SHAPE for an unknown stage. */
enum { MMATTN_STAGE_FWD = 0, MMATTN_STAGE_DKV = 1, MMATTN_STAGE_DQ = 2, MMATTN_STAGE_DKV_REDUCE = 3,
       MMATTN_STAGE_COUNT = 4 };
int mmattn_stage_events(int stage, void* ev_start, void* ev_stop);

/* Measurement aid (not part of the method): enqueue a kernel that only issues
 * the bf16 32x32x16 matrix instruction from registers (256 workgroups of 8
 * wavefronts, `iters` x 16 instructions per wavefront), so a harness can time
 * a matrix-pipe ceiling for this GPU beside the published peak.
 *   random_operands  0: constant operands; 1: pseudo-random bf16 operands
 *                    (realistic switching activity, lower sustained clock)
 *   d_sink           device, >= 2048 bytes, normally left untouched
 *   flops            host, optional: receives the floating-point operations
 *                    the launch performs
 * 1 <= iters <= 2^24. */
int mmattn_mfma_ceiling(int32_t iters, int32_t random_operands, void* d_sink, size_t sink_bytes,
                        double* flops, void* stream);

/* Library version string (static storage). */
const char* mmattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MMATTN_H */
