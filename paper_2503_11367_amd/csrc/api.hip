// C ABI of libmmattn: argument validation (host only, before any HIP call)
// and dispatch to the kernels.  See include/mmattn.h for the contract.
#include "common.h"

using namespace mm;

namespace {

bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

int check_attn(const void* q, const void* k, const void* v, const uint64_t* bits,
               const int32_t* blocks, int32_t n_blocks, int32_t block, int64_t S, int32_t Hq,
               int32_t Hkv, int32_t D, float scale, int dtype) {
    if (!k || !v || !bits || (n_blocks > 0 && (!q || !blocks))) return MMATTN_ERR_NULL;
    if (dtype != MMATTN_BF16) return MMATTN_ERR_UNSUPPORTED;
    if (S <= 0 || n_blocks < 0 || block <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0)
        return MMATTN_ERR_SHAPE;
    if (Hq % Hkv != 0 || S % block != 0 || (int64_t)n_blocks > S / block) return MMATTN_ERR_SHAPE;
    if (!(scale > 0.0f)) return MMATTN_ERR_SHAPE;
    if (D != 64 && D != 128) return MMATTN_ERR_UNSUPPORTED;
    if (S % 128 != 0 || block % 16 != 0) return MMATTN_ERR_UNSUPPORTED;
    if (S > ((int64_t)1 << 30) || Hq > 4096) return MMATTN_ERR_UNSUPPORTED;
    // the plans put one 64-row q-tile per grid row (at most 65535 of them)
    if ((int64_t)n_blocks * block > (int64_t)65535 * 64) return MMATTN_ERR_UNSUPPORTED;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(bits, 8) ||
        !aligned(blocks, 4))
        return MMATTN_ERR_SHAPE;
    return MMATTN_OK;
}

}  // namespace

namespace mm { StageEvents g_stage_events[MMATTN_STAGE_COUNT] = {}; }

extern "C" {

int mmattn_stage_events(int stage, void* ev_start, void* ev_stop) {
    if (stage < 0 || stage >= MMATTN_STAGE_COUNT) return MMATTN_ERR_SHAPE;
    g_stage_events[stage].start = (hipEvent_t)ev_start;
    g_stage_events[stage].stop = (hipEvent_t)ev_stop;
    return MMATTN_OK;
}

int mmattn_mfma_ceiling(int32_t iters, int32_t random_operands, void* d_sink, size_t sink_bytes,
                        double* flops, void* stream) {
    if (!d_sink) return MMATTN_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return MMATTN_ERR_SHAPE;
    if (sink_bytes < 2048) return MMATTN_ERR_WORKSPACE;
    return launch_mfma_ceiling(iters, random_operands, (float*)d_sink, flops, (hipStream_t)stream);
}

const char* mmattn_version(void) { return "mmattn 0.1 (gfx950)"; }

size_t mmattn_workspace_size(int op, int64_t S, int32_t n_blocks, int32_t block, int32_t Hq,
                             int32_t Hkv, int32_t D) {
    if (S <= 0 || n_blocks < 0 || block < 0) return 0;
    switch (op) {
        case MMATTN_OP_ENCODE:
            return align_up((size_t)n_blocks * sizeof(mmattn_span), 256) +
                   align_up(((size_t)block + 1) * sizeof(int64_t), 256);
        case MMATTN_OP_FWD:
            if (Hq <= 0 || Hkv <= 0 || D <= 0 || block <= 0 || n_blocks <= 0) return 0;
            return fwd_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D);
        case MMATTN_OP_FWD_HEADS:
            if (Hq <= 0 || Hkv <= 0 || D <= 0 || block <= 0 || n_blocks <= 0) return 0;
            if (Hq % Hkv != 0) return 0;
            return fwd_heads_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D);
        case MMATTN_OP_BWD:
            if (Hq <= 0 || Hkv <= 0 || D <= 0 || block <= 0 || n_blocks <= 0) return 0;
            return bwd_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D);
        default:
            return 0;
    }
}

int mmattn_mask_encode(const mmattn_span* spans, int32_t n_spans, const int64_t* sample_off,
                       int32_t n_samples, int64_t S, uint64_t* d_bits, void* ws, size_t ws_bytes,
                       void* stream) {
    if (!sample_off || !d_bits || (n_spans > 0 && !spans)) return MMATTN_ERR_NULL;
    if (S <= 0 || n_spans < 0 || n_samples < 1) return MMATTN_ERR_SHAPE;
    if (n_spans > MMATTN_MAX_SPANS || n_samples > MMATTN_MAX_SAMPLES) return MMATTN_ERR_UNSUPPORTED;
    if (sample_off[0] != 0 || sample_off[n_samples] != S) return MMATTN_ERR_LAYOUT;
    for (int i = 0; i < n_samples; ++i)
        if (sample_off[i + 1] <= sample_off[i]) return MMATTN_ERR_LAYOUT;
    int smp = 0;
    int64_t prev_end = 0;
    for (int j = 0; j < n_spans; ++j) {
        const mmattn_span& sp = spans[j];
        if (sp.len <= 0 || sp.start < prev_end || sp.start + sp.len > S) return MMATTN_ERR_LAYOUT;
        if (sp.modality < 1 || sp.modality > 7) return MMATTN_ERR_LAYOUT;     // one attend bit each
        if ((uint32_t)sp.flags & ~(uint32_t)(MMATTN_SPAN_NONCAUSAL | MMATTN_SPAN_NOBIDIR |
                                             (0xFFu << MMATTN_SPAN_DENY_SHIFT) |
                                             (0xFFFFu << MMATTN_SPAN_WINDOW_SHIFT)))
            return MMATTN_ERR_LAYOUT;
        // without the bidirectional term a token sees itself only through the
        // backward-looking term: causal bit set and own modality attended
        if ((sp.flags & MMATTN_SPAN_NOBIDIR) &&
            ((sp.flags & MMATTN_SPAN_NONCAUSAL) ||
             ((sp.flags >> MMATTN_SPAN_DENY_SHIFT) >> sp.modality & 1)))
            return MMATTN_ERR_LAYOUT;
        while (sample_off[smp + 1] <= sp.start) ++smp;
        if (sp.start + sp.len > sample_off[smp + 1]) return MMATTN_ERR_LAYOUT;   // crosses samples
        prev_end = sp.start + sp.len;
    }
    const size_t need = mmattn_workspace_size(MMATTN_OP_ENCODE, S, n_spans, n_samples, 0, 0, 0);
    if (!ws || !aligned(ws, 256) || ws_bytes < need) return MMATTN_ERR_WORKSPACE;
    return launch_encode(spans, n_spans, sample_off, n_samples, S, d_bits, ws, (hipStream_t)stream);
}

int mmattn_tile_map(const uint64_t* d_bits, int64_t S, int32_t tq, int32_t tk, uint8_t* d_cls,
                    uint32_t* d_cnt, uint64_t* d_rowpairs, void* stream) {
    if (!d_bits || !d_cnt) return MMATTN_ERR_NULL;
    if (S <= 0 || tq <= 0 || tk <= 0 || S % tq != 0 || S % tk != 0) return MMATTN_ERR_SHAPE;
    if ((int64_t)tq * tk > ((int64_t)1 << 31)) return MMATTN_ERR_SHAPE;
    if (S / tq > 65535 || S / tk > ((int64_t)1 << 24)) return MMATTN_ERR_UNSUPPORTED;
    return launch_tile_map(d_bits, S, nullptr, 1, S, tq, tk, d_cls, d_cnt, d_rowpairs,
                           (hipStream_t)stream);
}

int mmattn_balance(const uint64_t* d_W, int32_t nB, int32_t P, int32_t* d_rank_of_block,
                   uint64_t* d_load, int32_t* d_rank_off, int32_t* d_rank_blocks, void* stream) {
    if (!d_W || !d_rank_of_block || !d_load || !d_rank_off || !d_rank_blocks)
        return MMATTN_ERR_NULL;
    if (nB < 1 || P < 1) return MMATTN_ERR_SHAPE;
    if (nB > MMATTN_MAX_BLOCKS || P > MMATTN_MAX_RANKS) return MMATTN_ERR_UNSUPPORTED;
    return launch_balance(d_W, nB, P, d_rank_of_block, d_load, d_rank_off, d_rank_blocks,
                          (hipStream_t)stream);
}

int mmattn_fwd(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
               const int32_t* blocks, int32_t n_blocks, int32_t block, int64_t S, int32_t Hq,
               int32_t Hkv, int32_t D, float scale, int dtype, void* o_loc, float* lse, void* ws,
               size_t ws_bytes, void* stream) {
    if (n_blocks > 0 && (!o_loc || !lse)) return MMATTN_ERR_NULL;
    int rc = check_attn(q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, dtype);
    if (rc != MMATTN_OK) return rc;
    if (!aligned(o_loc, 16) || !aligned(lse, 4)) return MMATTN_ERR_SHAPE;
    if (n_blocks == 0) return MMATTN_OK;          // a rank that received no block: no rows, no output
    const size_t need = fwd_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D);
    if (!ws || !aligned(ws, 256) || ws_bytes < need) return MMATTN_ERR_WORKSPACE;
    AttnArgs a{q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, 0, Hkv, 0};
    return launch_fwd(a, o_loc, lse, ws, (hipStream_t)stream);
}

int mmattn_fwd_static(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
                      const int32_t* blocks, int32_t n_blocks, int32_t block, int64_t S, int32_t Hq,
                      int32_t Hkv, int32_t D, float scale, int dtype, void* o_loc, float* lse,
                      void* stream) {
    if (n_blocks > 0 && (!o_loc || !lse)) return MMATTN_ERR_NULL;
    int rc = check_attn(q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, dtype);
    if (rc != MMATTN_OK) return rc;
    if (!aligned(o_loc, 16) || !aligned(lse, 4)) return MMATTN_ERR_SHAPE;
    if (n_blocks == 0) return MMATTN_OK;
    if (fwd_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D) > (size_t)MMATTN_STATIC_SCRATCH_BYTES)
        return MMATTN_ERR_WORKSPACE;
    AttnArgs a{q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, 0, Hkv, 0};
    return launch_fwd_static(a, o_loc, lse, (hipStream_t)stream);
}

int mmattn_fwd_heads(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
                     const int32_t* blocks, int32_t n_blocks, int32_t block, int64_t S, int32_t Hq,
                     int32_t Hkv, int32_t D, float scale, int dtype, int32_t kv_head_begin,
                     int32_t kv_head_count, int32_t plan_ready, void* o_loc, float* lse, void* ws,
                     size_t ws_bytes, void* stream) {
    if (n_blocks > 0 && (!o_loc || !lse)) return MMATTN_ERR_NULL;
    int rc = check_attn(q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, dtype);
    if (rc != MMATTN_OK) return rc;
    if (kv_head_begin < 0 || kv_head_count < 1 || kv_head_begin > Hkv - kv_head_count)
        return MMATTN_ERR_SHAPE;
    if (!aligned(o_loc, 16) || !aligned(lse, 4)) return MMATTN_ERR_SHAPE;
    if (n_blocks == 0) return MMATTN_OK;
    const size_t need = fwd_heads_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D);
    if (!ws || !aligned(ws, 256) || ws_bytes < need) return MMATTN_ERR_WORKSPACE;
    AttnArgs a{q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale,
               kv_head_begin, kv_head_count, plan_ready != 0};
    return launch_fwd(a, o_loc, lse, ws, (hipStream_t)stream);
}

int mmattn_fwd_staged(const void* q_loc, const void* k_src, const void* v_src, void* k_stage,
                      void* v_stage, const uint64_t* bits, const int32_t* blocks, int32_t n_blocks,
                      int32_t block, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale,
                      int dtype, int32_t heads_per_stage, void* o_loc, float* lse, void* ws,
                      size_t ws_bytes, void* copy_stream, void* stream) {
    if (!k_src || !v_src || (n_blocks > 0 && (!o_loc || !lse))) return MMATTN_ERR_NULL;
    int rc = check_attn(q_loc, k_stage, v_stage, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, dtype);
    if (rc != MMATTN_OK) return rc;
    if (heads_per_stage < 1 || Hkv % heads_per_stage != 0) return MMATTN_ERR_SHAPE;
    if (!aligned(o_loc, 16) || !aligned(lse, 4) || !aligned(k_src, 16) || !aligned(v_src, 16))
        return MMATTN_ERR_SHAPE;
    if (copy_stream == stream) return MMATTN_ERR_SHAPE;          // nothing would overlap
    const size_t need = n_blocks > 0 ? fwd_heads_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D) : 0;
    if (n_blocks > 0 && (!ws || !aligned(ws, 256) || ws_bytes < need)) return MMATTN_ERR_WORKSPACE;

    hipStream_t cs = (hipStream_t)copy_stream, st = (hipStream_t)stream;
    const int n_stage = Hkv / heads_per_stage;
    const size_t pitch = (size_t)Hkv * D * 2, width = (size_t)heads_per_stage * D * 2;
    hipEvent_t ready = nullptr, arrived[MMATTN_MAX_STAGES] = {};
    if (n_stage > MMATTN_MAX_STAGES) return MMATTN_ERR_UNSUPPORTED;
    rc = MMATTN_OK;
    auto ok = [&](hipError_t e) { if (e != hipSuccess && rc == MMATTN_OK) rc = MMATTN_ERR_HIP; return e == hipSuccess; };
    // the copy stream starts once the inputs and the staging buffers are free on `stream`
    if (ok(hipEventCreateWithFlags(&ready, hipEventDisableTiming)) && ok(hipEventRecord(ready, st)))
        ok(hipStreamWaitEvent(cs, ready, 0));
    for (int i = 0; i < n_stage && rc == MMATTN_OK; ++i) {
        const size_t off = (size_t)i * width;
        if (k_src != k_stage)                   // already in place: nothing to move
            ok(hipMemcpy2DAsync((char*)k_stage + off, pitch, (const char*)k_src + off, pitch, width,
                                (size_t)S, hipMemcpyDeviceToDevice, cs));
        if (v_src != v_stage)
            ok(hipMemcpy2DAsync((char*)v_stage + off, pitch, (const char*)v_src + off, pitch, width,
                                (size_t)S, hipMemcpyDeviceToDevice, cs));
        if (ok(hipEventCreateWithFlags(&arrived[i], hipEventDisableTiming)))
            ok(hipEventRecord(arrived[i], cs));
    }
    for (int i = 0; i < n_stage && rc == MMATTN_OK; ++i) {
        if (!ok(hipStreamWaitEvent(st, arrived[i], 0))) break;
        if (n_blocks == 0) continue;
        AttnArgs a{q_loc, k_stage, v_stage, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale,
                   i * heads_per_stage, heads_per_stage, i > 0};
        rc = launch_fwd(a, o_loc, lse, ws, st);
    }
    // on an error part-way, `stream` still has to wait for whatever the copy stream was given
    if (rc != MMATTN_OK)
        for (int i = 0; i < n_stage; ++i)
            if (arrived[i]) (void)hipStreamWaitEvent(st, arrived[i], 0);
    // destroying a recorded event is deferred by the runtime until it has completed
    if (ready) (void)hipEventDestroy(ready);
    for (int i = 0; i < n_stage; ++i)
        if (arrived[i]) (void)hipEventDestroy(arrived[i]);
    return rc;
}

int mmattn_bwd(const void* q_loc, const void* k, const void* v, const uint64_t* bits,
               const int32_t* blocks, int32_t n_blocks, int32_t block, int64_t S, int32_t Hq,
               int32_t Hkv, int32_t D, float scale, int dtype, const void* o_loc, const float* lse,
               const void* do_loc, void* dq_loc, void* dk, void* dv, void* ws, size_t ws_bytes,
               void* stream) {
    if (!dk || !dv || (n_blocks > 0 && (!o_loc || !lse || !do_loc || !dq_loc))) return MMATTN_ERR_NULL;
    int rc = check_attn(q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, dtype);
    if (rc != MMATTN_OK) return rc;
    if (!aligned(o_loc, 16) || !aligned(do_loc, 16) || !aligned(dq_loc, 16) || !aligned(dk, 16) ||
        !aligned(dv, 16) || !aligned(lse, 4))
        return MMATTN_ERR_SHAPE;
    if (n_blocks == 0)                            // no rows: this rank's partial dK, dV are zero
        return launch_zero_kv(dk, dv, (size_t)S * Hkv * D * 2, (hipStream_t)stream);
    const size_t need = bwd_workspace(S, (int64_t)n_blocks * block, Hq, Hkv, D);
    if (!ws || !aligned(ws, 256) || ws_bytes < need) return MMATTN_ERR_WORKSPACE;
    AttnArgs a{q_loc, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale};
    return launch_bwd(a, o_loc, lse, do_loc, dq_loc, dk, dv, ws, (hipStream_t)stream);
}

}  // extern "C"
