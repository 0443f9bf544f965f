// mmattn_mask_encode: per-token 64-bit mask words from a span list and packed
// sample offsets (paper section 4.2, bitfield attention mask; App. C packing).
// One thread per token; binary search over the (sorted) sample offsets and
// span starts that were staged into the workspace.
#include <algorithm>
#include "common.h"

namespace mm {

struct DevSpan { int64_t start, len; int32_t modality, flags; };
static_assert(sizeof(DevSpan) == sizeof(mmattn_span), "span layout");

// the word of token t; spans / sample_off may live in global memory or in the
// kernel-argument segment
__device__ __forceinline__ void encode_token(const DevSpan* spans, int32_t n_spans,
                                             const int64_t* sample_off, int32_t n_samples, int64_t S,
                                             uint64_t* __restrict__ bits) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= S) return;
    // sample = last i with sample_off[i] <= t
    int lo = 0, hi = n_samples;              // invariant: off[lo] <= t < off[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (sample_off[mid] <= t) lo = mid; else hi = mid;
    }
    uint64_t w = 0xFFull | ((uint64_t)lo << kSampleShift);
    uint64_t causal = 1;
    // span = last j with start <= t, if t also lies before its end
    int a = -1, b = n_spans;                 // start[a] <= t < start[b]
    while (b - a > 1) {
        int mid = (a + b) >> 1;
        if (spans[mid].start <= t) a = mid; else b = mid;
    }
    if (a >= 0 && t < spans[a].start + spans[a].len) {
        if (!(spans[a].flags & MMATTN_SPAN_NOBIDIR)) w |= (uint64_t)(a + 1) << kSpanShift;
        w |= (uint64_t)(spans[a].modality & 0xF) << 8;
        if (spans[a].flags & MMATTN_SPAN_NONCAUSAL) causal = 0;
        // attend-set: all modalities minus the span's deny mask (flags bits 8-15)
        w &= ~(uint64_t)((spans[a].flags >> MMATTN_SPAN_DENY_SHIFT) & 0xFF);
        w |= (uint64_t)((uint32_t)spans[a].flags >> MMATTN_SPAN_WINDOW_SHIFT) << kWindowShift;
    }
    bits[t] = w | (causal << kCausalBit);
}

__global__ void __launch_bounds__(256)
encode_kernel(const DevSpan* __restrict__ spans, int32_t n_spans,
              const int64_t* __restrict__ sample_off, int32_t n_samples,
              int64_t S, uint64_t* __restrict__ bits) {
    encode_token(spans, n_spans, sample_off, n_samples, S, bits);
}

// Short lists travel by value in the kernel arguments: no staging copies, and the
// call can be captured into a graph.
constexpr int kInlineSpans = 64, kInlineSamples = 64;
struct InlineLayout {
    DevSpan spans[kInlineSpans];
    int64_t sample_off[kInlineSamples + 1];
};

__global__ void __launch_bounds__(256)
encode_inline_kernel(const InlineLayout lay, int32_t n_spans, int32_t n_samples, int64_t S,
                     uint64_t* __restrict__ bits) {
    encode_token(lay.spans, n_spans, lay.sample_off, n_samples, S, bits);
}

// one batch of the long lists: entries first .. first + ns - 1 of the spans and first ..
// first + no - 1 of the sample offsets, from the kernel arguments into the workspace
__global__ void __launch_bounds__(kInlineSpans)
stage_lists_kernel(const InlineLayout lay, int32_t first, int32_t ns, int32_t no,
                   DevSpan* __restrict__ d_spans, int64_t* __restrict__ d_off) {
    const int i = threadIdx.x;
    if (i < ns) d_spans[first + i] = lay.spans[i];
    if (i < no) d_off[first + i] = lay.sample_off[i];
}

int launch_encode(const mmattn_span* spans, int32_t n_spans, const int64_t* sample_off,
                  int32_t n_samples, int64_t S, uint64_t* d_bits, void* ws, hipStream_t st) {
    const unsigned n_wg = (unsigned)((S + 255) / 256);
    if (n_spans <= kInlineSpans && n_samples <= kInlineSamples) {
        InlineLayout lay{};
        for (int j = 0; j < n_spans; ++j)
            lay.spans[j] = DevSpan{spans[j].start, spans[j].len, spans[j].modality, spans[j].flags};
        for (int i = 0; i <= n_samples; ++i) lay.sample_off[i] = sample_off[i];
        hipLaunchKernelGGL(encode_inline_kernel, dim3(n_wg), dim3(256), 0, st, lay, n_spans, n_samples, S,
                           d_bits);
        MM_LAUNCH_CHECK();
        return MMATTN_OK;
    }
    // Long lists are staged into the workspace through kernel arguments as well, one batch of
    // entries per launch: the host lists are read here, before the call returns, whatever kind
    // of host memory they live in, and the call stays free of copy nodes.
    char* base = (char*)ws;
    DevSpan* d_spans = (DevSpan*)base;
    int64_t* d_off = (int64_t*)(base + align_up((size_t)n_spans * sizeof(DevSpan), 256));
    for (int32_t first = 0; first < n_spans || first <= n_samples; first += kInlineSpans) {
        InlineLayout lay{};
        const int32_t ns = std::max(0, std::min(kInlineSpans, n_spans - first));
        const int32_t no = std::max(0, std::min(kInlineSpans, n_samples + 1 - first));
        for (int j = 0; j < ns; ++j) {
            const mmattn_span& sp = spans[first + j];
            lay.spans[j] = DevSpan{sp.start, sp.len, sp.modality, sp.flags};
        }
        for (int i = 0; i < no; ++i) lay.sample_off[i] = sample_off[first + i];
        hipLaunchKernelGGL(stage_lists_kernel, dim3(1), dim3(kInlineSpans), 0, st, lay, first, ns, no,
                           d_spans, d_off);
    }
    MM_LAUNCH_CHECK();
    unsigned grid = (unsigned)((S + 255) / 256);
    hipLaunchKernelGGL(encode_kernel, dim3(grid), dim3(256), 0, st, d_spans, n_spans, d_off,
                       n_samples, S, d_bits);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

}  // namespace mm
