// Preparation kernels for the attention passes:
// compaction of the tile classes into per-tile work lists (so that fully masked tiles are never visited --
// the block skipping of paper section 3.2.1) ordered longest first (the
// intra-GPU balance concern of section 3.2.2: long query blocks start early so
// that the tail of the launch is short).
#include "attn_common.h"

namespace mm {

// ---- work lists ---------------------------------------------------------------
// One wavefront per line (a q-tile's row of classes, or a k-tile's column) compacts
// the line's non-empty tiles.  One launch serves up to two sets of lines (the second
// set's lines follow the first's in the grid).
struct CompactJob {
    const uint8_t* cls;
    int32_t n_lines, n_items;
    int64_t line_stride, item_stride;
    int32_t* count;
    uint32_t* list;
};
struct CompactJobs { CompactJob j[2]; };

__global__ void __launch_bounds__(64)
compact_kernel(const CompactJobs jobs) {
    const bool second = (int)blockIdx.x >= jobs.j[0].n_lines;     // workgroup-uniform
    const CompactJob& J = jobs.j[second ? 1 : 0];
    const uint8_t* __restrict__ cls = J.cls;
    const int32_t n_items = J.n_items;
    const int64_t line_stride = J.line_stride, item_stride = J.item_stride;
    int32_t* __restrict__ count = J.count;
    uint32_t* __restrict__ list = J.list;
    const int line = (int)blockIdx.x - (second ? jobs.j[0].n_lines : 0);
    const int lane = threadIdx.x;
    int base = 0;
    for (int j0 = 0; j0 < n_items; j0 += kWave) {
        const int j = j0 + lane;
        uint8_t c = MMATTN_TILE_EMPTY;
        if (j < n_items) c = cls[line * line_stride + j * item_stride];
        const bool act = c != MMATTN_TILE_EMPTY;
        const uint64_t m = __ballot(act);
        if (act) {
            const int pos = base + __popcll(m & ((1ull << lane) - 1));
            list[(int64_t)line * n_items + pos] =
                (uint32_t)j | (c == MMATTN_TILE_PARTIAL ? kPartialFlag : 0u);
        }
        base += __popcll(m);
    }
    if (lane == 0) count[line] = base;
}

// Slices of the key-outer lists.  One workgroup.
//   Slice length: the whole list (no slicing) unless the longest list's steps exceed half
//   of one CU's share of all steps; then a quarter of that share, at least 8 entries,
//   doubled until the slices beyond each list's first fit the table (`budget` entries).
//   pbase[kt]: first partial-sum slot of k-tile kt (slots per k-tile: slices x hc), or -1
//   when a single workgroup owns the k-tile's result and writes it directly.
//   extra[]: (k-tile, slice) of every slice beyond a list's first, by k-tile index; the
//   number of entries in use is slicing[kExtraUsed].
// Called by all threads of one workgroup of kSliceThreads.
constexpr int kSliceThreads = 256;
struct ColSlicing {
    int32_t hpc, hc, groups, budget;
    int32_t *slicing, *pbase, *extra;      // slicing == nullptr: no slicing wanted (row lists)
};
__device__ void slice_cols(const int32_t* __restrict__ count, int32_t nk, int32_t nq, const ColSlicing cs) {
    const int32_t hpc = cs.hpc, hc = cs.hc, groups = cs.groups, budget = cs.budget;
    int32_t* __restrict__ slicing = cs.slicing;
    int32_t* __restrict__ pbase = cs.pbase;
    int32_t* __restrict__ extra = cs.extra;
    constexpr int kWaves = kSliceThreads / kWave;
    __shared__ int64_t tot_s[kWaves];
    __shared__ int32_t max_s[kWaves], scan_s[kWaves];
    __shared__ int32_t csz_s, base_s, sliced_s;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    // workgroup sum and maximum: shuffles inside a wavefront, then one LDS exchange
    auto sum_and_max = [&](int64_t v, int32_t m, int64_t& total, int32_t& longest) {
        for (int off = kWave / 2; off > 0; off >>= 1) {
            v += __shfl_xor(v, off);
            m = max(m, __shfl_xor(m, off));
        }
        __syncthreads();                               // earlier readers of tot_s / max_s are done
        if (lane == 0) { tot_s[wave] = v; max_s[wave] = m; }
        __syncthreads();
        total = 0; longest = 0;
        for (int w = 0; w < kWaves; ++w) { total += tot_s[w]; longest = max(longest, max_s[w]); }
    };
    // exclusive prefix sum over the workgroup's threads, continued from base_s
    auto scan_step = [&](int32_t v) -> int32_t {
        int32_t inc = v;                               // inclusive scan inside the wavefront
        for (int off = 1; off < kWave; off <<= 1) {
            const int32_t up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        __syncthreads();                               // earlier readers of scan_s / base_s are done
        if (lane == kWave - 1) scan_s[wave] = inc;
        __syncthreads();
        int32_t before = base_s + inc - v, all = 0;
        for (int w = 0; w < kWaves; ++w) {
            if (w < wave) before += scan_s[w];
            all += scan_s[w];
        }
        __syncthreads();
        if (tid == 0) base_s += all;
        __syncthreads();
        return before;
    };

    int64_t v = 0, total;
    int32_t m = 0, longest;
    for (int b = tid; b < nk; b += kSliceThreads) { v += count[b]; m = max(m, count[b]); }
    sum_and_max(v, m, total, longest);
    if (tid == 0) {
        const int64_t share = total * hpc * groups / 256;          // steps per CU
        int64_t c = max(nq, 1);
        if (budget > 0 && (int64_t)longest * hpc * 2 > share) c = max((int64_t)8, share / (4 * hpc));
        csz_s = (int32_t)min(c, (int64_t)max(nq, 1));
    }
    __syncthreads();
    if (csz_s >= longest) {
        // nothing is sliced (the usual case): every k-tile has hc workgroups, closed forms
        for (int b = tid; b < nk; b += kSliceThreads) pbase[b] = hc > 1 ? b * hc : -1;
        if (tid == 0) {
            slicing[kSliceLen] = csz_s;
            slicing[kSlicedTiles] = 0;
            slicing[kExtraUsed] = 0;
        }
        return;                                                    // workgroup-uniform
    }
    for (int round = 0; round < 32; ++round) {                     // workgroup-uniform loop
        const int32_t c = csz_s;
        int64_t need = 0, need_all;
        int32_t unused;
        for (int b = tid; b < nk; b += kSliceThreads) need += max(0, (count[b] + c - 1) / c - 1);
        sum_and_max(need, 0, need_all, unused);
        if (need_all <= budget) break;
        if (tid == 0) csz_s = (int32_t)min((int64_t)c * 2, (int64_t)max(nq, 1));
        __syncthreads();
    }
    const int32_t c = csz_s;
    // partial-sum slots, k-tiles in index order
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int b0 = 0; b0 < nk; b0 += kSliceThreads) {
        const int b = b0 + tid;
        const int32_t pieces = b < nk ? max(1, (count[b] + c - 1) / c) * hc : 0;
        const int32_t slots = pieces > 1 ? pieces : 0;
        const int32_t before = scan_step(slots);
        if (b < nk) pbase[b] = slots ? before : -1;
    }
    // slices beyond the first
    if (tid == 0) { base_s = 0; sliced_s = 0; }
    __syncthreads();
    int32_t sliced = 0;
    for (int r0 = 0; r0 < nk; r0 += kSliceThreads) {
        const int kt = r0 + tid;
        const int32_t more = kt < nk ? max(0, (count[kt] + c - 1) / c - 1) : 0;
        const int32_t before = scan_step(more);
        for (int32_t s = 0; s < more; ++s)
            if (before + s < budget) {                             // always true after the loop above
                extra[2 * (before + s)] = kt;
                extra[2 * (before + s) + 1] = s + 1;
            }
        sliced += more > 0 ? 1 : 0;
    }
    atomicAdd(&sliced_s, sliced);
    __syncthreads();
    const int32_t used = min(base_s, budget);                      // entries past `used` are never read
    if (tid == 0) {
        slicing[kSliceLen] = c;
        slicing[kSlicedTiles] = sliced_s;
        slicing[kExtraUsed] = used;
    }
}

// Ranks the lines: order[rank] = line, by (count descending, line ascending), so that
// heavy lines are scheduled first.  One thread per line; every thread counts the lines
// that precede its own, reading the counts through LDS in chunks (all lanes the same
// address: a broadcast).  Workgroup 0 also derives the slice length for cutting the
// lists (csz_out, may be null) from the total, the longest and the non-empty lists.
constexpr int kRankThreads = 256;
static_assert(kRankThreads == kSliceThreads, "slice_cols runs in the ranking kernel's first workgroup");
constexpr int kRankChunk = 2048;
struct RankJob {
    const int32_t* count;
    int32_t n_lines, n_items, n_wgs;     // n_wgs: workgroups of this job in the grid
    int32_t* order;
    int32_t* csz_out;
    int32_t groups;
    ColSlicing cs;
};
struct RankJobs { RankJob j[2]; };

// One launch serves up to two sets of lines (the second set's workgroups follow the first's).
__global__ void __launch_bounds__(kRankThreads)
rank_lines_kernel(const RankJobs jobs) {
    const bool second = (int)blockIdx.x >= jobs.j[0].n_wgs;        // workgroup-uniform
    const RankJob& J = jobs.j[second ? 1 : 0];
    const int32_t* __restrict__ count = J.count;
    const int32_t n_lines = J.n_lines, n_items = J.n_items, groups = J.groups;
    int32_t* __restrict__ order = J.order;
    int32_t* __restrict__ csz_out = J.csz_out;
    const ColSlicing cs = J.cs;
    const int wg = (int)blockIdx.x - (second ? jobs.j[0].n_wgs : 0);
    __shared__ __attribute__((aligned(16))) int32_t cnt_s[kRankChunk];
    const int tid = threadIdx.x;
    const int a = wg * kRankThreads + tid;
    const int ca = a < n_lines ? count[a] : 0;
    int pos = 0;
    for (int b0 = 0; b0 < n_lines; b0 += kRankChunk) {
        const int nb = min(kRankChunk, n_lines - b0);
        __syncthreads();
        for (int b = tid; b < ((nb + 3) & ~3); b += kRankThreads) cnt_s[b] = b < nb ? count[b0 + b] : -1;
        __syncthreads();
        // four counts per LDS read; the tail of the last quad is padded with -1 (never ahead)
        for (int b = 0; b < nb; b += 4) {
            const int4 cb = *(const int4*)&cnt_s[b];
            pos += (cb.x > ca || (cb.x == ca && b0 + b < a)) ? 1 : 0;
            pos += (cb.y > ca || (cb.y == ca && b0 + b + 1 < a)) ? 1 : 0;
            pos += (cb.z > ca || (cb.z == ca && b0 + b + 2 < a)) ? 1 : 0;
            pos += (cb.w > ca || (cb.w == ca && b0 + b + 3 < a)) ? 1 : 0;
        }
    }
    if (a < n_lines) order[pos] = a;

    if (csz_out && wg == 0) {                  // workgroup-uniform
        __shared__ int64_t tot_s[kRankThreads];
        __shared__ int32_t max_s[kRankThreads], num_s[kRankThreads];
        int64_t total = 0;
        int longest = 0, lists = 0;
        for (int b = tid; b < n_lines; b += kRankThreads) {
            const int c = count[b];
            total += c;
            longest = max(longest, c);
            lists += c > 0 ? 1 : 0;
        }
        tot_s[tid] = total; max_s[tid] = longest; num_s[tid] = lists;
        __syncthreads();
        for (int off = kRankThreads / 2; off > 0; off >>= 1) {
            if (tid < off) {
                tot_s[tid] += tot_s[tid + off];
                max_s[tid] = max(max_s[tid], max_s[tid + off]);
                num_s[tid] += num_s[tid + off];
            }
            __syncthreads();
        }
        if (tid == 0) *csz_out = slice_length(tot_s[0], max_s[0], num_s[0], groups, n_items);
    }
    if (cs.slicing && wg == 0) slice_cols(count, n_lines, n_items, cs);            // workgroup-uniform
}

static const ColSlicing kNoSlicing = {0, 0, 0, 0, nullptr, nullptr, nullptr};

static CompactJob compact_job_rows(const TilePlan& p) {
    return CompactJob{p.cls, p.nq, p.nk, (int64_t)p.nk, (int64_t)1, p.kcount, p.klist};
}
static CompactJob compact_job_cols(const TilePlanT& p) {
    return CompactJob{p.cls, p.nk, p.nq, (int64_t)1, (int64_t)p.nk, p.qcount, p.qlist};
}
static RankJob rank_job_rows(const TilePlan& p) {
    return RankJob{p.kcount, p.nq, p.nk, (p.nq + kRankThreads - 1) / kRankThreads, p.qorder, p.csz, p.groups,
                   kNoSlicing};
}
static RankJob rank_job_cols(const TilePlanT& p) {
    return RankJob{p.qcount, p.nk, p.nq, (p.nk + kRankThreads - 1) / kRankThreads, p.korder, nullptr, 1,
                   ColSlicing{p.hpc, p.hc, p.groups, p.n_extra, p.slicing, p.pbase, p.extra}};
}
// compaction and ranking of one or two sets of lists: two launches
static int launch_lists(const CompactJob& ca, const RankJob& ra, const CompactJob* cb, const RankJob* rb,
                        hipStream_t st) {
    CompactJobs cj;
    RankJobs rj;
    cj.j[0] = ca; rj.j[0] = ra;
    cj.j[1] = cb ? *cb : ca; rj.j[1] = rb ? *rb : ra;
    const int lines = ca.n_lines + (cb ? cb->n_lines : 0);
    const int wgs = ra.n_wgs + (rb ? rb->n_wgs : 0);
    hipLaunchKernelGGL(compact_kernel, dim3(lines), dim3(64), 0, st, cj);
    hipLaunchKernelGGL(rank_lines_kernel, dim3(wgs), dim3(kRankThreads), 0, st, rj);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

// zero fill of two equally sized buffers (a kernel rather than a memset node, so
// that the call can sit inside a captured graph)
__global__ void __launch_bounds__(256)
zero_pair_kernel(u32x4* __restrict__ a, u32x4* __restrict__ b, size_t n16) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        a[i] = z;
        b[i] = z;
    }
}

int launch_zero_kv(void* dk, void* dv, size_t bytes_each, hipStream_t st) {
    const size_t n16 = bytes_each / 16;           // S*Hkv*D*2 with D in {64,128}: a multiple of 16
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 4096);
    hipLaunchKernelGGL(zero_pair_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)dk, (u32x4*)dv, n16);
    MM_LAUNCH_CHECK();
    return MMATTN_OK;
}

int launch_compact_rows(const TilePlan& p, hipStream_t st) {
    return launch_lists(compact_job_rows(p), rank_job_rows(p), nullptr, nullptr, st);
}

int launch_compact_cols(const TilePlanT& p, hipStream_t st) {
    return launch_lists(compact_job_cols(p), rank_job_cols(p), nullptr, nullptr, st);
}

// the query-outer and the key-outer plan of one share together
int launch_compact_both(const TilePlan& pa, const TilePlanT& pb, hipStream_t st) {
    const CompactJob cb = compact_job_cols(pb);
    const RankJob rb = rank_job_cols(pb);
    return launch_lists(compact_job_rows(pa), rank_job_rows(pa), &cb, &rb, st);
}

}  // namespace mm
