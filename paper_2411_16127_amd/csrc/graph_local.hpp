// Scheduler metadata for small graphs and for batches of small graphs in one to three launches.
//
// The preprocessing step of Sec. 5.3 (CSR for the forward pass, CSC for the backward pass) is paid once per
// mini-batch in the batch-graph setting of Sec. 5.1, so there it has to cost about what a training step
// costs.  A block-diagonal batch makes that possible: the CSC transpose of one graph of the batch touches
// only that graph's nodes and its contiguous slice of the CSR, so one workgroup per graph ("segment") does
// it in LDS with a stable radix sort of its own, and only the row / column order by degree class needs a
// (tiny) scan across segments.  A single graph of at most kSegMaxNodes nodes is a batch of one.
//   k_seg_phase1   per segment: validation, out-degrees, column pointers, stable transpose, degree-class counts
//   k_seg_offsets  per degree class: exclusive scan of the counts over the segments (and of the tile counts)
//   k_seg_phase3   per segment: stable scatter of its nodes into the row and column order; batch tile
//                  table and adjacency bit masks for the dense-tile kernels
//   k_seg_single   all three for one segment in one launch
// Results are bit-identical to those of the general builder in graph.hip (the tests compare both with the
// CPU reference).
#pragma once
#include "graph_device.hpp"

namespace dfgnn {

constexpr int kSegMaxNodes = 4096;      // nodes of one segment (two 6-bit radix passes cover its source ids)
constexpr int kSegMaxEdges = 1 << 18;   // edges of one segment (one workgroup walks them)
constexpr int kSegKeys = 72;            // 36 degree classes for rows, 36 for columns
constexpr int kSegBatchWaves = 4, kSegSingleWaves = 16;

struct SegArgs {
    const int* indptr;
    const int* indices;
    const int* batch_ptr;  // [n_seg + 1] first node of every segment; nullptr: one segment [0, n_nodes)
    int n_nodes, n_edges, n_seg, T;
    int *t_indptr, *t_indices, *t_eid, *row_order, *col_order;
    uint32_t* keys_tmp;  // [n_edges] sort scratch
    int* vals_tmp;       // [n_edges] sort scratch
    int* seg_hist;       // [n_seg][72] nodes per degree class (rows | columns)
    int* seg_off;        // [n_seg][72] the same, summed over the segments before
    int* key_total;      // [72] the same, summed over all segments
    int* counters;
    // batch tables for the dense-tile kernels (nullptr when the caller gave no batch structure)
    int* tile_ptr;       // [n_seg + 1]
    int* tile_graph;
    unsigned long long *mask, *mask_t;  // [n_nodes][words]
    int max_words;
};

template <int W> struct SegShared {
    int cnt[kSegMaxNodes];  // out-degree of the segment's nodes
    int hist[W][64];
    int base[64];
    int wave_sums[W];
    int keyhist[kSegKeys];
};

// exclusive prefix of v over the 64 * W threads of the workgroup, and the total
template <int W> __device__ inline int seg_block_scan(int v, int* wave_sums, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    __syncthreads();  // protects wave_sums against a previous call
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const int s = wave_sums[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + incl - v;
}

// A stable counting pass over m items with digits below 64, split in two calls.  Wave w owns the contiguous
// item range [w * quota, (w + 1) * quota) and places its items in index order, so equal digits keep their
// order.  digit_histogram leaves hist[w][d] = items of digit d in wave w's range; the caller then fills
// base[d] (start of digit d's output range) and calls ordered_scatter, which hands every item its position.
template <int W> __device__ inline int wave_quota(int m) { return ((m + W - 1) / W + 63) & ~63; }

template <int W, class DigitFn> __device__ inline void digit_histogram(int m, int (*hist)[64], DigitFn digit) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int i = tid; i < W * 64; i += 64 * W) (&hist[0][0])[i] = 0;
    __syncthreads();
    const int q = wave_quota<W>(m), lo = wave * q, hi = min(m, lo + q);
    for (int s = lo; s < hi; s += 64)
        if (s + lane < hi) atomicAdd(&hist[wave][digit(s + lane)], 1);
    __syncthreads();
}

template <int W, class DigitFn, class EmitFn>
__device__ inline void ordered_scatter(int m, int (*hist)[64], const int* base, DigitFn digit, EmitFn emit) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (tid < 64) {  // thread d owns digit d: counts become running output positions, wave after wave
        int run = base[tid];
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const int c = hist[w][tid];
            hist[w][tid] = run;
            run += c;
        }
    }
    __syncthreads();
    const int q = wave_quota<W>(m), lo = wave * q, hi = min(m, lo + q);
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int s = lo; s < hi; s += 64) {  // bounds are the same in all lanes of a wave
        const int idx = s + lane;
        const bool valid = idx < hi;
        const unsigned d = valid ? (unsigned)digit(idx) : 0u;
        const unsigned long long same = match_digit<6>(d, valid);
        if (valid) {
            const int rank = __popcll(same & below);
            const int first = hist[wave][d];
            emit(idx, first + rank);
            if (rank == 0) hist[wave][d] = first + __popcll(same);
        }
        // the next round reads the positions this round's first lanes just wrote
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
}

// base[d] = items with a smaller digit (one radix pass inside the segment)
template <int W> __device__ inline void radix_bases(int (*hist)[64], int* base) {
    if (threadIdx.x < 64) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) tot += hist[w][threadIdx.x];
        int incl = tot;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(incl, off);
            if ((int)threadIdx.x >= off) incl += t;
        }
        base[threadIdx.x] = incl - tot;
    }
    __syncthreads();
}

// Bounds of segment b, checked.  Returns false (the same in every thread) when the segment cannot be
// processed: a flag has been raised then and the host will report it or fall back to the general builder.
__device__ inline bool seg_bounds(const SegArgs& a, int b, int* first, int* n_b, int* e0, int* m) {
    int lo = 0, hi = a.n_nodes;
    if (a.batch_ptr) {
        lo = a.batch_ptr[b];
        hi = a.batch_ptr[b + 1];
        if (lo < 0 || hi < lo || hi > a.n_nodes || (b == 0 && lo != 0) || (b == a.n_seg - 1 && hi != a.n_nodes)) {
            if (threadIdx.x == 0) atomicOr(a.counters + CNT_BATCH, BATCH_BAD_PTR);
            return false;
        }
    }
    const int p0 = a.indptr[lo], p1 = a.indptr[hi];
    int bad = 0;
    if (lo == 0 && p0 != 0) bad |= CSR_FIRST_NOT_ZERO;
    if (hi == a.n_nodes && p1 != a.n_edges) bad |= CSR_LAST_NOT_E;
    if (p0 < 0 || p0 > a.n_edges || p1 < 0 || p1 > a.n_edges) bad |= CSR_PTR_RANGE;
    if (p1 < p0) bad |= CSR_DECREASES;
    if (bad) {
        if (threadIdx.x == 0) atomicOr(a.counters + CNT_ERROR, bad);
        return false;
    }
    if (hi - lo > kSegMaxNodes || p1 - p0 > kSegMaxEdges) {
        if (threadIdx.x == 0) atomicOr(a.counters + CNT_SEG_FLAGS, 1);
        return false;
    }
    *first = lo; *n_b = hi - lo; *e0 = p0; *m = p1 - p0;
    return true;
}

// row of CSR position e inside the segment's rows [first, first + n_b): the last row whose pointer is <= e
__device__ inline int seg_row_of(const int* __restrict__ indptr, int first, int n_b, int e) {
    int lo = first, hi = first + n_b;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (indptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

template <int W>
__device__ inline bool seg_phase1(const SegArgs& a, int b, SegShared<W>& S, int* first_, int* n_b_) {
    constexpr int T = 64 * W;
    const int tid = threadIdx.x;
    int first, n_b, e0, m;
    if (!seg_bounds(a, b, &first, &n_b, &e0, &m)) return false;
    *first_ = first; *n_b_ = n_b;
    if (a.tile_ptr && tid == 0) {  // batch statistics for the dense-tile kernels
        const int t = (n_b + 15) >> 4;
        a.tile_ptr[b] = t;  // tiles of this graph; k_seg_offsets turns the counts into pointers
        atomicMax(a.counters + CNT_BATCH_MAX, n_b);
        atomicAdd(reinterpret_cast<unsigned long long*>(a.counters + CNT_BATCH_PAIRS), (unsigned long long)t * t);
    }
    // rows: pointer checks and degree classes
    for (int i = tid; i < kSegKeys; i += T) S.keyhist[i] = 0;
    for (int i = tid; i < n_b; i += T) S.cnt[i] = 0;
    __syncthreads();
    int bad = 0;
    for (int i = tid; i < n_b; i += T) {
        const int p = a.indptr[first + i], p1 = a.indptr[first + i + 1];
        if (p1 < p) bad |= CSR_DECREASES;
        if (p < 0 || p > a.n_edges) bad |= CSR_PTR_RANGE;
        atomicAdd(&S.keyhist[degree_key(p1 - p, a.T)], 1);
    }
    // edges: range checks and out-degrees.  A source outside the segment is an error (reported by the
    // host); it is counted as the segment's first node here so that every index below stays in range.
    auto key_of = [&](int idx) {
        const unsigned k = (unsigned)(a.indices[e0 + idx] - first);
        return k < (unsigned)n_b ? (int)k : 0;
    };
    int cross = 0;
    for (int idx = tid; idx < m; idx += T) {
        const int j = a.indices[e0 + idx];
        if (j < 0 || j >= a.n_nodes) bad |= CSR_INDEX_RANGE;
        else if (j < first || j >= first + n_b) cross = 1;
        atomicAdd(&S.cnt[key_of(idx)], 1);
    }
    if (bad) atomicOr(a.counters + CNT_ERROR, bad);
    if (cross) atomicOr(a.counters + CNT_BATCH, BATCH_CROSS_EDGE);
    __syncthreads();
    // column pointers = exclusive scan of the out-degrees; column degree classes
    {
        const int per = (n_b + T - 1) / T, lo = min(n_b, tid * per), hi = min(n_b, lo + per);
        int s = 0;
        for (int i = lo; i < hi; ++i) {
            s += S.cnt[i];
            atomicAdd(&S.keyhist[36 + degree_key(S.cnt[i], a.T)], 1);
        }
        int total;
        int run = e0 + seg_block_scan<W>(s, S.wave_sums, &total);
        for (int i = lo; i < hi; ++i) {
            a.t_indptr[first + i] = run;
            run += S.cnt[i];
        }
        if (first + n_b == a.n_nodes && tid == 0) a.t_indptr[a.n_nodes] = a.n_edges;  // the last segment closes the array
    }
    __syncthreads();
    for (int i = tid; i < kSegKeys; i += T) a.seg_hist[(size_t)b * kSegKeys + i] = S.keyhist[i];
    // CSC entries: the segment's CSR positions sorted by source, stable (one or two 6-bit passes)
    const bool two = n_b > 64;
    auto emit_final = [&](int pos, int eid) {
        a.t_eid[e0 + pos] = eid;
        a.t_indices[e0 + pos] = seg_row_of(a.indptr, first, n_b, eid);
    };
    if (!two) {
        digit_histogram<W>(m, S.hist, key_of);
        radix_bases<W>(S.hist, S.base);
        ordered_scatter<W>(m, S.hist, S.base, key_of, [&](int idx, int pos) { emit_final(pos, e0 + idx); });
    } else {
        auto low = [&](int idx) { return key_of(idx) & 63; };
        digit_histogram<W>(m, S.hist, low);
        radix_bases<W>(S.hist, S.base);
        ordered_scatter<W>(m, S.hist, S.base, low, [&](int idx, int pos) {
            a.keys_tmp[e0 + pos] = (uint32_t)key_of(idx);
            a.vals_tmp[e0 + pos] = e0 + idx;
        });
        auto high = [&](int idx) { return (int)(a.keys_tmp[e0 + idx] >> 6); };
        digit_histogram<W>(m, S.hist, high);
        radix_bases<W>(S.hist, S.base);
        ordered_scatter<W>(m, S.hist, S.base, high, [&](int idx, int pos) { emit_final(pos, a.vals_tmp[e0 + idx]); });
    }
    return true;
}

// adjacency bits of node i's list (CSR row or CSC column) relative to the first node of its graph
__device__ inline void seg_node_mask(const int* __restrict__ ptr, const int* __restrict__ idx, int i, int first, int n_b,
                                     int words, unsigned long long* __restrict__ mask, int* flags) {
    unsigned long long w[kDenseMaxWords];
#pragma unroll
    for (int k = 0; k < kDenseMaxWords; ++k) w[k] = 0ull;
    int bad = 0;
    for (int e = ptr[i]; e < ptr[i + 1]; ++e) {
        const int rel = idx[e] - first;
        if (rel < 0 || rel >= n_b) continue;  // an edge that leaves the graph: reported by phase 1
        if (rel < 64 * words) {
            const unsigned long long bit = 1ull << (rel & 63);
#pragma unroll
            for (int k = 0; k < kDenseMaxWords; ++k) {
                if (k == (rel >> 6)) {
                    if (w[k] & bit) bad |= BATCH_DUPLICATE;
                    w[k] |= bit;
                }
            }
        }
    }
    for (int k = 0; k < words; ++k) mask[(size_t)i * words + k] = w[k];
    if (bad) atomicOr(flags, bad);
}

template <int W> __device__ inline void seg_phase3(const SegArgs& a, int b, SegShared<W>& S, int first, int n_b) {
    constexpr int T = 64 * W;
    const int tid = threadIdx.x;
    for (int side = 0; side < 2; ++side) {  // rows, then columns
        const int* ptr = side == 0 ? a.indptr : a.t_indptr;
        int* order = side == 0 ? a.row_order : a.col_order;
        if (tid < 64) {
            int s = 0;
            if (tid < 36) {
                for (int k = 0; k < tid; ++k) s += a.key_total[side * 36 + k];
                if (b == 0) a.counters[(side == 0 ? CNT_ROW_BUCKETS : CNT_COL_BUCKETS) + tid] = s;  // first position of class >= tid
                s += a.seg_off[(size_t)b * kSegKeys + side * 36 + tid];
            }
            S.base[tid] = s;
        }
        auto key = [&](int i) { return (int)degree_key(ptr[first + i + 1] - ptr[first + i], a.T); };
        digit_histogram<W>(n_b, S.hist, key);  // (its first barrier also publishes S.base)
        ordered_scatter<W>(n_b, S.hist, S.base, key, [&](int i, int pos) { order[pos] = first + i; });
    }
    if (a.tile_ptr) {
        for (int t = a.tile_ptr[b] + tid; t < a.tile_ptr[b + 1]; t += T) a.tile_graph[t] = b;
        const int max_nodes = a.counters[CNT_BATCH_MAX];
        int words = (max_nodes + 63) / 64;
        words = words < 1 ? 1 : (words > a.max_words ? a.max_words : words);
        for (int i = tid; i < n_b; i += T) {
            seg_node_mask(a.indptr, a.indices, first + i, first, n_b, words, a.mask, a.counters + CNT_BATCH);
            seg_node_mask(a.t_indptr, a.t_indices, first + i, first, n_b, words, a.mask_t, a.counters + CNT_BATCH);
        }
    }
}

template <int W> __global__ __launch_bounds__(64 * W) void k_seg_phase1(const SegArgs a) {
    __shared__ SegShared<W> S;
    int first, n_b;
    seg_phase1<W>(a, blockIdx.x, S, &first, &n_b);
}

// Block k < 72: exclusive scan over the segments of the node counts of degree class k.  Block 72: the same
// over the tile counts of the graphs (in place: counts become the tile pointer).
__global__ __launch_bounds__(256) void k_seg_offsets(const SegArgs a) {
    __shared__ int wave_sums[4];
    const int k = blockIdx.x;
    int carry = 0;
    for (int base = 0; base < a.n_seg; base += 256) {
        const int s = base + (int)threadIdx.x;
        int v = 0;
        if (s < a.n_seg) v = k < kSegKeys ? a.seg_hist[(size_t)s * kSegKeys + k] : a.tile_ptr[s];
        int total;
        const int ex = carry + seg_block_scan<4>(v, wave_sums, &total);
        if (s < a.n_seg) {
            if (k < kSegKeys) a.seg_off[(size_t)s * kSegKeys + k] = ex;
            else a.tile_ptr[s] = ex;
        }
        carry += total;
    }
    if (threadIdx.x == 0) {
        if (k < kSegKeys) a.key_total[k] = carry;
        else { a.tile_ptr[a.n_seg] = carry; a.counters[CNT_N_TILES] = carry; }
    }
}

template <int W> __global__ __launch_bounds__(64 * W) void k_seg_phase3(const SegArgs a) {
    __shared__ SegShared<W> S;
    int first, n_b, e0, m;
    // the bounds were checked by phase 1; a segment it refused raises the same flag again and is skipped
    if (!seg_bounds(a, blockIdx.x, &first, &n_b, &e0, &m)) return;
    seg_phase3<W>(a, blockIdx.x, S, first, n_b);
}

// one segment = the whole graph: the scan across segments is the identity
template <int W> __global__ __launch_bounds__(64 * W) void k_seg_single(const SegArgs a) {
    __shared__ SegShared<W> S;
    int first, n_b;
    if (!seg_phase1<W>(a, 0, S, &first, &n_b)) return;
    __syncthreads();
    for (int i = threadIdx.x; i < kSegKeys; i += 64 * W) {
        a.key_total[i] = S.keyhist[i];
        a.seg_off[i] = 0;
    }
    __syncthreads();  // the workgroup reads back what it just wrote to global memory (also the column pointers)
    seg_phase3<W>(a, 0, S, first, n_b);
}

// launches for n_seg segments; the caller has cleared the counters
static inline void launch_local(const SegArgs& a, hipStream_t st) {
    if (a.n_seg == 1 && a.tile_ptr == nullptr) {
        hipLaunchKernelGGL((k_seg_single<kSegSingleWaves>), dim3(1), dim3(64 * kSegSingleWaves), 0, st, a);
        return;
    }
    hipLaunchKernelGGL((k_seg_phase1<kSegBatchWaves>), dim3((unsigned)a.n_seg), dim3(64 * kSegBatchWaves), 0, st, a);
    hipLaunchKernelGGL(k_seg_offsets, dim3(kSegKeys + (a.tile_ptr ? 1 : 0)), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_seg_phase3<kSegBatchWaves>), dim3((unsigned)a.n_seg), dim3(64 * kSegBatchWaves), 0, st, a);
}

}  // namespace dfgnn
