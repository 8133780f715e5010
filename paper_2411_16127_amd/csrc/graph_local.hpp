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
constexpr int kSegMaxEdges = 1 << 16;   // edges of one segment (one workgroup walks them)
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
    int* edge_row;       // [n_edges] scratch: destination row of every CSR position
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
    int cnt[kSegMaxNodes];  // out-degree of the segment's nodes; later scratch (long rows)
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
    for (int s0 = lo; s0 < hi; s0 += 64 * 8) {  // the digits of eight rounds are requested together
        int d[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) d[r] = s0 + 64 * r + lane < hi ? digit(s0 + 64 * r + lane) : -1;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            if (d[r] >= 0) atomicAdd(&hist[wave][d[r]], 1);
    }
    __syncthreads();
}

// load(idx) -> Item {digit, payload, extra}: what the item needs from memory.  The loads of kScatterBatch
// rounds are requested together before the first of them is placed (a round's positions depend on the round
// before, its loads do not); emit(idx, item, position).
struct Item { int digit, payload, extra; };
constexpr int kScatterBatch = 8;
template <int W, class LoadFn, class EmitFn>
__device__ inline void ordered_scatter(int m, int (*hist)[64], const int* base, LoadFn load, EmitFn emit) {
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
    for (int s0 = lo; s0 < hi; s0 += 64 * kScatterBatch) {  // bounds are the same in all lanes of a wave
        Item it[kScatterBatch];
#pragma unroll
        for (int r = 0; r < kScatterBatch; ++r) {
            const int idx = s0 + 64 * r + lane;
            it[r] = idx < hi ? load(idx) : Item{0, 0, 0};
        }
        // All of the batch's loads are waited for here, once.  Left to itself the compiler waits for the first
        // round's item only, and then has to wait before every later round for everything outstanding, which by
        // then includes the stores of the rounds before (loads and stores share one counter): a store round
        // trip per round.
#pragma unroll
        for (int r = 0; r < kScatterBatch; ++r) asm volatile("" ::"v"(it[r].digit), "v"(it[r].payload), "v"(it[r].extra));
#pragma unroll
        for (int r = 0; r < kScatterBatch; ++r) {
            const int idx = s0 + 64 * r + lane;
            if (s0 + 64 * r >= hi) break;
            const bool valid = idx < hi;
            const unsigned d = (unsigned)it[r].digit;
            const unsigned long long same = match_digit<6>(d, valid);
            if (valid) {
                const int rank = __popcll(same & below);
                const int first = hist[wave][d];
                emit(idx, it[r], first + rank);
                if (rank == 0) hist[wave][d] = first + __popcll(same);
            }
            // the next round reads the positions this round's first lanes just wrote (LDS only: the stores to
            // global memory need no ordering here)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
            __builtin_amdgcn_wave_barrier();
        }
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

template <int W>
__device__ inline bool seg_phase1(const SegArgs& a, int b, SegShared<W>& S, int* first_, int* n_b_) {
    constexpr int T = 64 * W;
    const int tid = threadIdx.x;
    int first, n_b, e0, m;
    if (!seg_bounds(a, b, &first, &n_b, &e0, &m)) return false;
    *first_ = first; *n_b_ = n_b;
    // tiles of this graph for the dense-tile kernels; k_seg_offsets turns the counts into pointers and takes
    // the batch statistics from them
    if (a.tile_ptr && tid == 0) a.tile_ptr[b] = (n_b + 15) >> 4;
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
    for (int i0 = tid; i0 < m; i0 += 8 * T) {  // eight sources requested at a time
        int j[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) j[r] = i0 + r * T < m ? a.indices[e0 + i0 + r * T] : first;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (i0 + r * T >= m) break;
            if (j[r] < 0 || j[r] >= a.n_nodes) bad |= CSR_INDEX_RANGE;
            else if (j[r] < first || j[r] >= first + n_b) cross = 1;
            const unsigned k = (unsigned)(j[r] - first);
            atomicAdd(&S.cnt[k < (unsigned)n_b ? k : 0u], 1);
        }
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
    // destination row of every CSR position of the segment (what the CSC lists per entry): a thread walks a
    // short row alone; long rows are noted in LDS (row, begin, end: S.cnt is free by now) and walked by
    // whole wavefronts afterwards
    {
        constexpr int kMaxLong = kSegMaxNodes / 3;
        int* long_rows = S.cnt;
        if (tid == 0) S.base[0] = 0;
        __syncthreads();
        for (int i = tid; i < n_b; i += T) {
            const int p = a.indptr[first + i], p1 = a.indptr[first + i + 1];
            int slot = kMaxLong;
            if (p1 - p > 32 && p >= e0 && p1 <= e0 + m) slot = atomicAdd(&S.base[0], 1);  // (a malformed row is reported above)
            if (slot < kMaxLong) {
                long_rows[3 * slot] = first + i;
                long_rows[3 * slot + 1] = p;
                long_rows[3 * slot + 2] = p1;
            } else {
                for (int e = max(p, e0); e < min(p1, e0 + m); ++e) a.edge_row[e] = first + i;
            }
        }
        __syncthreads();
        const int n_long = min(S.base[0], kMaxLong);
        for (int k = tid >> 6; k < n_long; k += W) {
            const int row = long_rows[3 * k], p1 = long_rows[3 * k + 2];
            for (int e = long_rows[3 * k + 1] + (tid & 63); e < p1; e += 64) a.edge_row[e] = row;
        }
        __syncthreads();
    }
    // CSC entries: the segment's CSR positions sorted by source, stable (one or two 6-bit passes).  A single
    // workgroup is bound by the instruction issue of its compute unit here (about a hundred instructions per
    // round of 64 edges and pass), which is what limits a lone graph of several thousand edges.
    const bool two = n_b > 64;
    if (!two) {
        digit_histogram<W>(m, S.hist, key_of);
        radix_bases<W>(S.hist, S.base);
        ordered_scatter<W>(m, S.hist, S.base, [&](int idx) { return Item{key_of(idx), a.edge_row[e0 + idx], 0}; },
                           [&](int idx, const Item& it, int pos) {
                               a.t_eid[e0 + pos] = e0 + idx;
                               a.t_indices[e0 + pos] = it.payload;
                           });
    } else {
        auto low = [&](int idx) { return key_of(idx) & 63; };
        digit_histogram<W>(m, S.hist, low);
        radix_bases<W>(S.hist, S.base);
        ordered_scatter<W>(m, S.hist, S.base, [&](int idx) { const int k = key_of(idx); return Item{k & 63, k, 0}; },
                           [&](int idx, const Item& it, int pos) {
                               a.keys_tmp[e0 + pos] = (uint32_t)it.payload;
                               a.vals_tmp[e0 + pos] = e0 + idx;
                           });
        auto high = [&](int idx) { return (int)(a.keys_tmp[e0 + idx] >> 6); };
        digit_histogram<W>(m, S.hist, high);
        radix_bases<W>(S.hist, S.base);
        ordered_scatter<W>(m, S.hist, S.base,
                           [&](int idx) {
                               const int eid = a.vals_tmp[e0 + idx];
                               return Item{(int)(a.keys_tmp[e0 + idx] >> 6), eid, a.edge_row[eid]};
                           },
                           [&](int, const Item& it, int pos) {
                               a.t_eid[e0 + pos] = it.payload;
                               a.t_indices[e0 + pos] = it.extra;
                           });
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
    const int e1 = ptr[i + 1];
    for (int e0 = ptr[i]; e0 < e1; e0 += 8) {  // eight entries requested at a time
        int j[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) j[u] = e0 + u < e1 ? idx[e0 + u] : -1;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int rel = j[u] - first;
            if (j[u] < 0 || rel < 0 || rel >= n_b) continue;  // no entry, or an edge that leaves the graph (reported by phase 1)
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
    }
    for (int k = 0; k < words; ++k) mask[(size_t)i * words + k] = w[k];
    if (bad) atomicOr(flags, bad);
}

// rp / cp: CSR / CSC pointers of the segment's nodes, [n_b + 1] each
template <int W>
__device__ inline void seg_phase3(const SegArgs& a, int b, SegShared<W>& S, int first, int n_b, const int* rp, const int* cp) {
    constexpr int T = 64 * W;
    const int tid = threadIdx.x;
    for (int side = 0; side < 2; ++side) {  // rows, then columns
        const int* ptr = side == 0 ? rp : cp;
        int* order = side == 0 ? a.row_order : a.col_order;
        if (tid < 64) {  // (one wavefront) start of every degree class in the order: exclusive scan of the class totals
            const int tot = tid < 36 ? a.key_total[side * 36 + tid] : 0;
            int incl = tot;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int t = __shfl_up(incl, off);
                if (tid >= off) incl += t;
            }
            int s = incl - tot;
            if (tid < 36) {
                if (b == 0) a.counters[(side == 0 ? CNT_ROW_BUCKETS : CNT_COL_BUCKETS) + tid] = s;  // first position of class >= tid
                s += a.seg_off[(size_t)b * kSegKeys + side * 36 + tid];
            }
            S.base[tid] = s;
        }
        auto key = [&](int i) { return (int)degree_key(ptr[i + 1] - ptr[i], a.T); };
        digit_histogram<W>(n_b, S.hist, key);  // (its first barrier also publishes S.base)
        ordered_scatter<W>(n_b, S.hist, S.base, [&](int i) { return Item{key(i), 0, 0}; },
                           [&](int i, const Item&, int pos) { order[pos] = first + i; });
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
    if (!seg_phase1<W>(a, blockIdx.x, S, &first, &n_b)) {
        // a refused segment leaves defined (empty) counts behind: the scan over the segments reads them
        for (int i = threadIdx.x; i < kSegKeys; i += 64 * W) a.seg_hist[(size_t)blockIdx.x * kSegKeys + i] = 0;
        if (a.tile_ptr && threadIdx.x == 0) a.tile_ptr[blockIdx.x] = 0;
    }
}

// Block k < 72: exclusive scan over the segments of the node counts of degree class k.  Block 72: the same
// over the tile counts of the graphs (in place: counts become the tile pointer), and the batch statistics
// (largest graph, number of 16 x 16 score tiles a dense pass forms).
__global__ __launch_bounds__(256) void k_seg_offsets(const SegArgs a) {
    __shared__ int wave_sums[4];
    __shared__ int red_max[256];
    __shared__ unsigned long long red_pairs[256];
    const int k = blockIdx.x;
    int carry = 0, biggest = 0;
    unsigned long long pairs = 0;
    for (int base = 0; base < a.n_seg; base += 256) {
        const int s = base + (int)threadIdx.x;
        int v = 0;
        if (s < a.n_seg) {
            if (k < kSegKeys) {
                v = a.seg_hist[(size_t)s * kSegKeys + k];
            } else {
                v = a.tile_ptr[s];
                const int n_b = a.batch_ptr[s + 1] - a.batch_ptr[s];  // (checked by phase 1)
                biggest = max(biggest, n_b);
                pairs += (unsigned long long)v * (unsigned long long)v;
            }
        }
        int total;
        const int ex = carry + seg_block_scan<4>(v, wave_sums, &total);
        if (s < a.n_seg) {
            if (k < kSegKeys) a.seg_off[(size_t)s * kSegKeys + k] = ex;
            else a.tile_ptr[s] = ex;
        }
        carry += total;
    }
    if (k < kSegKeys) {
        if (threadIdx.x == 0) a.key_total[k] = carry;
        return;
    }
    red_max[threadIdx.x] = biggest;
    red_pairs[threadIdx.x] = pairs;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int t = 1; t < 256; ++t) { biggest = max(biggest, red_max[t]); pairs += red_pairs[t]; }
        a.tile_ptr[a.n_seg] = carry;
        a.counters[CNT_N_TILES] = carry;
        a.counters[CNT_BATCH_MAX] = biggest;
        *reinterpret_cast<unsigned long long*>(a.counters + CNT_BATCH_PAIRS) = pairs;
    }
}

template <int W> __global__ __launch_bounds__(64 * W) void k_seg_phase3(const SegArgs a) {
    __shared__ SegShared<W> S;
    int first, n_b, e0, m;
    // Any flag of phase 1 (a segment too large for this builder, a malformed CSR or batch pointer, an edge
    // between two graphs) means that the host discards the result: nothing is placed then, because the
    // positions of the other segments would be built on the counts of a segment that was not processed.
    if (a.counters[CNT_SEG_FLAGS] | a.counters[CNT_ERROR] | (a.counters[CNT_BATCH] & (BATCH_BAD_PTR | BATCH_CROSS_EDGE))) return;
    // the bounds were checked by phase 1; a segment it refused raises the same flag again and is skipped
    if (!seg_bounds(a, blockIdx.x, &first, &n_b, &e0, &m)) return;
    seg_phase3<W>(a, blockIdx.x, S, first, n_b, a.indptr + first, a.t_indptr + first);
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
    seg_phase3<W>(a, 0, S, first, n_b, a.indptr + first, a.t_indptr + first);
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
