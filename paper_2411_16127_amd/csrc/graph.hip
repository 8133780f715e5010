// Scheduler metadata for a CSR-by-destination graph, built on the GPU: row order by degree class,
// super-row chunk list, CSC transpose, and the same for columns.  This is the preprocessing step that
// Sec. 5.3 lists next to the fused kernels (CSR for the forward pass, CSC for the backward pass); the
// per-row split by neighbourhood size replaces the whole-graph strategy switch of Sec. 4.2.
//
// All integer work; results are unique and are compared bit for bit with a CPU reference in the tests.
// Primitives (exclusive scan, stable LSD radix sort) are written here so that buffer sizes are plain
// formulas and no device query is needed to size them.
#include "graph_device.hpp"
#include "graph_local.hpp"

#include <cstring>
#include <new>

namespace dfgnn {

// ------------------------------------------------------------------------------------------------
// exclusive scan (int32), three launches; in == out allowed
// ------------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

__device__ inline int block_exclusive_scan(int v, int* total) {
    // 256 threads; returns the exclusive prefix of v over the block and the block total
    __shared__ int wave_sums[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    __syncthreads();  // protects wave_sums against a previous call
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int s = wave_sums[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_block_sums(const int* __restrict__ in, int n, int* __restrict__ sums) {
    const int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    int s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n) s += in[base + k];
    int total;
    block_exclusive_scan(s, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_sums_inplace(int* sums, int nb) {
    int carry = 0;
    for (int base = 0; base < nb; base += kScanThreads) {
        const int i = base + threadIdx.x;
        const int v = i < nb ? sums[i] : 0;
        int total;
        const int ex = block_exclusive_scan(v, &total);
        if (i < nb) sums[i] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(kScanThreads) void k_scan_apply(const int* in, int* out, int n, const int* __restrict__ sums) {
    const int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    int v[kScanItems];
    int s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = base + k < n ? in[base + k] : 0;
        s += v[k];
    }
    int total;
    int run = block_exclusive_scan(s, &total) + sums[blockIdx.x];
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

// Short arrays: one workgroup walks the tiles with a running carry, one launch instead of three (the
// scheduler of a small graph is a chain of dependent launches, and their number is what it costs).
// in and out may be the same array.
constexpr int kScanSingleTiles = 32;
__global__ __launch_bounds__(kScanThreads) void k_scan_single(const int* in, int* out, int n) {
    int carry = 0;
    for (int tile = 0; tile * kScanTile < n; ++tile) {
        const int base = tile * kScanTile + threadIdx.x * kScanItems;
        int v[kScanItems];
        int s = 0;
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            v[k] = base + k < n ? in[base + k] : 0;
            s += v[k];
        }
        int total;
        int run = carry + block_exclusive_scan(s, &total);
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            if (base + k < n) out[base + k] = run;
            run += v[k];
        }
        carry += total;
    }
}

inline int64_t scan_blocks(int64_t n) { return (n + kScanTile - 1) / kScanTile; }

static int exclusive_scan(const int* in, int* out, int64_t n, int* sums_tmp, hipStream_t st) {
    if (n <= 0) return DFGNN_OK;
    const int nb = (int)scan_blocks(n);
    if (nb <= kScanSingleTiles) {
        hipLaunchKernelGGL(k_scan_single, dim3(1), dim3(kScanThreads), 0, st, in, out, (int)n);
        DFGNN_HIP(hipGetLastError());
        return DFGNN_OK;
    }
    hipLaunchKernelGGL(k_scan_block_sums, dim3(nb), dim3(kScanThreads), 0, st, in, (int)n, sums_tmp);
    hipLaunchKernelGGL(k_scan_sums_inplace, dim3(1), dim3(kScanThreads), 0, st, sums_tmp, nb);
    hipLaunchKernelGGL(k_scan_apply, dim3(nb), dim3(kScanThreads), 0, st, in, out, (int)n, sums_tmp);
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

// ------------------------------------------------------------------------------------------------
// stable LSD radix sort of (uint32 key, int32 value) pairs, 8-bit digits
// ------------------------------------------------------------------------------------------------
constexpr int kSortThreads = 256;
constexpr int kSortItems = 16;
constexpr int kSortTile = kSortThreads * kSortItems;  // 4096 keys per workgroup, 1024 per wave

inline int64_t sort_blocks(int64_t n) { return (n + kSortTile - 1) / kSortTile; }

__global__ __launch_bounds__(kSortThreads) void k_radix_hist(const uint32_t* __restrict__ keys, int n, int shift,
                                                             int* __restrict__ counts, int nblocks) {
    __shared__ int hist[256];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int base = blockIdx.x * kSortTile;
#pragma unroll
    for (int s = 0; s < kSortItems; ++s) {
        const int idx = base + s * kSortThreads + threadIdx.x;
        if (idx < n) atomicAdd(&hist[(keys[idx] >> shift) & 255u], 1);
    }
    __syncthreads();
    counts[threadIdx.x * nblocks + blockIdx.x] = hist[threadIdx.x];
}

// Each wave owns 1024 consecutive keys of the tile and places them in index order, so equal digits keep
// their relative order (stability).  values_in == nullptr means value = index (first pass).
__global__ __launch_bounds__(kSortThreads) void k_radix_scatter(const uint32_t* __restrict__ keys_in,
                                                                const int* __restrict__ vals_in,
                                                                uint32_t* __restrict__ keys_out, int* __restrict__ vals_out,
                                                                int n, int shift, const int* __restrict__ offsets,
                                                                int nblocks) {
    __shared__ int hist[4][256];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int base = blockIdx.x * kSortTile + wave * (kSortTile / 4);
    uint32_t k[kSortItems];
    int v[kSortItems];
#pragma unroll
    for (int s = 0; s < kSortItems; ++s) {
        const int idx = base + s * 64 + lane;
        const bool valid = idx < n;
        k[s] = valid ? keys_in[idx] : 0u;
        v[s] = valid ? (vals_in ? vals_in[idx] : idx) : 0;
    }
    for (int i = tid; i < 4 * 256; i += kSortThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < kSortItems; ++s)
        if (base + s * 64 + lane < n) atomicAdd(&hist[wave][(k[s] >> shift) & 255u], 1);
    __syncthreads();
    {
        int run = offsets[tid * nblocks + blockIdx.x];  // thread tid owns digit tid
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = hist[w][tid];
            hist[w][tid] = run;
            run += c;
        }
    }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int s = 0; s < kSortItems; ++s) {
        const bool valid = base + s * 64 + lane < n;
        const unsigned d = (k[s] >> shift) & 255u;
        const unsigned long long same = match_digit(d, valid);
        if (valid) {
            const int rank = __popcll(same & below);
            const int first = hist[wave][d];
            keys_out[first + rank] = k[s];
            vals_out[first + rank] = v[s];
            if (rank == 0) hist[wave][d] = first + __popcll(same);
        }
        // the next round reads the running offsets this round's first lanes just wrote: keep the LDS
        // accesses of the two rounds in program order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

struct SortBuffers {
    uint32_t* keys[2];
    int* vals[2];   // vals[final parity] is where the caller wants the sorted values
    int* counts;    // 256 * sort_blocks(n)
    int* scan_tmp;  // scan_blocks(256 * sort_blocks(n))
};

// Sorts by the low `bits` bits.  Returns (through *keys_sorted) the buffer holding the sorted keys;
// sorted values land in vals_final.  vals_other is a second value buffer of n ints.
static int radix_sort_pairs(const uint32_t* keys_in, int64_t n, int bits, uint32_t* keys_a, uint32_t* keys_b,
                            int* vals_final, int* vals_other, int* counts, int* scan_tmp, const uint32_t** keys_sorted,
                            hipStream_t st) {
    const int passes = bits <= 8 ? 1 : (bits + 7) / 8;
    const int nb = (int)sort_blocks(n);
    uint32_t* kb[2] = {keys_a, keys_b};
    int* vb[2];
    vb[(passes - 1) & 1] = vals_final;
    vb[passes & 1] = vals_other;
    const uint32_t* kin = keys_in;
    const int* vin = nullptr;
    for (int p = 0; p < passes; ++p) {
        hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(kSortThreads), 0, st, kin, (int)n, p * 8, counts, nb);
        int rc = exclusive_scan(counts, counts, (int64_t)256 * nb, scan_tmp, st);
        if (rc != DFGNN_OK) return rc;
        hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(kSortThreads), 0, st, kin, vin, kb[p & 1], vb[p & 1], (int)n,
                           p * 8, counts, nb);
        kin = kb[p & 1];
        vin = vb[p & 1];
    }
    DFGNN_HIP(hipGetLastError());
    *keys_sorted = kin;
    return DFGNN_OK;
}

// ------------------------------------------------------------------------------------------------
// scheduler kernels
// ------------------------------------------------------------------------------------------------

__global__ void k_validate(const int* __restrict__ indptr, const int* __restrict__ indices, int n, int e, int* flags) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int bad = 0;
    if (t <= n) {
        const int p = indptr[t];
        if (t == 0 && p != 0) bad |= 1;
        if (t == n && p != e) bad |= 2;
        if (t < n && indptr[t + 1] < p) bad |= 4;
        if (p < 0 || p > e) bad |= 8;
    }
    if (t < e) {
        const int j = indices[t];
        if (j < 0 || j >= n) bad |= 16;
    }
    if (bad) atomicOr(flags, bad);
}

// key 0 for super rows, else 33 - bit_length(degree): long rows sort before short ones
__global__ void k_degree_keys(const int* __restrict__ ptr, int n, int T, uint32_t* __restrict__ keys) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int deg = ptr[i + 1] - ptr[i];
    keys[i] = degree_key(deg, T);
}

// out[k] = position of the first key >= k in the sorted key array, k = 0..35
__global__ void k_bucket_ptr(const uint32_t* __restrict__ sorted, int n, int* __restrict__ out) {
    const int k = threadIdx.x;
    if (blockIdx.x || k >= 36) return;
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (sorted[mid] < (uint32_t)k) lo = mid + 1; else hi = mid;
    }
    out[k] = lo;
}

__global__ void k_chunk_counts(const int* __restrict__ order, const int* __restrict__ ptr, int n_super, int C,
                               int* __restrict__ cnt) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s > n_super) return;
    if (s == n_super) { cnt[s] = 0; return; }
    const int r = order[s];
    cnt[s] = (ptr[r + 1] - ptr[r] + C - 1) / C;
}

__global__ void k_fill_chunks(const int* __restrict__ order, const int* __restrict__ ptr,
                              const int* __restrict__ chunk_ptr, int n_super, const int* __restrict__ n_chunks, int C,
                              int* __restrict__ chunks) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= *n_chunks) return;
    int lo = 0, hi = n_super;  // last s with chunk_ptr[s] <= c
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (chunk_ptr[mid] <= c) lo = mid; else hi = mid;
    }
    const int r = order[lo];
    const int b = ptr[r] + (c - chunk_ptr[lo]) * C;
    const int e = min(b + C, ptr[r + 1]);
    chunks[3 * c + 0] = r;
    chunks[3 * c + 1] = b;
    chunks[3 * c + 2] = e;
}

// t_indptr[j] = number of edges whose source is < j = lower bound of j in the sorted source array
__global__ void k_pointer_from_sorted(const uint32_t* __restrict__ sorted, int e, int n, int* __restrict__ t_indptr) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j > n) return;
    int lo = 0, hi = e;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (sorted[mid] < (uint32_t)j) lo = mid + 1; else hi = mid;
    }
    t_indptr[j] = lo;
}

// Destination row of every CSR position (the COO row array of the CSR).  A thread finds the row of the
// first of its kRowsPerThread consecutive positions by binary search (the last row whose pointer is <= p)
// and walks the pointer array from there, so the search is paid once per 16 edges.
constexpr int kRowsPerThread = 16;
__global__ void k_edge_rows(const int* __restrict__ indptr, int n, int e, int* __restrict__ edge_row) {
    const int64_t p0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * kRowsPerThread;
    if (p0 >= e) return;
    int lo = 0, hi = n;  // invariant: indptr[lo] <= p0 < indptr[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (indptr[mid] <= p0) lo = mid; else hi = mid;
    }
    int row = lo, next = indptr[lo + 1];
    for (int k = 0; k < kRowsPerThread && p0 + k < e; ++k) {
        const int p = (int)(p0 + k);
        while (p >= next) next = indptr[++row + 1];  // p < e = indptr[n], so row stays below n
        edge_row[p] = row;
    }
}

// destination of every CSC entry: the row of its CSR position
__global__ void k_gather_rows(const int* __restrict__ t_eid, const int* __restrict__ edge_row, int e,
                              int* __restrict__ t_indices) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < e) t_indices[t] = edge_row[t_eid[t]];
}

// Locality of the numbering: how many of (up to) kLocalitySamples evenly spaced edges connect two nodes whose
// ids differ by less than kLocalityWindow.  Graphs numbered that way (batches of small graphs, meshes,
// clustered orderings) reuse neighbour rows among rows that are close in the work list; the layer launches
// then keep runs of the list on one XCD so that the reuse happens in that XCD's L2.
constexpr int kLocalitySamples = 1 << 16;
__global__ void k_edge_locality(const int* __restrict__ edge_row, const int* __restrict__ indices, int e, int stride,
                                int* __restrict__ near) {
    const int64_t p = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * stride;
    int hit = 0;
    if (p < e) {
        const int d = edge_row[p] - indices[p];
        hit = (d < 0 ? -d : d) < kLocalityWindow;
    }
    // one atomic per workgroup: wavefront counts meet in LDS first
    __shared__ int block_hits;
    if (threadIdx.x == 0) block_hits = 0;
    __syncthreads();
    const int n = __popcll(__ballot(hit));
    if (n > 0 && (threadIdx.x & 63) == 0) atomicAdd(&block_hits, n);
    __syncthreads();
    if (threadIdx.x == 0 && block_hits > 0) atomicAdd(near, block_hits);
}

// ------------------------------------------------------------------------------------------------
// layout of the caller's buffers
// ------------------------------------------------------------------------------------------------
MetaLayout meta_layout(int64_t N, int64_t E, int T, int C, int flags) {
    MetaLayout L{};
    size_t off = 0;
    auto take = [&](int64_t count) { size_t o = off; off += align_up((size_t)(count > 0 ? count : 1) * sizeof(int32_t)); return o; };
    const bool fwd_only = flags & DFGNN_SCHED_FORWARD_ONLY;  // no CSC, no column schedule
    L.row_order = take(N);
    L.col_order = take(fwd_only ? 0 : N);
    L.t_indptr = take(fwd_only ? 0 : N + 1);
    L.t_indices = take(fwd_only ? 0 : E);
    L.t_eid = take(fwd_only ? 0 : E);
    L.row_chunk_ptr = take(super_capacity(E, T) + 1);
    L.row_chunks = take(3 * chunk_capacity(E, T, C));
    L.col_chunk_ptr = take(fwd_only ? 0 : super_capacity(E, T) + 1);
    L.col_chunks = take(fwd_only ? 0 : 3 * chunk_capacity(E, T, C));
    L.counters = take(CNT_TOTAL);
    L.edge_row = take((flags & DFGNN_SCHED_SCORES_IN_MEMORY) ? E : 0);
    L.total = off;
    return L;
}

struct ScratchLayout {
    size_t keys_a, keys_b, vals, counts, scan_tmp, cnt, total;
};

static ScratchLayout scratch_layout(int64_t N, int64_t E, int T) {
    ScratchLayout L{};
    const int64_t M = N > E ? N : E;
    size_t off = 0;
    auto take = [&](int64_t count) { size_t o = off; off += align_up((size_t)(count > 0 ? count : 1) * sizeof(int32_t)); return o; };
    L.keys_a = take(M);
    L.keys_b = take(M);
    L.vals = take(M);
    const int64_t ncounts = 256 * sort_blocks(M);
    L.counts = take(ncounts);
    const int64_t cap = super_capacity(E, T) + 2;
    L.scan_tmp = take(scan_blocks(ncounts > cap ? ncounts : cap) + 1);
    L.cnt = take(cap);
    L.total = off;
    return L;
}

// Defaults grow with the graph: a chunk should be long enough to amortise its start-up and short enough
// that the chunks of the super rows alone can fill the GPU (256 CUs x 4 SIMDs x several wavefronts):
// chunk_edges = E / 16384 rounded up to a power of two, clamped to [128, 512]; super_threshold =
// 2 * chunk_edges.  Below 256 edges a row is not worth splitting: one wavefront walks it in a few
// microseconds, about what the merge launch costs that the first super row of a graph brings with it.
static int resolve_params(const dfgnn_sched_params* sched, int64_t E, int* T, int* C, int* flags = nullptr) {
    int c = 128;
    while (c < 512 && (int64_t)c * 16384 < E) c <<= 1;
    *C = c;
    *T = 0;
    if (sched) {
        for (int r : sched->reserved) DFGNN_REQUIRE(r == 0, DFGNN_EINVAL, "dfgnn_sched_params.reserved must be zero");
        DFGNN_REQUIRE(sched->super_threshold >= 0 && sched->chunk_edges >= 0, DFGNN_EINVAL,
                      "negative scheduling parameter");
        DFGNN_REQUIRE((sched->flags & ~(DFGNN_SCHED_NO_SHORT_ROWS | DFGNN_SCHED_NO_DENSE_BATCH | DFGNN_SCHED_FORCE_DENSE_BATCH |
                                         DFGNN_SCHED_SCORES_IN_MEMORY | DFGNN_SCHED_NO_XCD_GROUPS |
                                         DFGNN_SCHED_FORWARD_ONLY | DFGNN_SCHED_NO_PAIRED_PASSES)) == 0,
                      DFGNN_EINVAL, "unknown scheduling flag 0x%x", sched->flags);
        if (sched->chunk_edges > 0) *C = sched->chunk_edges;
        if (sched->super_threshold > 0) *T = sched->super_threshold;
        if (flags) *flags = sched->flags;
    }
    if (*T == 0) *T = *C > (1 << 29) ? *C : 2 * *C;
    return DFGNN_OK;
}

// Row (or column) order for one pointer array: the degree-class sort and, in the device counters, where
// each class starts in the order.  Nothing is read back here; the caller reads all counters at once.
static int schedule_order(const int* ptr, int64_t n, int T, int* order, int* d_counters, int slot_buckets, char* scratch,
                          const ScratchLayout& S, hipStream_t st) {
    if (n == 0) return DFGNN_OK;
    uint32_t* keys_a = (uint32_t*)(scratch + S.keys_a);
    uint32_t* keys_b = (uint32_t*)(scratch + S.keys_b);
    const int tpb = 256;
    hipLaunchKernelGGL(k_degree_keys, dim3((unsigned)((n + tpb - 1) / tpb)), dim3(tpb), 0, st, ptr, (int)n, T, keys_a);
    const uint32_t* sorted = nullptr;
    int rc = radix_sort_pairs(keys_a, n, 6, keys_b, keys_a, order, (int*)(scratch + S.vals), (int*)(scratch + S.counts),
                              (int*)(scratch + S.scan_tmp), &sorted, st);
    if (rc != DFGNN_OK) return rc;
    hipLaunchKernelGGL(k_bucket_ptr, dim3(1), dim3(64), 0, st, sorted, (int)n, d_counters + slot_buckets);
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

// Chunks of the n_super super rows (or columns) at the head of `order`.  The number of chunks stays on the
// device (counter slot_chunks, which k_fill_chunks reads; its grid covers max_chunks); the caller reads it
// back with the other counters.
static int schedule_chunks(const int* ptr, int n_super, int C, const int* order, int* chunk_ptr, int* chunks,
                           int64_t max_chunks, int* d_counters, int slot_chunks, char* scratch, const ScratchLayout& S,
                           hipStream_t st) {
    if (n_super == 0) return DFGNN_OK;
    int* cnt = (int*)(scratch + S.cnt);
    const int tpb = 256;
    hipLaunchKernelGGL(k_chunk_counts, dim3((unsigned)((n_super + 1 + tpb - 1) / tpb)), dim3(tpb), 0, st, order, ptr,
                       n_super, C, cnt);
    int rc = exclusive_scan(cnt, chunk_ptr, (int64_t)n_super + 1, (int*)(scratch + S.scan_tmp), st);
    if (rc != DFGNN_OK) return rc;
    DFGNN_HIP(hipMemcpyAsync(d_counters + slot_chunks, chunk_ptr + n_super, sizeof(int), hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(k_fill_chunks, dim3((unsigned)((max_chunks + tpb - 1) / tpb)), dim3(tpb), 0, st, order, ptr,
                       chunk_ptr, n_super, d_counters + slot_chunks, C, chunks);
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

}  // namespace dfgnn

using namespace dfgnn;

extern "C" int dfgnn_graph_meta_bytes(int64_t N, int64_t E, const dfgnn_sched_params* sched, size_t* meta_bytes,
                                      size_t* scratch_bytes) {
    clear_error();
    DFGNN_REQUIRE(N >= 0 && E >= 0, DFGNN_EINVAL, "negative graph size N=%lld E=%lld", (long long)N, (long long)E);
    DFGNN_REQUIRE(N < (int64_t)INT32_MAX - (1 << 20) && E < (int64_t)INT32_MAX - (1 << 20), DFGNN_EUNSUPPORTED,
                  "graph too large for int32 indexing");
    int T, C, flags = 0;
    int rc = resolve_params(sched, E, &T, &C, &flags);
    if (rc != DFGNN_OK) return rc;
    if (meta_bytes) *meta_bytes = meta_layout(N, E, T, C, flags).total;
    if (scratch_bytes) *scratch_bytes = scratch_layout(N, E, T).total;
    return DFGNN_OK;
}

namespace dfgnn {

// Everything a builder needs: the checked arguments, the layouts of the caller's buffers and the handle
// under construction (its arrays already point into the metadata buffer).
struct Build {
    dfgnn_graph g;
    MetaLayout M;
    ScratchLayout S;
    char* scratch;
    int* d_counters;
    hipStream_t st;
};

static int prepare_build(Build& B, dfgnn_graph** out, int64_t N, int64_t E, const int32_t* d_indptr,
                         const int32_t* d_indices, const dfgnn_sched_params* sched, void* d_meta, size_t meta_bytes,
                         void* d_scratch, size_t scratch_bytes, void* stream) {
    DFGNN_REQUIRE(out != nullptr, DFGNN_EINVAL, "out is NULL");
    *out = nullptr;
    size_t need_meta = 0, need_scratch = 0;
    int rc = dfgnn_graph_meta_bytes(N, E, sched, &need_meta, &need_scratch);
    if (rc != DFGNN_OK) return rc;
    DFGNN_REQUIRE(d_indptr != nullptr && (E == 0 || d_indices != nullptr), DFGNN_EINVAL, "indptr / indices is NULL");
    DFGNN_REQUIRE(d_meta != nullptr && d_scratch != nullptr, DFGNN_EINVAL, "metadata / scratch buffer is NULL");
    DFGNN_REQUIRE(((uintptr_t)d_meta % kAlign) == 0 && ((uintptr_t)d_scratch % kAlign) == 0, DFGNN_EUNSUPPORTED,
                  "metadata / scratch buffer must be 256-byte aligned");
    DFGNN_REQUIRE(meta_bytes >= need_meta, DFGNN_EWORKSPACE, "metadata buffer has %zu bytes, needs %zu", meta_bytes, need_meta);
    DFGNN_REQUIRE(scratch_bytes >= need_scratch, DFGNN_EWORKSPACE, "scratch buffer has %zu bytes, needs %zu",
                  scratch_bytes, need_scratch);
    int T, C, flags = 0;
    rc = resolve_params(sched, E, &T, &C, &flags);
    if (rc != DFGNN_OK) return rc;
    B.st = (hipStream_t)stream;
    B.M = meta_layout(N, E, T, C, flags);
    B.S = scratch_layout(N, E, T);
    char* meta = (char*)d_meta;
    B.scratch = (char*)d_scratch;
    dfgnn_graph& g = B.g;
    g = dfgnn_graph{};
    g.N = N; g.E = E; g.T = T; g.C = C; g.flags = flags;
    g.indptr = d_indptr; g.indices = d_indices;
    g.row_order = (int*)(meta + B.M.row_order);
    g.col_order = (int*)(meta + B.M.col_order);
    g.t_indptr = (int*)(meta + B.M.t_indptr);
    g.t_indices = (int*)(meta + B.M.t_indices);
    g.t_eid = (int*)(meta + B.M.t_eid);
    g.row_chunk_ptr = (int*)(meta + B.M.row_chunk_ptr);
    g.row_chunks = (int*)(meta + B.M.row_chunks);
    g.col_chunk_ptr = (int*)(meta + B.M.col_chunk_ptr);
    g.col_chunks = (int*)(meta + B.M.col_chunks);
    B.d_counters = (int*)(meta + B.M.counters);
    g.counters = B.d_counters;
    g.edge_row = (flags & DFGNN_SCHED_SCORES_IN_MEMORY) ? (int*)(meta + B.M.edge_row) : nullptr;
    return DFGNN_OK;
}

// Counters come back through a small page-locked staging block per host thread (allocated on first use and
// kept): a copy to pageable memory goes through the runtime's own staging and costs tens of microseconds.
static int* readback_block() {
    thread_local int* block = nullptr;
    if (block == nullptr) {
        void* p = nullptr;
        if (hipHostMalloc(&p, CNT_TOTAL * sizeof(int), hipHostMallocDefault) == hipSuccess) block = (int*)p;
        else (void)hipGetLastError();
    }
    return block;
}
// n ints from device memory to dst, then a synchronisation of the stream
static int read_back(int* dst, const int* d_src, int n, hipStream_t st) {
    int* block = readback_block();
    int* via = block ? block : dst;
    DFGNN_HIP(hipMemcpyAsync(via, d_src, (size_t)n * sizeof(int), hipMemcpyDeviceToHost, st));
    DFGNN_HIP(hipStreamSynchronize(st));
    if (via != dst) memcpy(dst, via, (size_t)n * sizeof(int));
    return DFGNN_OK;
}

static const char kCsrErrorText[] =
    "malformed CSR (flags 0x%x: 1 indptr[0]!=0, 2 indptr[N]!=E, 4 indptr decreases, 8 indptr out of range, 16 index out "
    "of range)";

// The general builder: any graph; global scans and radix sorts, about twenty launches.  Leaves the degree
// class pointers and the locality sample in the device counters.
static int build_general(Build& B, int* locality_stride) {
    dfgnn_graph& g = B.g;
    const int64_t N = g.N, E = g.E;
    const int T = g.T, flags = g.flags;
    hipStream_t st = B.st;
    char* scratch = B.scratch;
    const ScratchLayout& S = B.S;
    int* d_counters = B.d_counters;
    const int32_t *d_indptr = g.indptr, *d_indices = g.indices;
    const int tpb = 256;
    int rc;
    DFGNN_HIP(hipMemsetAsync(d_counters, 0, CNT_TOTAL * sizeof(int), st));
    {
        const int64_t span = (N + 1 > E ? N + 1 : E);
        hipLaunchKernelGGL(k_validate, dim3((unsigned)((span + tpb - 1) / tpb)), dim3(tpb), 0, st, d_indptr, d_indices,
                           (int)N, (int)E, d_counters + CNT_ERROR);
        int bad = 0;
        rc = read_back(&bad, d_counters + CNT_ERROR, 1, st);
        if (rc != DFGNN_OK) return rc;
        DFGNN_REQUIRE(bad == 0, DFGNN_EINVAL, kCsrErrorText, bad);
    }

    // rows: order (their chunks follow once the counters have been read)
    rc = schedule_order(d_indptr, N, T, g.row_order, d_counters, CNT_ROW_BUCKETS, scratch, S, st);
    if (rc != DFGNN_OK) return rc;

    // CSC transpose: stable sort of CSR positions by source id
    *locality_stride = 1;
    const bool fwd_only = flags & DFGNN_SCHED_FORWARD_ONLY;
    if (fwd_only) {
        g.col_order = g.t_indptr = g.t_indices = g.t_eid = g.col_chunk_ptr = g.col_chunks = nullptr;
        if (E > 0) {  // the COO row array is still needed for the locality sample
            int* edge_row = g.edge_row ? g.edge_row : (int*)(scratch + S.vals);
            const int64_t row_threads = (E + kRowsPerThread - 1) / kRowsPerThread;
            hipLaunchKernelGGL(k_edge_rows, dim3((unsigned)((row_threads + tpb - 1) / tpb)), dim3(tpb), 0, st, d_indptr,
                               (int)N, (int)E, edge_row);
            *locality_stride = (int)((E + kLocalitySamples - 1) / kLocalitySamples);
            const int64_t samples = (E + *locality_stride - 1) / *locality_stride;
            hipLaunchKernelGGL(k_edge_locality, dim3((unsigned)((samples + tpb - 1) / tpb)), dim3(tpb), 0, st, edge_row,
                               d_indices, (int)E, *locality_stride, d_counters + CNT_NEAR);
            DFGNN_HIP(hipGetLastError());
        }
    } else if (E > 0) {
        int bits = 1;
        while (((int64_t)1 << bits) < N) ++bits;
        const uint32_t* sorted = nullptr;
        rc = radix_sort_pairs((const uint32_t*)d_indices, E, bits, (uint32_t*)(scratch + S.keys_a),
                              (uint32_t*)(scratch + S.keys_b), g.t_eid, (int*)(scratch + S.vals),
                              (int*)(scratch + S.counts), (int*)(scratch + S.scan_tmp), &sorted, st);
        if (rc != DFGNN_OK) return rc;
        hipLaunchKernelGGL(k_pointer_from_sorted, dim3((unsigned)((N + 1 + tpb - 1) / tpb)), dim3(tpb), 0, st, sorted,
                           (int)E, (int)N, g.t_indptr);
        // COO row array of the CSR: kept when the edge-parallel comparator asked for it, else in sort scratch
        int* edge_row = g.edge_row ? g.edge_row : (int*)(scratch + S.vals);
        const int64_t row_threads = (E + kRowsPerThread - 1) / kRowsPerThread;
        hipLaunchKernelGGL(k_edge_rows, dim3((unsigned)((row_threads + tpb - 1) / tpb)), dim3(tpb), 0, st, d_indptr, (int)N,
                           (int)E, edge_row);
        hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)((E + tpb - 1) / tpb)), dim3(tpb), 0, st, g.t_eid, edge_row, (int)E,
                           g.t_indices);
        *locality_stride = (int)((E + kLocalitySamples - 1) / kLocalitySamples);
        const int64_t samples = (E + *locality_stride - 1) / *locality_stride;
        hipLaunchKernelGGL(k_edge_locality, dim3((unsigned)((samples + tpb - 1) / tpb)), dim3(tpb), 0, st, edge_row,
                           d_indices, (int)E, *locality_stride, d_counters + CNT_NEAR);
        DFGNN_HIP(hipGetLastError());
    } else {
        DFGNN_HIP(hipMemsetAsync(g.t_indptr, 0, (size_t)(N + 1) * sizeof(int), st));
    }

    // columns: order
    if (!fwd_only) {
        rc = schedule_order(g.t_indptr, N, T, g.col_order, d_counters, CNT_COL_BUCKETS, scratch, S, st);
        if (rc != DFGNN_OK) return rc;
    }
    return DFGNN_OK;
}

// A graph the segment-local builder takes: at most kSegMaxNodes nodes per segment is checked on the device
// for batches (batch_ptr lives there); a graph without batch structure is one segment.
static bool local_builder_applies(const dfgnn_graph& g, int64_t n_graphs) {
    if (g.flags & (DFGNN_SCHED_FORWARD_ONLY | DFGNN_SCHED_SCORES_IN_MEMORY)) return false;
    if (g.N <= 0 || g.E <= 0) return false;
    if (n_graphs == 0) return g.N <= kSegMaxNodes && g.E <= kSegMaxEdges;
    return true;
}

// The segment-local builder (graph_local.hpp): one launch for a small graph, three for a batch.  seg_tmp
// holds [n_seg][72] + [n_seg][72] + [72] ints.
static int build_local(Build& B, const int32_t* d_batch_ptr, int64_t n_graphs, int* seg_tmp, int* tile_ptr, int* tile_graph,
                       unsigned long long* mask, unsigned long long* mask_t) {
    dfgnn_graph& g = B.g;
    SegArgs a{};
    a.indptr = g.indptr; a.indices = g.indices; a.batch_ptr = d_batch_ptr;
    a.n_nodes = (int)g.N; a.n_edges = (int)g.E; a.n_seg = d_batch_ptr ? (int)n_graphs : 1; a.T = g.T;
    a.t_indptr = g.t_indptr; a.t_indices = g.t_indices; a.t_eid = g.t_eid;
    a.row_order = g.row_order; a.col_order = g.col_order;
    a.keys_tmp = (uint32_t*)(B.scratch + B.S.keys_a);
    a.vals_tmp = (int*)(B.scratch + B.S.vals);
    a.edge_row = (int*)(B.scratch + B.S.keys_b);
    a.seg_hist = seg_tmp;
    a.seg_off = seg_tmp + (size_t)a.n_seg * kSegKeys;
    a.key_total = seg_tmp + (size_t)a.n_seg * kSegKeys * 2;
    a.counters = B.d_counters;
    a.tile_ptr = tile_ptr; a.tile_graph = tile_graph; a.mask = mask; a.mask_t = mask_t;
    a.max_words = kDenseMaxWords;
    DFGNN_HIP(hipMemsetAsync(B.d_counters, 0, CNT_TOTAL * sizeof(int), B.st));
    launch_local(a, B.st);
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

// After either builder: one read-back of all counters (where the degree classes start, and with that the
// super rows and columns; the locality sample; error and batch flags), then the chunk lists of the super
// rows and columns if there are any, then the handle.
static int finish_build(Build& B, bool local, int locality_stride, int* host_counters) {
    dfgnn_graph& g = B.g;
    const int64_t N = g.N, E = g.E;
    hipStream_t st = B.st;
    int* d_counters = B.d_counters;
    const bool fwd_only = g.flags & DFGNN_SCHED_FORWARD_ONLY;
    int rc = read_back(host_counters, d_counters, CNT_TOTAL, st);
    if (rc != DFGNN_OK) return rc;
    if (local) {
        if (host_counters[CNT_SEG_FLAGS]) return DFGNN_OK;  // a segment was too large: the caller falls back
        DFGNN_REQUIRE(host_counters[CNT_ERROR] == 0, DFGNN_EINVAL, kCsrErrorText, host_counters[CNT_ERROR]);
        if (host_counters[CNT_BATCH] & (BATCH_BAD_PTR | BATCH_CROSS_EDGE)) return DFGNN_OK;  // reported by the caller
    }
    for (int k = 0; k < 36; ++k) {
        g.row_bucket_ptr[k] = N > 0 ? host_counters[CNT_ROW_BUCKETS + k] : 0;
        g.col_bucket_ptr[k] = (N > 0 && !fwd_only) ? host_counters[CNT_COL_BUCKETS + k] : 0;
    }
    g.n_super_rows = g.row_bucket_ptr[1];
    g.n_super_cols = g.col_bucket_ptr[1];
    if (g.n_super_rows > 0 || g.n_super_cols > 0) {
        const int64_t max_chunks = chunk_capacity(E, g.T, g.C);
        rc = schedule_chunks(g.indptr, g.n_super_rows, g.C, g.row_order, g.row_chunk_ptr, g.row_chunks, max_chunks,
                                 d_counters, CNT_ROW_CHUNKS, B.scratch, B.S, st);
        if (rc != DFGNN_OK) return rc;
        rc = schedule_chunks(g.t_indptr, g.n_super_cols, g.C, g.col_order, g.col_chunk_ptr, g.col_chunks, max_chunks,
                             d_counters, CNT_COL_CHUNKS, B.scratch, B.S, st);
        if (rc != DFGNN_OK) return rc;
        int n_chunks[4] = {0, 0, 0, 0};  // counters CNT_ROW_CHUNKS .. CNT_COL_CHUNKS
        rc = read_back(n_chunks, d_counters + CNT_ROW_CHUNKS, 3, st);
        if (rc != DFGNN_OK) return rc;
        g.n_row_chunks = n_chunks[0];
        g.n_col_chunks = n_chunks[CNT_COL_CHUNKS - CNT_ROW_CHUNKS];
    }
    // at least half of the sampled edges stay inside the window: runs of kXcdGroup workgroups share an XCD.
    // Every edge of a graph the local builder takes does (segments have at most kSegMaxNodes <= window nodes).
    static_assert(kSegMaxNodes <= kLocalityWindow, "edges inside a segment must count as local");
    const int64_t samples = E > 0 ? (E + locality_stride - 1) / locality_stride : 0;
    const int64_t near = local ? samples : host_counters[CNT_NEAR];
    g.xcd_group = (!(g.flags & DFGNN_SCHED_NO_XCD_GROUPS) && samples > 0 && 2 * near >= samples) ? kXcdGroup : 0;
    return DFGNN_OK;
}

static int publish(const dfgnn_graph& g, dfgnn_graph** out) {
    dfgnn_graph* h = new (std::nothrow) dfgnn_graph(g);
    DFGNN_REQUIRE(h != nullptr, DFGNN_EINVAL, "out of host memory");
    *out = h;
    return DFGNN_OK;
}

}  // namespace dfgnn

extern "C" int dfgnn_graph_create(dfgnn_graph** out, int64_t N, int64_t E, const int32_t* d_indptr,
                                  const int32_t* d_indices, const dfgnn_sched_params* sched, void* d_meta,
                                  size_t meta_bytes, void* d_scratch, size_t scratch_bytes, void* stream) {
    clear_error();
    Build B;
    int rc = prepare_build(B, out, N, E, d_indptr, d_indices, sched, d_meta, meta_bytes, d_scratch, scratch_bytes, stream);
    if (rc != DFGNN_OK) return rc;
    int host_counters[CNT_TOTAL];
    int locality_stride = 1;
    const bool local = local_builder_applies(B.g, 0);
    if (local) {
        // one segment: its 3 x 72 ints of degree-class counts fit the sort's counter area (at least 256 ints)
        rc = build_local(B, nullptr, 0, (int*)(B.scratch + B.S.counts), nullptr, nullptr, nullptr, nullptr);
    } else {
        rc = build_general(B, &locality_stride);
    }
    if (rc != DFGNN_OK) return rc;
    rc = finish_build(B, local, locality_stride, host_counters);
    if (rc != DFGNN_OK) return rc;
    return publish(B.g, out);
}

// ------------------------------------------------------------------------------------------------
// block-diagonal batches of small graphs
// ------------------------------------------------------------------------------------------------
namespace dfgnn {

// per graph: pointer checks, largest graph, and the number of 16-node tiles (for the tile pointer)
__global__ void k_batch_check_ptr(const int* __restrict__ bp, int n_graphs, int n_nodes, int* __restrict__ tiles,
                                  int* flags, int* max_nodes, unsigned long long* tile_pairs) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g > n_graphs) return;
    int bad = 0;
    const int p = bp[g];
    if (g == 0 && p != 0) bad |= BATCH_BAD_PTR;
    if (g == n_graphs && p != n_nodes) bad |= BATCH_BAD_PTR;
    if (p < 0 || p > n_nodes) bad |= BATCH_BAD_PTR;
    int t = 0;
    if (g < n_graphs) {
        const int sz = bp[g + 1] - p;
        if (sz < 0) bad |= BATCH_BAD_PTR;
        else { atomicMax(max_nodes, sz); t = (sz + 15) >> 4; atomicAdd(tile_pairs, (unsigned long long)t * t); }
    }
    tiles[g] = t;
    if (bad) atomicOr(flags, bad);
}

// graph of every 16-row tile
__global__ void k_batch_tile_graph(const int* __restrict__ tile_ptr, int n_graphs, int* __restrict__ tile_graph) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_graphs) return;
    for (int t = tile_ptr[g]; t < tile_ptr[g + 1]; ++t) tile_graph[t] = g;
}

// One thread per node: adjacency bits of its row (from the CSR) and of its column (from the CSC), both
// relative to the first node of its graph, `words` 64-bit words each.
__global__ void k_batch_masks(const int* __restrict__ bp, int n_graphs, const int* __restrict__ ptr,
                              const int* __restrict__ idx, int n_nodes, int words, unsigned long long* __restrict__ mask,
                              int* flags) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_nodes) return;
    int lo = 0, hi = n_graphs;  // last graph whose first node is <= i
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (bp[mid] <= i) lo = mid; else hi = mid;
    }
    const int first = bp[lo], last = bp[lo + 1];
    unsigned long long w[kDenseMaxWords];
#pragma unroll
    for (int k = 0; k < kDenseMaxWords; ++k) w[k] = 0ull;
    int bad = 0;
    for (int e = ptr[i]; e < ptr[i + 1]; ++e) {
        const int j = idx[e];
        if (j < first || j >= last) { bad |= BATCH_CROSS_EDGE; continue; }
        const int rel = j - first;
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

struct BatchLayout {
    size_t adj_mask, adj_mask_t, tile_ptr, tile_graph, scan_tmp, seg_tmp, total;
};
static BatchLayout batch_layout(int64_t N, int64_t n_graphs) {
    BatchLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes ? bytes : 1); return o; };
    L.adj_mask = take((size_t)N * kDenseMaxWords * 8);
    L.adj_mask_t = take((size_t)N * kDenseMaxWords * 8);
    L.tile_ptr = take((size_t)(n_graphs + 2) * 4);
    L.tile_graph = take((size_t)(N / 16 + n_graphs + 2) * 4);  // every graph has at most nodes/16 + 1 tiles
    L.scan_tmp = take((size_t)(scan_blocks(n_graphs + 2) + 1) * 4);
    L.seg_tmp = take(((size_t)(n_graphs + 1) * 2 + 1) * kSegKeys * 4);  // degree-class counts per graph (dfgnn_graph_create_batch)
    L.total = off;
    return L;
}
}  // namespace dfgnn

extern "C" int dfgnn_graph_batch_bytes(int64_t N, int64_t n_graphs, size_t* batch_bytes) {
    clear_error();
    DFGNN_REQUIRE(N >= 0 && n_graphs >= 0 && batch_bytes != nullptr, DFGNN_EINVAL, "negative size or NULL");
    *batch_bytes = batch_layout(N, n_graphs).total;
    return DFGNN_OK;
}

extern "C" int dfgnn_graph_set_batch(dfgnn_graph* g, const int32_t* d_batch_ptr, int64_t n_graphs, void* d_batch,
                                     size_t batch_bytes, void* stream) {
    clear_error();
    DFGNN_REQUIRE(g != nullptr, DFGNN_EINVAL, "graph is NULL");
    g->batch_dense = false;
    g->batch_ptr = nullptr;
    g->n_graphs = 0;
    g->n_tiles = 0;
    if (d_batch_ptr == nullptr && n_graphs == 0) return DFGNN_OK;  // forget the batch structure
    DFGNN_REQUIRE(d_batch_ptr != nullptr && n_graphs >= 0 && n_graphs <= g->N + 1, DFGNN_EINVAL,
                  "batch_ptr is NULL or n_graphs = %lld is out of range", (long long)n_graphs);
    DFGNN_REQUIRE(n_graphs > 0 || g->N == 0, DFGNN_EINVAL, "a graph with nodes needs at least one batch entry");
    const BatchLayout B = batch_layout(g->N, n_graphs);
    DFGNN_REQUIRE(d_batch != nullptr && ((uintptr_t)d_batch % kAlign) == 0, DFGNN_EINVAL,
                  "batch buffer is NULL or not 256-byte aligned");
    DFGNN_REQUIRE(batch_bytes >= B.total, DFGNN_EWORKSPACE, "batch buffer has %zu bytes, needs %zu", batch_bytes, B.total);
    hipStream_t st = (hipStream_t)stream;
    char* buf = (char*)d_batch;
    int* flags = g->counters + CNT_BATCH;
    int* tile_ptr = (int*)(buf + B.tile_ptr);
    const int tpb = 256;
    DFGNN_HIP(hipMemsetAsync(flags, 0, 6 * sizeof(int), st));  // flags, running maximum, (pad), 64-bit tile-pair count
    unsigned long long* d_pairs = (unsigned long long*)(g->counters + CNT_BATCH_PAIRS);
    hipLaunchKernelGGL(k_batch_check_ptr, dim3((unsigned)((n_graphs + 1 + tpb - 1) / tpb)), dim3(tpb), 0, st, d_batch_ptr,
                       (int)n_graphs, (int)g->N, tile_ptr, flags, flags + 1, d_pairs);
    int rc = exclusive_scan(tile_ptr, tile_ptr, n_graphs + 1, (int*)(buf + B.scan_tmp), st);
    if (rc != DFGNN_OK) return rc;
    int host[2] = {0, 0};
    int n_tiles = 0;
    DFGNN_HIP(hipMemcpyAsync(host, flags, 2 * sizeof(int), hipMemcpyDeviceToHost, st));
    unsigned long long pairs = 0;
    DFGNN_HIP(hipMemcpyAsync(&n_tiles, tile_ptr + n_graphs, sizeof(int), hipMemcpyDeviceToHost, st));
    DFGNN_HIP(hipMemcpyAsync(&pairs, d_pairs, sizeof(pairs), hipMemcpyDeviceToHost, st));
    DFGNN_HIP(hipStreamSynchronize(st));
    DFGNN_REQUIRE(!(host[0] & BATCH_BAD_PTR), DFGNN_EINVAL, "batch_ptr must start at 0, end at N and be non-decreasing");
    int* tile_graph = (int*)(buf + B.tile_graph);  // a valid pointer array has at most N / 16 + n_graphs tiles
    if (n_graphs > 0)
        hipLaunchKernelGGL(k_batch_tile_graph, dim3((unsigned)((n_graphs + tpb - 1) / tpb)), dim3(tpb), 0, st, tile_ptr,
                           (int)n_graphs, tile_graph);
    const int max_nodes = host[1];
    int words = (max_nodes + 63) / 64;
    if (words < 1) words = 1;
    const bool small_enough = max_nodes <= kDenseMaxGraphNodes;
    if (words > kDenseMaxWords) words = kDenseMaxWords;  // larger graphs: masks are not used, edges are still checked
    unsigned long long* mask = (unsigned long long*)(buf + B.adj_mask);
    unsigned long long* mask_t = (unsigned long long*)(buf + B.adj_mask_t);
    if (g->N > 0) {
        const dim3 grid((unsigned)((g->N + tpb - 1) / tpb));
        hipLaunchKernelGGL(k_batch_masks, grid, dim3(tpb), 0, st, d_batch_ptr, (int)n_graphs, g->indptr, g->indices,
                           (int)g->N, words, mask, flags);
        if (!(g->flags & DFGNN_SCHED_FORWARD_ONLY))  // the column masks serve the backward kernels only
            hipLaunchKernelGGL(k_batch_masks, grid, dim3(tpb), 0, st, d_batch_ptr, (int)n_graphs, g->t_indptr, g->t_indices,
                               (int)g->N, words, mask_t, flags);
        DFGNN_HIP(hipMemcpyAsync(host, flags, sizeof(int), hipMemcpyDeviceToHost, st));
        DFGNN_HIP(hipStreamSynchronize(st));
    }
    DFGNN_REQUIRE(!(host[0] & BATCH_CROSS_EDGE), DFGNN_EINVAL, "an edge connects nodes of different graphs of the batch");
    g->batch_ptr = d_batch_ptr;
    g->n_graphs = n_graphs;
    g->tile_ptr = tile_ptr;
    g->tile_graph = tile_graph;
    g->n_tiles = n_tiles;
    g->tile_pairs = (int64_t)pairs;
    g->max_graph_nodes = max_nodes;
    g->mask_words = words;
    g->adj_mask = mask;
    g->adj_mask_t = mask_t;
    g->batch_dense = small_enough && !(host[0] & BATCH_DUPLICATE);
    return DFGNN_OK;
}

// Graph metadata and batch structure in one call (see graph_local.hpp); falls back to the two general calls
// for what the segment-local builder does not take.
extern "C" int dfgnn_graph_create_batch(dfgnn_graph** out, int64_t N, int64_t E, const int32_t* d_indptr,
                                        const int32_t* d_indices, const int32_t* d_batch_ptr, int64_t n_graphs,
                                        const dfgnn_sched_params* sched, void* d_meta, size_t meta_bytes, void* d_batch,
                                        size_t batch_bytes, void* d_scratch, size_t scratch_bytes, void* stream) {
    clear_error();
    Build B;
    int rc = prepare_build(B, out, N, E, d_indptr, d_indices, sched, d_meta, meta_bytes, d_scratch, scratch_bytes, stream);
    if (rc != DFGNN_OK) return rc;
    DFGNN_REQUIRE(d_batch_ptr != nullptr && n_graphs >= 0 && n_graphs <= N + 1, DFGNN_EINVAL,
                  "batch_ptr is NULL or n_graphs = %lld is out of range", (long long)n_graphs);
    DFGNN_REQUIRE(n_graphs > 0 || N == 0, DFGNN_EINVAL, "a graph with nodes needs at least one batch entry");
    const BatchLayout L = batch_layout(N, n_graphs);
    DFGNN_REQUIRE(d_batch != nullptr && ((uintptr_t)d_batch % kAlign) == 0, DFGNN_EINVAL,
                  "batch buffer is NULL or not 256-byte aligned");
    DFGNN_REQUIRE(batch_bytes >= L.total, DFGNN_EWORKSPACE, "batch buffer has %zu bytes, needs %zu", batch_bytes, L.total);
    char* buf = (char*)d_batch;
    bool done = false;
    if (local_builder_applies(B.g, n_graphs) && n_graphs > 0) {
        int* tile_ptr = (int*)(buf + L.tile_ptr);
        int* tile_graph = (int*)(buf + L.tile_graph);
        unsigned long long* mask = (unsigned long long*)(buf + L.adj_mask);
        unsigned long long* mask_t = (unsigned long long*)(buf + L.adj_mask_t);
        rc = build_local(B, d_batch_ptr, n_graphs, (int*)(buf + L.seg_tmp), tile_ptr, tile_graph, mask, mask_t);
        if (rc != DFGNN_OK) return rc;
        int host_counters[CNT_TOTAL];
        rc = finish_build(B, true, 1, host_counters);
        if (rc != DFGNN_OK) return rc;
        if (!host_counters[CNT_SEG_FLAGS]) {  // every graph of the batch fitted a segment
            const int bf = host_counters[CNT_BATCH];
            DFGNN_REQUIRE(!(bf & BATCH_BAD_PTR), DFGNN_EINVAL, "batch_ptr must start at 0, end at N and be non-decreasing");
            DFGNN_REQUIRE(!(bf & BATCH_CROSS_EDGE), DFGNN_EINVAL, "an edge connects nodes of different graphs of the batch");
            dfgnn_graph& g = B.g;
            const int max_nodes = host_counters[CNT_BATCH_MAX];
            int words = (max_nodes + 63) / 64;
            words = words < 1 ? 1 : (words > kDenseMaxWords ? kDenseMaxWords : words);
            unsigned long long pairs;
            memcpy(&pairs, host_counters + CNT_BATCH_PAIRS, sizeof(pairs));
            g.batch_ptr = d_batch_ptr;
            g.n_graphs = n_graphs;
            g.tile_ptr = tile_ptr;
            g.tile_graph = tile_graph;
            g.n_tiles = host_counters[CNT_N_TILES];
            g.tile_pairs = (int64_t)pairs;
            g.max_graph_nodes = max_nodes;
            g.mask_words = words;
            g.adj_mask = mask;
            g.adj_mask_t = mask_t;
            g.batch_dense = max_nodes <= kDenseMaxGraphNodes && !(bf & BATCH_DUPLICATE);
            done = true;
        }
    }
    if (done) return publish(B.g, out);
    // the general route: any graph sizes, forward-only graphs, the comparator's extra array
    rc = dfgnn_graph_create(out, N, E, d_indptr, d_indices, sched, d_meta, meta_bytes, d_scratch, scratch_bytes, stream);
    if (rc != DFGNN_OK) return rc;
    rc = dfgnn_graph_set_batch(*out, d_batch_ptr, n_graphs, d_batch, batch_bytes, stream);
    if (rc != DFGNN_OK) {
        delete *out;
        *out = nullptr;
    }
    return rc;
}

extern "C" int dfgnn_graph_destroy(dfgnn_graph* graph) {
    clear_error();
    delete graph;
    return DFGNN_OK;
}

extern "C" int dfgnn_graph_query(const dfgnn_graph* g, int what, const void** d_ptr, int64_t* count) {
    clear_error();
    DFGNN_REQUIRE(g != nullptr && count != nullptr, DFGNN_EINVAL, "NULL argument");
    const void* p = nullptr;
    int64_t c = 0;
    switch (what) {
    case DFGNN_Q_ROW_ORDER: p = g->row_order; c = g->N; break;
    case DFGNN_Q_ROW_CHUNK_PTR: p = g->row_chunk_ptr; c = g->n_super_rows ? g->n_super_rows + 1 : 0; break;
    case DFGNN_Q_ROW_CHUNKS: p = g->row_chunks; c = 3 * (int64_t)g->n_row_chunks; break;
    case DFGNN_Q_T_INDPTR: p = g->t_indptr; c = p ? g->N + 1 : 0; break;  // absent in a forward-only graph
    case DFGNN_Q_T_INDICES: p = g->t_indices; c = p ? g->E : 0; break;
    case DFGNN_Q_T_EID: p = g->t_eid; c = p ? g->E : 0; break;
    case DFGNN_Q_COL_ORDER: p = g->col_order; c = p ? g->N : 0; break;
    case DFGNN_Q_COL_CHUNK_PTR: p = g->col_chunk_ptr; c = g->n_super_cols ? g->n_super_cols + 1 : 0; break;
    case DFGNN_Q_COL_CHUNKS: p = g->col_chunks; c = 3 * (int64_t)g->n_col_chunks; break;
    case DFGNN_Q_N_SUPER_ROWS: c = g->n_super_rows; break;
    case DFGNN_Q_N_SUPER_COLS: c = g->n_super_cols; break;
    case DFGNN_Q_SUPER_THRESHOLD: c = g->T; break;
    case DFGNN_Q_CHUNK_EDGES: c = g->C; break;
    case DFGNN_Q_BATCH_DENSE: c = g->batch_dense ? 1 : 0; break;
    case DFGNN_Q_XCD_GROUP: c = g->xcd_group; break;
    default: DFGNN_REQUIRE(false, DFGNN_EINVAL, "unknown query item %d", what);
    }
    if (d_ptr) *d_ptr = p;
    *count = c;
    return DFGNN_OK;
}
