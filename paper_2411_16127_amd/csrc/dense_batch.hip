// Dense-tile kernels for batches of small graphs (block-diagonal CSR; the batch-graph workloads of
// Sec. 5.1 at batch size 1024), GT model, bf16 tensors.
//
// A graph of n <= 64 nodes is small enough that one wavefront can hold one head of it: Q_h, K_h, V_h
// (n x D values each) are staged once into LDS with coalesced loads, the n x n score block is formed with
// MFMA (v_mfma_f32_16x16x16_bf16) in 16 x 16 tiles, missing edges are masked with a per-row adjacency
// bit mask, and the softmax and the aggregation P V run on the tiles in registers.  Every K/V row is
// read from memory once per graph instead of once per edge, which is what makes this path pay: the
// gather kernels move E*R bytes through the caches, this one N*R.  The backward kernel handles the row
// side (dQ) and the column side (dK, dV) of Appendix B in one launch, because both fit in LDS.
//
// MFMA 16x16x16 operand layout (lane l, q = l / 16): A[m = l % 16][k = 4q .. 4q+3],
// B[k = 4q .. 4q+3][n = l % 16], C/D[m = 4q + r][n = l % 16] for r = 0..3.  The score tile is computed
// transposed (S^T = K Q^T), so that a lane owns one query row i = l % 16 and the keys j = 4q + r: this
// is already the A-operand layout of P for the second product, and no transpose through LDS is needed.
#include "common.hpp"
#include "layer_device.hpp"
#include "dense_bf16.hpp"

namespace dfgnn {

constexpr int kDenseMaxNodes = kDenseSmallNodes;  // nodes per graph these kernels cover (4 tiles of 16)
constexpr int kDenseTiles = kDenseMaxNodes / 16;
constexpr int kTStride = kDenseMaxNodes + 8;  // row stride (elements) of transposed copies: breaks bank conflicts

struct DenseArgs {
    const int* batch_ptr;
    const unsigned long long* adj_mask;  // bit j of adj_mask[i]: edge i <- (first node of i's graph + j)
    const uint16_t *q, *k, *v, *out, *d_out;
    uint16_t *o, *d_q, *d_k, *d_v;
    const float *row_max, *row_sum;
    float *o_max, *o_sum;
    int n_graphs, H, D, HD, W;  // W: 64-bit words per mask row (only word 0 is used: graphs have <= 64 nodes)
    float c_score, scale;
};

__device__ inline float sum_over_q(float x) { x += __shfl_xor(x, 16); x += __shfl_xor(x, 32); return x; }
__device__ inline float max_over_q(float x) { x = fmaxf(x, __shfl_xor(x, 16)); x = fmaxf(x, __shfl_xor(x, 32)); return x; }

// Stage one head of one node tensor: rows [0, n) of the graph into plain[row][d] (row stride D) and, if
// wanted, transposed[d][row] (row stride kTStride); rows [n, 16 * tiles) are zero-filled.
template <int D, bool PLAIN, bool TRANS>
__device__ inline void stage_head(const uint16_t* __restrict__ src, size_t first_elem, int HD, int n, int tiles,
                                  uint16_t* plain, uint16_t* trans, int lane) {
    constexpr int LR = D / 8;        // lanes per row (8 bf16 = 16 bytes each)
    constexpr int ROWS = 64 / LR;    // rows per load instruction
    const int part = lane % LR;
    for (int r0 = 0; r0 < tiles * 16; r0 += ROWS) {
        const int row = r0 + lane / LR;
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (row < n) raw = *reinterpret_cast<const u32x4*>(src + first_elem + (size_t)row * HD + part * 8);
        if (PLAIN) *reinterpret_cast<u32x4*>(plain + row * D + part * 8) = raw;
        if (TRANS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                trans[(part * 8 + 2 * e) * kTStride + row] = (uint16_t)(raw[e] & 0xffffu);
                trans[(part * 8 + 2 * e + 1) * kTStride + row] = (uint16_t)(raw[e] >> 16);
            }
        }
    }
}

template <int D> __device__ inline s16x4 frag_plain(const uint16_t* x, int row, int ks, int q) {
    return *reinterpret_cast<const s16x4*>(x + row * D + ks * 16 + 4 * q);
}
__device__ inline s16x4 frag_trans(const uint16_t* xt, int d, int col0) {
    return *reinterpret_cast<const s16x4*>(xt + d * kTStride + col0);
}

// ---------------------------------------------------------------------------------------------
// forward: one wavefront per (graph, head)
// ---------------------------------------------------------------------------------------------
template <int D, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_dense_gt_forward(const DenseArgs a) {
    constexpr int KS = D / 16;
    __shared__ __attribute__((aligned(16))) uint16_t lds[WAVES][2 * kDenseMaxNodes * D + D * kTStride];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int gh = blockIdx.x * WAVES + wave;
    if (gh >= a.n_graphs * a.H) return;
    const int g = gh / a.H, h = gh - g * a.H;
    const int base = a.batch_ptr[g], n = a.batch_ptr[g + 1] - base;
    const int tiles = (n + 15) >> 4;
    const int l16 = lane & 15, q = lane >> 4;
    uint16_t* Qs = lds[wave];
    uint16_t* Ks = Qs + kDenseMaxNodes * D;
    uint16_t* Vt = Ks + kDenseMaxNodes * D;
    const size_t first = (size_t)base * a.HD + (size_t)h * D;
    stage_head<D, true, false>(a.q, first, a.HD, n, tiles, Qs, nullptr, lane);
    stage_head<D, true, false>(a.k, first, a.HD, n, tiles, Ks, nullptr, lane);
    stage_head<D, false, true>(a.v, first, a.HD, n, tiles, nullptr, Vt, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    for (int it = 0; it < tiles; ++it) {
        const int i = it * 16 + l16;  // the query row this lane owns in the transposed score tile
        const unsigned long long mask = i < n ? a.adj_mask[(size_t)(base + i) * a.W] : 0ull;
        float s[kDenseTiles][4];
        float m = -INFINITY;
#pragma unroll
        for (int jt = 0; jt < kDenseTiles; ++jt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            if (jt < tiles) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag_plain<D>(Ks, jt * 16 + l16, ks, q),
                                                                     frag_plain<D>(Qs, i, ks, q), acc, 0, 0, 0);
            }
            const uint32_t bits = (uint32_t)(mask >> (jt * 16 + 4 * q)) & 0xfu;  // keys 4q .. 4q+3 of this tile
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[jt][r] = ((bits >> r) & 1u) ? acc[r] * a.c_score : -INFINITY;
                m = fmaxf(m, s[jt][r]);
            }
        }
        m = max_over_q(m);
        float lsum = 0.f;
        SplitFrag pf[kDenseTiles];
#pragma unroll
        for (int jt = 0; jt < kDenseTiles; ++jt) {
            float p[4] = {0.f, 0.f, 0.f, 0.f};
            if (jt < tiles) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p[r] = s[jt][r] == -INFINITY ? 0.f : fast_exp2(s[jt][r] - m);
                    lsum += p[r];
                }
            }
            pf[jt] = split_bf16x4(p[0], p[1], p[2], p[3]);
        }
        lsum = sum_over_q(lsum);
        if (q == 0 && i < n) {
            a.o_max[(size_t)(base + i) * a.H + h] = m * kLn2;
            a.o_sum[(size_t)(base + i) * a.H + h] = lsum;
        }
        // O rows of the result tile are 4q + r: fetch their denominators from the lanes that own them
        float inv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float lr = __shfl(lsum, 4 * q + r);
            inv[r] = lr > 0.f ? 1.f / lr : 0.f;
        }
#pragma unroll
        for (int nt = 0; nt < KS; ++nt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jt = 0; jt < kDenseTiles; ++jt)
                if (jt < tiles)
                    acc = mfma_split(pf[jt], frag_trans(Vt, nt * 16 + l16, jt * 16 + 4 * q), acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = it * 16 + 4 * q + r;
                if (row < n) a.o[(size_t)(base + row) * a.HD + h * D + nt * 16 + l16] = to_bf16(acc[r] * inv[r]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// backward: row side (dQ) and column side (dK, dV) of one (graph, head) in one wavefront
// ---------------------------------------------------------------------------------------------
template <int D, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_dense_gt_backward(const DenseArgs a) {
    constexpr int KS = D / 16;
    constexpr int PLAIN = kDenseMaxNodes * D, TRANS = D * kTStride;
    __shared__ __attribute__((aligned(16))) uint16_t lds[WAVES][4 * PLAIN + 3 * TRANS];
    __shared__ __attribute__((aligned(16))) float lse_s[WAVES][kDenseMaxNodes], delta_s[WAVES][kDenseMaxNodes];
    __shared__ unsigned long long mask_s[WAVES][kDenseMaxNodes];
    __shared__ unsigned long long maskt_s[WAVES][kDenseMaxNodes];  // bit i of maskt_s[j]: edge i <- j
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int gh = blockIdx.x * WAVES + wave;
    if (gh >= a.n_graphs * a.H) return;
    const int g = gh / a.H, h = gh - g * a.H;
    const int base = a.batch_ptr[g], n = a.batch_ptr[g + 1] - base;
    const int tiles = (n + 15) >> 4;
    const int l16 = lane & 15, q = lane >> 4;
    uint16_t* Qs = lds[wave];
    uint16_t* Ks = Qs + PLAIN;
    uint16_t* Vs = Ks + PLAIN;
    uint16_t* Gs = Vs + PLAIN;
    uint16_t* Qt = Gs + PLAIN;
    uint16_t* Kt = Qt + TRANS;
    uint16_t* Gt = Kt + TRANS;
    const size_t first = (size_t)base * a.HD + (size_t)h * D;
    stage_head<D, true, true>(a.q, first, a.HD, n, tiles, Qs, Qt, lane);
    stage_head<D, true, true>(a.k, first, a.HD, n, tiles, Ks, Kt, lane);
    stage_head<D, true, false>(a.v, first, a.HD, n, tiles, Vs, nullptr, lane);
    stage_head<D, true, true>(a.d_out, first, a.HD, n, tiles, Gs, Gt, lane);
    {
        const int i = lane;  // one row per lane (n <= 64)
        float lse = 0.f;
        unsigned long long mk = 0ull;
        if (i < n) {
            lse = a.row_max[(size_t)(base + i) * a.H + h] * kLog2e + fast_log2(a.row_sum[(size_t)(base + i) * a.H + h]);
            mk = a.adj_mask[(size_t)(base + i) * a.W];
        }
        lse_s[wave][i] = lse;
        mask_s[wave][i] = mk;
        delta_s[wave][i] = 0.f;
        // column masks: a ballot over the 64 rows for every key column of the graph
        unsigned long long mine = 0ull;
        for (int j = 0; j < tiles * 16; ++j) {
            const unsigned long long col = __ballot((mk >> j) & 1ull);
            if (lane == j) mine = col;
        }
        maskt_s[wave][lane] = mine;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // ---- row side: lane owns query row i; dQ_i = scale sum_j dS_ij k_j; delta_i goes to LDS ----
    for (int it = 0; it < tiles; ++it) {
        const int i = it * 16 + l16;
        const unsigned long long mask = mask_s[wave][i];
        const float lse = lse_s[wave][i];
        float p[kDenseTiles][4], dp[kDenseTiles][4];
        float dsum = 0.f;
#pragma unroll
        for (int jt = 0; jt < kDenseTiles; ++jt) {
            f32x4 sa = {0.f, 0.f, 0.f, 0.f}, da = {0.f, 0.f, 0.f, 0.f};
            if (jt < tiles) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    sa = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag_plain<D>(Ks, jt * 16 + l16, ks, q),
                                                                    frag_plain<D>(Qs, i, ks, q), sa, 0, 0, 0);
                    da = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag_plain<D>(Vs, jt * 16 + l16, ks, q),
                                                                    frag_plain<D>(Gs, i, ks, q), da, 0, 0, 0);
                }
            }
            const uint32_t bits = (uint32_t)(mask >> (jt * 16 + 4 * q)) & 0xfu;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[jt][r] = ((bits >> r) & 1u) ? fast_exp2(sa[r] * a.c_score - lse) : 0.f;
                dp[jt][r] = da[r];
                dsum = fmaf(p[jt][r], da[r], dsum);
            }
        }
        const float delta = sum_over_q(dsum);
        if (q == 0) delta_s[wave][i] = delta;
        SplitFrag dsf[kDenseTiles];
#pragma unroll
        for (int jt = 0; jt < kDenseTiles; ++jt)
            dsf[jt] = split_bf16x4(p[jt][0] * (dp[jt][0] - delta), p[jt][1] * (dp[jt][1] - delta),
                                  p[jt][2] * (dp[jt][2] - delta), p[jt][3] * (dp[jt][3] - delta));
#pragma unroll
        for (int nt = 0; nt < KS; ++nt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jt = 0; jt < kDenseTiles; ++jt)
                if (jt < tiles)
                    acc = mfma_split(dsf[jt], frag_trans(Kt, nt * 16 + l16, jt * 16 + 4 * q), acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = it * 16 + 4 * q + r;
                if (row < n) a.d_q[(size_t)(base + row) * a.HD + h * D + nt * 16 + l16] = to_bf16(a.scale * acc[r]);
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // ---- column side: lane owns key column j; rows i = 4q + r of the plain score tile ----
    for (int jt = 0; jt < tiles; ++jt) {
        const int j = jt * 16 + l16;
        const unsigned long long maskt = maskt_s[wave][j];
        f32x4 acc_v[KS], acc_k[KS];
#pragma unroll
        for (int nt = 0; nt < KS; ++nt) { acc_v[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; acc_k[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        for (int it = 0; it < tiles; ++it) {
            f32x4 sa = {0.f, 0.f, 0.f, 0.f}, da = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                sa = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag_plain<D>(Qs, it * 16 + l16, ks, q),
                                                                frag_plain<D>(Ks, j, ks, q), sa, 0, 0, 0);
                da = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag_plain<D>(Gs, it * 16 + l16, ks, q),
                                                                frag_plain<D>(Vs, j, ks, q), da, 0, 0, 0);
            }
            float p[4], ds[4];
            const uint32_t bits = (uint32_t)(maskt >> (it * 16 + 4 * q)) & 0xfu;  // rows 4q .. 4q+3 of this tile
            const f32x4 lse4 = *reinterpret_cast<const f32x4*>(&lse_s[wave][it * 16 + 4 * q]);
            const f32x4 del4 = *reinterpret_cast<const f32x4*>(&delta_s[wave][it * 16 + 4 * q]);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = ((bits >> r) & 1u) ? fast_exp2(sa[r] * a.c_score - lse4[r]) : 0.f;
                ds[r] = p[r] * (da[r] - del4[r]);
            }
            const SplitFrag pf = split_bf16x4(p[0], p[1], p[2], p[3]);
            const SplitFrag dsf = split_bf16x4(ds[0], ds[1], ds[2], ds[3]);
#pragma unroll
            for (int nt = 0; nt < KS; ++nt) {
                acc_v[nt] = mfma_split(pf, frag_trans(Gt, nt * 16 + l16, it * 16 + 4 * q), acc_v[nt]);
                acc_k[nt] = mfma_split(dsf, frag_trans(Qt, nt * 16 + l16, it * 16 + 4 * q), acc_k[nt]);
            }
        }
#pragma unroll
        for (int nt = 0; nt < KS; ++nt) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = jt * 16 + 4 * q + r;
                if (row < n) {
                    const size_t o = (size_t)(base + row) * a.HD + h * D + nt * 16 + l16;
                    a.d_v[o] = to_bf16(acc_v[nt][r]);
                    a.d_k[o] = to_bf16(a.scale * acc_k[nt][r]);
                }
            }
        }
    }
}

// The dense kernels form every 16 x 16 score tile of a graph whatever its density, the gather kernels pay
// per edge, so what decides is how full the tiles are: fill = E / (256 * tile pairs).  Measured on MI355X
// against the gather kernels:
//   bf16 kernels of this file:   0.83x at fill 0.19, 1.5x at 0.24, 3.5x at 0.94   -> used from 0.22
//   fp32 streaming kernels:      0.70x at 0.10, 0.91x at 0.18, 1.04x at 0.23, 1.2x at 0.28, 1.5x at 0.39
//                                -> used from 0.22
//   bf16 streaming kernels:      0.53x at 0.10, 1.06x at 0.18, 1.16x at 0.23, 1.5x at 0.39 (2.5x for one head
//                                of 64 features)   -> used from 0.20
// The streaming kernels gain less because they fetch their operands again for every row tile and spend
// most of their time on the softmax arithmetic of masked-out tile entries.
constexpr int64_t kDenseMinEdgesPerTileBf16 = 56;        // 0.22 * 256
constexpr int64_t kDenseMinEdgesPerTileBf16Stream = 52;  // 0.20 * 256
constexpr int64_t kDenseMinEdgesPerTileF32 = 56;         // 0.22 * 256

// 1: bf16 kernels of this file (graphs of at most 64 nodes, staged in LDS); 2: fp32 streaming kernels
// (dense_batch_f32.hip); 3: bf16 streaming kernels (dense_batch_bf16.hip); 0: general kernels
int dense_batch_kind(const dfgnn_graph* g, const dfgnn_layer* L) {
    if (!g->batch_dense || (g->flags & DFGNN_SCHED_NO_DENSE_BATCH) || L->model != DFGNN_GT) return 0;
    const bool force = g->flags & DFGNN_SCHED_FORCE_DENSE_BATCH;
    const bool width_ok = L->D == 16 || L->D == 32 || L->D == 64;
    if (L->dtype == DFGNN_BF16 && width_ok) {
        const bool small = L->D <= 32 && g->max_graph_nodes <= kDenseSmallNodes;
        const int64_t need = small ? kDenseMinEdgesPerTileBf16 : kDenseMinEdgesPerTileBf16Stream;
        if (!force && g->E < need * g->tile_pairs) return 0;
        return small ? 1 : 3;
    }
    if (L->dtype == DFGNN_F32 && width_ok)
        return (force || g->E >= kDenseMinEdgesPerTileF32 * g->tile_pairs) ? 2 : 0;
    return 0;
}

static DenseArgs dense_args(const dfgnn_graph* g, const dfgnn_layer* L) {
    DenseArgs a{};
    a.batch_ptr = g->batch_ptr;
    a.adj_mask = g->adj_mask;
    a.n_graphs = (int)g->n_graphs;
    a.W = g->mask_words;
    a.H = L->H; a.D = L->D; a.HD = L->H * L->D;
    a.scale = L->scale;
    a.c_score = L->scale * kLog2e;
    return a;
}

int dense_gt_forward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v, void* out,
                     float* row_max, float* row_sum, hipStream_t st) {
    DenseArgs a = dense_args(g, L);
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
    a.o = (uint16_t*)out; a.o_max = row_max; a.o_sum = row_sum;
    const int64_t waves = g->n_graphs * L->H;
    if (waves == 0) return DFGNN_OK;
    KernelTimer t("dense_fwd", st);
    if (L->D == 16) hipLaunchKernelGGL((k_dense_gt_forward<16, 4>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((k_dense_gt_forward<32, 4>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, a);
    return DFGNN_OK;
}

int dense_gt_backward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v,
                      const float* row_max, const float* row_sum, const void* d_out, void* d_q, void* d_k, void* d_v,
                      hipStream_t st) {
    DenseArgs a = dense_args(g, L);
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_out = (const uint16_t*)d_out;
    a.row_max = row_max; a.row_sum = row_sum;
    a.d_q = (uint16_t*)d_q; a.d_k = (uint16_t*)d_k; a.d_v = (uint16_t*)d_v;
    const int64_t waves = g->n_graphs * L->H;
    if (waves == 0) return DFGNN_OK;
    KernelTimer t("dense_bwd", st);
    // LDS per wavefront: 15 KB (D = 16) or 30 KB (D = 32) of staged tiles plus 1 KB of row statistics
    if (L->D == 16) hipLaunchKernelGGL((k_dense_gt_backward<16, 2>), dim3((unsigned)((waves + 1) / 2)), dim3(128), 0, st, a);
    else hipLaunchKernelGGL((k_dense_gt_backward<32, 1>), dim3((unsigned)waves), dim3(64), 0, st, a);
    return DFGNN_OK;
}

}  // namespace dfgnn
