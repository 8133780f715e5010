// Dense-tile kernels for batches of small graphs, GT model, fp32 tensors, graphs of up to 512 nodes
// (the batch-graph workloads of Sec. 5.1: 70-480 nodes per graph at batch size 1024).
//
// One wavefront works on one (graph, head, tile of 16 rows): it streams over the graph's 16-node
// column tiles, forms each 16 x 16 score tile with four v_mfma_f32_16x16x4_f32 per 16 features, masks
// missing edges with the row's adjacency bits, and feeds the attention weights straight back into
// MFMA for the aggregation.  Operands are read from memory (the L2, after a graph's first touch) in
// exactly the per-lane layout the instruction wants, so no LDS is used at all:
//   lane l, q = l / 16:  A[m = l % 16][k = q],  B[k = q][n = l % 16],  C[m = 4q + r][n = l % 16].
// The contraction over the features is order-free, so MFMA number ks of a 16-feature block is given
// feature 4q + ks: a lane then needs 4 consecutive features of one row, i.e. one 16-byte load.
// Score tiles are computed transposed (S^T = K Q^T): a lane owns query row i = l % 16 and keys
// j = 4q + r, which is the A-operand layout of the second product (k index q <-> key 4q + r in MFMA
// number r, whose B operand is the single element V[4q + r][l % 16]).
// The forward kernel makes two sweeps over the column tiles (row maximum and sum, then weights and
// aggregation); recomputing the score tile costs four MFMAs and avoids rescaling the accumulator.
#include "common.hpp"
#include "layer_device.hpp"

namespace dfgnn {

struct DenseF32Args {
    const int* batch_ptr;
    const int* tile_ptr;                   // first 16-row tile of every graph
    const unsigned long long* adj_mask;    // [N][W]: bit j of row i's words = edge i <- (first node of the graph + j)
    const unsigned long long* adj_mask_t;  // [N][W]: bit i of column j's words = edge (first + i) <- j
    const float *q, *k, *v, *out, *d_out, *row_max, *row_sum;
    float *o, *o_max, *o_sum, *d_q, *d_k, *d_v, *stats;
    int n_graphs, n_tiles, W, H, HD;
    float c_score, scale;
};

struct Unit {
    int base, n, tiles, t, h;  // graph's first node, node count, tile count; this wave's tile and head
};

__device__ inline Unit find_unit(const DenseF32Args& a, int u) {
    const int tile = u / a.H;
    Unit r;
    r.h = u - tile * a.H;
    int lo = 0, hi = a.n_graphs;  // last graph whose first tile is <= tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tile_ptr[mid] <= tile) lo = mid; else hi = mid;
    }
    r.base = a.batch_ptr[lo];
    r.n = a.batch_ptr[lo + 1] - r.base;
    r.tiles = (r.n + 15) >> 4;
    r.t = tile - a.tile_ptr[lo];
    return r;
}

// features kb*16 + 4q .. +3 of node `row` of the unit's graph and head (zeros past the graph's end)
__device__ inline f32x4 row_frag(const float* x, const DenseF32Args& a, const Unit& u, int row, int kb, int q, int D) {
    f32x4 z = {0.f, 0.f, 0.f, 0.f};
    if (row < u.n) z = *reinterpret_cast<const f32x4*>(x + (size_t)(u.base + row) * a.HD + u.h * D + kb * 16 + 4 * q);
    return z;
}
__device__ inline float elem(const float* x, const DenseF32Args& a, const Unit& u, int row, int d, int D) {
    return row < u.n ? x[(size_t)(u.base + row) * a.HD + u.h * D + d] : 0.f;
}
// bits for entries 4q .. 4q+3 of 16-wide tile `t` in a row of mask words (nullptr: no bits)
__device__ inline uint32_t tile_bits(const unsigned long long* words, int t, int q) {
    return words ? (uint32_t)(words[t >> 2] >> ((t & 3) * 16 + 4 * q)) & 0xfu : 0u;
}

template <int KB> __device__ inline f32x4 tile_product(const f32x4 (&a)[KB], const f32x4 (&b)[KB]) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[kb][ks], b[kb][ks], acc, 0, 0, 0);
    return acc;
}

__device__ inline float sum_q(float x) { x += __shfl_xor(x, 16); x += __shfl_xor(x, 32); return x; }

constexpr int kDenseWaves = 4;

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense32_forward(const DenseF32Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = blockIdx.x * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const int i = u.t * 16 + l16;
    f32x4 qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) qf[kb] = row_frag(a.q, a, u, i, kb, q, D) * a.c_score;
    const unsigned long long* mrow = i < u.n ? a.adj_mask + (size_t)(u.base + i) * a.W : nullptr;

    // sweep 1: maximum and sum of the row's exponentials, each lane over its own keys
    float m = -INFINITY, l = 0.f;
    for (int jt = 0; jt < u.tiles; ++jt) {
        f32x4 kf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = row_frag(a.k, a, u, jt * 16 + l16, kb, q, D);
        const f32x4 s = tile_product<KB>(kf, qf);
        const uint32_t bits = tile_bits(mrow, jt, q);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if ((bits >> r) & 1u) {
                const float mn = fmaxf(m, s[r]);
                l = l * fast_exp2(m - mn) + fast_exp2(s[r] - mn);
                m = mn;
            }
        }
    }
#pragma unroll
    for (int o = 16; o < 64; o <<= 1) {
        const float mo = __shfl_xor(m, o), lo = __shfl_xor(l, o);
        const float mn = fmaxf(m, mo);
        l = (m == mn ? l : l * fast_exp2(m - mn)) + (mo == mn ? lo : lo * fast_exp2(mo - mn));
        m = mn;
    }
    if (q == 0 && i < u.n) {
        a.o_max[(size_t)(u.base + i) * a.H + u.h] = m * kLn2;
        a.o_sum[(size_t)(u.base + i) * a.H + u.h] = l;
    }

    // sweep 2: weights and aggregation
    f32x4 acc[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int jt = 0; jt < u.tiles; ++jt) {
        f32x4 kf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = row_frag(a.k, a, u, jt * 16 + l16, kb, q, D);
        float vv[KB][4];
#pragma unroll
        for (int nt = 0; nt < KB; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) vv[nt][r] = elem(a.v, a, u, jt * 16 + 4 * q + r, nt * 16 + l16, D);
        const f32x4 s = tile_product<KB>(kf, qf);
        const uint32_t bits = tile_bits(mrow, jt, q);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = ((bits >> r) & 1u) ? fast_exp2(s[r] - m) : 0.f;
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(p, vv[nt][r], acc[nt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float lr = __shfl(l, 4 * q + r);  // denominator of result row 4q + r
        const float inv = lr > 0.f ? 1.f / lr : 0.f;
        const int row = u.t * 16 + 4 * q + r;
        if (row < u.n) {
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) a.o[(size_t)(u.base + row) * a.HD + u.h * D + nt * 16 + l16] = acc[nt][r] * inv;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// backward, row side: dQ and the row statistics {lse2, delta} for the column side
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense32_backward_rows(const DenseF32Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = blockIdx.x * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const int i = u.t * 16 + l16;
    f32x4 qf[KB], gf[KB];
    float dsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = row_frag(a.q, a, u, i, kb, q, D) * a.c_score;
        gf[kb] = row_frag(a.d_out, a, u, i, kb, q, D);
        const f32x4 of = row_frag(a.out, a, u, i, kb, q, D);
#pragma unroll
        for (int e = 0; e < 4; ++e) dsum = fmaf(gf[kb][e], of[e], dsum);
    }
    const float delta = sum_q(dsum);  // dO_i . O_i = sum_j p_ij dP_ij
    float lse = 0.f;
    if (i < u.n)
        lse = a.row_max[(size_t)(u.base + i) * a.H + u.h] * kLog2e + fast_log2(a.row_sum[(size_t)(u.base + i) * a.H + u.h]);
    const unsigned long long* mrow = i < u.n ? a.adj_mask + (size_t)(u.base + i) * a.W : nullptr;
    if (q == 0 && i < u.n) {
        f32x2 st = {lse, delta};
        *reinterpret_cast<f32x2*>(a.stats + 2 * ((size_t)(u.base + i) * a.H + u.h)) = st;
    }
    f32x4 acc[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int jt = 0; jt < u.tiles; ++jt) {
        f32x4 kf[KB], vf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            kf[kb] = row_frag(a.k, a, u, jt * 16 + l16, kb, q, D);
            vf[kb] = row_frag(a.v, a, u, jt * 16 + l16, kb, q, D);
        }
        float kk[KB][4];
#pragma unroll
        for (int nt = 0; nt < KB; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) kk[nt][r] = elem(a.k, a, u, jt * 16 + 4 * q + r, nt * 16 + l16, D);
        const f32x4 s = tile_product<KB>(kf, qf);
        const f32x4 dp = tile_product<KB>(vf, gf);
        const uint32_t bits = tile_bits(mrow, jt, q);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = ((bits >> r) & 1u) ? fast_exp2(s[r] - lse) : 0.f;
            const float ds = p * (dp[r] - delta);
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(ds, kk[nt][r], acc[nt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = u.t * 16 + 4 * q + r;
        if (row < u.n) {
#pragma unroll
            for (int nt = 0; nt < KB; ++nt)
                a.d_q[(size_t)(u.base + row) * a.HD + u.h * D + nt * 16 + l16] = a.scale * acc[nt][r];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// backward, column side: dK and dV of one tile of 16 key columns
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense32_backward_cols(const DenseF32Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = blockIdx.x * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const int j = u.t * 16 + l16;
    f32x4 kf[KB], vf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        kf[kb] = row_frag(a.k, a, u, j, kb, q, D) * a.c_score;
        vf[kb] = row_frag(a.v, a, u, j, kb, q, D);
    }
    const unsigned long long* mcol = j < u.n ? a.adj_mask_t + (size_t)(u.base + j) * a.W : nullptr;
    f32x4 acc_v[KB], acc_k[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) { acc_v[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; acc_k[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    for (int it = 0; it < u.tiles; ++it) {
        f32x4 qf[KB], gf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            qf[kb] = row_frag(a.q, a, u, it * 16 + l16, kb, q, D);
            gf[kb] = row_frag(a.d_out, a, u, it * 16 + l16, kb, q, D);
        }
        float qq[KB][4], gg[KB][4], lse[4], delta[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = it * 16 + 4 * q + r;
            f32x2 st = {0.f, 0.f};
            if (row < u.n) st = *reinterpret_cast<const f32x2*>(a.stats + 2 * ((size_t)(u.base + row) * a.H + u.h));
            lse[r] = st[0];
            delta[r] = st[1];
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) {
                qq[nt][r] = elem(a.q, a, u, row, nt * 16 + l16, D);
                gg[nt][r] = elem(a.d_out, a, u, row, nt * 16 + l16, D);
            }
        }
        const f32x4 s = tile_product<KB>(qf, kf);    // s[r] = score of (row 4q + r of the tile, column j)
        const f32x4 dp = tile_product<KB>(gf, vf);
        const uint32_t bits = tile_bits(mcol, it, q);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = ((bits >> r) & 1u) ? fast_exp2(s[r] - lse[r]) : 0.f;
            const float ds = p * (dp[r] - delta[r]);
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) {
                acc_v[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(p, gg[nt][r], acc_v[nt], 0, 0, 0);
                acc_k[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(ds, qq[nt][r], acc_k[nt], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = u.t * 16 + 4 * q + r;
        if (row < u.n) {
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) {
                const size_t o = (size_t)(u.base + row) * a.HD + u.h * D + nt * 16 + l16;
                a.d_v[o] = acc_v[nt][r];
                a.d_k[o] = a.scale * acc_k[nt][r];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static DenseF32Args dense32_args(const dfgnn_graph* g, const dfgnn_layer* L) {
    DenseF32Args a{};
    a.batch_ptr = g->batch_ptr;
    a.tile_ptr = g->tile_ptr;
    a.adj_mask = g->adj_mask;
    a.adj_mask_t = g->adj_mask_t;
    a.n_graphs = (int)g->n_graphs;
    a.n_tiles = (int)g->n_tiles;
    a.W = g->mask_words;
    a.H = L->H;
    a.HD = L->H * L->D;
    a.scale = L->scale;
    a.c_score = L->scale * kLog2e;
    return a;
}

template <typename F16, typename F32, typename F64>
static void launch_by_width(int D, F16 f16, F32 f32, F64 f64) {
    if (D == 16) f16();
    else if (D == 32) f32();
    else f64();
}

int dense32_gt_forward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v, void* out,
                       float* row_max, float* row_sum, hipStream_t st) {
    DenseF32Args a = dense32_args(g, L);
    a.q = (const float*)q; a.k = (const float*)k; a.v = (const float*)v;
    a.o = (float*)out; a.o_max = row_max; a.o_sum = row_sum;
    const int64_t waves = g->n_tiles * L->H;
    if (waves == 0) return DFGNN_OK;
    const dim3 grid((unsigned)((waves + kDenseWaves - 1) / kDenseWaves)), block(64 * kDenseWaves);
    KernelTimer t("dense_fwd", st);
    launch_by_width(L->D, [&] { hipLaunchKernelGGL((k_dense32_forward<1>), grid, block, 0, st, a); },
                    [&] { hipLaunchKernelGGL((k_dense32_forward<2>), grid, block, 0, st, a); },
                    [&] { hipLaunchKernelGGL((k_dense32_forward<4>), grid, block, 0, st, a); });
    return DFGNN_OK;
}

int dense32_gt_backward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v,
                        const void* out, const float* row_max, const float* row_sum, const void* d_out, void* d_q,
                        void* d_k, void* d_v, float* stats, hipStream_t st) {
    DenseF32Args a = dense32_args(g, L);
    a.q = (const float*)q; a.k = (const float*)k; a.v = (const float*)v; a.out = (const float*)out;
    a.d_out = (const float*)d_out; a.row_max = row_max; a.row_sum = row_sum;
    a.d_q = (float*)d_q; a.d_k = (float*)d_k; a.d_v = (float*)d_v; a.stats = stats;
    const int64_t waves = g->n_tiles * L->H;
    if (waves == 0) return DFGNN_OK;
    const dim3 grid((unsigned)((waves + kDenseWaves - 1) / kDenseWaves)), block(64 * kDenseWaves);
    {
        KernelTimer t("dense_bwd_rows", st);
        launch_by_width(L->D, [&] { hipLaunchKernelGGL((k_dense32_backward_rows<1>), grid, block, 0, st, a); },
                        [&] { hipLaunchKernelGGL((k_dense32_backward_rows<2>), grid, block, 0, st, a); },
                        [&] { hipLaunchKernelGGL((k_dense32_backward_rows<4>), grid, block, 0, st, a); });
    }
    {
        KernelTimer t("dense_bwd_cols", st);
        launch_by_width(L->D, [&] { hipLaunchKernelGGL((k_dense32_backward_cols<1>), grid, block, 0, st, a); },
                        [&] { hipLaunchKernelGGL((k_dense32_backward_cols<2>), grid, block, 0, st, a); },
                        [&] { hipLaunchKernelGGL((k_dense32_backward_cols<4>), grid, block, 0, st, a); });
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
