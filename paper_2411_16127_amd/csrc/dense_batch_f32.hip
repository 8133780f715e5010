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
// The forward kernel makes two sweeps over the column tiles (row maximum, then weights, their sum and the
// aggregation); recomputing the score tile costs four MFMAs and avoids rescaling the accumulator.
// All loads of the tile loops are buffer loads against a view of the wavefront's own graph and head
// (rows past the graph's end read as zero), so the loops have no bounds checks and no branches.
#include "common.hpp"
#include "layer_device.hpp"
#include "dense_stream.hpp"

namespace dfgnn {

struct DenseF32Args {
    const int* batch_ptr;
    const int* tile_ptr;                   // first 16-row tile of every graph
    const int* tile_graph;                 // graph of every 16-row tile
    const unsigned long long* adj_mask;    // [N][W]: bit j of row i's words = edge i <- (first node of the graph + j)
    const unsigned long long* adj_mask_t;  // [N][W]: bit i of column j's words = edge (first + i) <- j
    const float *q, *k, *v, *out, *d_out, *row_max, *row_sum;
    float *o, *o_max, *o_sum, *d_q, *d_k, *d_v, *stats;
    int n_graphs, n_tiles, W, H, HD;
    float c_score, scale;
};

// Per-lane byte offsets into a unit's tensor view for column (or row) tile 0; a tile step adds 16 rows.
struct LaneOffsets32 {
    uint32_t frag;  // features 4q .. 4q+3 of row l16 (operands of a score product)
    uint32_t col;   // feature l16 of row 4q (B operand of a second product: rows 4q .. 4q+3)
    uint32_t row_bytes, tile_bytes;
};
__device__ inline LaneOffsets32 lane_offsets32(int HD, int l16, int q) {
    LaneOffsets32 o;
    o.row_bytes = (uint32_t)HD * 4u;
    o.tile_bytes = 16u * o.row_bytes;
    o.frag = (uint32_t)l16 * o.row_bytes + (uint32_t)q * 16u;
    o.col = (uint32_t)(4 * q) * o.row_bytes + (uint32_t)l16 * 4u;
    return o;
}

template <int KB> __device__ inline f32x4 tile_product(const f32x4 (&a)[KB], const f32x4 (&b)[KB]) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[kb][ks], b[kb][ks], acc, 0, 0, 0);
    return acc;
}

// ---------------------------------------------------------------------------------------------
// forward: a sweep for the row maximum, then a sweep for weights, their sum and the aggregation
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense32_forward(const DenseF32Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = xcd_block(blockIdx.x, gridDim.x) * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const LaneOffsets32 lo = lane_offsets32(a.HD, l16, q);
    const rsrc_t rq = unit_tensor(a.q, u, a.HD, D, 4), rk = unit_tensor(a.k, u, a.HD, D, 4), rv = unit_tensor(a.v, u, a.HD, D, 4);
    const rsrc_t rm = unit_rows(a.adj_mask, u, a.W * 8, 0, a.W * 8);
    const int i = u.t * 16 + l16;
    const uint32_t moff = (uint32_t)i * (uint32_t)(a.W * 8);
    f32x4 qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) qf[kb] = buf_load_f32x4(rq, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 64u) * a.c_score;

    float m = -INFINITY;
    for (int jt = 0; jt < u.tiles; ++jt) {
        f32x4 kf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = buf_load_f32x4(rk, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 64u);
        const uint32_t bits = tile_bits(rm, moff, jt, q);
        const f32x4 s = tile_product<KB>(kf, qf);
#pragma unroll
        for (int r = 0; r < 4; ++r) m = fmaxf(m, ((bits >> r) & 1u) ? s[r] : -INFINITY);
    }
    m = max_q(m);

    float l = 0.f;
    f32x4 acc[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int jt = 0; jt < u.tiles; ++jt) {
        f32x4 kf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = buf_load_f32x4(rk, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 64u);
        float vv[KB][4];
#pragma unroll
        for (int nt = 0; nt < KB; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) vv[nt][r] = buf_load_f32(rv, lo.col + (uint32_t)jt * lo.tile_bytes + r * lo.row_bytes + nt * 64u);
        const uint32_t bits = tile_bits(rm, moff, jt, q);
        const f32x4 s = tile_product<KB>(kf, qf);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = ((bits >> r) & 1u) ? fast_exp2(s[r] - m) : 0.f;
            l += p;
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(p, vv[nt][r], acc[nt], 0, 0, 0);
        }
    }
    l = sum_q(l);
    if (q == 0 && i < u.n) {
        a.o_max[(size_t)(u.base + i) * a.H + u.h] = m * kLn2;
        a.o_sum[(size_t)(u.base + i) * a.H + u.h] = l;
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
    const int uidx = xcd_block(blockIdx.x, gridDim.x) * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const LaneOffsets32 lo = lane_offsets32(a.HD, l16, q);
    const rsrc_t rq = unit_tensor(a.q, u, a.HD, D, 4), rk = unit_tensor(a.k, u, a.HD, D, 4), rv = unit_tensor(a.v, u, a.HD, D, 4);
    const rsrc_t rg = unit_tensor(a.d_out, u, a.HD, D, 4), ro = unit_tensor(a.out, u, a.HD, D, 4);
    const rsrc_t rm = unit_rows(a.adj_mask, u, a.W * 8, 0, a.W * 8);
    const int i = u.t * 16 + l16;
    const uint32_t moff = (uint32_t)i * (uint32_t)(a.W * 8);
    f32x4 qf[KB], gf[KB];
    float dsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        const uint32_t off = lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 64u;
        qf[kb] = buf_load_f32x4(rq, off) * a.c_score;
        gf[kb] = buf_load_f32x4(rg, off);
        const f32x4 of = buf_load_f32x4(ro, off);
#pragma unroll
        for (int e = 0; e < 4; ++e) dsum = fmaf(gf[kb][e], of[e], dsum);
    }
    const float delta = sum_q(dsum);  // dO_i . O_i = sum_j p_ij dP_ij
    float lse = 0.f;
    if (i < u.n)
        lse = a.row_max[(size_t)(u.base + i) * a.H + u.h] * kLog2e + fast_log2(a.row_sum[(size_t)(u.base + i) * a.H + u.h]);
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
            kf[kb] = buf_load_f32x4(rk, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 64u);
            vf[kb] = buf_load_f32x4(rv, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 64u);
        }
        float kk[KB][4];
#pragma unroll
        for (int nt = 0; nt < KB; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) kk[nt][r] = buf_load_f32(rk, lo.col + (uint32_t)jt * lo.tile_bytes + r * lo.row_bytes + nt * 64u);
        const uint32_t bits = tile_bits(rm, moff, jt, q);
        const f32x4 s = tile_product<KB>(kf, qf);
        const f32x4 dp = tile_product<KB>(vf, gf);
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
    const int uidx = xcd_block(blockIdx.x, gridDim.x) * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const LaneOffsets32 lo = lane_offsets32(a.HD, l16, q);
    const rsrc_t rq = unit_tensor(a.q, u, a.HD, D, 4), rk = unit_tensor(a.k, u, a.HD, D, 4), rv = unit_tensor(a.v, u, a.HD, D, 4);
    const rsrc_t rg = unit_tensor(a.d_out, u, a.HD, D, 4);
    const rsrc_t rm = unit_rows(a.adj_mask_t, u, a.W * 8, 0, a.W * 8);
    const rsrc_t rs = unit_rows(a.stats, u, a.H * 8, u.h * 8, 8);  // {lse2, delta} of (row, this head)
    const int j = u.t * 16 + l16;
    const uint32_t moff = (uint32_t)j * (uint32_t)(a.W * 8);
    const uint32_t soff = (uint32_t)(4 * q) * (uint32_t)(a.H * 8);
    f32x4 kf[KB], vf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        kf[kb] = buf_load_f32x4(rk, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 64u) * a.c_score;
        vf[kb] = buf_load_f32x4(rv, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 64u);
    }
    f32x4 acc_v[KB], acc_k[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) { acc_v[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; acc_k[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    for (int it = 0; it < u.tiles; ++it) {
        f32x4 qf[KB], gf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            qf[kb] = buf_load_f32x4(rq, lo.frag + (uint32_t)it * lo.tile_bytes + kb * 64u);
            gf[kb] = buf_load_f32x4(rg, lo.frag + (uint32_t)it * lo.tile_bytes + kb * 64u);
        }
        float qq[KB][4], gg[KB][4];
        f32x2 st[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            st[r] = buf_load_f32x2(rs, soff + (uint32_t)(it * 16 + r) * (uint32_t)(a.H * 8));
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) {
                const uint32_t off = lo.col + (uint32_t)it * lo.tile_bytes + r * lo.row_bytes + nt * 64u;
                qq[nt][r] = buf_load_f32(rq, off);
                gg[nt][r] = buf_load_f32(rg, off);
            }
        }
        const uint32_t bits = tile_bits(rm, moff, it, q);
        const f32x4 s = tile_product<KB>(qf, kf);    // s[r] = score of (row 4q + r of the tile, column j)
        const f32x4 dp = tile_product<KB>(gf, vf);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = ((bits >> r) & 1u) ? fast_exp2(s[r] - st[r][0]) : 0.f;
            const float ds = p * (dp[r] - st[r][1]);
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
    a.tile_graph = g->tile_graph;
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
