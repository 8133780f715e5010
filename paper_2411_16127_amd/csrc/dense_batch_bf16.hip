// Dense-tile kernels for batches of small graphs, GT model, bf16 tensors, graphs of up to 512 nodes
// (the batch-graph workloads of Sec. 5.1: 70-480 nodes per graph at batch size 1024).
//
// Same decomposition as the fp32 streaming kernels: one wavefront works on one (graph, head, tile of 16
// rows) and walks over the graph's 16-node column tiles.  Products use
// v_mfma_f32_16x16x16_bf16, whose per-lane operand layout is
//   lane l, q = l / 16:  A[m = l % 16][k = 4q .. 4q+3],  B[k = 4q .. 4q+3][n = l % 16],  C[m = 4q + r][n = l % 16].
// A score tile is computed transposed (S^T = K Q^T): both operands are 8-byte loads of 4 consecutive
// features of one row, and a lane ends up with query row i = l % 16 and keys j = 4q + r, which is the
// A-operand layout of the second product (k index 4q + r <-> key), so the attention weights go back
// into MFMA from registers.  The B operand of a second product holds one feature of 4 consecutive rows:
// four 2-byte loads in the forward kernel, a transpose of the row-fragment tile through a 640-byte patch
// of LDS per wavefront in the backward kernels.  Attention weights and their gradients are fp32 values: they are fed as a bf16
// head plus a bf16 remainder (two MFMAs), so the second products keep about 16 bits of them.
// All loads of the tile loops are buffer loads against a view of the wavefront's own graph and head
// (rows past the graph's end read as zero), so the loops have no bounds checks and no branches.
// The row statistics are exact: delta_i = sum_j p_ij dP_ij is accumulated by the row kernel itself
// (sum_j p (dP - delta) k_j = sum_j p dP k_j - delta sum_j p k_j), not read off the bf16-rounded output.
#include "common.hpp"
#include "layer_device.hpp"
#include "dense_bf16.hpp"
#include "dense_stream.hpp"

namespace dfgnn {

struct DenseBf16Args {
    const int* batch_ptr;
    const int* tile_ptr;                   // first 16-row tile of every graph
    const int* tile_graph;                 // graph of every 16-row tile
    const unsigned long long* adj_mask;    // [N][W]: bit j of row i's words = edge i <- (first node of the graph + j)
    const unsigned long long* adj_mask_t;  // [N][W]: bit i of column j's words = edge (first + i) <- j
    const uint16_t *q, *k, *v, *d_out;
    const float *row_max, *row_sum;
    uint16_t *o, *d_q, *d_k, *d_v;
    float *o_max, *o_sum, *stats;
    int n_graphs, n_tiles, W, H, HD;
    float c_score, scale;
};

// Per-lane byte offsets into a unit's tensor view for column (or row) tile 0; a tile step adds 16 rows.
struct LaneOffsets {
    uint32_t frag;  // 4 consecutive features 4q .. 4q+3 of row l16 (A / B operand of a score product)
    uint32_t col;   // feature l16 of row 4q (B operand of a second product: rows 4q .. 4q+3)
    uint32_t row_bytes, tile_bytes;
};
__device__ inline LaneOffsets lane_offsets16(int HD, int l16, int q) {
    LaneOffsets o;
    o.row_bytes = (uint32_t)HD * 2u;
    o.tile_bytes = 16u * o.row_bytes;
    o.frag = (uint32_t)l16 * o.row_bytes + (uint32_t)q * 8u;
    o.col = (uint32_t)(4 * q) * o.row_bytes + (uint32_t)l16 * 2u;
    return o;
}
__device__ inline s16x4 load_frag16(rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(s16x4, __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0));
}
// one feature of 4 consecutive rows, straight from memory (four 2-byte loads)
__device__ inline s16x4 load_col16(rsrc_t r, uint32_t off, uint32_t row_bytes) {
    s16x4 z;
#pragma unroll
    for (int k = 0; k < 4; ++k) z[k] = (short)__builtin_amdgcn_raw_buffer_load_b16(r, off + (uint32_t)k * row_bytes, 0, 0);
    return z;
}
// A 16 x 16 tile held as row fragments (lane (l16, q): features 4q .. 4q+3 of row l16) turned into column
// fragments (lane (l16, q): feature l16 of rows 4q .. 4q+3), the B-operand layout of a second product,
// through a patch of the wavefront's own LDS.  Rows are 20 elements apart: the 8-byte writes stay aligned
// and the four row groups of a transposed read fall into different banks.  The backward kernels, which
// need the transposed form of tiles they hold as row fragments anyway, use this instead of 2-byte loads
// (measured 8-14 % faster); the forward kernel, which would have to fetch the V tile twice, does not.
constexpr int kPatchStride = 20;
constexpr int kPatchElems = 16 * kPatchStride;
__device__ inline s16x4 transpose_tile(uint16_t* patch, s16x4 frag, int l16, int q) {
    *reinterpret_cast<s16x4*>(patch + l16 * kPatchStride + 4 * q) = frag;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    s16x4 z;
#pragma unroll
    for (int r = 0; r < 4; ++r) z[r] = (short)patch[(4 * q + r) * kPatchStride + l16];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return z;
}
template <int KB> __device__ inline f32x4 tile_product16(const s16x4 (&a)[KB], const s16x4 (&b)[KB]) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[kb], b[kb], acc, 0, 0, 0);
    return acc;
}

// ---------------------------------------------------------------------------------------------
// forward: a sweep for the row maximum, then a sweep for weights, their sum and the aggregation
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense16_forward(const DenseBf16Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = xcd_block(blockIdx.x, gridDim.x) * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const LaneOffsets lo = lane_offsets16(a.HD, l16, q);
    const rsrc_t rq = unit_tensor(a.q, u, a.HD, D, 2), rk = unit_tensor(a.k, u, a.HD, D, 2), rv = unit_tensor(a.v, u, a.HD, D, 2);
    const rsrc_t rm = unit_rows(a.adj_mask, u, a.W * 8, 0, a.W * 8);
    const int i = u.t * 16 + l16;
    const uint32_t moff = (uint32_t)i * (uint32_t)(a.W * 8);
    s16x4 qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) qf[kb] = load_frag16(rq, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 32u);

    // The operands of tile jt + 1 are requested before tile jt is worked on (a tile past the end reads as
    // zeros and is never used), so the loads of one iteration overlap the arithmetic of the previous one.
    struct Tile1 { s16x4 kf[KB]; uint32_t bits; };
    auto fetch1 = [&](int jt, Tile1& t) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) t.kf[kb] = load_frag16(rk, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 32u);
        t.bits = tile_bits(rm, moff, jt, q);
    };
    float m = -INFINITY;
    Tile1 c1, n1;
    fetch1(0, c1);
    for (int jt = 0; jt < u.tiles; ++jt) {
        fetch1(jt + 1, n1);
        const f32x4 s = tile_product16<KB>(c1.kf, qf) * a.c_score;
#pragma unroll
        for (int r = 0; r < 4; ++r) m = fmaxf(m, ((c1.bits >> r) & 1u) ? s[r] : -INFINITY);
        c1 = n1;
    }
    m = max_q(m);

    float l = 0.f;
    f32x4 acc[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    struct Tile2 { s16x4 kf[KB], vc[KB]; uint32_t bits; };
    auto fetch2 = [&](int jt, Tile2& t) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) t.kf[kb] = load_frag16(rk, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 32u);
#pragma unroll
        for (int nt = 0; nt < KB; ++nt) t.vc[nt] = load_col16(rv, lo.col + (uint32_t)jt * lo.tile_bytes + nt * 32u, lo.row_bytes);
        t.bits = tile_bits(rm, moff, jt, q);
    };
    Tile2 c2, n2;
    fetch2(0, c2);
    for (int jt = 0; jt < u.tiles; ++jt) {
        fetch2(jt + 1, n2);
        const f32x4 s = tile_product16<KB>(c2.kf, qf);
        float p[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p[r] = ((c2.bits >> r) & 1u) ? fast_exp2(fmaf(s[r], a.c_score, -m)) : 0.f;
            l += p[r];
        }
        const SplitFrag pf = split_bf16x4(p[0], p[1], p[2], p[3]);  // bf16 head + remainder: the sum l above is of the fp32 weights
#pragma unroll
        for (int nt = 0; nt < KB; ++nt) acc[nt] = mfma_split(pf, c2.vc[nt], acc[nt]);
        c2 = n2;
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
            for (int nt = 0; nt < KB; ++nt)
                a.o[(size_t)(u.base + row) * a.HD + u.h * D + nt * 16 + l16] = to_bf16(acc[nt][r] * inv);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// backward, row side: dQ and the row statistics {lse2, delta} for the column side
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense16_backward_rows(const DenseBf16Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = xcd_block(blockIdx.x, gridDim.x) * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const LaneOffsets lo = lane_offsets16(a.HD, l16, q);
    const rsrc_t rq = unit_tensor(a.q, u, a.HD, D, 2), rk = unit_tensor(a.k, u, a.HD, D, 2), rv = unit_tensor(a.v, u, a.HD, D, 2);
    const rsrc_t rg = unit_tensor(a.d_out, u, a.HD, D, 2);
    const rsrc_t rm = unit_rows(a.adj_mask, u, a.W * 8, 0, a.W * 8);
    const int i = u.t * 16 + l16;
    const uint32_t moff = (uint32_t)i * (uint32_t)(a.W * 8);
    s16x4 qf[KB], gf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = load_frag16(rq, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 32u);
        gf[kb] = load_frag16(rg, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 32u);
    }
    float lse = 0.f;
    if (i < u.n)
        lse = a.row_max[(size_t)(u.base + i) * a.H + u.h] * kLog2e + fast_log2(a.row_sum[(size_t)(u.base + i) * a.H + u.h]);
    f32x4 acc_t[KB], acc_p[KB];  // sum_j p dP k_j and sum_j p k_j
    float dsum = 0.f;            // this lane's share of delta_i = sum_j p dP
    int edges = 0;               // this lane's share of the row's neighbour count
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) { acc_t[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; acc_p[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    // operands of tile jt + 1 are requested before tile jt is worked on (a tile past the end reads as zeros)
    __shared__ uint16_t patches[kDenseWaves][kPatchElems];
    uint16_t* patch = patches[wave];
    struct Tile { s16x4 kf[KB], vf[KB]; uint32_t bits; };
    auto fetch = [&](int jt, Tile& t) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            t.kf[kb] = load_frag16(rk, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 32u);
            t.vf[kb] = load_frag16(rv, lo.frag + (uint32_t)jt * lo.tile_bytes + kb * 32u);
        }
        t.bits = tile_bits(rm, moff, jt, q);
    };
    Tile c, nx;
    fetch(0, c);
    for (int jt = 0; jt < u.tiles; ++jt) {
        fetch(jt + 1, nx);
        const f32x4 s = tile_product16<KB>(c.kf, qf);
        const f32x4 dp = tile_product16<KB>(c.vf, gf);
        float p[4], t[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p[r] = ((c.bits >> r) & 1u) ? fast_exp2(fmaf(s[r], a.c_score, -lse)) : 0.f;
            t[r] = p[r] * dp[r];
            dsum += t[r];
        }
        edges += __popc(c.bits & 0xfu);
        const SplitFrag pf = split_bf16x4(p[0], p[1], p[2], p[3]);
        const SplitFrag tf = split_bf16x4(t[0], t[1], t[2], t[3]);
#pragma unroll
        for (int nt = 0; nt < KB; ++nt) {
            const s16x4 kc = transpose_tile(patch, c.kf[nt], l16, q);  // the K tile again, as B operand
            acc_t[nt] = mfma_split(tf, kc, acc_t[nt]);
            acc_p[nt] = mfma_split(pf, kc, acc_p[nt]);
        }
        c = nx;
    }
    const float delta = sum_q(dsum);
    const int degree = (int)sum_q((float)edges);  // at most 512 neighbours: exact in fp32
    if (q == 0 && i < u.n) {
        f32x2 st = {lse, delta};
        *reinterpret_cast<f32x2*>(a.stats + 2 * ((size_t)(u.base + i) * a.H + u.h)) = st;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float dr = __shfl(delta, 4 * q + r);  // delta of result row 4q + r
        // a row with a single neighbour has dS = 0 exactly; the difference below would leave the fp32
        // rounding of two equal terms instead
        const bool single = __shfl(degree, 4 * q + r) <= 1;
        const int row = u.t * 16 + 4 * q + r;
        if (row < u.n) {
#pragma unroll
            for (int nt = 0; nt < KB; ++nt)
                a.d_q[(size_t)(u.base + row) * a.HD + u.h * D + nt * 16 + l16] =
                    to_bf16(single ? 0.f : a.scale * (acc_t[nt][r] - dr * acc_p[nt][r]));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// backward, column side: dK and dV of one tile of 16 key columns
// ---------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense16_backward_cols(const DenseBf16Args a) {
    constexpr int D = KB * 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int uidx = xcd_block(blockIdx.x, gridDim.x) * kDenseWaves + wave;
    if (uidx >= a.n_tiles * a.H) return;
    const Unit u = find_unit(a, uidx);
    const int l16 = lane & 15, q = lane >> 4;
    const LaneOffsets lo = lane_offsets16(a.HD, l16, q);
    const rsrc_t rq = unit_tensor(a.q, u, a.HD, D, 2), rk = unit_tensor(a.k, u, a.HD, D, 2), rv = unit_tensor(a.v, u, a.HD, D, 2);
    const rsrc_t rg = unit_tensor(a.d_out, u, a.HD, D, 2);
    const rsrc_t rm = unit_rows(a.adj_mask_t, u, a.W * 8, 0, a.W * 8);
    const rsrc_t rs = unit_rows(a.stats, u, a.H * 8, u.h * 8, 8);  // {lse2, delta} of (row, this head)
    const int j = u.t * 16 + l16;
    const uint32_t moff = (uint32_t)j * (uint32_t)(a.W * 8);
    const uint32_t soff = (uint32_t)(4 * q) * (uint32_t)(a.H * 8);
    s16x4 kf[KB], vf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        kf[kb] = load_frag16(rk, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 32u);
        vf[kb] = load_frag16(rv, lo.frag + (uint32_t)u.t * lo.tile_bytes + kb * 32u);
    }
    f32x4 acc_v[KB], acc_k[KB];
#pragma unroll
    for (int nt = 0; nt < KB; ++nt) { acc_v[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; acc_k[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    // operands of tile it + 1 are requested before tile it is worked on (a tile past the end reads as zeros)
    __shared__ uint16_t patches[kDenseWaves][kPatchElems];
    uint16_t* patch = patches[wave];
    struct Tile { s16x4 qf[KB], gf[KB]; f32x2 st[4]; uint32_t bits; };
    auto fetch = [&](int it, Tile& t) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            t.qf[kb] = load_frag16(rq, lo.frag + (uint32_t)it * lo.tile_bytes + kb * 32u);
            t.gf[kb] = load_frag16(rg, lo.frag + (uint32_t)it * lo.tile_bytes + kb * 32u);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) t.st[r] = buf_load_f32x2(rs, soff + (uint32_t)(it * 16 + r) * (uint32_t)(a.H * 8));
        t.bits = tile_bits(rm, moff, it, q);
    };
    Tile c, nx;
    fetch(0, c);
    for (int it = 0; it < u.tiles; ++it) {
        fetch(it + 1, nx);
        const f32x4 s = tile_product16<KB>(c.qf, kf);  // s[r] = score of (row 4q + r of the tile, column j)
        const f32x4 dp = tile_product16<KB>(c.gf, vf);
        float p[4], ds[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p[r] = ((c.bits >> r) & 1u) ? fast_exp2(fmaf(s[r], a.c_score, -c.st[r][0])) : 0.f;
            ds[r] = p[r] * (dp[r] - c.st[r][1]);
        }
        const SplitFrag pf = split_bf16x4(p[0], p[1], p[2], p[3]);
        const SplitFrag dsf = split_bf16x4(ds[0], ds[1], ds[2], ds[3]);
#pragma unroll
        for (int nt = 0; nt < KB; ++nt) {
            acc_v[nt] = mfma_split(pf, transpose_tile(patch, c.gf[nt], l16, q), acc_v[nt]);
            acc_k[nt] = mfma_split(dsf, transpose_tile(patch, c.qf[nt], l16, q), acc_k[nt]);
        }
        c = nx;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = u.t * 16 + 4 * q + r;
        if (row < u.n) {
#pragma unroll
            for (int nt = 0; nt < KB; ++nt) {
                const size_t o = (size_t)(u.base + row) * a.HD + u.h * D + nt * 16 + l16;
                a.d_v[o] = to_bf16(acc_v[nt][r]);
                a.d_k[o] = to_bf16(a.scale * acc_k[nt][r]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static DenseBf16Args dense16_args(const dfgnn_graph* g, const dfgnn_layer* L) {
    DenseBf16Args a{};
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

#define DFGNN_LAUNCH_BY_WIDTH(KERNEL)                                                      \
    do {                                                                                   \
        if (L->D == 16) hipLaunchKernelGGL((KERNEL<1>), grid, block, 0, st, a);            \
        else if (L->D == 32) hipLaunchKernelGGL((KERNEL<2>), grid, block, 0, st, a);       \
        else hipLaunchKernelGGL((KERNEL<4>), grid, block, 0, st, a);                       \
    } while (0)

int dense16_gt_forward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v, void* out,
                       float* row_max, float* row_sum, hipStream_t st) {
    DenseBf16Args a = dense16_args(g, L);
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
    a.o = (uint16_t*)out; a.o_max = row_max; a.o_sum = row_sum;
    const int64_t waves = g->n_tiles * L->H;
    if (waves == 0) return DFGNN_OK;
    const dim3 grid((unsigned)((waves + kDenseWaves - 1) / kDenseWaves)), block(64 * kDenseWaves);
    KernelTimer t("dense_fwd", st);
    DFGNN_LAUNCH_BY_WIDTH(k_dense16_forward);
    return DFGNN_OK;
}

int dense16_gt_backward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v,
                        const float* row_max, const float* row_sum, const void* d_out, void* d_q, void* d_k, void* d_v,
                        float* stats, hipStream_t st) {
    DenseBf16Args a = dense16_args(g, L);
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
    a.d_out = (const uint16_t*)d_out; a.row_max = row_max; a.row_sum = row_sum;
    a.d_q = (uint16_t*)d_q; a.d_k = (uint16_t*)d_k; a.d_v = (uint16_t*)d_v; a.stats = stats;
    const int64_t waves = g->n_tiles * L->H;
    if (waves == 0) return DFGNN_OK;
    const dim3 grid((unsigned)((waves + kDenseWaves - 1) / kDenseWaves)), block(64 * kDenseWaves);
    {
        KernelTimer t("dense_bwd_rows", st);
        DFGNN_LAUNCH_BY_WIDTH(k_dense16_backward_rows);
    }
    {
        KernelTimer t("dense_bwd_cols", st);
        DFGNN_LAUNCH_BY_WIDTH(k_dense16_backward_cols);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
