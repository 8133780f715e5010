// Launch side shared by the per-model translation units: the table of lane geometries, the launch of one
// pass (chunks of super rows, whole rows and short rows in one kernel, then the merge of chunk partials)
// and the entry points each unit defines.  The kernels of one model and direction are instantiated in
// one unit each, so that the library builds in parallel.
#pragma once
#include "common.hpp"
#include "layer_device.hpp"

namespace dfgnn {

constexpr int kUnroll = 4;  // neighbour rows requested per edge slot before the first is consumed

// (id, type, LPE, LPH): LPH = 0 handles any head width at run time (ids 0-4 fp32, 5-9 bf16, 28-32 fp16, by
// LPE); the others are full rows of 64 or 128 features split into 1 to 16 heads, with compile-time DPP
// reductions over the lanes of a head.
#define DFGNN_GEOMETRIES(X)                                                                          \
    X(0, float, 4, 0) X(1, float, 8, 0) X(2, float, 16, 0) X(3, float, 32, 0) X(4, float, 64, 0)     \
    X(5, bf16_t, 4, 0) X(6, bf16_t, 8, 0) X(7, bf16_t, 16, 0) X(8, bf16_t, 32, 0) X(9, bf16_t, 64, 0) \
    X(10, float, 16, 16) X(11, float, 16, 8) X(12, float, 16, 4) X(13, float, 16, 2)                 \
    X(14, float, 32, 32) X(15, float, 32, 16) X(16, float, 32, 8) X(17, float, 32, 4) X(18, float, 32, 2) \
    X(19, bf16_t, 16, 16) X(20, bf16_t, 16, 8) X(21, bf16_t, 16, 4) X(22, bf16_t, 16, 2) X(23, bf16_t, 16, 1) \
    X(24, bf16_t, 8, 8) X(25, bf16_t, 8, 4) X(26, bf16_t, 8, 2) X(27, bf16_t, 8, 1)                  \
    X(28, f16_t, 4, 0) X(29, f16_t, 8, 0) X(30, f16_t, 16, 0) X(31, f16_t, 32, 0) X(32, f16_t, 64, 0) \
    X(33, f16_t, 16, 16) X(34, f16_t, 16, 8) X(35, f16_t, 16, 4) X(36, f16_t, 16, 2) X(37, f16_t, 16, 1) \
    X(38, f16_t, 8, 8) X(39, f16_t, 8, 4) X(40, f16_t, 8, 2) X(41, f16_t, 8, 1)

// storage type of a geometry's element type as the ABI numbers it (dfgnn_dtype)
template <typename T> struct dtype_of;
template <> struct dtype_of<float> { static constexpr int value = DFGNN_F32; };
template <> struct dtype_of<bf16_t> { static constexpr int value = DFGNN_BF16; };
template <> struct dtype_of<f16_t> { static constexpr int value = DFGNN_F16; };

// the same geometry with the code for the optional additive edge term compiled in
template <class G> using with_edge_term = Geo<typename G::T, G::LPE, G::LPH, true>;

// ---------------------------------------------------------------------------------------------
// launch sequences
// ---------------------------------------------------------------------------------------------
static inline unsigned blocks_for(int64_t waves) { return (unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock); }

// Work list of one pass over the rows (or columns) of a graph: chunk items of super rows, whole-row items,
// short rows (fewer than EPW * U neighbours, i.e. less than one load round of a whole wavefront: one per edge
// slot; they are the tail of the degree-ordered list).
struct PassShape {
    int n_super, n_chunks;
    int64_t first_small, n_direct, n_small, waves;
};
template <class G> static PassShape pass_shape(const dfgnn_graph* g, bool columns) {
    PassShape s{};
    s.n_super = columns ? g->n_super_cols : g->n_super_rows;
    s.n_chunks = columns ? g->n_col_chunks : g->n_row_chunks;
    const int32_t* bucket = columns ? g->col_bucket_ptr : g->row_bucket_ptr;
    s.first_small = g->N;
    if (G::EPW > 1 && !(g->flags & DFGNN_SCHED_NO_SHORT_ROWS)) {
        int lg = 0;
        while ((1 << (lg + 1)) <= G::EPW * kUnroll) ++lg;  // degree < 2^lg  <=>  bit_length(degree) <= lg
        s.first_small = bucket[33 - lg];
        if (s.first_small < s.n_super) s.first_small = s.n_super;
    }
    s.n_direct = s.first_small - s.n_super;
    s.n_small = g->N - s.first_small;
    const int64_t small_waves = G::EPW > 1 ? (s.n_small + G::EPW - 1) / G::EPW : 0;
    s.waves = s.n_chunks + s.n_direct + small_waves;
    return s;
}
// small launches spread their wavefronts over more compute units with smaller workgroups
// (2,708-node graph: 25.2 us per training step with 4 wavefronts per workgroup, 23.5 with 1); graphs whose
// numbering is local (mini-batches of small graphs: short rows, XCD-local runs of the work list) take
// single-wavefront workgroups at any size, which fill free wave slots one by one (1,024 graphs of 10-40
// nodes: 47.8 -> 46.6 us per step, 4,096 graphs: 158 -> 148 us; a 169,343-node power-law graph loses 1.5 %)
static inline int waves_per_block(int64_t waves, bool local_numbering) {
    if (local_numbering) return 1;
    return waves <= 1024 ? 1 : (waves <= 4096 ? 2 : kWavesPerBlock);
}

// fills the work-list fields of `a` for workgroups of wpb wavefronts; returns the number of workgroups
template <class G> static unsigned bind_pass(const dfgnn_graph* g, bool columns, const PassShape& s, int wpb, Args& a) {
    a.ptr = columns ? g->t_indptr : g->indptr;
    a.idx = columns ? g->t_indices : g->indices;
    a.order = columns ? g->col_order : g->row_order;
    a.chunks = columns ? g->col_chunks : g->row_chunks;
    a.chunk_ptr = columns ? g->col_chunk_ptr : g->row_chunk_ptr;
    a.eid = (columns && a.bias) ? g->t_eid : nullptr;  // the edge term is stored in CSR edge order
    auto blocks_for = [&](int64_t waves) { return (unsigned)((waves + wpb - 1) / wpb); };
    a.n_chunks = s.n_chunks;
    a.blocks_chunk = (int)blocks_for(s.n_chunks);
    a.n_direct = (int)s.n_direct;
    a.blocks_direct = (int)blocks_for(s.n_direct);
    a.first_direct = s.n_super;
    a.n_small = (int)s.n_small;
    a.first_small = (int)s.first_small;
    a.xcd_group = g->xcd_group;
    return (unsigned)a.blocks_chunk + (unsigned)a.blocks_direct + blocks_for((s.n_small + G::EPW - 1) / G::EPW);
}

// chunk pass over super rows, direct pass over the rest, then the merge of the chunk partials
template <class G, template <class, int> class PassT>
static void run_pass(const dfgnn_graph* g, bool columns, Args a, const char* const (&labels)[2], hipStream_t st,
                     bool merge = true) {
    const PassShape s = pass_shape<G>(g, columns);
    const int wpb = waves_per_block(s.waves, g->xcd_group > 0);
    const unsigned total = bind_pass<G>(g, columns, s, wpb, a);
    const int n_super = s.n_super, n_chunks = s.n_chunks;
    const dim3 block(64 * wpb);
    if (total > 0) {
        KernelTimer t(labels[0], st);
        if (a.bias) hipLaunchKernelGGL((k_pass<with_edge_term<G>, PassT, kUnroll>), dim3(total), block, 0, st, a);
        else hipLaunchKernelGGL((k_pass<G, PassT, kUnroll>), dim3(total), block, 0, st, a);
    }
    if (n_super > 0 && merge) {
        a.n_items = n_super;
        // rows with very many chunks are merged in two levels; the group count follows the mean chunk count
        // of the super rows (a power of two, at most 64), so graphs whose super rows have a few chunks each
        // launch the final merge only
        int groups = 1;
        while (groups < 64 && (int64_t)groups * kMergeGroupChunks * n_super < n_chunks) groups <<= 1;
        a.merge_groups = groups;
        KernelTimer t(labels[1], st);
        if (groups > 1)
            hipLaunchKernelGGL((k_merge_groups<G, PassT, kUnroll>), dim3(dfgnn::blocks_for((int64_t)n_super * groups)),
                               dim3(64 * kWavesPerBlock), 0, st, a);
        hipLaunchKernelGGL((k_merge<G, PassT, kUnroll>), dim3(dfgnn::blocks_for(n_super)), dim3(64 * kWavesPerBlock), 0, st, a);
    }
}

// Row pass and column pass of a backward call in one launch, for graphs without super rows or columns whose
// passes do not depend on each other (the column pass recomputes what the row pass would hand over).
template <class G, template <class, int> class RowPass, template <class, int> class ColPass>
static void run_pass_pair(const dfgnn_graph* g, const Args& a, const char* label, hipStream_t st) {
    const PassShape sr = pass_shape<G>(g, false), sc = pass_shape<G>(g, true);
    const int wpb = waves_per_block(sr.waves + sc.waves, g->xcd_group > 0);
    Args ar = a, ac = a;
    const unsigned blocks_r = bind_pass<G>(g, false, sr, wpb, ar), blocks_c = bind_pass<G>(g, true, sc, wpb, ac);
    if (blocks_r + blocks_c == 0) return;
    KernelTimer t(label, st);
    hipLaunchKernelGGL((k_pass_pair<G, RowPass, ColPass, kUnroll>), dim3(blocks_r + blocks_c), dim3(64 * wpb), 0, st, ar, ac,
                       (int)blocks_r);
}

[[maybe_unused]] static const char* const kFwdLabels[2] = {"fwd", "fwd_merge"};
[[maybe_unused]] static const char* const kStoredLabels[2] = {"fwd_softmax_spmm", "fwd_softmax_spmm_merge"};
[[maybe_unused]] static const char* const kAttentionLabels[2] = {"attention_weights", "attention_weights"};
[[maybe_unused]] static const char* const kRowLabels[2] = {"bwd_row", "bwd_row_merge"};
[[maybe_unused]] static const char* const kColLabels[2] = {"bwd_col", "bwd_col_merge"};


// One entry point per model and direction; `geo` is an id of the table above.  Each returns a status.
int launch_forward_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_forward_gat(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_forward_gatv2(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_forward_agnn(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
// attention weights of every edge from the statistics of a finished forward call (a.p_out)
int launch_attention_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_attention_gat(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_attention_gatv2(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_attention_agnn(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_backward_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st);
int launch_backward_gat(int geo, const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_a_l, float* d_a_r,
                        hipStream_t st);
int launch_backward_gatv2(int geo, const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_a_l, hipStream_t st);
int launch_backward_agnn(int geo, const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_scale, bool add_to_scale,
                         hipStream_t st);

}  // namespace dfgnn
