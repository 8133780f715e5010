// GT backward kernels (Appendix B: row pass over the CSR, column pass over the CSC).
#include "layer_launch.hpp"
#include "pass_gt.hpp"

namespace dfgnn {

// Graphs small enough that a launch costs as much as a pass (all tensors cache-resident), fp32, no super rows
// or columns, no edge term: row side and column side run as one launch.  The column side then gathers the
// output row of every edge as well (one more row per edge), which a graph that streams from HBM cannot afford.
constexpr int64_t kPairedPassMaxEdges = 1 << 18;
template <class G> static bool paired(const dfgnn_graph* g, const Args& a) {
    return sizeof(typename G::T) == 4 && a.bias == nullptr && g->n_super_rows == 0 && g->n_super_cols == 0 &&
           g->E <= kPairedPassMaxEdges && !(g->flags & DFGNN_SCHED_NO_PAIRED_PASSES);
}

template <class G> static void run(const dfgnn_graph* g, const Args& a, hipStream_t st) {
    if constexpr (sizeof(typename G::T) == 4) {
        if (paired<G>(g, a)) {
            run_pass_pair<G, GtBwdRow, GtBwdColSelf>(g, a, "bwd_row_col", st);
            return;
        }
    }
    run_pass<G, GtBwdRow>(g, false, a, kRowLabels, st);
    run_pass<G, GtBwdCol>(g, true, a, kColLabels, st);
}

int launch_backward_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run<Geo<T, LPE, LPH>>(g, a, st); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
