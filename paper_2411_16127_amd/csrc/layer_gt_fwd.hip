// GT forward kernels (Eq. 1 with the dot-product score of Sec. 5.1) and the two-kernel comparator of Sec. 3.
#include "layer_launch.hpp"
#include "pass_gt.hpp"

namespace dfgnn {

template <class G> static void run(const dfgnn_graph* g, const Args& a, hipStream_t st) {
    if (a.scores) {  // comparator: scores through memory (Sec. 3, parallelism maximization fusion)
        const int64_t per_wave = (int64_t)G::EPW * kUnroll * kScoreRounds;
        const dim3 grid(blocks_for((g->E + per_wave - 1) / per_wave)), block(64 * kWavesPerBlock);
        {
            KernelTimer t("fwd_scores", st);
            if (a.bias) hipLaunchKernelGGL((k_edge_scores<with_edge_term<G>, kUnroll>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((k_edge_scores<G, kUnroll>), grid, block, 0, st, a);
        }
        Args b = a;
        b.bias = nullptr;  // the stored scores already contain the edge term
        run_pass<G, GtFwdStored>(g, false, b, kStoredLabels, st);
    } else {
        run_pass<G, GtFwd>(g, false, a, kFwdLabels, st);
    }
}

int launch_forward_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run<Geo<T, LPE, LPH>>(g, a, st); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

// chunks of super rows write their own edges, so there is nothing to merge
int launch_attention_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run_pass<Geo<T, LPE, LPH>, GtAttention>(g, false, a, kAttentionLabels, st, false); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
