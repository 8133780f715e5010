// GATv2 forward kernels (the second member of the GAT family cited in Sec. 1).
#include "layer_launch.hpp"
#include "pass_gatv2.hpp"

namespace dfgnn {

int launch_forward_gatv2(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run_pass<Geo<T, LPE, LPH>, GatV2Fwd>(g, false, a, kFwdLabels, st); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

// chunks of super rows write their own edges, so there is nothing to merge
int launch_attention_gatv2(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run_pass<Geo<T, LPE, LPH>, GatV2Attention>(g, false, a, kAttentionLabels, st, false); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
