// GT backward kernels (Appendix B: row pass over the CSR, column pass over the CSC).
#include "layer_launch.hpp"
#include "pass_gt.hpp"

namespace dfgnn {

int launch_backward_gt(int geo, const dfgnn_graph* g, const Args& a, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH)                                                  \
    case ID:                                                                \
        run_pass<Geo<T, LPE, LPH>, GtBwdRow>(g, false, a, kRowLabels, st);  \
        run_pass<Geo<T, LPE, LPH>, GtBwdCol>(g, true, a, kColLabels, st);   \
        break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
