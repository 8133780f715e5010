// AGNN backward kernels (Appendix B with the derivative of the L2 normalisation) and the reduction of dbeta.
#include "layer_launch.hpp"
#include "pass_agnn.hpp"

namespace dfgnn {

template <class G>
static void run(const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_scale, bool add_to_scale, hipStream_t st) {
    run_pass<G, AgnnBwdRow>(g, false, a, kRowLabels, st);
    run_pass<G, AgnnBwdCol>(g, true, a, kColLabels, st);
    KernelTimer t("param_reduce", st);
    hipLaunchKernelGGL(k_sum_partial, dim3(kReduceBlocks), dim3(256), 0, st, a.dbeta_row, (int64_t)a.n_nodes * a.H,
                       reduce_tmp);
    hipLaunchKernelGGL(k_sum_final, dim3(1), dim3(256), 0, st, reduce_tmp, kReduceBlocks, add_to_scale,
                       reduce_tmp + kReduceBlocks, d_scale);
}

int launch_backward_agnn(int geo, const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_scale, bool add_to_scale,
                         hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run<Geo<T, LPE, LPH>>(g, a, reduce_tmp, d_scale, add_to_scale, st); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
