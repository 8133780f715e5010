// GAT backward kernels (Appendix B with the chain rule through LeakyReLU) and the reduction of da_l, da_r.
#include "layer_launch.hpp"
#include "pass_gat.hpp"

namespace dfgnn {

template <class G>
static void run(const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_a_l, float* d_a_r, hipStream_t st) {
    run_pass<G, GatBwdRow>(g, false, a, kRowLabels, st);
    run_pass<G, GatBwdCol>(g, true, a, kColLabels, st);
    KernelTimer t("param_reduce", st);
    // one workgroup per 4 load rounds of its wavefronts, at most kReduceBlocks (the partial buffer's size)
    const int64_t rows_per_block = (int64_t)kReduceWaves * G::EPW * 16;
    int blocks = (int)((a.n_nodes + rows_per_block - 1) / rows_per_block);
    blocks = blocks < 1 ? 1 : (blocks > kReduceBlocks ? kReduceBlocks : blocks);
    hipLaunchKernelGGL((k_gat_param_partial<G>), dim3(blocks), dim3(64 * kReduceWaves), 0, st, a, reduce_tmp);
    int wf = 8;  // columns of the second stage: a power of two >= 2 * HD (HD <= 512)
    while (wf < 2 * a.HD) wf <<= 1;
    hipLaunchKernelGGL(k_gat_param_final, dim3(1), dim3(1024), 0, st, reduce_tmp, blocks, a.HD, wf, d_a_l, d_a_r);
}

int launch_backward_gat(int geo, const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_a_l, float* d_a_r,
                        hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run<Geo<T, LPE, LPH>>(g, a, reduce_tmp, d_a_l, d_a_r, st); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
