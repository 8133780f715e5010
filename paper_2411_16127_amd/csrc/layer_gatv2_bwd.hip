// GATv2 backward kernels and the column sum that finishes the gradient of the attention vector.
#include "layer_launch.hpp"
#include "pass_gatv2.hpp"

namespace dfgnn {

template <class G> static void run(const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_a, hipStream_t st) {
    run_pass<G, GatV2BwdRow>(g, false, a, kRowLabels, st);
    run_pass<G, GatV2BwdCol>(g, true, a, kColLabels, st);
    KernelTimer t("param_reduce", st);
    int w = 1;  // threads per row, 4 columns each (a power of two, so that it divides 256)
    while (4 * w < a.HD && w < 256) w <<= 1;
    // about 16 rows per thread of the first stage, at most kRowsumBlocks workgroups
    int64_t blocks = ((int64_t)a.n_nodes + (256 / w) * 16 - 1) / ((256 / w) * 16);
    if (blocks > kRowsumBlocks) blocks = kRowsumBlocks;
    int wf = 4;
    while (wf < a.HD && wf < 256) wf <<= 1;
    hipLaunchKernelGGL(k_rowsum_partial, dim3((unsigned)blocks), dim3(256), 0, st, a.da_row, (int64_t)a.n_nodes, a.HD, w,
                       reduce_tmp);
    hipLaunchKernelGGL(k_rowsum_final, dim3(1), dim3(256), 0, st, reduce_tmp, (int)blocks, a.HD, wf, d_a);
}

int launch_backward_gatv2(int geo, const dfgnn_graph* g, const Args& a, double* reduce_tmp, float* d_a_l, hipStream_t st) {
    switch (geo) {
#define X(ID, T, LPE, LPH) case ID: run<Geo<T, LPE, LPH>>(g, a, reduce_tmp, d_a_l, st); break;
        DFGNN_GEOMETRIES(X)
#undef X
    default: DFGNN_REQUIRE(false, DFGNN_EUNSUPPORTED, "no kernel for geometry %d", geo);
    }
    return DFGNN_OK;
}

}  // namespace dfgnn
