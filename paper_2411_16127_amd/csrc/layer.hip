// Host side of the layer calls: argument checks, workspace carving, lane-geometry selection and the
// launch sequence of the fused kernels (Eq. 1 forward; Appendix B backward as a CSR row pass and a CSC
// column pass).  Every launch goes to the caller's stream; nothing here synchronises or allocates.
#include "layer_launch.hpp"

#include <mutex>

// Library-owned scratch memory for dfgnn_forward_static: callers that cannot provide (allocate) a workspace
// get the forward pass's chunk partials placed here.  The array exists once per GPU that loads the library;
// in host code its name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[DFGNN_STATIC_SCRATCH_BYTES];

namespace dfgnn {

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, resolved on first use

// Device address of this GPU's copy of `scratch` (the calling thread's current device).
static int static_scratch(void** out) {
    int dev = -1;
    DFGNN_HIP(hipGetDevice(&dev));
    DFGNN_REQUIRE(dev >= 0 && dev < kMaxDevices, DFGNN_EUNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        DFGNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        DFGNN_REQUIRE(p != nullptr && ((uintptr_t)p % kAlign) == 0, DFGNN_EHIP, "static scratch resolved to %p", p);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DFGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// lane geometry
// ---------------------------------------------------------------------------------------------
// A wavefront covers at most 64 lanes x 16 bytes of a node row.  A layer whose rows are wider is run as
// `groups` launches sequences over `heads` heads each (heads are independent): the kernels see a layer
// of `heads` heads whose tensors have the strides of the whole layer.
struct Geometry {
    int vec;     // elements per lane
    int lph;     // lanes per head
    int lpe;     // lanes per neighbour row (power of two, >= 4)
    int id;      // index into the instantiation table
    int heads;   // heads per group (a divisor of H)
    int groups;  // H / heads
    bool wide;   // node tensors of 4 GiB and more: run-time geometry with 64-bit gather addresses
};

static int elem_bytes(int dtype) { return dtype == DFGNN_F32 ? 4 : 2; }

static int pick_geometry(const dfgnn_layer* L, bool wide, Geometry* out) {
    DFGNN_REQUIRE(L->dtype == DFGNN_F32 || L->dtype == DFGNN_BF16 || L->dtype == DFGNN_F16, DFGNN_EINVAL, "unknown dtype %d",
                  L->dtype);
    DFGNN_REQUIRE(L->H >= 1 && L->D >= 1, DFGNN_EINVAL, "H and D must be positive (H=%d D=%d)", L->H, L->D);
    Geometry g{};
    g.vec = 16 / elem_bytes(L->dtype);
    DFGNN_REQUIRE(L->D % g.vec == 0, DFGNN_EUNSUPPORTED, "D=%d: a head must be a multiple of 16 bytes", L->D);
    g.lph = L->D / g.vec;
    DFGNN_REQUIRE((g.lph & (g.lph - 1)) == 0, DFGNN_EUNSUPPORTED, "D=%d: D/%d must be a power of two", L->D, g.vec);
    DFGNN_REQUIRE(g.lph <= 64, DFGNN_EUNSUPPORTED, "D=%d: one head exceeds one wavefront of 16-byte lanes", L->D);
    g.heads = 1;
    for (int h = 1; h <= L->H && h * g.lph <= 64; ++h)
        if (L->H % h == 0) g.heads = h;
    g.groups = L->H / g.heads;
    const int lanes = g.heads * g.lph;
    g.lpe = 4;
    while (g.lpe < lanes) g.lpe <<= 1;
    // a compile-time geometry needs the row to fill its lanes exactly; otherwise the run-time one of that width
    struct Entry { int id, dtype, lpe, lph; };
    static const Entry table[] = {
#define X(ID, T, LPE, LPH) {ID, dtype_of<T>::value, LPE, LPH},
        DFGNN_GEOMETRIES(X)
#undef X
    };
    g.id = -1;
    for (const Entry& e : table)
        if (e.lph == 0 && e.dtype == L->dtype && e.lpe == g.lpe) g.id = e.id;
    for (const Entry& e : table)
        if (!wide && e.lph != 0 && e.dtype == L->dtype && e.lpe == g.lpe && lanes == g.lpe && e.lph == g.lph) g.id = e.id;
    g.wide = wide;
    DFGNN_REQUIRE(g.id >= 0, DFGNN_EUNSUPPORTED, "no kernel for dtype %d with %d lanes per row", L->dtype, g.lpe);
    *out = g;
    return DFGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// workspace layout (float offsets turned into pointers)
// ---------------------------------------------------------------------------------------------
struct Workspace {
    size_t stats, d_el, d_er, g_row, dbeta_row, part_v0, part_v1, part_v2, part_v3, part_s0, part_s1, part_s2, reduce, scores, total;
};

// the two-kernel forward comparator applies (GT on the general kernels)
static bool scores_in_memory(const dfgnn_graph* g, const dfgnn_layer* L) {
    return (g->flags & DFGNN_SCHED_SCORES_IN_MEMORY) && L->model == DFGNN_GT && g->E > 0;
}

// sized for one group of `heads` heads: the groups of a wide layer run one after the other and reuse it
static Workspace workspace_layout(const dfgnn_graph* g, const dfgnn_layer* L, bool backward, int heads) {
    Workspace W{};
    size_t off = 0;
    auto take = [&](size_t floats) { size_t o = off; off += align_up((floats ? floats : 1) * sizeof(float)); return o; };
    const size_t N = (size_t)g->N, H = (size_t)heads, HD = (size_t)heads * L->D;
    const size_t chunks = backward ? (size_t)(g->n_row_chunks > g->n_col_chunks ? g->n_row_chunks : g->n_col_chunks)
                                   : (size_t)g->n_row_chunks;
    const bool gat = L->model == DFGNN_GAT, agnn = L->model == DFGNN_AGNN, v2 = L->model == DFGNN_GATV2;
    W.part_v0 = take(chunks * HD);
    W.part_s0 = take(chunks * H);
    W.part_s1 = take(chunks * H);
    if (backward) {
        W.stats = take(N * H * (L->model == DFGNN_GT || v2 ? 2 : 4));
        W.part_v1 = take(chunks * HD);
        W.part_v2 = take(v2 ? chunks * HD : 0);
        W.part_v3 = take(v2 ? chunks * HD : 0);
        W.part_s2 = take(chunks * H);
        W.d_el = take(gat ? N * H : 0);
        W.d_er = take(gat ? N * H : 0);
        W.g_row = take(agnn || v2 ? N * HD : 0);
        W.dbeta_row = take(agnn ? N * H : 0);
        // double-precision partials of the parameter-gradient reductions (AGNN: plus the running total)
        W.reduce = take(2 * (gat ? (size_t)kReduceBlocks * 2 * HD : (v2 ? (size_t)kRowsumBlocks * HD : (agnn ? (size_t)kReduceBlocks + 1 : 0))));
    }
    if (!backward && scores_in_memory(g, L)) W.scores = take((size_t)g->E * H);
    W.total = off;
    return W;
}

static void bind_workspace(Args& a, const Workspace& W, void* ws, bool backward) {
    char* b = (char*)ws;
    a.part_v0 = (float*)(b + W.part_v0);
    a.part_s0 = (float*)(b + W.part_s0);
    a.part_s1 = (float*)(b + W.part_s1);
    if (!backward && W.scores) a.scores = (float*)(b + W.scores);
    if (backward) {
        a.stats = (float*)(b + W.stats);
        a.part_v1 = (float*)(b + W.part_v1);
        a.part_v2 = (float*)(b + W.part_v2);
        a.part_v3 = (float*)(b + W.part_v3);
        a.da_row = (float*)(b + W.g_row);
        a.part_s2 = (float*)(b + W.part_s2);
        a.d_el = (float*)(b + W.d_el);
        a.d_er = (float*)(b + W.d_er);
        a.g_row = (float*)(b + W.g_row);
        a.dbeta_row = (float*)(b + W.dbeta_row);
    }
}

// ---------------------------------------------------------------------------------------------
// launch sequences: one translation unit per model and direction holds the kernels
// ---------------------------------------------------------------------------------------------
static int dispatch_forward(int geo, const dfgnn_graph* g, int model, const Args& a, hipStream_t st) {
    switch (model) {
    case DFGNN_GT: return launch_forward_gt(geo, g, a, st);
    case DFGNN_GAT: return launch_forward_gat(geo, g, a, st);
    case DFGNN_GATV2: return launch_forward_gatv2(geo, g, a, st);
    default: return launch_forward_agnn(geo, g, a, st);
    }
}

static int dispatch_attention(int geo, const dfgnn_graph* g, int model, const Args& a, hipStream_t st) {
    switch (model) {
    case DFGNN_GT: return launch_attention_gt(geo, g, a, st);
    case DFGNN_GAT: return launch_attention_gat(geo, g, a, st);
    case DFGNN_GATV2: return launch_attention_gatv2(geo, g, a, st);
    default: return launch_attention_agnn(geo, g, a, st);
    }
}

static int dispatch_backward(int geo, const dfgnn_graph* g, int model, const Args& a, double* reduce_tmp, float* d_a_l,
                             float* d_a_r, float* d_scale, bool add_to_scale, hipStream_t st) {
    switch (model) {
    case DFGNN_GT: return launch_backward_gt(geo, g, a, st);
    case DFGNN_GAT: return launch_backward_gat(geo, g, a, reduce_tmp, d_a_l, d_a_r, st);
    case DFGNN_GATV2: return launch_backward_gatv2(geo, g, a, reduce_tmp, d_a_l, st);
    default: return launch_backward_agnn(geo, g, a, reduce_tmp, d_scale, add_to_scale, st);
    }
}

__global__ void k_zero(float* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}
static void launch_zero(float* p, int n, hipStream_t st) {
    hipLaunchKernelGGL(k_zero, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
}

// the edge term is read with 32-bit byte offsets
static bool edge_term_fits(const dfgnn_graph* g, const dfgnn_layer* L) {
    return (int64_t)g->E * L->H * 4 < ((int64_t)1 << 32) - 4096;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

static int check_layer(const dfgnn_graph* g, const dfgnn_layer* L, Geometry* geo) {
    DFGNN_REQUIRE(g != nullptr && L != nullptr, DFGNN_EINVAL, "graph / layer is NULL");
    DFGNN_REQUIRE(L->model == DFGNN_GT || L->model == DFGNN_GAT || L->model == DFGNN_AGNN || L->model == DFGNN_GATV2,
                  DFGNN_EINVAL, "unknown model %d", L->model);
    DFGNN_REQUIRE(L->reserved[0] == 0, DFGNN_EINVAL, "dfgnn_layer.reserved must be zero");
    // Gathers address node rows with 32-bit byte offsets against a buffer resource, and an absent neighbour is
    // read at offset 2^32 - row_bytes + ..., which must fall outside the tensor: tensors up to 2^32 - row_bytes
    // bytes take that path.  Larger ones run on the run-time-geometry kernels with 64-bit gather addresses.
    const int64_t elem = elem_bytes(L->dtype);
    const int64_t row_bytes = (int64_t)L->H * L->D * elem;
    const bool wide = (int64_t)g->N * row_bytes > ((int64_t)1 << 32) - row_bytes;
    int rc = pick_geometry(L, wide, geo);
    if (rc != DFGNN_OK) return rc;
    if (wide) {
        // the packed per-(row, head) records of the backward pass are still gathered with 32-bit offsets
        DFGNN_REQUIRE((int64_t)g->N * L->H * 16 < ((int64_t)1 << 32) - 4096, DFGNN_EUNSUPPORTED,
                      "N * H = %lld: the per-row statistics records exceed 4 GiB", (long long)((int64_t)g->N * L->H));
        DFGNN_REQUIRE(!(g->flags & DFGNN_SCHED_SCORES_IN_MEMORY), DFGNN_EUNSUPPORTED,
                      "the scores-in-memory comparator does not take node tensors of 4 GiB and more");
    }
    if (L->model == DFGNN_AGNN) DFGNN_REQUIRE(L->eps > 0.f, DFGNN_EINVAL, "AGNN eps must be positive");
    return DFGNN_OK;
}

static void fill_common(Args& a, const dfgnn_graph* g, const dfgnn_layer* L, const Geometry& geo) {
    a.n_nodes = (int)g->N;
    a.wide = geo.wide ? 1 : 0;
    a.row_bytes = (uint32_t)(L->H * L->D * elem_bytes(L->dtype));
    a.tensor_bytes = (uint32_t)((uint64_t)g->N * a.row_bytes);
    a.nh_bytes = (uint32_t)((uint64_t)g->N * geo.heads * 4u);
    a.H = geo.heads;
    a.D = L->D;
    a.HD = geo.heads * L->D;
    a.row_stride = L->H * L->D;
    a.stat_stride = L->H;
    a.bias_stride = L->H;
    a.lph = geo.lph;
    a.scale = (L->model == DFGNN_GAT || L->model == DFGNN_GATV2) ? 1.f : L->scale;
    a.c_score = a.scale * kLog2e;
    a.neg_slope = L->neg_slope;
    a.eps = L->eps;
    a.inv_eps = L->eps > 0.f ? 1.f / L->eps : 0.f;
}

// Pointers of head group `gi`: the caller's tensors start at the group's first head; buffer ranges shrink by
// the same amount so that the hardware range check still ends at the end of the allocation.
template <typename T> static T* shift(T* p, size_t bytes) { return p ? (T*)((char*)p + bytes) : nullptr; }
template <typename T> static const T* shift(const T* p, size_t bytes) { return p ? (const T*)((const char*)p + bytes) : nullptr; }

static void select_group(Args& a, const Args& whole, const dfgnn_layer* L, const Geometry& geo, int gi) {
    a = whole;
    const size_t elem = (size_t)elem_bytes(L->dtype);
    const size_t first = (size_t)gi * geo.heads;      // first head of the group
    const size_t tb = first * L->D * elem;            // byte offset inside a node row
    const size_t pb = first * L->D * sizeof(float);   // inside an [H, D] fp32 parameter
    const size_t sb = first * sizeof(float);          // inside an [.., H] fp32 record
    a.x = shift(whole.x, tb); a.k = shift(whole.k, tb); a.v = shift(whole.v, tb);
    a.out = shift(whole.out, tb); a.d_out = shift(whole.d_out, tb);
    a.o = shift(whole.o, tb); a.d_x = shift(whole.d_x, tb); a.d_k = shift(whole.d_k, tb); a.d_v = shift(whole.d_v, tb);
    a.a_l = shift(whole.a_l, pb); a.a_r = shift(whole.a_r, pb);
    a.row_max = shift(whole.row_max, sb); a.row_sum = shift(whole.row_sum, sb);
    a.o_max = shift(whole.o_max, sb); a.o_sum = shift(whole.o_sum, sb);
    a.bias = shift(whole.bias, sb); a.d_bias = shift(whole.d_bias, sb); a.p_out = shift(whole.p_out, sb);
    a.tensor_bytes = whole.tensor_bytes - (uint32_t)tb;
    a.bias_bytes = whole.bias_bytes - (uint32_t)sb;
}

}  // namespace dfgnn

using namespace dfgnn;

extern "C" int dfgnn_workspace_bytes(const dfgnn_graph* graph, const dfgnn_layer* layer, size_t* fwd_bytes,
                                     size_t* bwd_bytes) {
    clear_error();
    Geometry geo;
    int rc = check_layer(graph, layer, &geo);
    if (rc != DFGNN_OK) return rc;
    if (fwd_bytes) *fwd_bytes = workspace_layout(graph, layer, false, geo.heads).total;
    if (bwd_bytes) *bwd_bytes = workspace_layout(graph, layer, true, geo.heads).total;
    return DFGNN_OK;
}

static int forward_impl(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                        const void* v, const float* a_l, const float* a_r, const float* edge_bias, void* out,
                        float* row_max, float* row_sum, void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    Geometry geo;
    int rc = check_layer(graph, layer, &geo);
    if (rc != DFGNN_OK) return rc;
    const bool gt = layer->model == DFGNN_GT, gat = layer->model == DFGNN_GAT, v2 = layer->model == DFGNN_GATV2,
               agnn = layer->model == DFGNN_AGNN;
    if (graph->N == 0) return DFGNN_OK;  // nothing to compute; node tensors have no elements and may be NULL
    DFGNN_REQUIRE(x && out && row_max && row_sum, DFGNN_EINVAL, "x / out / row_max / row_sum is NULL");
    DFGNN_REQUIRE(!gt || (k && v), DFGNN_EINVAL, "GT needs k and v");
    DFGNN_REQUIRE(!v2 || (k && !v), DFGNN_EINVAL, "GATv2 needs k, and v must be NULL");
    DFGNN_REQUIRE(gt || v2 || (!k && !v), DFGNN_EINVAL, "k and v must be NULL unless the model is GT or GATv2");
    DFGNN_REQUIRE(!gat || (a_l && a_r), DFGNN_EINVAL, "GAT needs a_l and a_r");
    DFGNN_REQUIRE(!v2 || (a_l && !a_r), DFGNN_EINVAL, "GATv2 needs a_l, and a_r must be NULL");
    DFGNN_REQUIRE(gat || v2 || agnn || (!a_l && !a_r), DFGNN_EINVAL, "a_l and a_r must be NULL unless the model is GAT or GATv2");
    DFGNN_REQUIRE(!agnn || !a_r, DFGNN_EINVAL, "AGNN: a_r must be NULL (a_l may point to beta on the device)");
    DFGNN_REQUIRE(aligned16(x) && aligned16(k) && aligned16(v) && aligned16(out) && (agnn || aligned16(a_l)) && aligned16(a_r),
                  DFGNN_EUNSUPPORTED, "device pointers must be 16-byte aligned");
    DFGNN_REQUIRE(((uintptr_t)a_l & 3u) == 0, DFGNN_EUNSUPPORTED, "beta must be 4-byte aligned");
    DFGNN_REQUIRE(((uintptr_t)edge_bias & 3u) == 0, DFGNN_EUNSUPPORTED, "edge_bias must be 4-byte aligned");
    DFGNN_REQUIRE(!edge_bias || edge_term_fits(graph, layer), DFGNN_EUNSUPPORTED,
                  "edge term of E*H*4 bytes must stay below 4 GiB");
    if (const int kind = edge_bias ? 0 : dense_batch_kind(graph, layer)) {  // the dense-tile kernels have no edge term
        hipStream_t st = (hipStream_t)stream;
        rc = kind == 1   ? dense_gt_forward(graph, layer, x, k, v, out, row_max, row_sum, st)
             : kind == 2 ? dense32_gt_forward(graph, layer, x, k, v, out, row_max, row_sum, st)
                         : dense16_gt_forward(graph, layer, x, k, v, out, row_max, row_sum, st);
        if (rc != DFGNN_OK) return rc;
        DFGNN_HIP(hipGetLastError());
        return DFGNN_OK;
    }
    const Workspace W = workspace_layout(graph, layer, false, geo.heads);
    DFGNN_REQUIRE(workspace != nullptr, DFGNN_EINVAL, "workspace is NULL");
    DFGNN_REQUIRE(((uintptr_t)workspace % kAlign) == 0, DFGNN_EUNSUPPORTED, "workspace must be 256-byte aligned");
    DFGNN_REQUIRE(workspace_bytes >= W.total, DFGNN_EWORKSPACE, "workspace has %zu bytes, forward needs %zu",
                  workspace_bytes, W.total);
    Args a{};
    fill_common(a, graph, layer, geo);
    a.x = x; a.k = k; a.v = v; a.a_l = agnn ? nullptr : a_l; a.a_r = a_r;
    a.scale_dev = agnn ? a_l : nullptr;
    a.o = out; a.o_max = row_max; a.o_sum = row_sum;
    a.idx = graph->indices; a.edge_row = graph->edge_row; a.n_edges = (int)graph->E;
    a.bias = edge_bias;
    a.bias_bytes = (uint32_t)((uint64_t)graph->E * layer->H * 4u);
    bind_workspace(a, W, workspace, false);
    for (int gi = 0; gi < geo.groups; ++gi) {
        Args ag;
        select_group(ag, a, layer, geo, gi);
        rc = dispatch_forward(geo.id, graph, layer->model, ag, (hipStream_t)stream);
        if (rc != DFGNN_OK) return rc;
    }
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

extern "C" int dfgnn_attention_weights(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                                       const float* a_l, const float* a_r, const float* edge_bias,
                                       const float* row_max, const float* row_sum, float* p, void* stream) {
    clear_error();
    Geometry geo;
    int rc = check_layer(graph, layer, &geo);
    if (rc != DFGNN_OK) return rc;
    const bool gt = layer->model == DFGNN_GT, gat = layer->model == DFGNN_GAT, v2 = layer->model == DFGNN_GATV2,
               agnn = layer->model == DFGNN_AGNN;
    if (graph->N == 0 || graph->E == 0) return DFGNN_OK;  // no edge, nothing to write
    DFGNN_REQUIRE(x && row_max && row_sum && p, DFGNN_EINVAL, "x / row_max / row_sum / p is NULL");
    DFGNN_REQUIRE((gt || v2) == (k != nullptr), DFGNN_EINVAL, "k is needed by GT and GATv2 and by no other model");
    DFGNN_REQUIRE((agnn || (gat || v2) == (a_l != nullptr)) && gat == (a_r != nullptr), DFGNN_EINVAL,
                  "GAT needs a_l and a_r, GATv2 a_l, GT neither; AGNN may pass beta on the device in a_l");
    DFGNN_REQUIRE(aligned16(x) && aligned16(k) && (agnn || aligned16(a_l)) && aligned16(a_r) && ((uintptr_t)a_l & 3u) == 0,
                  DFGNN_EUNSUPPORTED, "device pointers must be 16-byte aligned (beta: 4-byte)");
    DFGNN_REQUIRE((((uintptr_t)edge_bias | (uintptr_t)p) & 3u) == 0, DFGNN_EUNSUPPORTED, "edge_bias / p must be 4-byte aligned");
    DFGNN_REQUIRE(!edge_bias || edge_term_fits(graph, layer), DFGNN_EUNSUPPORTED,
                  "edge term of E*H*4 bytes must stay below 4 GiB");
    Args a{};
    fill_common(a, graph, layer, geo);
    a.x = x; a.k = k; a.v = k;  // no value tensor is read; GT's value gathers are dropped by the compiler
    a.a_l = agnn ? nullptr : a_l; a.a_r = a_r;
    a.scale_dev = agnn ? a_l : nullptr;
    a.row_max = row_max; a.row_sum = row_sum;
    a.bias = edge_bias;
    a.bias_bytes = (uint32_t)((uint64_t)graph->E * layer->H * 4u);
    a.p_out = p;
    for (int gi = 0; gi < geo.groups; ++gi) {
        Args ag;
        select_group(ag, a, layer, geo, gi);
        rc = dispatch_attention(geo.id, graph, layer->model, ag, (hipStream_t)stream);
        if (rc != DFGNN_OK) return rc;
    }
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

extern "C" int dfgnn_forward(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                             const void* v, const float* a_l, const float* a_r, void* out, float* row_max,
                             float* row_sum, void* workspace, size_t workspace_bytes, void* stream) {
    return forward_impl(graph, layer, x, k, v, a_l, a_r, nullptr, out, row_max, row_sum, workspace, workspace_bytes,
                        stream);
}

extern "C" int dfgnn_forward_static(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                                    const void* v, const float* a_l, const float* a_r, void* out, float* row_max,
                                    float* row_sum, void* stream) {
    clear_error();
    Geometry geo;
    int rc = check_layer(graph, layer, &geo);
    if (rc != DFGNN_OK) return rc;
    const size_t need = workspace_layout(graph, layer, false, geo.heads).total;
    DFGNN_REQUIRE(need <= (size_t)DFGNN_STATIC_SCRATCH_BYTES, DFGNN_EWORKSPACE,
                  "this graph and layer need %zu bytes of forward workspace, the library's static scratch holds %zu: "
                  "use dfgnn_forward with a caller-provided workspace",
                  need, (size_t)DFGNN_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != DFGNN_OK) return rc;
    // nothing in the forward workspace has to start at zero: every chunk partial is written by the pass
    // kernel before the merge kernel of the same call reads it
    return forward_impl(graph, layer, x, k, v, a_l, a_r, nullptr, out, row_max, row_sum, ws,
                        (size_t)DFGNN_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int dfgnn_forward_edge_bias(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                                       const void* v, const float* a_l, const float* a_r, const float* edge_bias,
                                       void* out, float* row_max, float* row_sum, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    return forward_impl(graph, layer, x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum, workspace, workspace_bytes,
                        stream);
}

static int backward_impl(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                         const void* v, const float* a_l, const float* a_r, const float* edge_bias, const void* out,
                         const float* row_max, const float* row_sum, const void* d_out, void* d_x, void* d_k, void* d_v,
                         float* d_a_l, float* d_a_r, float* d_scale, float* d_edge_bias, void* workspace,
                         size_t workspace_bytes, void* stream) {
    clear_error();
    Geometry geo;
    int rc = check_layer(graph, layer, &geo);
    if (rc != DFGNN_OK) return rc;
    const bool gt = layer->model == DFGNN_GT, gat = layer->model == DFGNN_GAT, agnn = layer->model == DFGNN_AGNN,
               v2 = layer->model == DFGNN_GATV2;
    DFGNN_REQUIRE(!(graph->flags & DFGNN_SCHED_FORWARD_ONLY), DFGNN_EINVAL,
                  "the graph was created forward-only (DFGNN_SCHED_FORWARD_ONLY): it has no CSC for the backward pass");
    if (graph->N == 0) {  // no nodes: node tensors have no elements and may be NULL; parameter gradients are zero
        // cleared by a kernel, not a memset: layer calls may be recorded into a HIP graph
        if ((gat || v2) && d_a_l) launch_zero(d_a_l, layer->H * layer->D, (hipStream_t)stream);
        if (gat && d_a_r) launch_zero(d_a_r, layer->H * layer->D, (hipStream_t)stream);
        if (agnn && d_scale) launch_zero(d_scale, 1, (hipStream_t)stream);
        DFGNN_HIP(hipGetLastError());
        return DFGNN_OK;
    }
    DFGNN_REQUIRE(x && out && row_max && row_sum && d_out && d_x, DFGNN_EINVAL,
                  "x / out / row_max / row_sum / d_out / d_x is NULL");
    DFGNN_REQUIRE(!gt || (k && v && d_k && d_v), DFGNN_EINVAL, "GT needs k, v, d_k and d_v");
    DFGNN_REQUIRE(!v2 || (k && d_k && !v && !d_v), DFGNN_EINVAL, "GATv2 needs k and d_k; v and d_v must be NULL");
    DFGNN_REQUIRE(gt || v2 || (!k && !v && !d_k && !d_v), DFGNN_EINVAL,
                  "k, v, d_k, d_v must be NULL unless the model is GT or GATv2");
    DFGNN_REQUIRE(!gat || (a_l && a_r && d_a_l && d_a_r), DFGNN_EINVAL, "GAT needs a_l, a_r, d_a_l and d_a_r");
    DFGNN_REQUIRE(!v2 || (a_l && d_a_l && !a_r && !d_a_r), DFGNN_EINVAL,
                  "GATv2 needs a_l and d_a_l; a_r and d_a_r must be NULL");
    DFGNN_REQUIRE(gat || v2 || (!a_r && !d_a_l && !d_a_r && (agnn || !a_l)), DFGNN_EINVAL,
                  "a_l, a_r, d_a_l, d_a_r must be NULL unless the model is GAT or GATv2 (AGNN: a_l may point to beta)");
    DFGNN_REQUIRE(!agnn || d_scale, DFGNN_EINVAL, "AGNN needs d_scale");
    DFGNN_REQUIRE(agnn || !d_scale, DFGNN_EINVAL, "d_scale must be NULL unless the model is AGNN");
    DFGNN_REQUIRE(aligned16(x) && aligned16(k) && aligned16(v) && aligned16(out) && aligned16(d_out) && aligned16(d_x) &&
                      aligned16(d_k) && aligned16(d_v) && (agnn || aligned16(a_l)) && aligned16(a_r) && ((uintptr_t)a_l & 3u) == 0,
                  DFGNN_EUNSUPPORTED, "device pointers must be 16-byte aligned (beta: 4-byte)");
    DFGNN_REQUIRE((((uintptr_t)edge_bias | (uintptr_t)d_edge_bias) & 3u) == 0, DFGNN_EUNSUPPORTED,
                  "edge_bias / d_edge_bias must be 4-byte aligned");
    DFGNN_REQUIRE(edge_bias || !d_edge_bias, DFGNN_EINVAL, "d_edge_bias without edge_bias");
    DFGNN_REQUIRE(!edge_bias || edge_term_fits(graph, layer), DFGNN_EUNSUPPORTED,
                  "edge term of E*H*4 bytes must stay below 4 GiB");
    const int dense_kind = edge_bias ? 0 : dense_batch_kind(graph, layer);
    if (dense_kind == 1) {
        rc = dense_gt_backward(graph, layer, x, k, v, row_max, row_sum, d_out, d_x, d_k, d_v, (hipStream_t)stream);
        if (rc != DFGNN_OK) return rc;
        DFGNN_HIP(hipGetLastError());
        return DFGNN_OK;
    }
    const Workspace W = workspace_layout(graph, layer, true, geo.heads);
    DFGNN_REQUIRE(workspace != nullptr, DFGNN_EINVAL, "workspace is NULL");
    DFGNN_REQUIRE(((uintptr_t)workspace % kAlign) == 0, DFGNN_EUNSUPPORTED, "workspace must be 256-byte aligned");
    DFGNN_REQUIRE(workspace_bytes >= W.total, DFGNN_EWORKSPACE, "workspace has %zu bytes, backward needs %zu",
                  workspace_bytes, W.total);
    hipStream_t st = (hipStream_t)stream;
    if (dense_kind != 0) {  // the row kernel hands {lse2, delta} to the column kernel through the workspace
        float* stats = (float*)((char*)workspace + W.stats);
        rc = dense_kind == 2 ? dense32_gt_backward(graph, layer, x, k, v, out, row_max, row_sum, d_out, d_x, d_k, d_v,
                                                   stats, st)
                             : dense16_gt_backward(graph, layer, x, k, v, row_max, row_sum, d_out, d_x, d_k, d_v, stats, st);
        if (rc != DFGNN_OK) return rc;
        DFGNN_HIP(hipGetLastError());
        return DFGNN_OK;
    }

    Args a{};
    fill_common(a, graph, layer, geo);
    a.x = x; a.k = k; a.v = v; a.a_l = agnn ? nullptr : a_l; a.a_r = a_r;
    a.scale_dev = agnn ? a_l : nullptr;
    a.out = out; a.row_max = row_max; a.row_sum = row_sum; a.d_out = d_out;
    a.d_x = d_x; a.d_k = d_k; a.d_v = d_v;
    a.bias = edge_bias; a.d_bias = d_edge_bias;
    a.bias_bytes = (uint32_t)((uint64_t)graph->E * layer->H * 4u);
    bind_workspace(a, W, workspace, true);
    double* reduce_tmp = (double*)((char*)workspace + W.reduce);
    for (int gi = 0; gi < geo.groups; ++gi) {
        Args ag;
        select_group(ag, a, layer, geo, gi);
        const size_t pb = (size_t)gi * geo.heads * layer->D * sizeof(float);
        // d_scale (AGNN) is one number for all heads: the first group writes it, the others add to it
        rc = dispatch_backward(geo.id, graph, layer->model, ag, reduce_tmp, shift(d_a_l, pb), shift(d_a_r, pb), d_scale,
                               gi > 0, st);
        if (rc != DFGNN_OK) return rc;
    }
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}

extern "C" int dfgnn_backward(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                              const void* v, const float* a_l, const float* a_r, const void* out, const float* row_max,
                              const float* row_sum, const void* d_out, void* d_x, void* d_k, void* d_v, float* d_a_l,
                              float* d_a_r, float* d_scale, void* workspace, size_t workspace_bytes, void* stream) {
    return backward_impl(graph, layer, x, k, v, a_l, a_r, nullptr, out, row_max, row_sum, d_out, d_x, d_k, d_v, d_a_l,
                         d_a_r, d_scale, nullptr, workspace, workspace_bytes, stream);
}

extern "C" int dfgnn_backward_edge_bias(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x,
                                        const void* k, const void* v, const float* a_l, const float* a_r,
                                        const float* edge_bias, const void* out, const float* row_max,
                                        const float* row_sum, const void* d_out, void* d_x, void* d_k, void* d_v,
                                        float* d_a_l, float* d_a_r, float* d_scale, float* d_edge_bias,
                                        void* workspace, size_t workspace_bytes, void* stream) {
    return backward_impl(graph, layer, x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum, d_out, d_x, d_k, d_v,
                         d_a_l, d_a_r, d_scale, d_edge_bias, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// Yardstick for the gather kernels: the rows idx[e] of a table are read with the same instruction the
// passes gather with (16 bytes per lane, row_bytes / 16 lanes per row, four rows of an edge slot in
// flight) and nothing else happens to them, so the rate of this kernel is what the memory system gives
// to random row reads of that size on this machine.
// ---------------------------------------------------------------------------------------------
namespace dfgnn {
constexpr int kProbeRows = 4;  // rows requested per edge slot before the first is used (as in the passes)
static __global__ __launch_bounds__(64 * kWavesPerBlock) void k_probe_gather(const void* __restrict__ table, uint32_t table_bytes,
                                                                             uint32_t row_bytes, int lpe_shift,
                                                                             const int* __restrict__ idx, int64_t n,
                                                                             u32x4* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t thread = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t wave = thread >> 6, waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int epw = 64 >> lpe_shift, slot = lane >> lpe_shift;
    const uint32_t part = (uint32_t)(lane & ((1 << lpe_shift) - 1)) * 16u;
    const rsrc_t r = make_rsrc(table, table_bytes);
    u32x4 acc = {0u, 0u, 0u, 0u};
    // wave w takes the rounds w, w + waves, ...; a round is epw * kProbeRows consecutive entries of idx
    for (int64_t e0 = wave * epw * kProbeRows; e0 < n; e0 += waves * epw * kProbeRows) {
        u32x4 v[kProbeRows];
#pragma unroll
        for (int u = 0; u < kProbeRows; ++u) {
            const int64_t e = e0 + (int64_t)u * epw + slot;
            const int j = e < n ? idx[e] : -1;
            v[u] = buf_load16(r, j >= 0 ? (uint32_t)j * row_bytes + part : 0xffffffffu);  // (out of range: zeros)
        }
#pragma unroll
        for (int u = 0; u < kProbeRows; ++u) acc ^= v[u];
    }
    out[thread] = acc;
}
}  // namespace dfgnn

extern "C" int dfgnn_probe_gather(const void* table, int64_t n_rows, int32_t row_bytes, const int32_t* idx, int64_t n_idx,
                                  void* out, size_t out_bytes, void* stream) {
    clear_error();
    DFGNN_REQUIRE(table && idx && out && n_rows > 0 && n_idx >= 0, DFGNN_EINVAL, "NULL pointer, n_rows <= 0 or n_idx < 0");
    int lpe_shift = 0;
    while (lpe_shift < 6 && (16 << lpe_shift) != row_bytes) ++lpe_shift;
    DFGNN_REQUIRE((16 << lpe_shift) == row_bytes, DFGNN_EINVAL, "row_bytes = %d is not 16, 32, ..., 1024", row_bytes);
    DFGNN_REQUIRE((uint64_t)n_rows * (uint64_t)row_bytes < (1ull << 32), DFGNN_EUNSUPPORTED, "the table must stay below 4 GiB");
    const size_t block_bytes = (size_t)64 * kWavesPerBlock * 16;  // a workgroup writes 16 bytes per thread
    DFGNN_REQUIRE(out_bytes >= block_bytes && out_bytes / block_bytes <= 0x7fffffffu, DFGNN_EINVAL,
                  "out_bytes = %zu is below one workgroup's %zu bytes (or absurdly large)", out_bytes, block_bytes);
    DFGNN_REQUIRE(aligned16(table) && aligned16(out) && ((uintptr_t)idx & 3u) == 0, DFGNN_EUNSUPPORTED,
                  "table and out must be 16-byte aligned, idx 4-byte");
    hipLaunchKernelGGL(dfgnn::k_probe_gather, dim3((unsigned)(out_bytes / block_bytes)), dim3(64 * kWavesPerBlock), 0,
                       (hipStream_t)stream, table, (uint32_t)((uint64_t)n_rows * (uint64_t)row_bytes), (uint32_t)row_bytes,
                       lpe_shift, idx, n_idx, (dfgnn::u32x4*)out);
    DFGNN_HIP(hipGetLastError());
    return DFGNN_OK;
}
