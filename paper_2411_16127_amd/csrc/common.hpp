// Internal host-side definitions shared by the translation units of libdfgnn (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "../../include/dfgnn.h"

namespace dfgnn {

constexpr size_t kAlign = 256;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Thread-local error text behind dfgnn_last_error().
void set_error(const char* fmt, ...);
void clear_error();

#define DFGNN_HIP(expr)                                                                         \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            ::dfgnn::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return DFGNN_EHIP;                                                                  \
        }                                                                                       \
    } while (0)

#define DFGNN_REQUIRE(cond, status, ...)   \
    do {                                   \
        if (!(cond)) {                     \
            ::dfgnn::set_error(__VA_ARGS__); \
            return (status);               \
        }                                  \
    } while (0)

// Capacity of the chunk arrays for a graph with E edges: a super row has at least T edges, and a row of
// deg edges has ceil(deg / C) <= deg / C + 1 chunks.
inline int64_t super_capacity(int64_t E, int T) { return E / T + 1; }
inline int64_t chunk_capacity(int64_t E, int T, int C) { return E / C + super_capacity(E, T) + 1; }

// Byte offsets of the arrays inside the caller's metadata buffer.
struct MetaLayout {
    size_t row_order, col_order, t_indptr, t_indices, t_eid;
    size_t row_chunk_ptr, row_chunks, col_chunk_ptr, col_chunks, counters, edge_row, total;
};
MetaLayout meta_layout(int64_t N, int64_t E, int T, int C, int flags);

// Optional per-kernel timing (dfgnn_timing_enable): a pair of HIP events around a launch.
struct KernelTimer {
    KernelTimer(const char* label, hipStream_t st);
    ~KernelTimer();
    int slot;
    hipStream_t stream;
};

}  // namespace dfgnn

// The opaque handle of the ABI.
struct dfgnn_graph {
    int64_t N, E;
    int T, C, flags;
    const int32_t* indptr;
    const int32_t* indices;
    int32_t *row_order, *col_order, *t_indptr, *t_indices, *t_eid;
    int32_t *row_chunk_ptr, *row_chunks, *col_chunk_ptr, *col_chunks;
    int32_t n_super_rows, n_row_chunks, n_super_cols, n_col_chunks;
    // [k] = position in row_order / col_order of the first entry with sort key >= k (key 0 = super,
    // key 33 - b = bit_length(degree) b); [35] = N
    int32_t row_bucket_ptr[36], col_bucket_ptr[36];
    // block-diagonal batch of small graphs (dfgnn_graph_set_batch); arrays live in the caller's batch buffer
    const int32_t* batch_ptr;
    int64_t n_graphs;
    int32_t* tile_ptr;               // [n_graphs + 1] first 16-node tile of every graph
    int32_t* tile_graph;             // [n_tiles] graph of every 16-node tile
    int64_t n_tiles;
    int64_t tile_pairs;              // sum over graphs of (tiles of the graph)^2: 16 x 16 score tiles a dense pass forms
    int32_t max_graph_nodes;
    int32_t mask_words;              // 64-bit words per row of the adjacency bit masks
    unsigned long long* adj_mask;    // [N][mask_words] bit j: edge row <- (first node of the graph + j)
    unsigned long long* adj_mask_t;  // [N][mask_words] bit i: edge (first node + i) <- column
    int32_t* counters;               // device scratch words inside the metadata buffer
    int32_t* edge_row;               // [E] destination row of every CSR position (only with SCORES_IN_MEMORY)
    bool batch_dense;                // no repeated edge and every graph has at most 512 nodes
    int32_t xcd_group;               // workgroups per XCD-local run of a pass's work list (0: plain round-robin)
};

namespace dfgnn {
int dense_batch_kind(const dfgnn_graph* g, const dfgnn_layer* L);
int dense_gt_forward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v, void* out,
                     float* row_max, float* row_sum, hipStream_t st);
int dense_gt_backward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v,
                      const float* row_max, const float* row_sum, const void* d_out, void* d_q, void* d_k, void* d_v,
                      hipStream_t st);
int dense16_gt_forward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v, void* out,
                       float* row_max, float* row_sum, hipStream_t st);
int dense16_gt_backward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v,
                        const float* row_max, const float* row_sum, const void* d_out, void* d_q, void* d_k, void* d_v,
                        float* stats, hipStream_t st);
int dense32_gt_forward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v, void* out,
                       float* row_max, float* row_sum, hipStream_t st);
int dense32_gt_backward(const dfgnn_graph* g, const dfgnn_layer* L, const void* q, const void* k, const void* v,
                        const void* out, const float* row_max, const float* row_sum, const void* d_out, void* d_q,
                        void* d_k, void* d_v, float* stats, hipStream_t st);
constexpr int kXcdGroup = 32;          // run length used for graphs whose numbering is local
constexpr int kDenseSmallNodes = 64;   // bf16 kernels: a whole graph head per wavefront
constexpr int kDenseMaxGraphNodes = 512;
constexpr int kDenseMaxWords = kDenseMaxGraphNodes / 64;
}  // namespace dfgnn
