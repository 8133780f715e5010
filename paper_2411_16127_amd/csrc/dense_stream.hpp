// Work decomposition and memory access shared by the streaming dense-tile kernels (fp32 and bf16): one
// wavefront per (graph, head, tile of 16 rows or columns) that walks over the graph's other 16-node
// tiles.  Everything a wavefront reads goes through buffer loads against a view of its own graph (and
// head): offsets are relative to the graph's first node, and a row past the graph's end is out of range
// and reads as zero, so the tile loops contain no bounds checks and no branches.
#pragma once
#include "layer_device.hpp"

namespace dfgnn {

struct Unit {
    int base, n, tiles, t, h;  // graph's first node, node count, tile count; this wave's tile and head
};

// u must be the same in all lanes (it is made so here); the result lives in scalar registers
template <class ArgsT> __device__ inline Unit find_unit(const ArgsT& a, int u) {
    u = __builtin_amdgcn_readfirstlane(u);
    const int tile = u / a.H;
    Unit r;
    r.h = u - tile * a.H;
    const int lo = a.tile_graph[tile];
    r.base = a.batch_ptr[lo];
    r.n = a.batch_ptr[lo + 1] - r.base;
    r.tiles = (r.n + 15) >> 4;
    r.t = tile - a.tile_ptr[lo];
    return r;
}

// view of the unit's head in a node tensor [N, H*D]: byte offset = row_in_graph * HD * elem + feature * elem
__device__ inline rsrc_t unit_tensor(const void* x, const Unit& u, int HD, int D, int elem) {
    const char* p = static_cast<const char*>(x) + ((size_t)u.base * HD + (size_t)u.h * D) * elem;
    return make_rsrc(p, u.n > 0 ? (uint32_t)(((u.n - 1) * HD + D) * elem) : 0u);
}
// view of the unit's graph in a per-node array of `stride` bytes per node, starting `first` bytes into a node's record
__device__ inline rsrc_t unit_rows(const void* x, const Unit& u, int stride, int first, int bytes) {
    const char* p = static_cast<const char*>(x) + (size_t)u.base * stride + first;
    return make_rsrc(p, u.n > 0 ? (uint32_t)((u.n - 1) * stride + bytes) : 0u);
}

// The hardware deals workgroups to the 8 XCDs round-robin, and every XCD has an L2 of its own.  This maps
// block b to the (b % 8)-th contiguous eighth of the work list, so that the units of one graph (all its
// heads and row tiles, which read the same rows over and over) run on one XCD and share one L2.
__device__ inline int xcd_block(int b, int nb) {
    const int per = nb >> 3;
    return b < (per << 3) ? (b & 7) * per + (b >> 3) : b;
}

// adjacency bits of entries 4q .. 4q+3 of 16-wide tile t, from the mask words of one row (or column)
__device__ inline uint32_t tile_bits(rsrc_t masks, uint32_t row_off, int t, int q) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 w = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(masks, row_off + (uint32_t)(t >> 2) * 8u, 0, 0));
    const unsigned long long word = ((unsigned long long)w[1] << 32) | w[0];
    return (uint32_t)(word >> ((t & 3) * 16 + 4 * q)) & 0xfu;
}

__device__ inline float sum_q(float x) { x += __shfl_xor(x, 16); x += __shfl_xor(x, 32); return x; }
__device__ inline float max_q(float x) { x = fmaxf(x, __shfl_xor(x, 16)); x = fmaxf(x, __shfl_xor(x, 32)); return x; }

constexpr int kDenseWaves = 4;

}  // namespace dfgnn
