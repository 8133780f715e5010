// Device-side building blocks of the fused attention-GNN layer kernels (gfx950, wave64).
//
// Work mapping (the node-parallel / edge-parallel choice of Sec. 2.2 and Sec. 4.1, taken per row):
//   * one wavefront processes one work item: a whole row (node-parallel) or one chunk of a super row
//     (edge-parallel split); chunk partials are combined by a merge kernel;
//   * inside the wavefront, LPE adjacent lanes cover one neighbour's feature row with one 16-byte load
//     each, so 64/LPE neighbours are in flight per load instruction (coalesced, vectorised access of
//     Sec. 4.2 "SpMM"); U such instructions are issued back to back before any is consumed;
//   * a head's dot product is reduced over its LPH lanes with DPP cross-lane moves; the softmax is kept
//     online per edge slot (max / sum / accumulator in registers), so no score or attention weight is
//     ever stored (Sec. 4.2 "Softmax": no duplicated work, no recomputation inside a pass).
// This file holds what all models share (element types, buffer loads, reductions, the online softmax,
// the kernels that drive a pass); the passes of a model are in pass_gt.hpp, pass_gat.hpp,
// pass_gatv2.hpp and pass_agnn.hpp.  A pass is a struct with init / issue / consume / combine_slots /
// store_partial / load_partial / fold_partial / finalize; k_pass and k_merge are templates over it.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace dfgnn {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct bf16_t { uint16_t bits; };
struct f16_t { uint16_t bits; };  // IEEE half

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---------------------------------------------------------------------------------------------
// element types: a lane owns VEC consecutive elements = 16 bytes of a node row
// ---------------------------------------------------------------------------------------------
template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int VEC = 4;
    __device__ static void unpack(const u32x4& r, float (&x)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = __builtin_bit_cast(float, (uint32_t)r[i]);
    }
    __device__ static void store(float* p, const float (&x)[4]) {
        f32x4 t = {x[0], x[1], x[2], x[3]};
        *reinterpret_cast<f32x4*>(p) = t;
    }
};

template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    __device__ static void unpack(const u32x4& r, float (&x)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w = r[i];
            x[2 * i] = __builtin_bit_cast(float, w << 16);
            x[2 * i + 1] = __builtin_bit_cast(float, w & 0xffff0000u);
        }
    }
    __device__ static uint32_t round_bits(float f) {  // round to nearest even, keep the high half
        uint32_t u = __builtin_bit_cast(uint32_t, f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    __device__ static void store(bf16_t* p, const float (&x)[8]) {
        u32x4 t;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = round_bits(x[2 * i]) | (round_bits(x[2 * i + 1]) << 16);
        *reinterpret_cast<u32x4*>(p) = t;
    }
};

template <> struct Elem<f16_t> {
    static constexpr int VEC = 8;
    typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
    __device__ static void unpack(const u32x4& r, float (&x)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const h16x2 h = __builtin_bit_cast(h16x2, (uint32_t)r[i]);
            x[2 * i] = (float)h[0];
            x[2 * i + 1] = (float)h[1];
        }
    }
    __device__ static void store(f16_t* p, const float (&x)[8]) {  // round to nearest even
        u32x4 t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const h16x2 h = {(_Float16)x[2 * i], (_Float16)x[2 * i + 1]};
            t[i] = __builtin_bit_cast(uint32_t, h);
        }
        *reinterpret_cast<u32x4*>(p) = t;
    }
};

// Gathers go through buffer loads: a 32-bit byte offset per lane against a base held in scalar
// registers, with the hardware range check returning zeros past the end of the tensor.  An absent
// neighbour (index -1) wraps to an offset beyond any tensor (tensors are kept below 4 GiB), so tail
// rounds need no per-lane branches.
using rsrc_t = __amdgpu_buffer_rsrc_t;
__device__ inline rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline u32x4 buf_load16(rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
}
__device__ inline f32x4 buf_load_f32x4(rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
}
__device__ inline f32x2 buf_load_f32x2(rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(f32x2, __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0));
}
__device__ inline float buf_load_f32(rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
}

template <typename T> __device__ inline u32x4 load_raw(const void* base, size_t elem_offset) {
    return *reinterpret_cast<const u32x4*>(static_cast<const T*>(base) + elem_offset);
}

template <int VEC> __device__ inline void load_f32(const float* p, float (&x)[VEC]) {
#pragma unroll
    for (int i = 0; i < VEC; i += 4) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(p + i);
        x[i] = t[0]; x[i + 1] = t[1]; x[i + 2] = t[2]; x[i + 3] = t[3];
    }
}
template <int VEC> __device__ inline void store_f32(float* p, const float (&x)[VEC]) {
#pragma unroll
    for (int i = 0; i < VEC; i += 4) {
        f32x4 t = {x[i], x[i + 1], x[i + 2], x[i + 3]};
        *reinterpret_cast<f32x4*>(p + i) = t;
    }
}

template <int VEC> __device__ inline float dotv(const float (&a)[VEC], const float (&b)[VEC]) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) s = fmaf(a[i], b[i], s);
    return s;
}

// ---------------------------------------------------------------------------------------------
// cross-lane reductions
// ---------------------------------------------------------------------------------------------
template <int CTRL> __device__ inline float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over the LPH adjacent lanes of one head; every lane of the head gets the total.
// LPH = 0: the head width is the run-time value lph (a power of two).
template <int LPH> __device__ inline float head_sum(float x, int lph) {
    if constexpr (LPH == 0) {
        for (int o = 1; o < lph; o <<= 1) x += __shfl_xor(x, o);
    } else {
        if constexpr (LPH >= 2) x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
        if constexpr (LPH >= 4) x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
        if constexpr (LPH >= 8) x += dpp_move<0x141>(x);  // row_half_mirror
        if constexpr (LPH >= 16) x += dpp_move<0x140>(x); // row_mirror
        if constexpr (LPH >= 32) x += __shfl_xor(x, 16);
        if constexpr (LPH >= 64) x += __shfl_xor(x, 32);
    }
    return x;
}

// Sum over the 64/LPE edge slots of the wavefront (lanes that own the same features).
template <int LPE> __device__ inline float slot_sum(float x) {
#pragma unroll
    for (int o = LPE; o < 64; o <<= 1) x += __shfl_xor(x, o);
    return x;
}

// ---------------------------------------------------------------------------------------------
// kernel arguments
// ---------------------------------------------------------------------------------------------
struct Args {
    // work list: CSR (rows) for forward / backward row pass, CSC (columns) for the backward column pass
    const int* ptr;
    const int* idx;
    const int* order;
    const int* chunks;
    const int* chunk_ptr;
    int n_chunks, blocks_chunk;             // chunk items (super rows), and the workgroups that hold them
    int n_direct, blocks_direct;            // whole-row items: order[first_direct + item]
    int n_small, first_small, first_direct; // short rows: order[first_small + r], one per edge slot
    int n_items;                            // merge kernel: super rows
    int merge_groups;                       // merge kernels: largest number of chunk groups per super row (1: one level)
    int xcd_group;                          // workgroups per XCD-local run of the work list (0: no remapping)
    int n_nodes;
    int wide;               // node tensors of 4 GiB and more: gathers use 64-bit addresses (run-time geometries only)
    uint32_t row_bytes;     // bytes of one node row
    uint32_t tensor_bytes;  // bytes of one node tensor (unused when wide)
    uint32_t nh_bytes;      // bytes of one [N, H] fp32 array
    // shape and constants.  H, HD describe the heads this launch works on; when a layer has more features
    // than one wavefront covers, the host runs it in groups of heads, and the caller's tensors keep the
    // strides of the whole layer (row_stride, stat_stride, bias_stride: elements between consecutive nodes
    // or edges), while workspace arrays are compact ([.., HD] or [.., H] of the group).
    int H, D, HD, lph;
    int row_stride, stat_stride, bias_stride;
    float c_score;  // GT scale*log2(e); AGNN beta*log2(e); GAT log2(e)
    float scale;    // GT scale; AGNN beta
    const float* scale_dev;  // AGNN: beta read from device memory instead (nullptr: the value above)
    float neg_slope, eps, inv_eps;
    // tensors in the layer dtype
    const void *x, *k, *v, *out, *d_out;
    void *o, *d_x, *d_k, *d_v;
    // fp32 tensors
    const float *a_l, *a_r, *row_max, *row_sum;
    float *o_max, *o_sum;
    // workspace
    float* stats;      // per (row, head): GT {lse2, delta}; GAT {el2, lse2, delta, 0}; AGNN {rn, lse2, delta, 0}
    float* d_el;       // GAT [N,H]
    float* d_er;       // GAT [N,H]
    float* g_row;      // AGNN [N,HD] row-side gradient w.r.t. normalised features
    float* dbeta_row;  // AGNN [N,H]
    float* part_v0;    // [chunks, HD]
    float* part_v1;    // [chunks, HD]
    float* part_v2;    // [chunks, HD] (GATv2 backward)
    float* part_v3;    // [chunks, HD] (GATv2 backward)
    float* da_row;     // GATv2 [N,HD] per-row contribution to the gradient of the attention vector
    float* part_s0;    // [chunks, H]
    float* part_s1;    // [chunks, H]
    float* part_s2;    // [chunks, H]
    // optional additive edge term of the score (edge features, Sec. 1): [E, H] fp32 in CSR edge order
    const float* bias;
    uint32_t bias_bytes;  // E * H * 4 (< 4 GiB)
    float* d_bias;   // its gradient dS (may be null)
    const int* eid;  // column pass only, when there is an edge term: CSR position of every CSC entry
    float* p_out;    // attention-weight output [E, bias_stride] (dfgnn_attention_weights)
    // scores-through-memory comparator
    float* scores;        // [E, H] scaled scores in log2 units
    const int* edge_row;  // [E] destination row of every CSR position
    int n_edges;
};

// AGNN's beta: a layer field, or one float in device memory (so that a trained beta never has to visit the host)
__device__ inline float agnn_beta(const Args& a) { return a.scale_dev ? *a.scale_dev : a.scale; }

// Lane geometry: LPE lanes per neighbour row, LPH lanes per head (0 = run-time), element type T.
// EDGE_TERM: the kernels also handle the optional additive edge term of the score (kept out of the
// ordinary kernels at compile time, so that they pay nothing for it).
template <typename T_, int LPE_, int LPH_, bool EDGE_TERM_ = false> struct Geo {
    using T = T_;
    static constexpr int LPE = LPE_, LPH = LPH_, VEC = Elem<T_>::VEC, EPW = 64 / LPE_;
    static constexpr bool kEdgeTerm = EDGE_TERM_;
};

struct Ctx {
    int lane, c, g, f0, h, node;
    int deg;      // neighbours of the row this lane finishes (a large value where a row is merged from chunks)
    bool active;  // this lane's features exist (f0 < HD)
    bool head0;   // first lane of its head
    bool writer;  // this lane stores results: edge slot 0 when the wave shares one row, every live slot otherwise
    uint32_t fbyte;  // byte offset of this lane's features inside a node row
    uint32_t hbyte;  // byte offset of this lane's head inside a [.., H] fp32 record
    size_t off;   // node*row_stride + f0: this lane's features in a caller's node tensor
    size_t woff;  // node*HD + f0: the same in a compact workspace array
};

// Where a lane reads chunk partials: lanes without features of their own read feature 0 / head 0, so
// the merge loop has no per-lane branch (its loads can overlap); such lanes never store anything.
struct PartialIndex {
    int f0, h;
    __device__ explicit PartialIndex(const Ctx& c) : f0(c.active ? c.f0 : 0), h(c.h) {}
};

// One chunk's partial results as loaded by a merge wavefront: up to four feature vectors and three
// per-head scalars (each pass uses the ones it stored; chunks of an absent index are masked when folded).
template <int VEC> struct PartialRegs {
    float v0[VEC], v1[VEC], v2[VEC], v3[VEC], s0, s1, s2;
};

template <class G> __device__ inline Ctx make_ctx(const Args& a, int lane, int node) {
    Ctx c;
    c.lane = lane;
    c.c = lane % G::LPE;
    c.g = lane / G::LPE;
    c.f0 = c.c * G::VEC;
    c.active = c.f0 < a.HD;
    // head of this lane: lanes per head is a power of two (a compile-time one where the geometry fixes it)
    const int lph = G::LPH > 0 ? G::LPH : a.lph;
    c.h = c.active ? c.c >> __builtin_ctz(lph) : 0;
    c.head0 = c.active && (c.c & (lph - 1)) == 0;
    c.node = node;
    c.deg = 0x7fffffff;
    c.off = (size_t)node * a.row_stride + c.f0;
    c.woff = (size_t)node * a.HD + c.f0;
    c.writer = c.g == 0;
    c.fbyte = (uint32_t)c.f0 * (uint32_t)sizeof(typename G::T);
    c.hbyte = (uint32_t)c.h * 4u;
    return c;
}

template <class G> __device__ inline void load_row(const void* base, const Ctx& c, float (&x)[G::VEC]) {
    if (c.active) {
        Elem<typename G::T>::unpack(load_raw<typename G::T>(base, c.off), x);
    } else {
#pragma unroll
        for (int i = 0; i < G::VEC; ++i) x[i] = 0.f;
    }
}

// neighbour row j of a node tensor (zeros for j = -1).  Tensors of 4 GiB and more are beyond a buffer
// resource's 32-bit range: the kernels whose head width is a run-time value (LPH = 0) then form a 64-bit
// address per lane and skip the load for an absent neighbour (and for lanes without features of their own,
// which the range check would otherwise cover at the end of the tensor).  The branch is the same in every
// lane of the launch; the kernels with compile-time geometries, which the host never picks for such tensors,
// do not carry it.
template <class G> __device__ inline u32x4 gather_raw(const void* base, const Args& a, const Ctx& c, int j) {
    if constexpr (G::LPH == 0) {
        if (a.wide) {
            u32x4 r = {0u, 0u, 0u, 0u};
            if (j >= 0 && c.active)
                r = *reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + (size_t)(uint32_t)j * a.row_bytes + c.fbyte);
            return r;
        }
    }
    return buf_load16(make_rsrc(base, a.tensor_bytes), (uint32_t)j * a.row_bytes + c.fbyte);
}
// one fp32 value of (i, head) from an [N, stat_stride] array (zero for i = -1)
__device__ inline float gather_stat(const float* p, const Args& a, const Ctx& c, int i) {
    return buf_load_f32(make_rsrc(p, (uint32_t)a.n_nodes * (uint32_t)a.stat_stride * 4u),
                        i >= 0 ? (uint32_t)i * (uint32_t)(a.stat_stride * 4) + c.hbyte : 0xffffffffu);
}
// packed row statistics of (i, head): 2 or 4 floats per record (zeros for i = -1)
__device__ inline f32x2 gather_stats2(const Args& a, const Ctx& c, int i) {
    return buf_load_f32x2(make_rsrc(a.stats, a.nh_bytes * 2u), (uint32_t)i * (uint32_t)(a.H * 8) + c.hbyte * 2u);
}
__device__ inline f32x4 gather_stats4(const Args& a, const Ctx& c, int i) {
    return buf_load_f32x4(make_rsrc(a.stats, a.nh_bytes * 4u), (uint32_t)i * (uint32_t)(a.H * 16) + c.hbyte * 4u);
}

// additive edge term of edge e (CSR position); 0 for an empty slot (the offset is then out of range and
// the buffer load returns zero; the [E, H] array is kept below 4 GiB)
template <class G> __device__ inline float load_bias(const Args& a, const Ctx& c, int j, int e) {
    if constexpr (G::kEdgeTerm)
        return buf_load_f32(make_rsrc(a.bias, a.bias_bytes), j >= 0 ? (uint32_t)e * (uint32_t)(a.bias_stride * 4) + c.hbyte : 0xffffffffu);
    else return 0.f;
}
// score in log2 units plus the edge term (given in natural units)
template <class G> __device__ inline float with_bias(float s, float b) {
    if constexpr (G::kEdgeTerm) return fmaf(b, kLog2e, s);
    else return s;
}
// Gradient of the edge term = dS of the edge.  Both backward passes know dS of every edge; the row pass
// writes it (in CSR order, i.e. sequentially) when it has the final delta during its sweep (fp32
// tensors), otherwise the column pass does (bf16 tensors, where delta is only known at the end of a row).
template <class G, bool ROW_PASS> __device__ inline void store_dbias(const Args& a, const Ctx& c, bool valid, int e, float ds) {
    if constexpr (G::kEdgeTerm && ROW_PASS == (sizeof(typename G::T) == 4)) {
        if (a.d_bias != nullptr && valid && c.head0) a.d_bias[(size_t)e * a.bias_stride + c.h] = ds;
    }
}

// ---------------------------------------------------------------------------------------------
// online softmax accumulator shared by the three forward passes (edge softmax of Appendix A in its
// streaming form: running maximum m, running sum l and running weighted value sum acc, in log2 units)
// ---------------------------------------------------------------------------------------------
template <class G, int U> struct SoftmaxAcc {
    static constexpr int VEC = G::VEC;
    float m, l, acc[VEC];

    __device__ void reset() {
        m = -INFINITY;
        l = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    }
    // the interface a forward pass drives (see also AttentionOut below)
    __device__ void init(const Args&, const Ctx&) { reset(); }
    __device__ void absorb(const Args&, const Ctx&, const float (&s)[U], const u32x4 (&val)[U], const int (&)[U],
                           const int (&)[U]) {
        update(s, val);
    }
    // s[u] = -inf for slots without an edge (their value registers hold zeros); s[0] must be finite
    __device__ void update(const float (&s)[U], const u32x4 (&val)[U]) {
        float mn = m;
#pragma unroll
        for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u]);
        const float corr = fast_exp2(m - mn);
        l *= corr;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] *= corr;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float p = fast_exp2(s[u] - mn);
            float vf[VEC];
            Elem<typename G::T>::unpack(val[u], vf);
            l += p;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaf(p, vf[i], acc[i]);
        }
        m = mn;
    }
    __device__ void merge(float mo, float lo, const float (&ao)[VEC]) {
        const float mn = fmaxf(m, mo);
        const float c1 = (m == mn) ? 1.f : fast_exp2(m - mn);
        const float c2 = (mo == mn) ? 1.f : fast_exp2(mo - mn);
        l = l * c1 + lo * c2;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = acc[i] * c1 + ao[i] * c2;
        m = mn;
    }
    __device__ void combine_slots() {
#pragma unroll
        for (int o = G::LPE; o < 64; o <<= 1) {
            const float mo = __shfl_xor(m, o);
            const float lo = __shfl_xor(l, o);
            float ao[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) ao[i] = __shfl_xor(acc[i], o);
            merge(mo, lo, ao);
        }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) const {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, acc);
        if (c.head0) {
            a.part_s0[(size_t)item * a.H + c.h] = m;
            a.part_s1[(size_t)item * a.H + c.h] = l;
        }
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        P.s0 = a.part_s0[(size_t)chunk * a.H + c.h];
        P.s1 = a.part_s1[(size_t)chunk * a.H + c.h];
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
        float ao[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) ao[i] = w * P.v0[i];
        merge(valid ? P.s0 : -INFINITY, w * P.s1, ao);
    }
    // O = acc / l; statistics back in natural-log units
    __device__ void finalize(const Args& a, const Ctx& c) const {
        if (!c.writer || !c.active) return;
        const float inv = l > 0.f ? 1.f / l : 0.f;
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = acc[i] * inv;
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.o) + c.off, o);
        if (c.head0) {
            a.o_max[(size_t)c.node * a.stat_stride + c.h] = m * kLn2;
            a.o_sum[(size_t)c.node * a.stat_stride + c.h] = l;
        }
    }
};

// Drop-in for SoftmaxAcc that turns a forward pass into "write the attention weights": with the row
// statistics of a finished forward call, p_ij = exp(s_ij - max_i) / sum_i is stored for every edge at its
// CSR position (the normalised scores P of Eq. 1, which the fused layer itself never materialises).
// Nothing is accumulated, so there is nothing to combine, merge or finalise.
template <class G, int U> struct AttentionOut {
    static constexpr int VEC = G::VEC;
    float lse2;
    __device__ void init(const Args& a, const Ctx& c) {
        float mx = 0.f, sm = 1.f;
        if (c.active) {
            mx = a.row_max[(size_t)c.node * a.stat_stride + c.h];
            sm = a.row_sum[(size_t)c.node * a.stat_stride + c.h];
        }
        lse2 = mx * kLog2e + fast_log2(sm);
    }
    __device__ void absorb(const Args& a, const Ctx& c, const float (&s)[U], const u32x4 (&)[U], const int (&ep)[U],
                           const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (j[u] >= 0 && c.head0) a.p_out[(size_t)ep[u] * a.bias_stride + c.h] = fast_exp2(s[u] - lse2);
    }
    __device__ void combine_slots() {}
    __device__ void store_partial(const Args&, const Ctx&, int) const {}
    __device__ void load_partial(const Args&, const Ctx&, int, PartialRegs<VEC>&) const {}
    __device__ void fold_partial(const PartialRegs<VEC>&, bool) {}
    __device__ void finalize(const Args&, const Ctx&) const {}
};

// Row-side quantities every backward row pass starts from: lse2 = log2 of the softmax denominator
// including the maximum, and delta_i = sum_j p_ij dP_ij per head.
//   fp32 tensors: delta_i = dO_i . O_i (the same number, read off the forward output);
//   bf16 tensors: O was rounded to bf16, which would put a 2^-9 relative error into delta, so the
//   pass accumulates dsum = sum_j p_ij dP_ij itself and uses  sum_j p (dP - delta) y_j
//   = sum_j p dP y_j - delta sum_j p y_j  to finish in one sweep (kExact).
//   A row with a single edge has p = 1 and dS = 0 exactly, while its computed p is 1 only to rounding (the
//   statistics went through a logarithm).  kExact passes therefore finish such a row with delta = dP of its
//   edge (dp0, which the column pass recomputes bit for bit, so that its dS is exactly zero too) and write
//   zeros for every score-side gradient of the row (single_edge / exact_delta below).
template <class G> struct RowBackwardBase {
    static constexpr int VEC = G::VEC;
    static constexpr bool kExact = sizeof(typename G::T) == 2;
    float g[VEC];  // dO_i
    float delta, lse2, dsum;
    float dp0;     // kExact: dP of the first edge of this lane's slot in the latest round
    __device__ static bool single_edge(const Ctx& c) { return c.deg == 1; }
    __device__ float exact_delta(const Ctx& c) const { return single_edge(c) ? dp0 : dsum; }
    __device__ void init_row(const Args& a, const Ctx& c) {
        load_row<G>(a.d_out, c, g);
        dsum = 0.f;
        delta = 0.f;
        dp0 = 0.f;
        if constexpr (!kExact) {
            float o[VEC];
            load_row<G>(a.out, c, o);
            delta = head_sum<G::LPH>(dotv<VEC>(g, o), a.lph);
        }
        float mx = 0.f, sm = 1.f;
        if (c.active) {
            mx = a.row_max[(size_t)c.node * a.stat_stride + c.h];
            sm = a.row_sum[(size_t)c.node * a.stat_stride + c.h];
        }
        lse2 = mx * kLog2e + fast_log2(sm);
    }
};

// ---------------------------------------------------------------------------------------------
// helpers shared by the GAT-family passes
// ---------------------------------------------------------------------------------------------
__device__ inline float leaky(float z, float slope) { return z > 0.f ? z : slope * z; }

// this lane's slice of a [H, D] fp32 attention vector, times mul (zeros for lanes without features)
template <class G> __device__ inline void load_attention(const float* v, const Ctx& c, float mul, float (&out)[G::VEC]) {
#pragma unroll
    for (int i = 0; i < G::VEC; ++i) out[i] = 0.f;
    if (c.active) {
        load_f32<G::VEC>(v + c.f0, out);
#pragma unroll
        for (int i = 0; i < G::VEC; ++i) out[i] *= mul;
    }
}

// =============================================================================================
// kernels
// =============================================================================================
constexpr int kWavesPerBlock = 4;

// neighbour ids of one load round and the CSR position of their edges: the list position itself for a
// row pass, the stored CSR position of the CSC entry for a column pass that needs it (a.eid set)
template <class G, int U>
__device__ inline void load_indices(const Args& a, const Ctx& c, int base, int ee, int (&j)[U], int (&ep)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int e = base + u * G::EPW + c.g;
        j[u] = e < ee ? a.idx[e] : -1;
        if constexpr (G::kEdgeTerm) ep[u] = (a.eid != nullptr && e < ee) ? a.eid[e] : e;
        else ep[u] = e;
    }
}

// A whole wavefront on one work item.  PARTIAL: the item is a chunk of a super row and its result goes
// to the workspace; otherwise the item is a whole row and the wavefront finishes it.
template <class G, template <class, int> class PassT, int U, bool PARTIAL>
__device__ inline void wave_item(const Args& a, int item, int lane) {
    int node, eb, ee;
    if (PARTIAL) {
        node = a.chunks[3 * item];
        eb = a.chunks[3 * item + 1];
        ee = a.chunks[3 * item + 2];
    } else {
        node = a.order[a.first_direct + item];
        eb = a.ptr[node];
        ee = a.ptr[node + 1];
    }
    // the whole wavefront works on one item: keep its bounds in scalar registers
    node = __builtin_amdgcn_readfirstlane(node);
    eb = __builtin_amdgcn_readfirstlane(eb);
    ee = __builtin_amdgcn_readfirstlane(ee);
    Ctx c = make_ctx<G>(a, lane, node);
    if (!PARTIAL) c.deg = ee - eb;
    PassT<G, U> p;
    p.init(a, c);
    constexpr int STEP = G::EPW * U;
    int j[U], jn[U], ep[U], epn[U];
    load_indices<G, U>(a, c, eb, ee, j, ep);
    for (int base = eb; base < ee; base += STEP) {
#pragma unroll
        for (int u = 0; u < U; ++u) p.issue(a, c, u, j[u], ep[u]);
        load_indices<G, U>(a, c, base + STEP, ee, jn, epn);
        if (base + STEP <= ee) p.template consume<true>(a, c, j);
        else p.template consume<false>(a, c, j);
#pragma unroll
        for (int u = 0; u < U; ++u) { j[u] = jn[u]; ep[u] = epn[u]; }
    }
    p.combine_slots(a, c);
    if (PARTIAL) p.store_partial(a, c, item);
    else p.finalize(a, c);
}

// Rows shorter than one load round of a whole wavefront: every edge slot (LPE lanes) owns a row of
// its own, so a wavefront finishes 64/LPE rows at once and nothing has to be merged across slots.
// Rows come from the degree-ordered list, so the slots of a wavefront have similar trip counts.
template <class G, template <class, int> class PassT, int U>
__device__ inline void wave_small_rows(const Args& a, int item, int lane) {
    const int r = item * G::EPW + lane / G::LPE;
    const bool live = r < a.n_small;
    const int node = a.order[a.first_small + (live ? r : 0)];
    const int eb = live ? a.ptr[node] : 0;
    const int ee = live ? a.ptr[node + 1] : 0;
    Ctx c = make_ctx<G>(a, lane, node);
    c.writer = live;
    c.deg = ee - eb;
    PassT<G, U> p;
    p.init(a, c);
    int j[U], jn[U], ep[U], epn[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        j[u] = eb + u < ee ? a.idx[eb + u] : -1;
        if constexpr (G::kEdgeTerm) ep[u] = (a.eid != nullptr && eb + u < ee) ? a.eid[eb + u] : eb + u;
        else ep[u] = eb + u;
    }
    for (int pos = eb; __any(pos < ee); pos += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) p.issue(a, c, u, j[u], ep[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = pos + U + u;
            jn[u] = e < ee ? a.idx[e] : -1;
            if constexpr (G::kEdgeTerm) epn[u] = (a.eid != nullptr && e < ee) ? a.eid[e] : e;
            else epn[u] = e;
        }
        if (__all(pos + U <= ee)) p.template consume<true>(a, c, j);
        else p.template consume<false>(a, c, j);
#pragma unroll
        for (int u = 0; u < U; ++u) { j[u] = jn[u]; ep[u] = epn[u]; }
    }
    p.finalize(a, c);
}

// One launch per pass.  Workgroups are handed out in the order of their work: first the chunks of
// super rows (edge-parallel split), then whole rows by descending degree class (node-parallel, one
// wavefront each), then the short rows, one per edge slot.  Each of the 4 wavefronts of a workgroup
// works alone; the kind of work depends only on blockIdx, so a wavefront never diverges on it.
template <class G, template <class, int> class PassT, int U>
__device__ inline void pass_block(const Args& a, int b, int grid) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wpb = (int)blockDim.x >> 6;  // wavefronts per workgroup (the host picks 1, 2 or 4)
    // The hardware deals workgroups to the 8 XCDs round-robin.  For graphs whose numbering is local the
    // work list is cut into runs of xcd_group workgroups and run r of every 8 goes to XCD r, so that rows
    // which are neighbours in the list (and share neighbour rows) meet in one L2, while all XCDs still
    // advance through the degree-ordered list at the same pace.
    if (a.xcd_group > 0) {
        const int sh = __builtin_ctz(a.xcd_group) + 3;  // the run length is a power of two
        if (b < (int)((grid >> sh) << sh)) {
            const int r = b & ((1 << sh) - 1);
            b = (b - r) + (r & 7) * a.xcd_group + (r >> 3);
        }
    }
    if (b < a.blocks_chunk) {
        const int item = b * wpb + wave;
        if (item < a.n_chunks) wave_item<G, PassT, U, true>(a, item, lane);
        return;
    }
    b -= a.blocks_chunk;
    if (b < a.blocks_direct) {
        const int item = b * wpb + wave;
        if (item < a.n_direct) wave_item<G, PassT, U, false>(a, item, lane);
        return;
    }
    b -= a.blocks_direct;
    if constexpr (G::EPW > 1) {
        const int item = b * wpb + wave;
        if (item * G::EPW < a.n_small) wave_small_rows<G, PassT, U>(a, item, lane);
    }
}

template <class G, template <class, int> class PassT, int U>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_pass(const Args a) {
    pass_block<G, PassT, U>(a, (int)blockIdx.x, (int)gridDim.x);
}

// Two passes that do not depend on each other in one launch (the row side and the column side of the
// backward pass of a small graph, where a launch costs as much as the work it starts): the first blocks_a
// workgroups run pass A over its work list, the others pass B over its own.
template <class G, template <class, int> class PassA, template <class, int> class PassB, int U>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_pass_pair(const Args a, const Args b, int blocks_a) {
    if ((int)blockIdx.x < blocks_a) pass_block<G, PassA, U>(a, (int)blockIdx.x, blocks_a);
    else pass_block<G, PassB, U>(b, (int)blockIdx.x - blocks_a, (int)gridDim.x - blocks_a);
}

// chunks a merge wavefront loads per edge slot before folding them in (a pass may ask for fewer)
template <class P, class = void> struct merge_batch { static constexpr int value = 8; };
template <class P> struct merge_batch<P, std::void_t<decltype(P::kMergeBatch)>> { static constexpr int value = P::kMergeBatch; };

// A super row with very many chunks (a hub with 10^5 neighbours) is merged in two levels, so that its merge
// is not one wavefront's work: the row's chunks are cut into at most merge_groups groups of equal size, one
// wavefront per group folds the group's partials into the slot of the group's first chunk (k_merge_groups),
// and the final merge reads one partial per group.  Both kernels derive the grouping from the row's chunk count
// alone, so the summation order is fixed.
constexpr int kMergeGroupChunks = 32;  // a group is worth a wavefront from this many chunks on
__device__ inline int merge_groups_of(int chunks, int max_groups) {
    const int want = (chunks + kMergeGroupChunks - 1) / kMergeGroupChunks;
    return want < max_groups ? (want < 1 ? 1 : want) : max_groups;
}

// the partials [cb, ce) with stride `step` folded into p (kMergeBatch per edge slot are loaded before any is
// folded in; absent ones read the first and are masked, so the loop has no per-lane branch and its loads overlap)
template <class G, class P> __device__ inline void fold_range(const Args& a, const Ctx& c, P& p, int cb, int ce, int step) {
    constexpr int kMergeBatch = merge_batch<P>::value;
    for (int base = cb; base < ce; base += G::EPW * kMergeBatch * step) {
        PartialRegs<G::VEC> R[kMergeBatch];
#pragma unroll
        for (int m = 0; m < kMergeBatch; ++m) {
            const int ch = base + (m * G::EPW + c.g) * step;
            p.load_partial(a, c, ch < ce ? ch : cb, R[m]);
        }
#pragma unroll
        for (int m = 0; m < kMergeBatch; ++m) p.fold_partial(R[m], base + (m * G::EPW + c.g) * step < ce);
    }
}

// first level: wavefront (s, g) folds group g of super row s into the partial slot of the group's first chunk
template <class G, template <class, int> class PassT, int U>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_merge_groups(const Args a) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int w = blockIdx.x * kWavesPerBlock + wave;
    const int s = w / a.merge_groups, g = w - s * a.merge_groups;
    if (s >= a.n_items) return;
    const int node = __builtin_amdgcn_readfirstlane(a.order[s]);
    const int c0 = __builtin_amdgcn_readfirstlane(a.chunk_ptr[s]);
    const int c1 = __builtin_amdgcn_readfirstlane(a.chunk_ptr[s + 1]);
    const int ng = merge_groups_of(c1 - c0, a.merge_groups);
    if (ng <= 1 || g >= ng) return;  // a row with one group is merged by the final kernel alone
    const int gs = (c1 - c0 + ng - 1) / ng;
    const int cb = c0 + g * gs, ce = min(c1, cb + gs);
    if (cb >= ce) return;
    const Ctx c = make_ctx<G>(a, lane, node);
    PassT<G, U> p;
    p.init(a, c);
    fold_range<G>(a, c, p, cb, ce, 1);
    p.combine_slots(a, c);
    p.store_partial(a, c, cb);
}

// One wavefront per super row / column: the edge slots take the row's chunks (or the partials of its chunk
// groups) round-robin and sum (or, for the forward pass, softmax-merge) their partial results, the slots are
// combined as in the direct pass, and the row is finished exactly as the direct pass would.  Summation order
// is fixed.
template <class G, template <class, int> class PassT, int U>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_merge(const Args a) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int s = blockIdx.x * kWavesPerBlock + wave;
    if (s >= a.n_items) return;
    const int node = __builtin_amdgcn_readfirstlane(a.order[s]);
    const int c0 = __builtin_amdgcn_readfirstlane(a.chunk_ptr[s]);
    const int c1 = __builtin_amdgcn_readfirstlane(a.chunk_ptr[s + 1]);
    const Ctx c = make_ctx<G>(a, lane, node);
    PassT<G, U> p;
    p.init(a, c);
    const int ng = merge_groups_of(c1 - c0, a.merge_groups);
    const int step = ng <= 1 ? 1 : (c1 - c0 + ng - 1) / ng;  // one partial per group, at the group's first chunk
    fold_range<G>(a, c, p, c0, c1, step);
    p.combine_slots(a, c);
    p.finalize(a, c);
}

// Edge-parallel SDDMM of the two-kernel comparator: the CSR positions are dealt out evenly, EPW * U per
// round and kScoreRounds rounds per wavefront, whatever rows they belong to; each edge slot gathers
// q of its edge's row (COO row array) and k of its neighbour and stores the scaled score of every head.
constexpr int kScoreRounds = 4;
template <class G, int U>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_edge_scores(const Args a) {
    const int wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    const Ctx c = make_ctx<G>(a, lane, 0);
    constexpr int STEP = G::EPW * U;
    const int64_t first = (int64_t)wave * STEP * kScoreRounds;
    for (int r = 0; r < kScoreRounds; ++r) {
        const int64_t base = first + (int64_t)r * STEP;
        if (base >= a.n_edges) return;
        int i[U], j[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + u * G::EPW + c.g;
            const bool live = e < a.n_edges;
            i[u] = live ? a.edge_row[e] : -1;
            j[u] = live ? a.idx[e] : -1;
        }
        u32x4 Q[U], K[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            Q[u] = gather_raw<G>(a.x, a, c, i[u]);
            K[u] = gather_raw<G>(a.k, a, c, j[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float qf[G::VEC], kf[G::VEC];
            Elem<typename G::T>::unpack(Q[u], qf);
            Elem<typename G::T>::unpack(K[u], kf);
            const int64_t e = base + u * G::EPW + c.g;
            const float s = with_bias<G>(head_sum<G::LPH>(dotv<G::VEC>(qf, kf), a.lph) * a.c_score, load_bias<G>(a, c, j[u], (int)e));
            if (c.head0 && j[u] >= 0) a.scores[(size_t)e * a.H + c.h] = s;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// small deterministic reductions (two stages, fixed summation order).  The parameter gradients are signed
// sums over all nodes and edges whose terms largely cancel, so both stages add in double precision: the
// result then carries the rounding of its fp32 terms only, not of the summation.
// ---------------------------------------------------------------------------------------------
constexpr int kReduceBlocks = 256;
constexpr int kReduceWaves = 16;  // wavefronts per workgroup of the first stage over node rows

template <int LPE> __device__ inline double slot_sum_f64(double x) {
#pragma unroll
    for (int o = LPE; o < 64; o <<= 1) x += __shfl_xor(x, o);
    return x;
}

// stage 1 of da_l[h,d] = sum_v d_el[v,h] Wh[v,h,d] and da_r likewise.  Same lane geometry as the passes:
// an edge slot reads one node row per step; wave w of the grid takes node groups w, w + W, ...;
// one partial per workgroup.  Workgroups of 16 wavefronts: the 256 partials of the second stage then come
// from 4,096 wavefronts, enough loads in flight to stream the node tensor at memory speed.
template <class G>
__global__ __launch_bounds__(64 * kReduceWaves) void k_gat_param_partial(const Args a, double* __restrict__ partial) {
    __shared__ double red[kReduceWaves][2][G::LPE * G::VEC];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int waves = gridDim.x * kReduceWaves;
    double sl[G::VEC], sr[G::VEC];
#pragma unroll
    for (int i = 0; i < G::VEC; ++i) { sl[i] = 0.0; sr[i] = 0.0; }
    constexpr int B = 4;  // node rows requested per edge slot before the first is used
    const int stride = waves * G::EPW;
    for (int base = (blockIdx.x * kReduceWaves + wave) * G::EPW; base < a.n_nodes; base += stride * B) {
        float x[B][G::VEC], del[B], der[B];
#pragma unroll
        for (int k = 0; k < B; ++k) {
            const int v = base + k * stride + lane / G::LPE;
            const bool live = v < a.n_nodes;
            const Ctx c = make_ctx<G>(a, lane, live ? v : 0);
            load_row<G>(a.x, c, x[k]);
            del[k] = live ? a.d_el[(size_t)c.node * a.H + c.h] : 0.f;
            der[k] = live ? a.d_er[(size_t)c.node * a.H + c.h] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < B; ++k) {
#pragma unroll
            for (int i = 0; i < G::VEC; ++i) {
                sl[i] = fma((double)del[k], (double)x[k][i], sl[i]);
                sr[i] = fma((double)der[k], (double)x[k][i], sr[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < G::VEC; ++i) { sl[i] = slot_sum_f64<G::LPE>(sl[i]); sr[i] = slot_sum_f64<G::LPE>(sr[i]); }
    const int f0 = (lane % G::LPE) * G::VEC;
    if (lane < G::LPE) {
#pragma unroll
        for (int i = 0; i < G::VEC; ++i) { red[wave][0][f0 + i] = sl[i]; red[wave][1][f0 + i] = sr[i]; }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * a.HD; t += blockDim.x) {
        const int which = t / a.HD, f = t % a.HD;
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < kReduceWaves; ++w) sum += red[w][which][f];
        partial[((size_t)blockIdx.x * 2 + which) * a.HD + f] = sum;
    }
}

// second stage: 1024 threads; thread t owns column t % wf of the 2 * HD columns (a_l | a_r) and every
// (1024 / wf)-th partial row, the groups are then added in order through LDS (wf = a power of two >= 2 * HD)
[[maybe_unused]] static __global__ __launch_bounds__(1024) void k_gat_param_final(const double* __restrict__ partial, int nblocks, int HD,
                                                          int wf, float* __restrict__ d_a_l, float* __restrict__ d_a_r) {
    __shared__ double red[1024];
    const int groups = 1024 / wf, bs = threadIdx.x / wf, t = threadIdx.x % wf;
    double sum = 0.0;
    if (t < 2 * HD) {
        for (int b = bs; b < nblocks; b += 16 * groups) {
            double v[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = b + k * groups < nblocks ? partial[(size_t)(b + k * groups) * 2 * HD + t] : 0.0;
#pragma unroll
            for (int k = 0; k < 16; ++k) sum += v[k];
        }
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    if (bs == 0 && t < 2 * HD) {
        double total = 0.0;
        for (int k = 0; k < groups; ++k) total += red[k * wf + t];
        (t < HD ? d_a_l : d_a_r)[t < HD ? t : t - HD] = (float)total;
    }
}

__device__ inline double block_sum_256(double v) {
    __shared__ double red[256];
    red[threadIdx.x] = v;
    __syncthreads();
#pragma unroll
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
}

[[maybe_unused]] static __global__ __launch_bounds__(256) void k_sum_partial(const float* __restrict__ in, int64_t n, double* __restrict__ partial) {
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) s += (double)in[i];
    const double t = block_sum_256(s);
    if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

// `carry` (one double, device) holds the running total in double across the head groups of a wide layer:
// the first group writes it, the others add to it; *out always receives the fp32 rounding of the total
[[maybe_unused]] static __global__ __launch_bounds__(256) void k_sum_final(const double* __restrict__ partial, int n, bool add,
                                                   double* __restrict__ carry, float* __restrict__ out) {
    const double t = block_sum_256((int)threadIdx.x < n ? partial[threadIdx.x] : 0.0);
    if (threadIdx.x == 0) {
        const double total = add ? *carry + t : t;
        *carry = total;
        *out = (float)total;
    }
}

// Column sums of a row-major [n, hd] fp32 array (hd a multiple of 4) in two stages with a fixed summation
// order: thread t of a workgroup owns the 4 columns 4 * (t % w) .. +3 and every (256 / w)-th row of the
// workgroup's rows, four rows in flight at a time.
typedef double f64x4 __attribute__((ext_vector_type(4)));
__device__ inline f64x4 widen(const f32x4& v) { return f64x4{(double)v[0], (double)v[1], (double)v[2], (double)v[3]}; }
constexpr int kRowsumBlocks = 1024;
[[maybe_unused]] static __global__ __launch_bounds__(256) void k_rowsum_partial(const float* __restrict__ in, int64_t n, int hd, int w,
                                                        double* __restrict__ partial) {
    __shared__ f64x4 red[256];
    const int rows_par = 256 / w, rs = threadIdx.x / w, fc = threadIdx.x % w;
    const int64_t stride = (int64_t)gridDim.x * rows_par;
    for (int f0 = 0; f0 < hd; f0 += 4 * w) {
        const int f = f0 + 4 * fc;
        f64x4 acc = {0.0, 0.0, 0.0, 0.0};
        if (f < hd) {
            int64_t r = (int64_t)blockIdx.x * rows_par + rs;
            for (; r + 3 * stride < n; r += 4 * stride) {
                f32x4 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const f32x4*>(in + (r + k * stride) * hd + f);
#pragma unroll
                for (int k = 0; k < 4; ++k) acc += widen(v[k]);
            }
            for (; r < n; r += stride) acc += widen(*reinterpret_cast<const f32x4*>(in + r * hd + f));
        }
        red[threadIdx.x] = acc;
        __syncthreads();
        if (rs == 0 && f < hd) {
            f64x4 t = {0.0, 0.0, 0.0, 0.0};
            for (int k = 0; k < rows_par; ++k) t += red[k * w + fc];
            *reinterpret_cast<f64x4*>(partial + (size_t)blockIdx.x * hd + f) = t;
        }
        __syncthreads();
    }
}

// second stage: thread t owns column t % wf and every (256 / wf)-th partial row; fixed order
[[maybe_unused]] static __global__ __launch_bounds__(256) void k_rowsum_final(const double* __restrict__ partial, int nblocks, int hd,
                                                      int wf, float* __restrict__ out) {
    __shared__ double red[256];
    const int groups = 256 / wf, bs = threadIdx.x / wf, fc = threadIdx.x % wf;
    for (int f0 = 0; f0 < hd; f0 += wf) {
        const int f = f0 + fc;
        double sum = 0.0;
        if (f < hd) {
            for (int b = bs; b < nblocks; b += 16 * groups) {
                double v[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) v[k] = b + k * groups < nblocks ? partial[(size_t)(b + k * groups) * hd + f] : 0.0;
#pragma unroll
                for (int k = 0; k < 16; ++k) sum += v[k];
            }
        }
        red[threadIdx.x] = sum;
        __syncthreads();
        if (bs == 0 && f < hd) {
            double t = 0.0;
            for (int k = 0; k < groups; ++k) t += red[k * wf + fc];
            out[f] = (float)t;
        }
        __syncthreads();
    }
}

}  // namespace dfgnn
