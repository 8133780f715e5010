// Passes of the GAT layer.
#pragma once
#include "layer_device.hpp"

namespace dfgnn {

// =============================================================================================
// GAT (add-SDDMM, Sec. 5.1): s_ij = LeakyReLU(el_i + er_j); el, er are per-node scalars per head
// =============================================================================================
template <class G, int U, class Acc> struct GatFwdT {
    static constexpr int VEC = G::VEC;
    float el2, ar2[VEC];  // el_i * log2e; this lane's slice of a_r * log2e
    float B[U];
    Acc sm;  // SoftmaxAcc: the layer itself; AttentionOut: write the attention weights instead
    int Ep[U];
    u32x4 V[U];
    // el_i comes from the row's own features and er_j from the gathered neighbour row (one dot product
    // over the head's lanes), so no per-node scalar has to be gathered from memory
    __device__ void init(const Args& a, const Ctx& c) {
        float x[VEC], al[VEC];
        load_row<G>(a.x, c, x);
        load_attention<G>(a.a_l, c, kLog2e, al);
        load_attention<G>(a.a_r, c, kLog2e, ar2);
        el2 = head_sum<G::LPH>(dotv<VEC>(x, al), a.lph);
        sm.init(a, c);
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        V[u] = gather_raw<G>(a.x, a, c, j);
        B[u] = load_bias<G>(a, c, j, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[VEC];
            Elem<typename G::T>::unpack(V[u], vf);
            s[u] = with_bias<G>(leaky(el2 + head_sum<G::LPH>(dotv<VEC>(vf, ar2), a.lph), a.neg_slope), B[u]);
            if (!FULL && j[u] < 0) s[u] = -INFINITY;
        }
        if (!FULL && j[0] < 0) return;
        sm.absorb(a, c, s, V, Ep, j);
    }
    __device__ void combine_slots(const Args&, const Ctx&) { sm.combine_slots(); }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) { sm.store_partial(a, c, item); }
    __device__ void load_partial(const Args& a, const Ctx& c, int chunk, PartialRegs<VEC>& P) const { sm.load_partial(a, c, chunk, P); }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) { sm.fold_partial(P, valid); }
    __device__ void finalize(const Args& a, const Ctx& c) { sm.finalize(a, c); }
};
template <class G, int U> using GatFwd = GatFwdT<G, U, SoftmaxAcc<G, U>>;
template <class G, int U> using GatAttention = GatFwdT<G, U, AttentionOut<G, U>>;


// d_el_i = sum_j dS_ij LeakyReLU'(z_ij)
template <class G, int U> struct GatBwdRow : RowBackwardBase<G> {
    static constexpr int VEC = G::VEC;
    static constexpr bool kExact = RowBackwardBase<G>::kExact;
    float el2, ar2[VEC], d_el, pl;  // pl = sum_j p LeakyReLU'(z) (kExact only)
    float B[U];
    int Ep[U];
    u32x4 V[U];
    __device__ void init(const Args& a, const Ctx& c) {
        float x[VEC], al[VEC];
        load_row<G>(a.x, c, x);
        load_attention<G>(a.a_l, c, kLog2e, al);
        load_attention<G>(a.a_r, c, kLog2e, ar2);
        el2 = head_sum<G::LPH>(dotv<VEC>(x, al), a.lph);
        d_el = 0.f;
        pl = 0.f;
        this->init_row(a, c);
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        V[u] = gather_raw<G>(a.x, a, c, j);
        B[u] = load_bias<G>(a, c, j, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[VEC];
            Elem<typename G::T>::unpack(V[u], vf);
            const float dp = head_sum<G::LPH>(dotv<VEC>(this->g, vf), a.lph);
            const float z = el2 + head_sum<G::LPH>(dotv<VEC>(vf, ar2), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(with_bias<G>(leaky(z, a.neg_slope), B[u]) - this->lse2) : 0.f;
            const float slope = z > 0.f ? 1.f : a.neg_slope;
            if constexpr (kExact) {
                const float t = p * dp;
                if (u == 0 && (FULL || j[0] >= 0)) this->dp0 = dp;  // (a slot that has run out of edges keeps its value)
                this->dsum += t;
                d_el = fmaf(t, slope, d_el);
                pl = fmaf(p, slope, pl);
            } else {
                const float ds = p * (dp - this->delta);
                store_dbias<G, true>(a, c, FULL || j[u] >= 0, Ep[u], ds);
                d_el = fmaf(ds, slope, d_el);
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
        d_el = slot_sum<G::LPE>(d_el);
        if constexpr (kExact) {
            pl = slot_sum<G::LPE>(pl);
            this->dsum = slot_sum<G::LPE>(this->dsum);
        }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.head0) return;
        a.part_s0[(size_t)item * a.H + c.h] = d_el;
        if constexpr (kExact) {
            a.part_s1[(size_t)item * a.H + c.h] = pl;
            a.part_s2[(size_t)item * a.H + c.h] = this->dsum;
        }
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        P.s0 = a.part_s0[(size_t)chunk * a.H + c.h];
        if constexpr (kExact) {
            P.s1 = a.part_s1[(size_t)chunk * a.H + c.h];
            P.s2 = a.part_s2[(size_t)chunk * a.H + c.h];
        }
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
        d_el = fmaf(w, P.s0, d_el);
        if constexpr (kExact) {
            pl = fmaf(w, P.s1, pl);
            this->dsum = fmaf(w, P.s2, this->dsum);
        }
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.head0) return;
        if constexpr (kExact) {
            this->delta = this->exact_delta(c);
            d_el = this->single_edge(c) ? 0.f : d_el - this->delta * pl;
        }
        const size_t nh = (size_t)c.node * a.H + c.h;
        a.d_el[nh] = d_el;
        f32x4 st = {el2, this->lse2, this->delta, 0.f};
        *reinterpret_cast<f32x4*>(a.stats + 4 * nh) = st;
    }
};

// dWh_j = sum_i p_ij dO_i + d_el_j a_l + d_er_j a_r ;  d_er_j = sum_i dS_ij LeakyReLU'(z_ij)
template <class G, int U> struct GatBwdCol {
    static constexpr int VEC = G::VEC;
    float wh[VEC], dwh[VEC];
    float er2, d_er;
    float B[U];
    int Ep[U];
    u32x4 Gd[U];
    f32x4 St[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, wh);
        float ar[VEC];
        load_attention<G>(a.a_r, c, kLog2e, ar);
        er2 = head_sum<G::LPH>(dotv<VEC>(wh, ar), a.lph);
        d_er = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) dwh[i] = 0.f;
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int i, int e) {
        Gd[u] = gather_raw<G>(a.d_out, a, c, i);
        St[u] = gather_stats4(a, c, i);
        B[u] = load_bias<G>(a, c, i, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float gf[VEC];
            Elem<typename G::T>::unpack(Gd[u], gf);
            const float dp = head_sum<G::LPH>(dotv<VEC>(gf, wh), a.lph);
            const float z = St[u][0] + er2;
            const float p = (FULL || j[u] >= 0) ? fast_exp2(with_bias<G>(leaky(z, a.neg_slope), B[u]) - St[u][1]) : 0.f;
            const float ds = p * (dp - St[u][2]);
            store_dbias<G, false>(a, c, FULL || j[u] >= 0, Ep[u], ds);
            d_er += ds * (z > 0.f ? 1.f : a.neg_slope);
#pragma unroll
            for (int i = 0; i < VEC; ++i) dwh[i] = fmaf(p, gf[i], dwh[i]);
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
        d_er = slot_sum<G::LPE>(d_er);
#pragma unroll
        for (int i = 0; i < VEC; ++i) dwh[i] = slot_sum<G::LPE>(dwh[i]);
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, dwh);
        if (c.head0) a.part_s0[(size_t)item * a.H + c.h] = d_er;
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        P.s0 = a.part_s0[(size_t)chunk * a.H + c.h];
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) dwh[i] = fmaf(w, P.v0[i], dwh[i]);
        d_er = fmaf(w, P.s0, d_er);
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        const size_t nh = (size_t)c.node * a.H + c.h;
        const float del = a.d_el[nh];
        float al[VEC], ar[VEC], o[VEC];
        load_f32<VEC>(a.a_l + c.f0, al);
        load_f32<VEC>(a.a_r + c.f0, ar);
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = dwh[i] + del * al[i] + d_er * ar[i];
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_x) + c.off, o);
        if (c.head0) a.d_er[nh] = d_er;
    }
};

}  // namespace dfgnn
