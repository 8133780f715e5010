// Passes of the GATv2 layer.
#pragma once
#include "layer_device.hpp"

namespace dfgnn {

// =============================================================================================
// GATv2 (the second member of the GAT family cited in Sec. 1): s_ij = sum_d a_d LeakyReLU(x_i,d + k_j,d),
// x = destination-side and k = source-side projection; the aggregated value is k_j.  The score is not a
// sum of two per-node scalars, so every edge costs a D-wide elementwise pass over the gathered row; the
// memory traffic is that of GAT (one neighbour row per edge).
// =============================================================================================
template <class G, int U, class Acc> struct GatV2FwdT {
    static constexpr int VEC = G::VEC;
    float x[VEC], al2[VEC];  // destination features; this lane's slice of a * log2e
    float B[U];
    Acc sm;  // SoftmaxAcc: the layer itself; AttentionOut: write the attention weights instead
    int Ep[U];
    u32x4 K[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, x);
        load_attention<G>(a.a_l, c, kLog2e, al2);
        sm.init(a, c);
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        K[u] = gather_raw<G>(a.k, a, c, j);
        B[u] = load_bias<G>(a, c, j, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[VEC], t = 0.f;
            Elem<typename G::T>::unpack(K[u], kf);
#pragma unroll
            for (int i = 0; i < VEC; ++i) t = fmaf(al2[i], leaky(x[i] + kf[i], a.neg_slope), t);
            s[u] = with_bias<G>(head_sum<G::LPH>(t, a.lph), B[u]);
            if (!FULL && j[u] < 0) s[u] = -INFINITY;
        }
        if (!FULL && j[0] < 0) return;
        sm.absorb(a, c, s, K, Ep, j);
    }
    __device__ void combine_slots(const Args&, const Ctx&) { sm.combine_slots(); }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) { sm.store_partial(a, c, item); }
    __device__ void load_partial(const Args& a, const Ctx& c, int chunk, PartialRegs<VEC>& P) const { sm.load_partial(a, c, chunk, P); }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) { sm.fold_partial(P, valid); }
    __device__ void finalize(const Args& a, const Ctx& c) { sm.finalize(a, c); }
};
template <class G, int U> using GatV2Fwd = GatV2FwdT<G, U, SoftmaxAcc<G, U>>;
template <class G, int U> using GatV2Attention = GatV2FwdT<G, U, AttentionOut<G, U>>;


// Row side: with z_d = x_i,d + k_j,d,  dX_i,d = a_d sum_j dS_ij LeakyReLU'(z_d)  and the row's share of
// da_d = sum_ij dS_ij LeakyReLU(z_d)  (summed over rows afterwards).  The factor a_d is applied once at the end.
template <class G, int U> struct GatV2BwdRow : RowBackwardBase<G> {
    static constexpr int VEC = G::VEC;
    static constexpr bool kExact = RowBackwardBase<G>::kExact;
    static constexpr int kMergeBatch = kExact ? 2 : 4;  // four partial vectors per chunk: keep the merge in registers
    float x[VEC], al2[VEC], dx[VEC], da[VEC];
    float px[VEC], pa[VEC];  // sum_j p LeakyReLU'(z), sum_j p LeakyReLU(z)  (kExact only)
    float B[U];
    int Ep[U];
    u32x4 K[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, x);
        load_attention<G>(a.a_l, c, kLog2e, al2);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dx[i] = 0.f; da[i] = 0.f; px[i] = 0.f; pa[i] = 0.f; }
        this->init_row(a, c);
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        K[u] = gather_raw<G>(a.k, a, c, j);
        B[u] = load_bias<G>(a, c, j, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[VEC], lr[VEC], sl[VEC], t = 0.f;
            Elem<typename G::T>::unpack(K[u], kf);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float z = x[i] + kf[i];
                sl[i] = z > 0.f ? 1.f : a.neg_slope;
                lr[i] = z * sl[i];
                t = fmaf(al2[i], lr[i], t);
            }
            const float s = with_bias<G>(head_sum<G::LPH>(t, a.lph), B[u]);
            const float dp = head_sum<G::LPH>(dotv<VEC>(this->g, kf), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(s - this->lse2) : 0.f;
            if constexpr (kExact) {
                const float w = p * dp;
                if (u == 0 && (FULL || j[0] >= 0)) this->dp0 = dp;  // (a slot that has run out of edges keeps its value)
                this->dsum += w;
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    dx[i] = fmaf(w, sl[i], dx[i]); da[i] = fmaf(w, lr[i], da[i]);
                    px[i] = fmaf(p, sl[i], px[i]); pa[i] = fmaf(p, lr[i], pa[i]);
                }
            } else {
                const float ds = p * (dp - this->delta);
                store_dbias<G, true>(a, c, FULL || j[u] >= 0, Ep[u], ds);
#pragma unroll
                for (int i = 0; i < VEC; ++i) { dx[i] = fmaf(ds, sl[i], dx[i]); da[i] = fmaf(ds, lr[i], da[i]); }
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dx[i] = slot_sum<G::LPE>(dx[i]); da[i] = slot_sum<G::LPE>(da[i]); }
        if constexpr (kExact) {
            this->dsum = slot_sum<G::LPE>(this->dsum);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { px[i] = slot_sum<G::LPE>(px[i]); pa[i] = slot_sum<G::LPE>(pa[i]); }
        }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        const size_t o = (size_t)item * a.HD + c.f0;
        store_f32<VEC>(a.part_v0 + o, dx);
        store_f32<VEC>(a.part_v1 + o, da);
        if constexpr (kExact) {
            store_f32<VEC>(a.part_v2 + o, px);
            store_f32<VEC>(a.part_v3 + o, pa);
            if (c.head0) a.part_s2[(size_t)item * a.H + c.h] = this->dsum;
        }
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        const size_t o = (size_t)chunk * a.HD + c.f0;
        load_f32<VEC>(a.part_v0 + o, P.v0);
        load_f32<VEC>(a.part_v1 + o, P.v1);
        if constexpr (kExact) {
            load_f32<VEC>(a.part_v2 + o, P.v2);
            load_f32<VEC>(a.part_v3 + o, P.v3);
            P.s2 = a.part_s2[(size_t)chunk * a.H + c.h];
        }
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dx[i] = fmaf(w, P.v0[i], dx[i]); da[i] = fmaf(w, P.v1[i], da[i]); }
        if constexpr (kExact) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) { px[i] = fmaf(w, P.v2[i], px[i]); pa[i] = fmaf(w, P.v3[i], pa[i]); }
            this->dsum = fmaf(w, P.s2, this->dsum);
        }
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        if constexpr (kExact) {
            this->delta = this->exact_delta(c);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                dx[i] = this->single_edge(c) ? 0.f : dx[i] - this->delta * px[i];
                da[i] = this->single_edge(c) ? 0.f : da[i] - this->delta * pa[i];
            }
        }
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = al2[i] * kLn2 * dx[i];
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_x) + c.off, o);
        store_f32<VEC>(a.da_row + c.woff, da);
        if (c.head0) {
            f32x2 st = {this->lse2, this->delta};
            *reinterpret_cast<f32x2*>(a.stats + 2 * ((size_t)c.node * a.H + c.h)) = st;
        }
    }
};

// Column side: dK_j = sum_i p_ij dO_i + a (.) sum_i dS_ij LeakyReLU'(z_ij), p and dS recomputed per edge
template <class G, int U> struct GatV2BwdCol {
    static constexpr int VEC = G::VEC;
    float kk[VEC], al2[VEC], dk[VEC], dz[VEC];
    float B[U];
    int Ep[U];
    u32x4 X[U], Gd[U];
    f32x2 St[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.k, c, kk);
        load_attention<G>(a.a_l, c, kLog2e, al2);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dk[i] = 0.f; dz[i] = 0.f; }
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int i, int e) {
        X[u] = gather_raw<G>(a.x, a, c, i);
        Gd[u] = gather_raw<G>(a.d_out, a, c, i);
        St[u] = gather_stats2(a, c, i);
        B[u] = load_bias<G>(a, c, i, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float xf[VEC], gf[VEC], sl[VEC], t = 0.f;
            Elem<typename G::T>::unpack(X[u], xf);
            Elem<typename G::T>::unpack(Gd[u], gf);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float z = xf[i] + kk[i];
                sl[i] = z > 0.f ? 1.f : a.neg_slope;
                t = fmaf(al2[i], z * sl[i], t);
            }
            const float s = with_bias<G>(head_sum<G::LPH>(t, a.lph), B[u]);
            const float dp = head_sum<G::LPH>(dotv<VEC>(gf, kk), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(s - St[u][0]) : 0.f;
            const float ds = p * (dp - St[u][1]);
            store_dbias<G, false>(a, c, FULL || j[u] >= 0, Ep[u], ds);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { dk[i] = fmaf(p, gf[i], dk[i]); dz[i] = fmaf(ds, sl[i], dz[i]); }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dk[i] = slot_sum<G::LPE>(dk[i]); dz[i] = slot_sum<G::LPE>(dz[i]); }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, dk);
        store_f32<VEC>(a.part_v1 + (size_t)item * a.HD + c.f0, dz);
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        load_f32<VEC>(a.part_v1 + (size_t)chunk * a.HD + c.f0, P.v1);
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dk[i] = fmaf(w, P.v0[i], dk[i]); dz[i] = fmaf(w, P.v1[i], dz[i]); }
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = fmaf(al2[i] * kLn2, dz[i], dk[i]);
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_k) + c.off, o);
    }
};

}  // namespace dfgnn
