// Passes of the AGNN layer.
#pragma once
#include "layer_device.hpp"

namespace dfgnn {

// =============================================================================================
// AGNN (Sec. 5.1): s_ij = beta * cos(h_i, h_j); aggregated value is the raw feature row
// =============================================================================================
// 1 / max(|h|, eps) from the squared norm.  The norm of a neighbour is taken from its gathered row
// (one more dot product over the head's lanes) instead of being gathered as a 4-byte scalar, which
// would cost a whole memory sector per edge.
__device__ inline float inv_norm(float n2, float inv_eps) { return fminf(__builtin_amdgcn_rsqf(n2), inv_eps); }

template <class G, int U, class Acc> struct AgnnFwdT {
    static constexpr int VEC = G::VEC;
    float x2[VEC], B[U];
    Acc sm;  // SoftmaxAcc: the layer itself; AttentionOut: write the attention weights instead
    int Ep[U];
    u32x4 V[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, x2);
        const float rn = inv_norm(head_sum<G::LPH>(dotv<VEC>(x2, x2), a.lph), a.inv_eps);
#pragma unroll
        for (int i = 0; i < VEC; ++i) x2[i] *= agnn_beta(a) * kLog2e * rn;
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
            const float rnj = inv_norm(head_sum<G::LPH>(dotv<VEC>(vf, vf), a.lph), a.inv_eps);
            s[u] = with_bias<G>(head_sum<G::LPH>(dotv<VEC>(x2, vf), a.lph) * rnj, B[u]);
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
template <class G, int U> using AgnnFwd = AgnnFwdT<G, U, SoftmaxAcc<G, U>>;
template <class G, int U> using AgnnAttention = AgnnFwdT<G, U, AttentionOut<G, U>>;


// row side: g_i = beta sum_j dS_ij xhat_j ;  dbeta_i = sum_j dS_ij cos_ij
template <class G, int U> struct AgnnBwdRow : RowBackwardBase<G> {
    static constexpr int VEC = G::VEC;
    static constexpr bool kExact = RowBackwardBase<G>::kExact;
    float xh[VEC], ga[VEC], px[VEC];  // px = sum_j p xhat_j (kExact only)
    float rn, dbeta, pc;              // pc = sum_j p cos_ij (kExact only)
    float beta, beta2;                // beta and beta * log2(e)
    float B[U];
    int Ep[U];
    u32x4 V[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, xh);
        rn = inv_norm(head_sum<G::LPH>(dotv<VEC>(xh, xh), a.lph), a.inv_eps);
        beta = agnn_beta(a);
        beta2 = beta * kLog2e;
        dbeta = 0.f;
        pc = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) { xh[i] *= rn; ga[i] = 0.f; px[i] = 0.f; }
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
            const float rnj = inv_norm(head_sum<G::LPH>(dotv<VEC>(vf, vf), a.lph), a.inv_eps);
            const float cs = head_sum<G::LPH>(dotv<VEC>(xh, vf), a.lph) * rnj;
            const float dp = head_sum<G::LPH>(dotv<VEC>(this->g, vf), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(with_bias<G>(cs * beta2, B[u]) - this->lse2) : 0.f;
            if constexpr (kExact) {
                const float t = p * dp;
                if (u == 0 && (FULL || j[0] >= 0)) this->dp0 = dp;  // (a slot that has run out of edges keeps its value)
                this->dsum += t;
                dbeta = fmaf(t, cs, dbeta);
                pc = fmaf(p, cs, pc);
                const float w1 = t * rnj, w2 = p * rnj;
#pragma unroll
                for (int i = 0; i < VEC; ++i) { ga[i] = fmaf(w1, vf[i], ga[i]); px[i] = fmaf(w2, vf[i], px[i]); }
            } else {
                const float ds = p * (dp - this->delta);
                store_dbias<G, true>(a, c, FULL || j[u] >= 0, Ep[u], ds);
                dbeta = fmaf(ds, cs, dbeta);
                const float w = ds * rnj;
#pragma unroll
                for (int i = 0; i < VEC; ++i) ga[i] = fmaf(w, vf[i], ga[i]);
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
        dbeta = slot_sum<G::LPE>(dbeta);
#pragma unroll
        for (int i = 0; i < VEC; ++i) ga[i] = slot_sum<G::LPE>(ga[i]);
        if constexpr (kExact) {
            pc = slot_sum<G::LPE>(pc);
            this->dsum = slot_sum<G::LPE>(this->dsum);
#pragma unroll
            for (int i = 0; i < VEC; ++i) px[i] = slot_sum<G::LPE>(px[i]);
        }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, ga);
        if constexpr (kExact) store_f32<VEC>(a.part_v1 + (size_t)item * a.HD + c.f0, px);
        if (c.head0) {
            a.part_s0[(size_t)item * a.H + c.h] = dbeta;
            if constexpr (kExact) {
                a.part_s1[(size_t)item * a.H + c.h] = pc;
                a.part_s2[(size_t)item * a.H + c.h] = this->dsum;
            }
        }
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        P.s0 = a.part_s0[(size_t)chunk * a.H + c.h];
        if constexpr (kExact) {
            load_f32<VEC>(a.part_v1 + (size_t)chunk * a.HD + c.f0, P.v1);
            P.s1 = a.part_s1[(size_t)chunk * a.H + c.h];
            P.s2 = a.part_s2[(size_t)chunk * a.H + c.h];
        }
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) ga[i] = fmaf(w, P.v0[i], ga[i]);
        dbeta = fmaf(w, P.s0, dbeta);
        if constexpr (kExact) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) px[i] = fmaf(w, P.v1[i], px[i]);
            pc = fmaf(w, P.s1, pc);
            this->dsum = fmaf(w, P.s2, this->dsum);
        }
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        if constexpr (kExact) {
            this->delta = this->exact_delta(c);
            dbeta = this->single_edge(c) ? 0.f : dbeta - this->delta * pc;
#pragma unroll
            for (int i = 0; i < VEC; ++i) ga[i] = this->single_edge(c) ? 0.f : ga[i] - this->delta * px[i];
        }
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = beta * ga[i];
        store_f32<VEC>(a.g_row + c.woff, o);
        if (c.head0) {
            const size_t nh = (size_t)c.node * a.H + c.h;
            a.dbeta_row[nh] = dbeta;
            f32x4 st = {rn, this->lse2, this->delta, 0.f};
            *reinterpret_cast<f32x4*>(a.stats + 4 * nh) = st;
        }
    }
};

// column side: value term sum_i p_ij dO_i, key term beta sum_i dS_ij xhat_i, then the derivative of the
// normalisation x -> x / max(|x|, eps) applied to the summed row+column gradient of xhat_j
template <class G, int U> struct AgnnBwdCol {
    static constexpr int VEC = G::VEC;
    float hj[VEC], xh[VEC], val[VEC], ga[VEC];
    float rn, beta;
    float B[U];
    int Ep[U];
    u32x4 Xi[U], Gd[U];
    f32x4 St[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, hj);
        rn = inv_norm(head_sum<G::LPH>(dotv<VEC>(hj, hj), a.lph), a.inv_eps);
        beta = agnn_beta(a);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { xh[i] = hj[i] * rn; val[i] = 0.f; ga[i] = 0.f; }
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int i, int e) {
        Xi[u] = gather_raw<G>(a.x, a, c, i);
        Gd[u] = gather_raw<G>(a.d_out, a, c, i);
        St[u] = gather_stats4(a, c, i);
        B[u] = load_bias<G>(a, c, i, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float xf[VEC], gf[VEC];
            Elem<typename G::T>::unpack(Xi[u], xf);
            Elem<typename G::T>::unpack(Gd[u], gf);
            const float cs = head_sum<G::LPH>(dotv<VEC>(xf, xh), a.lph) * St[u][0];
            const float dp = head_sum<G::LPH>(dotv<VEC>(gf, hj), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(with_bias<G>(cs * (beta * kLog2e), B[u]) - St[u][1]) : 0.f;
            const float ds = p * (dp - St[u][2]);
            store_dbias<G, false>(a, c, FULL || j[u] >= 0, Ep[u], ds);
            const float w = ds * St[u][0];
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                val[i] = fmaf(p, gf[i], val[i]);
                ga[i] = fmaf(w, xf[i], ga[i]);
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) { val[i] = slot_sum<G::LPE>(val[i]); ga[i] = slot_sum<G::LPE>(ga[i]); }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, val);
        store_f32<VEC>(a.part_v1 + (size_t)item * a.HD + c.f0, ga);
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        load_f32<VEC>(a.part_v1 + (size_t)chunk * a.HD + c.f0, P.v1);
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) { val[i] = fmaf(w, P.v0[i], val[i]); ga[i] = fmaf(w, P.v1[i], ga[i]); }
    }
    // all lanes of the wave must call this (it reduces over the head's lanes)
    __device__ void finalize(const Args& a, const Ctx& c) {
        float gt[VEC];
        if (c.active) {
            load_f32<VEC>(a.g_row + c.woff, gt);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) gt[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) gt[i] = fmaf(beta, ga[i], gt[i]);
        const float proj = head_sum<G::LPH>(dotv<VEC>(gt, xh), a.lph);
        const float nrm2 = head_sum<G::LPH>(dotv<VEC>(hj, hj), a.lph);
        const bool clamped = !(sqrtf(nrm2) > a.eps);
        if (!c.writer || !c.active) return;
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = (clamped ? gt[i] * rn : rn * (gt[i] - proj * xh[i])) + val[i];
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_x) + c.off, o);
    }
};

}  // namespace dfgnn
