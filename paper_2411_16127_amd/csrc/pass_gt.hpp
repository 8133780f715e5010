// Passes of the GT layer (forward, backward row side, backward column side) and of the two-kernel comparator.
#pragma once
#include "layer_device.hpp"

namespace dfgnn {

// =============================================================================================
// GT (dot-SDDMM, Sec. 5.1): s_ij = scale q_i.k_j
// =============================================================================================
template <class G, int U, class Acc> struct GtFwdT {
    static constexpr int VEC = G::VEC;
    float q[VEC], B[U];
    Acc sm;  // SoftmaxAcc: the layer itself; AttentionOut: write the attention weights instead
    int Ep[U];
    u32x4 K[U], V[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, q);
#pragma unroll
        for (int i = 0; i < VEC; ++i) q[i] *= a.c_score;
        sm.init(a, c);
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        K[u] = gather_raw<G>(a.k, a, c, j);
        V[u] = gather_raw<G>(a.v, a, c, j);
        B[u] = load_bias<G>(a, c, j, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[VEC];
            Elem<typename G::T>::unpack(K[u], kf);
            s[u] = with_bias<G>(head_sum<G::LPH>(dotv<VEC>(q, kf), a.lph), B[u]);
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
template <class G, int U> using GtFwd = GtFwdT<G, U, SoftmaxAcc<G, U>>;
template <class G, int U> using GtAttention = GtFwdT<G, U, AttentionOut<G, U>>;


// Forward pass of the two-kernel comparator (Sec. 3, parallelism maximization fusion): the scores were
// written by k_edge_scores; this pass reads them back and does the softmax and the aggregation.
template <class G, int U> struct GtFwdStored {
    static constexpr int VEC = G::VEC;
    SoftmaxAcc<G, U> sm;
    float S[U];
    u32x4 V[U];
    __device__ void init(const Args&, const Ctx&) { sm.reset(); }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        S[u] = j >= 0 ? a.scores[(size_t)e * a.H + c.h] : -INFINITY;
        V[u] = gather_raw<G>(a.v, a, c, j);
    }
    template <bool FULL> __device__ void consume(const Args&, const Ctx&, const int (&j)[U]) {
        if (!FULL && j[0] < 0) return;
        sm.update(S, V);
    }
    __device__ void combine_slots(const Args&, const Ctx&) { sm.combine_slots(); }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) { sm.store_partial(a, c, item); }
    __device__ void load_partial(const Args& a, const Ctx& c, int chunk, PartialRegs<VEC>& P) const { sm.load_partial(a, c, chunk, P); }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) { sm.fold_partial(P, valid); }
    __device__ void finalize(const Args& a, const Ctx& c) { sm.finalize(a, c); }
};

// dQ_i = scale sum_j dS_ij k_j with dS_ij = p_ij (dO_i.v_j - delta_i)   (Appendix B; fused chain of Sec. 4.3)
template <class G, int U> struct GtBwdRow : RowBackwardBase<G> {
    static constexpr int VEC = G::VEC;
    static constexpr bool kExact = RowBackwardBase<G>::kExact;
    float q[VEC], dq[VEC], pk[VEC];  // pk = sum_j p k_j (kExact only)
    float B[U];
    int Ep[U];
    u32x4 K[U], V[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.x, c, q);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { q[i] *= a.c_score; dq[i] = 0.f; pk[i] = 0.f; }
        this->init_row(a, c);
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int j, int e) {
        K[u] = gather_raw<G>(a.k, a, c, j);
        V[u] = gather_raw<G>(a.v, a, c, j);
        B[u] = load_bias<G>(a, c, j, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[VEC], vf[VEC];
            Elem<typename G::T>::unpack(K[u], kf);
            Elem<typename G::T>::unpack(V[u], vf);
            const float s = with_bias<G>(head_sum<G::LPH>(dotv<VEC>(q, kf), a.lph), B[u]);
            const float dp = head_sum<G::LPH>(dotv<VEC>(this->g, vf), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(s - this->lse2) : 0.f;
            if constexpr (kExact) {
                const float t = p * dp;
                if (u == 0 && (FULL || j[0] >= 0)) this->dp0 = dp;  // (a slot that has run out of edges keeps its value)
                this->dsum += t;
#pragma unroll
                for (int i = 0; i < VEC; ++i) { dq[i] = fmaf(t, kf[i], dq[i]); pk[i] = fmaf(p, kf[i], pk[i]); }
            } else {
                const float ds = p * (dp - this->delta);
                store_dbias<G, true>(a, c, FULL || j[u] >= 0, Ep[u], ds);
#pragma unroll
                for (int i = 0; i < VEC; ++i) dq[i] = fmaf(ds, kf[i], dq[i]);
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) dq[i] = slot_sum<G::LPE>(dq[i]);
        if constexpr (kExact) {
            this->dsum = slot_sum<G::LPE>(this->dsum);
#pragma unroll
            for (int i = 0; i < VEC; ++i) pk[i] = slot_sum<G::LPE>(pk[i]);
        }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, dq);
        if constexpr (kExact) {
            store_f32<VEC>(a.part_v1 + (size_t)item * a.HD + c.f0, pk);
            if (c.head0) a.part_s2[(size_t)item * a.H + c.h] = this->dsum;
        }
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        if constexpr (kExact) {
            load_f32<VEC>(a.part_v1 + (size_t)chunk * a.HD + c.f0, P.v1);
            P.s2 = a.part_s2[(size_t)chunk * a.H + c.h];
        }
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) dq[i] = fmaf(w, P.v0[i], dq[i]);
        if constexpr (kExact) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) pk[i] = fmaf(w, P.v1[i], pk[i]);
            this->dsum = fmaf(w, P.s2, this->dsum);
        }
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        if constexpr (kExact) {
            this->delta = this->exact_delta(c);
#pragma unroll
            for (int i = 0; i < VEC; ++i) dq[i] = this->single_edge(c) ? 0.f : dq[i] - this->delta * pk[i];
        }
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = a.scale * dq[i];
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_x) + c.off, o);
        if (c.head0) {
            f32x2 st = {this->lse2, this->delta};
            *reinterpret_cast<f32x2*>(a.stats + 2 * ((size_t)c.node * a.H + c.h)) = st;
        }
    }
};

// Column pass over the CSC (transposed products of Appendix B): for source j and every edge i <- j,
// dV_j += p_ij dO_i,  dK_j += scale dS_ij q_i, with p and dS recomputed from the row statistics.
template <class G, int U> struct GtBwdCol {
    static constexpr int VEC = G::VEC;
    float k2[VEC], vv[VEC], dk[VEC], dv[VEC];
    float B[U];
    int Ep[U];
    u32x4 Q[U], Gd[U];
    f32x2 St[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.k, c, k2);
        load_row<G>(a.v, c, vv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { k2[i] *= a.c_score; dk[i] = 0.f; dv[i] = 0.f; }
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int i, int e) {
        Q[u] = gather_raw<G>(a.x, a, c, i);
        Gd[u] = gather_raw<G>(a.d_out, a, c, i);
        St[u] = gather_stats2(a, c, i);
        B[u] = load_bias<G>(a, c, i, e);
        Ep[u] = e;
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx& c, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float qf[VEC], gf[VEC];
            Elem<typename G::T>::unpack(Q[u], qf);
            Elem<typename G::T>::unpack(Gd[u], gf);
            const float s = with_bias<G>(head_sum<G::LPH>(dotv<VEC>(qf, k2), a.lph), B[u]);
            const float dp = head_sum<G::LPH>(dotv<VEC>(gf, vv), a.lph);
            const float p = (FULL || j[u] >= 0) ? fast_exp2(s - St[u][0]) : 0.f;
            const float ds = p * (dp - St[u][1]);
            store_dbias<G, false>(a, c, FULL || j[u] >= 0, Ep[u], ds);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                dv[i] = fmaf(p, gf[i], dv[i]);
                dk[i] = fmaf(ds, qf[i], dk[i]);
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dk[i] = slot_sum<G::LPE>(dk[i]); dv[i] = slot_sum<G::LPE>(dv[i]); }
    }
    __device__ void store_partial(const Args& a, const Ctx& c, int item) {
        if (!c.writer || !c.active) return;
        store_f32<VEC>(a.part_v0 + (size_t)item * a.HD + c.f0, dk);
        store_f32<VEC>(a.part_v1 + (size_t)item * a.HD + c.f0, dv);
    }
    __device__ void load_partial(const Args& a, const Ctx& c0, int chunk, PartialRegs<VEC>& P) const {
        const PartialIndex c(c0);
        load_f32<VEC>(a.part_v0 + (size_t)chunk * a.HD + c.f0, P.v0);
        load_f32<VEC>(a.part_v1 + (size_t)chunk * a.HD + c.f0, P.v1);
    }
    __device__ void fold_partial(const PartialRegs<VEC>& P, bool valid) {
        const float w = valid ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dk[i] = fmaf(w, P.v0[i], dk[i]); dv[i] = fmaf(w, P.v1[i], dv[i]); }
    }
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = a.scale * dk[i];
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_k) + c.off, o);
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_v) + c.off, dv);
    }
};

// The column pass without the row pass's hand-over: log-sum-exp and delta_i = dO_i.O_i of every edge's row are
// recomputed from the forward statistics and the gathered output row (one more row per edge, which only a
// cache-resident graph can afford), so that the row side and the column side of a small graph's backward
// pass run as one launch (k_pass_pair).  fp32 tensors only: a 16-bit output row does not give delta to fp32
// accuracy.  The row pass computes delta with the same instructions, so both sides see the same bits.
template <class G, int U> struct GtBwdColSelf {
    static constexpr int VEC = G::VEC;
    float k2[VEC], vv[VEC], dk[VEC], dv[VEC];
    u32x4 Q[U], Gd[U], O[U];
    float Mx[U], Sm[U];
    __device__ void init(const Args& a, const Ctx& c) {
        load_row<G>(a.k, c, k2);
        load_row<G>(a.v, c, vv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { k2[i] *= a.c_score; dk[i] = 0.f; dv[i] = 0.f; }
    }
    __device__ void issue(const Args& a, const Ctx& c, int u, int i, int) {
        Q[u] = gather_raw<G>(a.x, a, c, i);
        Gd[u] = gather_raw<G>(a.d_out, a, c, i);
        O[u] = gather_raw<G>(a.out, a, c, i);
        Mx[u] = gather_stat(a.row_max, a, c, i);
        Sm[u] = gather_stat(a.row_sum, a, c, i);
    }
    template <bool FULL> __device__ void consume(const Args& a, const Ctx&, const int (&j)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float qf[VEC], gf[VEC], of[VEC];
            Elem<typename G::T>::unpack(Q[u], qf);
            Elem<typename G::T>::unpack(Gd[u], gf);
            Elem<typename G::T>::unpack(O[u], of);
            const bool live = FULL || j[u] >= 0;
            const float lse2 = Mx[u] * kLog2e + fast_log2(live ? Sm[u] : 1.f);
            const float delta = head_sum<G::LPH>(dotv<VEC>(gf, of), a.lph);
            const float s = head_sum<G::LPH>(dotv<VEC>(qf, k2), a.lph);
            const float dp = head_sum<G::LPH>(dotv<VEC>(gf, vv), a.lph);
            const float p = live ? fast_exp2(s - lse2) : 0.f;
            const float ds = p * (dp - delta);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                dv[i] = fmaf(p, gf[i], dv[i]);
                dk[i] = fmaf(ds, qf[i], dk[i]);
            }
        }
    }
    __device__ void combine_slots(const Args&, const Ctx&) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) { dk[i] = slot_sum<G::LPE>(dk[i]); dv[i] = slot_sum<G::LPE>(dv[i]); }
    }
    // graphs with super columns do not take this pass (the host checks), so there are no partials
    __device__ void store_partial(const Args&, const Ctx&, int) {}
    __device__ void load_partial(const Args&, const Ctx&, int, PartialRegs<VEC>&) const {}
    __device__ void fold_partial(const PartialRegs<VEC>&, bool) {}
    __device__ void finalize(const Args& a, const Ctx& c) {
        if (!c.writer || !c.active) return;
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = a.scale * dk[i];
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_k) + c.off, o);
        Elem<typename G::T>::store(static_cast<typename G::T*>(a.d_v) + c.off, dv);
    }
};

}  // namespace dfgnn
