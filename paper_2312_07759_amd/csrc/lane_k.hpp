// Lane <-> codeword kernels for large (or odd-sized) codebooks: lane l of a
// wavefront owns codewords l, l+64, ... (KPL per lane), a wavefront walks over
// weight vectors one at a time (broadcast from a lane with v_readlane), the row
// softmax is a wavefront reduction, and the M-step sums stay in lane registers.
#pragma once
#include "common.hpp"
#include "small_k.hpp"

namespace idkm {

__device__ __forceinline__ float lane_bcast(float x, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}

// Per-wavefront state of one pass: this lane's codewords and accumulators.
template <int KPL, int D, int DIST, int PASS>
struct LaneWave {
    static constexpr bool STATS = (PASS == PASS_FWD || PASS == PASS_FIN);
    static constexpr bool BACK = (PASS == PASS_B1 || PASS == PASS_B2 || PASS == PASS_B3);
    static constexpr bool USE_G = (PASS == PASS_B1 || PASS == PASS_B3);
    static constexpr bool USE_H = (PASS == PASS_B2 || PASS == PASS_B3);
    static constexpr int ACCW = STATS ? (D + 1) : D;
    static constexpr int NA = (PASS == PASS_B3) ? 1 : KPL * ACCW;  // accumulators per lane
    // passes that work in scaled coordinates t = s (w - c): the forward loop, and the (dF/dC)^T pass of the
    // squared energy
    static constexpr bool SCALED = (PASS == PASS_FWD) || (PASS == PASS_B2 && DIST == DIST_SQL2);

    float c[KPL][D], hs[KPL][D], ff[KPL][D];
    float cs[KPL][D];  // scaled passes only: codewords in scaled coordinates, padding lanes far away
    float hf[KPL];     // scaled (dF/dC)^T pass: sum_r hs_r F_r, so that h.(w - F) = (hs/s).t_w - hf
    bool valid[KPL];
    float acc[NA];

    // Cf/Hs/Ff may point to global memory or LDS.
    __device__ __forceinline__ void init(int k, const float* Cf, const float* Hs, const float* Ff, float escale = 0.f) {
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int q = 0; q < KPL; ++q) {
            const int j = lane + 64 * q;
            valid[q] = j < k;
#pragma unroll
            for (int r = 0; r < D; ++r) {
                c[q][r] = valid[q] ? Cf[j * D + r] : 0.f;
                // a padding codeword sits 1e18 away: its weight underflows to exactly zero without a select
                cs[q][r] = valid[q] ? Cf[j * D + r] * escale : 1e18f;
                hs[q][r] = (USE_H && valid[q]) ? Hs[j * D + r] : 0.f;
                ff[q][r] = (USE_H && valid[q]) ? Ff[j * D + r] : 0.f;
            }
            hf[q] = 0.f;
            if (PASS == PASS_B2 && DIST == DIST_SQL2) {
                const float inv = 1.0f / escale;
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    hf[q] = fmaf(hs[q][r], ff[q][r], hf[q]);
                    hs[q][r] *= inv;  // meets the scaled vector
                }
            }
        }
#pragma unroll
        for (int q = 0; q < NA; ++q) acc[q] = 0.f;
    }

    // Processes vectors gbase .. gbase+cnt-1 (cnt <= 64); lane l holds vector gbase+l in wv (and dL/dWq in gv).
    // Per-vector outputs (Wq, assignment, dW) are collected in lane l and stored coalesced.
    __device__ __forceinline__ void batch(const Args& a, int64_t gbase, int cnt, const float (&wv)[D],
                                          const float (&gv)[D]) {
        const int lane = threadIdx.x & 63;
        const int k = a.k;
        const float inf = __builtin_inff();
        const float nscale = a.nscale;
        float ov[D];
        int oa = 0;
#pragma unroll
        for (int r = 0; r < D; ++r) ov[r] = 0.f;
        // forward loop: the lane's vector is moved to scaled coordinates once per batch
        float wb[D];
#pragma unroll
        for (int r = 0; r < D; ++r) wb[r] = SCALED ? wv[r] * a.escale : wv[r];
        const float inv_escale = SCALED ? 1.0f / a.escale : 0.f;
        for (int l = 0; l < cnt; ++l) {
            float w[D], g[D], gs[D];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                w[r] = lane_bcast(wb[r], l);
                g[r] = USE_G ? lane_bcast(gv[r], l) : 0.f;
                gs[r] = g[r] * a.inv_tau;
            }
            if (PASS == PASS_FWD) {
                // forward loop in scaled coordinates t = s w - s c (s^2 = log2(e)/tau for the squared energy,
                // s = log2(e)/tau for the plain norm): exp(-e/tau) = exp2(-|t|^2) resp. exp2(-|t|); the
                // normalisation is folded into the M-step FMAs.  wv was scaled before the loop, so the
                // broadcast value feeds the subtraction straight from its scalar register.
                float ev[KPL];
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    float t = w[0] - cs[q][0];
                    float e2 = t * t;
#pragma unroll
                    for (int r = 1; r < D; ++r) {
                        t = w[r] - cs[q][r];
                        e2 = fmaf(t, t, e2);
                    }
                    if (DIST == DIST_SQL2)
                        ev[q] = e2;
                    else
                        ev[q] = (D == 1) ? fabsf(w[0] - cs[q][0]) : fast_sqrt(e2);
                }
                // Squared energy: exp2(-e) cannot overflow and the row shift of the softmax is only needed when the
                // whole row underflows (a vector many kernel widths from every codeword).  That is decided from the
                // unshifted row sum, which is wave-uniform; only then is the row minimum found and the row redone.
                // With the plain norm rows underflow routinely (e/tau is large at small tau): always shifted.
                float p[KPL], S = 0.f;
                if (DIST == DIST_SQL2) {
#pragma unroll
                    for (int q = 0; q < KPL; ++q) {
                        p[q] = fast_exp2(-ev[q]);
                        S = (q == 0) ? p[0] : S + p[q];
                    }
                    S = wave_sum(S);
                }
                if (DIST != DIST_SQL2 || S < 7.9e-31f) {  // below 2^-100
                    float emin = ev[0];
#pragma unroll
                    for (int q = 1; q < KPL; ++q) emin = fminf(emin, ev[q]);
                    emin = wave_min_nonneg(emin);
                    S = 0.f;
#pragma unroll
                    for (int q = 0; q < KPL; ++q) {
                        p[q] = fast_exp2(emin - ev[q]);
                        S += p[q];
                    }
                    S = wave_sum(S);
                }
                const float rS = fast_rcp(S);
                const float rSu = rS * inv_escale;  // undoes the scaling of w in the first-moment sums
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    acc[q * ACCW] = fmaf(p[q], rS, acc[q * ACCW]);
#pragma unroll
                    for (int r = 0; r < D; ++r) acc[q * ACCW + 1 + r] = fmaf(p[q], w[r] * rSu, acc[q * ACCW + 1 + r]);
                }
                continue;
            }
            if (PASS == PASS_B2 && DIST == DIST_SQL2) {
                // (dF/dC)^T pass in scaled coordinates, squared energy: the row softmax as in the forward loop
                // (unshifted unless the whole row underflows); with t = s (w - c): delta = 2 (w - c) = (2/s) t and
                // h.(w - F) = (h/s).(s w) - h.F, so the factor 2/(s S) joins the row's scalar and nothing per
                // codeword is rescaled.
                float t[KPL][D], ev[KPL], p[KPL], qv[KPL];
                float S = 0.f;
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    t[q][0] = w[0] - cs[q][0];
                    float e2 = t[q][0] * t[q][0];
                    float sq = fmaf(hs[q][0], w[0], -hf[q]);
#pragma unroll
                    for (int r = 1; r < D; ++r) {
                        t[q][r] = w[r] - cs[q][r];
                        e2 = fmaf(t[q][r], t[q][r], e2);
                        sq = fmaf(hs[q][r], w[r], sq);
                    }
                    ev[q] = e2;
                    qv[q] = sq;
                    p[q] = fast_exp2(-e2);
                    S = (q == 0) ? p[0] : S + p[q];
                }
                S = wave_sum(S);
                if (S < 7.9e-31f) {  // below 2^-100: redo the row shifted by its minimum
                    float emin = ev[0];
#pragma unroll
                    for (int q = 1; q < KPL; ++q) emin = fminf(emin, ev[q]);
                    emin = wave_min_nonneg(emin);
                    S = 0.f;
#pragma unroll
                    for (int q = 0; q < KPL; ++q) {
                        p[q] = fast_exp2(emin - ev[q]);
                        S += p[q];
                    }
                    S = wave_sum(S);
                }
                const float rS = fast_rcp(S);
                float qb = 0.f;
#pragma unroll
                for (int q = 0; q < KPL; ++q) qb = fmaf(p[q], qv[q], qb);
                qb = wave_sum(qb) * rS;
                const float f = 2.f * rS * inv_escale;
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    const float th = (p[q] * f) * (qv[q] - qb);
#pragma unroll
                    for (int r = 0; r < D; ++r) acc[q * ACCW + r] = fmaf(th, t[q][r], acc[q * ACCW + r]);
                }
                continue;
            }
            // E-step: energies of this lane's codewords, wavefront softmax (Eq. "aterms")
            float df[KPL][D], ri[KPL], u[KPL], at[KPL];
            float umax = -inf;
#pragma unroll
            for (int q = 0; q < KPL; ++q) {
#pragma unroll
                for (int r = 0; r < D; ++r) df[q][r] = w[r] - c[q][r];
                float e;
                ri[q] = 0.f;
                if (D == 1) {
                    e = (DIST == DIST_SQL2) ? df[q][0] * df[q][0] : fabsf(df[q][0]);
                } else {
                    float e2 = df[q][0] * df[q][0];
#pragma unroll
                    for (int r = 1; r < D; ++r) e2 = fmaf(df[q][r], df[q][r], e2);
                    if (DIST == DIST_SQL2) {
                        e = e2;
                    } else if (BACK) {
                        float rs = (e2 > 0.f) ? fast_rsq(e2) : 0.f;
                        ri[q] = rs;
                        e = e2 * rs;
                    } else {
                        e = fast_sqrt(e2);
                    }
                }
                u[q] = valid[q] ? e * nscale : -inf;
                umax = fmaxf(umax, u[q]);
            }
            umax = wave_max(umax);
            float S = 0.f;
#pragma unroll
            for (int q = 0; q < KPL; ++q) {
                at[q] = fast_exp2(u[q] - umax);
                S += at[q];
            }
            S = wave_sum(S);
            const float rS = fast_rcp(S);
#pragma unroll
            for (int q = 0; q < KPL; ++q) at[q] *= rS;

            if (STATS) {
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    acc[q * ACCW] += at[q];
#pragma unroll
                    for (int r = 0; r < D; ++r) acc[q * ACCW + 1 + r] = fmaf(at[q], w[r], acc[q * ACCW + 1 + r]);
                }
            }
            if (PASS == PASS_FIN) {
                if (a.Wq_out) {
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        float s = 0.f;
#pragma unroll
                        for (int q = 0; q < KPL; ++q) s = fmaf(at[q], c[q][r], s);
                        s = wave_sum(s);
                        if (lane == l) ov[r] = s;
                    }
                }
                if (a.A_out) {
#pragma unroll
                    for (int q = 0; q < KPL; ++q)
                        if (valid[q]) a.A_out[(gbase + l) * (int64_t)k + lane + 64 * q] = at[q];
                }
                if (a.assign_out) {
                    // closest codeword on a float32 key with separately rounded operations; lowest index on ties
                    float key[KPL], bk = inf;
#pragma unroll
                    for (int q = 0; q < KPL; ++q) {
                        if (D == 1) {
                            key[q] = fabsf(df[q][0]);
                        } else {
                            key[q] = sum_sq_unfused<D>(df[q]);
                        }
                        if (!valid[q]) key[q] = inf;
                        bk = fminf(bk, key[q]);
                    }
                    const float kmin = wave_min(bk);
                    int cand = 0x7fffffff;
#pragma unroll
                    for (int q = KPL - 1; q >= 0; --q)
                        if (valid[q] && key[q] == kmin) cand = lane + 64 * q;
                    const int jmin = wave_min_i(cand);
                    if (lane == l) oa = jmin;
                }
            }
            if (BACK) {
                float qv[KPL], qb = 0.f;
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    float s = 0.f;
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        if (USE_G) s = fmaf(gs[r], c[q][r], s);
                        if (USE_H) s = fmaf(hs[q][r], w[r] - ff[q][r], s);
                    }
                    qv[q] = s;
                    qb = fmaf(at[q], s, qb);
                }
                qb = wave_sum(qb);
                float out[D];
#pragma unroll
                for (int r = 0; r < D; ++r) out[r] = 0.f;
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    const float th = at[q] * (qv[q] - qb);
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        float dl;
                        if (DIST == DIST_SQL2)
                            dl = 2.f * df[q][r];
                        else if (D == 1)
                            dl = (df[q][0] > 0.f) ? 1.f : ((df[q][0] < 0.f) ? -1.f : 0.f);
                        else
                            dl = df[q][r] * ri[q];
                        if (PASS == PASS_B3) {
                            out[r] = fmaf(at[q], hs[q][r] * a.tau, out[r]);
                            out[r] = fmaf(-th, dl, out[r]);
                        } else {
                            float t = acc[q * ACCW + r];
                            if (PASS == PASS_B1) t = fmaf(at[q], g[r], t);
                            acc[q * ACCW + r] = fmaf(th, dl, t);
                        }
                    }
                }
                if (PASS == PASS_B3) {
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        const float s = wave_sum(out[r]);
                        if (lane == l) ov[r] = s;
                    }
                }
            }
        }
        if (lane < cnt) {
            const int64_t i = gbase + lane;
            if (PASS == PASS_FIN && a.Wq_out) VecLoad<D>::store(a.Wq_out, i, ov);
            if (PASS == PASS_FIN && a.assign_out) a.assign_out[i] = oa;
            if (PASS == PASS_B3) VecLoad<D>::store(a.dW_out, i, ov);
        }
    }
};

template <int KPL, int D, int DIST, int PASS>
__global__ __launch_bounds__(WG) void lane_pass(const Args a) {
    using LW = LaneWave<KPL, D, DIST, PASS>;
    constexpr int ACCW = LW::ACCW;
    constexpr int NA = LW::NA;

    if (PASS == PASS_FWD && a.ctrl->done) return;
    if (PASS == PASS_B2 && a.ctrl->b_done) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = a.k;
    LW st;
    st.init(k, a.Cf, a.Hs, a.Ff, a.escale);

    const int64_t vpw = a.vec_per_wg / (WG / 64);
    const int64_t wbase = (int64_t)blockIdx.x * a.vec_per_wg + (int64_t)wave * vpw;
    int64_t wend = wbase + vpw;
    if (wend > a.m) wend = a.m;

    // float32 sums absorb at most 256 vectors before they are folded into float64 ones
    double acc64[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) acc64[q] = 0.0;
    int since = 0;
    for (int64_t b = wbase; b < wend; b += 64) {
        const int64_t i = b + lane;
        float wv[D], gv[D];
#pragma unroll
        for (int r = 0; r < D; ++r) wv[r] = gv[r] = 0.f;
        if (i < wend) {
            VecLoad<D>::load(a.W, i, wv);
            if (LW::USE_G) VecLoad<D>::load(a.G, i, gv);
        }
        const int cnt = (wend - b < 64) ? (int)(wend - b) : 64;
        st.batch(a, b, cnt, wv, gv);
        if (PASS != PASS_B3 && ++since == 4) {
            since = 0;
#pragma unroll
            for (int q = 0; q < NA; ++q) {
                acc64[q] += (double)st.acc[q];
                st.acc[q] = 0.f;
            }
        }
    }

    if (PASS == PASS_B3) return;

    // workgroup partial: wavefronts add into LDS one after the other (fixed order), float64
    __shared__ double s_acc[64][NA];
    for (int wv = 0; wv < WG / 64; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int q = 0; q < NA; ++q) {
                const double v = acc64[q] + (double)st.acc[q];
                if (wv == 0)
                    s_acc[lane][q] = v;
                else
                    s_acc[lane][q] += v;
            }
        }
        __syncthreads();
    }
    // the partials of this family (k (d+1) values per workgroup) are reduced by reduce_rows + lane_tail
    const int nacc = k * ACCW;
    for (int idx = threadIdx.x; idx < nacc; idx += WG) {
        const int j = idx / ACCW, comp = idx - j * ACCW;
        a.partials[(size_t)blockIdx.x * nacc + idx] = s_acc[j & 63][(j >> 6) * ACCW + comp];
    }
}

// tot[acc] = sum over workgroups of partials[wg][acc], fixed order.  One workgroup per 64 accumulators; the four
// wavefronts take interleaved quarters of the workgroups with eight loads in flight each.
template <int UNUSED>  // a template only so that the header can be included by several translation units
__global__ __launch_bounds__(WG) void reduce_rows(const Args a, int nacc, int nwg, int pass) {
    if (pass == PASS_FWD && a.ctrl->done) return;
    if (pass == PASS_B2 && a.ctrl->b_done) return;
    __shared__ double s_q[WG / 64][64];
    const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int acc = blockIdx.x * 64 + lane;
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (acc < nacc) {
        const double* __restrict__ p = a.partials + acc;
        int wg = part;
        for (; wg + 7 * 4 < nwg; wg += 8 * 4) {
            double x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = p[(size_t)(wg + 4 * u) * nacc];
#pragma unroll
            for (int u = 0; u < 8; ++u) s[u] += x[u];
        }
        for (; wg < nwg; wg += 4) s[0] += p[(size_t)wg * nacc];
    }
    s_q[part][lane] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
    __syncthreads();
    if (part == 0 && acc < nacc) a.tot[acc] = (s_q[0][lane] + s_q[1][lane]) + (s_q[2][lane] + s_q[3][lane]);
}

// The O(k d) update and stop logic of a pass whose totals are already in a.tot (single workgroup).
template <int PASS>
__global__ __launch_bounds__(WG) void lane_tail(const Args a) {
    if (PASS == PASS_FWD && a.ctrl->done) return;
    if (PASS == PASS_B2 && a.ctrl->b_done) return;
    if (PASS == PASS_FWD) tail_forward(a, a.tot);
    if (PASS == PASS_FIN) tail_final(a, a.tot);
    if (PASS == PASS_B1) tail_b1(a, a.tot);
    if (PASS == PASS_B2) tail_b2(a, a.tot);
}

// The same tail with 16 wavefronts, for the minimal-residual solve at large k d: its inner products and vector
// updates over the Krylov basis are spread over the threads of this one workgroup.
template <int UNUSED>
__global__ __launch_bounds__(1024) void lane_tail_b2_wide(const Args a) {
    if (a.ctrl->b_done) return;
    tail_b2(a, a.tot);
}

}  // namespace idkm
