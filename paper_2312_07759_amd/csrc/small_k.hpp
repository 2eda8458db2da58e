// Lane <-> weight-vector kernels for small codebooks (K <= 16): each lane owns
// whole vectors, the K codewords are wave-uniform, and the K (D+1) partial sums
// of the M-step live in the lane's registers.
#pragma once
#include "common.hpp"

namespace idkm {

template <int D>
struct VecLoad {
    static __device__ __forceinline__ void load(const float* __restrict__ p, int64_t i, float (&w)[D]) {
#pragma unroll
        for (int r = 0; r < D; ++r) w[r] = p[i * D + r];
    }
    static __device__ __forceinline__ void store(float* __restrict__ p, int64_t i, const float (&w)[D]) {
#pragma unroll
        for (int r = 0; r < D; ++r) p[i * D + r] = w[r];
    }
};
template <>
struct VecLoad<2> {
    static __device__ __forceinline__ void load(const float* __restrict__ p, int64_t i, float (&w)[2]) {
        float2 v = reinterpret_cast<const float2*>(p)[i];
        w[0] = v.x, w[1] = v.y;
    }
    static __device__ __forceinline__ void store(float* __restrict__ p, int64_t i, const float (&w)[2]) {
        reinterpret_cast<float2*>(p)[i] = make_float2(w[0], w[1]);
    }
};
template <>
struct VecLoad<4> {
    static __device__ __forceinline__ void load(const float* __restrict__ p, int64_t i, float (&w)[4]) {
        float4 v = reinterpret_cast<const float4*>(p)[i];
        w[0] = v.x, w[1] = v.y, w[2] = v.z, w[3] = v.w;
    }
    static __device__ __forceinline__ void store(float* __restrict__ p, int64_t i, const float (&w)[4]) {
        reinterpret_cast<float4*>(p)[i] = make_float4(w[0], w[1], w[2], w[3]);
    }
};

// E-step for one vector against K uniform codewords (Eq. "aterms"): fills the
// attention row a[K], the differences df = w - c and, for the plain norm with
// D > 1 when derivatives are needed, ri = 1/||w - c|| (0 at coincidence).
//
// Scalar weights in the backward passes (D == 1, DERIV): scaled coordinates relative to the first codeword,
// t_j = (w - c_0) s - (c_j - c_0) s with s = sqrt(log2(e)/tau) (squared energy) or log2(e)/tau (plain norm), so that
// exp(-e_j/tau) = exp2(-t_j^2) resp. exp2(-|t_j|); the row is shifted by the smallest |t_j|.  Three operations fewer
// per codeword than the general form.  df receives t_j and ri the factor that turns it into d e_j / d w for the squared
// energy (2/s); for the plain norm only the sign of t_j is used, and t_j = 0 exactly where w = c_j (the two products
// are rounded on their own).  The reference point keeps layers far from the origin free of cancellation.
template <int K, int D, int DIST, bool DERIV>
__device__ __forceinline__ void estep_small(const float (&w)[D], const float (&c)[K][D], float nscale, float escale,
                                            float (&a)[K], float (&df)[K][D], float (&ri)[K]) {
    if constexpr (D == 1 && DERIV) {
        const float c0 = c[0][0];
        const float wr = w[0] - c0;
        float t[K];
#pragma unroll
        for (int j = 0; j < K; ++j) t[j] = scaled_minus_unfused(wr, escale, (c[j][0] - c0) * escale);  // (c_j - c_0) s is loop-invariant
        float tmin = fabsf(t[0]);
#pragma unroll
        for (int j = 1; j < K; ++j) tmin = fminf(tmin, fabsf(t[j]));
        const float qmin = tmin * tmin;
        float S = 0.f;
#pragma unroll
        for (int j = 0; j < K; ++j) {
            a[j] = (DIST == DIST_SQL2) ? fast_exp2(fmaf(-t[j], t[j], qmin)) : fast_exp2(tmin - fabsf(t[j]));
            S = (j == 0) ? a[0] : S + a[j];
        }
        const float rS = fast_rcp(S);
        const float dfac = (DIST == DIST_SQL2) ? 2.f / escale : 0.f;  // loop-invariant
#pragma unroll
        for (int j = 0; j < K; ++j) {
            a[j] *= rS;
            df[j][0] = t[j];
            ri[j] = dfac;
        }
        return;
    }
    float u[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
#pragma unroll
        for (int r = 0; r < D; ++r) df[j][r] = w[r] - c[j][r];
        float e;
        if (D == 1) {
            e = (DIST == DIST_SQL2) ? df[j][0] * df[j][0] : fabsf(df[j][0]);
            ri[j] = 0.f;
        } else {
            float e2 = df[j][0] * df[j][0];
#pragma unroll
            for (int r = 1; r < D; ++r) e2 = fmaf(df[j][r], df[j][r], e2);
            if (DIST == DIST_SQL2) {
                e = e2;
                ri[j] = 0.f;
            } else if (DERIV) {
                float rs = (e2 > 0.f) ? fast_rsq(e2) : 0.f;
                ri[j] = rs;
                e = e2 * rs;
            } else {
                e = fast_sqrt(e2);
                ri[j] = 0.f;
            }
        }
        u[j] = e * nscale;
    }
    float umax = u[0];
#pragma unroll
    for (int j = 1; j < K; ++j) umax = fmaxf(umax, u[j]);
    float S = 0.f;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        a[j] = fast_exp2(u[j] - umax);
        S += a[j];
    }
    const float rS = fast_rcp(S);
#pragma unroll
    for (int j = 0; j < K; ++j) a[j] *= rS;
}

// delta_jr = d e_j / d w_r
template <int K, int D, int DIST>
__device__ __forceinline__ float delta_small(const float (&df)[K][D], const float (&ri)[K], int j, int r) {
    if (DIST == DIST_SQL2 && D > 1) return 2.f * df[j][r];
    if (DIST == DIST_L2 && D == 1) return (df[j][0] > 0.f) ? 1.f : ((df[j][0] < 0.f) ? -1.f : 0.f);
    return df[j][r] * ri[j];  // plain norm, D > 1: unit vector; squared energy, D == 1: df is scaled, ri = 2/s
}

// Everything one pass does for one weight vector i: E-step, then the pass's own
// accumulation or per-vector output.  acc has K*(D+1) entries for the forward
// passes ((n_j, s_j) interleaved), K*D for B1/B2, and is unused for B3.
template <int K, int D, int DIST, int PASS>
struct SmallItem {
    static constexpr bool STATS = (PASS == PASS_FWD || PASS == PASS_FIN);
    static constexpr bool BACK = (PASS == PASS_B1 || PASS == PASS_B2 || PASS == PASS_B3 || PASS == PASS_BJ);
    static constexpr bool USE_G = (PASS == PASS_B1 || PASS == PASS_B3 || PASS == PASS_BJ);
    static constexpr bool USE_H = (PASS == PASS_B2 || PASS == PASS_B3);
    static constexpr bool USE_F = USE_H || PASS == PASS_BJ;  // needs F* = F(C*, W)
    static constexpr int ACCW = STATS ? (D + 1) : D;
    static constexpr int KD = K * D;
    // dense backward: T[KD][KD], U[KD][D], V[KD]
    static constexpr int NACC = (PASS == PASS_B3) ? 1 : (PASS == PASS_BJ ? KD * KD + KD * D + KD : K * ACCW);

    // (dF/dC)^T pass, squared energy, d >= 2 (the pass an implicit solve repeats): in coordinates relative to the mean
    // codeword mu, wm = w - mu and cm_j = c_j - mu, the exponents of the row are products as in the forward loop
    // (FWD_DOT below), l_j = 2 s^2 cm_j.wm - s^2 |cm_j|^2, and  sum_i theta_ij (w_i - c_j)  is accumulated as
    // sum_i theta_ij wm_i  -  cm_j sum_i theta_ij :  k more sums per lane (registers [K D, K D + K)), folded in by
    // finish(), instead of d subtractions per (vector, codeword) pair; 2 d + 6 operations per pair and 10 per vector
    // instead of 5 d + 9 and 2.  prepare() leaves cm in c, h_j.(F*_j - mu) in ff[j][0], mu_r in ff[r][1] and
    // -s^2 |cm_j|^2 in ff[j][D].
    static constexpr bool B2_DOT = (PASS == PASS_B2 && DIST == DIST_SQL2 && D >= 2 && K >= D);
    // accumulators a lane keeps in registers; the first NACC of them are the pass's partial sums after finish()
    static constexpr int NREG = NACC + (B2_DOT ? K : 0);

    // k d >= 32 with d >= 2, (dF/dC)^T pass and last pass: codebook, h and F* (up to 192 values) plus the sums and a
    // vector's own state do not fit 256 registers, and what the compiler moves to the accumulation registers costs a
    // vector-ALU move per use.  There h_j . (w - F*_j) is taken as h_j . (w - mu) - h_j . (F*_j - mu), mu the mean
    // codeword (so that layers far from the origin lose nothing to cancellation): prepare() leaves the k products in
    // ff[j][0] and mu_r in ff[r][1] (the other values of F* are not used again) and run() expects them there; d
    // subtractions per vector instead of d per codeword.
    static constexpr bool FOLD_HF = ((PASS == PASS_B2 || PASS == PASS_B3) && D >= 2 && K * D >= 32) && !B2_DOT;

    // Forward loop, squared energy, d >= 2: the exponent of a weight of the row softmax (Eq. "aterms") is taken as a
    // product.  With s^2 = log2(e)/tau and a reference point mu (the mean codeword; the energy does not change when w
    // and c move together),  -s^2 |w - c_j|^2 = -s^2 |w - mu|^2 + 2 s^2 (c_j - mu).(w - mu) - s^2 |c_j - mu|^2 :  the
    // first term is the same for every codeword and drops out of the row, the rest is d multiply-adds per codeword
    // (2 d + 1 operations for differences, squares and scale) at the price of d subtractions per vector.  The row is
    // shifted by its largest exponent, and the normalisation is folded into the multiply-adds of the M-step (Eq.
    // "centers").  prepare() leaves 2 s^2 (c_j - mu) in hs[j][.], -s^2 |c_j - mu|^2 in ff[j][0] and mu_r in ff[r][1]
    // (this pass uses neither h nor F*).  The rounding error of an exponent is a few float32 ulps of
    // s^2 |c - mu| |w - mu|, i.e. of the exponents themselves; the closest-codeword key of the last pass is not formed
    // this way.
    static constexpr bool FWD_DOT = (PASS == PASS_FWD && DIST == DIST_SQL2 && D >= 2 && K >= D);

    // Called once per pass by every caller of run(), after it has loaded the tables into registers.
    static __device__ __forceinline__ void prepare(const Args& a, float (&c)[K][D], float (&hs)[K][D], float (&ff)[K][D + 1]) {
        if constexpr (B2_DOT) {
            const float s2 = -a.nscale;
            float mu[D];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < K; ++j) s += c[j][r];
                mu[r] = s * (1.f / K);
            }
#pragma unroll
            for (int j = 0; j < K; ++j) {
                float q = 0.f, hf = 0.f;
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    hf = fmaf(hs[j][r], ff[j][r] - mu[r], hf);
                    c[j][r] -= mu[r];
                    q = fmaf(c[j][r], c[j][r], q);
                }
                ff[j][0] = hf;
                ff[j][D] = -s2 * q;
            }
#pragma unroll
            for (int r = 0; r < D; ++r) ff[r][1] = mu[r];
        }
        if constexpr (FWD_DOT) {
            const float s2 = -a.nscale;
            float mu[D];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < K; ++j) s += c[j][r];
                mu[r] = s * (1.f / K);
            }
#pragma unroll
            for (int j = 0; j < K; ++j) {
                float q = 0.f;
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    const float dc = c[j][r] - mu[r];
                    hs[j][r] = 2.f * s2 * dc;
                    q = fmaf(dc, dc, q);
                }
                ff[j][0] = -s2 * q;
            }
#pragma unroll
            for (int r = 0; r < D; ++r) ff[r][1] = mu[r];
        }
        if constexpr (FOLD_HF) {
            static_assert(K >= D, "mu is kept in ff[0..D)[1]");
            float mu[D];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < K; ++j) s += c[j][r];
                mu[r] = s * (1.f / K);
            }
#pragma unroll
            for (int j = 0; j < K; ++j) {
                float s = 0.f;
#pragma unroll
                for (int r = 0; r < D; ++r) s = fmaf(hs[j][r], ff[j][r] - mu[r], s);
                ff[j][0] = s;
            }
#pragma unroll
            for (int r = 0; r < D; ++r) ff[r][1] = mu[r];
        }
    }

    // Scalar weights, (dF/dC)^T pass (the pass an implicit solve repeats): written out in scaled coordinates with ten
    // instructions per codeword; for the squared energy the sums lack the constant factor 2/s of d e / d w, which
    // finish() applies once per pass.
    static constexpr bool SCALAR_B2 = (PASS == PASS_B2 && D == 1);

    // Called once per pass by every caller of run(), after the last vector.
    static __device__ __forceinline__ void finish(const Args& a, const float (&c)[K][D], float (&acc)[NREG]) {
        if constexpr (B2_DOT) {
            // d e / d w = 2 (w - c) = 2 (wm - cm)
#pragma unroll
            for (int j = 0; j < K; ++j)
#pragma unroll
                for (int r = 0; r < D; ++r) acc[j * D + r] = 2.f * fmaf(-c[j][r], acc[KD + j], acc[j * D + r]);
        }
        if constexpr (SCALAR_B2 && DIST == DIST_SQL2) {
            const float f = 2.f / a.escale;
#pragma unroll
            for (int q = 0; q < NACC; ++q) acc[q] *= f;
        }
        (void)c;
    }

    static __device__ __forceinline__ void run(const Args& a, int64_t i, const float (&w)[D], const float (&g)[D],
                                               const float (&c)[K][D], const float (&hs)[K][D],
                                               const float (&ff)[K][D + 1], float (&acc)[NREG]) {
        if constexpr (B2_DOT) {
            const float two_s2 = -2.f * a.nscale;
            float wm[D];
#pragma unroll
            for (int r = 0; r < D; ++r) wm[r] = w[r] - ff[r][1];
            float l[K], q[K];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                float dot = wm[0] * c[j][0], qq = fmaf(hs[j][0], wm[0], -ff[j][0]);
#pragma unroll
                for (int r = 1; r < D; ++r) {
                    dot = fmaf(wm[r], c[j][r], dot);
                    qq = fmaf(hs[j][r], wm[r], qq);
                }
                l[j] = fmaf(dot, two_s2, ff[j][D]);
                q[j] = qq;  // (h_j/tau) . (w - F*_j)
            }
            float lmax = l[0];
#pragma unroll
            for (int j = 1; j < K; ++j) lmax = fmaxf(lmax, l[j]);
            float p[K], S = 0.f, pq = 0.f;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                p[j] = fast_exp2(l[j] - lmax);
                S = (j == 0) ? p[0] : S + p[j];
                pq = fmaf(p[j], q[j], pq);
            }
            const float rS = fast_rcp(S);
            const float nqb = -(pq * rS) * rS;  // -qbar / S
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const float th = p[j] * fmaf(q[j], rS, nqb);  // a_j (q_j - qbar)
                acc[KD + j] += th;
#pragma unroll
                for (int r = 0; r < D; ++r) acc[j * D + r] = fmaf(th, wm[r], acc[j * D + r]);
            }
            return;
        }
        if constexpr (SCALAR_B2) {
            // t_j = (w - c_0) s - (c_j - c_0) s (both products rounded on their own: exactly zero where w = c_j),
            // p_j = exp2(-t_j^2 + min t^2) resp. exp2(-|t_j| + min |t|), S = sum p
            const float sc = a.escale;
            const float c0 = c[0][0];
            const float wr = w[0] - c0;
            float t[K];
#pragma unroll
            for (int j = 0; j < K; ++j) t[j] = scaled_minus_unfused(wr, sc, (c[j][0] - c0) * sc);  // loop-invariant product
            float tmin = fabsf(t[0]);
#pragma unroll
            for (int j = 1; j < K; ++j) tmin = fminf(tmin, fabsf(t[j]));
            const float qmin = tmin * tmin;
            // q_j = (h_j/tau) (w - F_j) = hs_j (w - c_0) - hs_j (F_j - c_0); pq = sum p q
            float p[K], q[K], S = 0.f, pq = 0.f;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                p[j] = (DIST == DIST_SQL2) ? fast_exp2(fmaf(-t[j], t[j], qmin)) : fast_exp2(tmin - fabsf(t[j]));
                S = (j == 0) ? p[0] : S + p[j];
                q[j] = fmaf(hs[j][0], wr, -(hs[j][0] * (ff[j][0] - c0)));  // loop-invariant product
                pq = fmaf(p[j], q[j], pq);
            }
            const float rS = fast_rcp(S);
            const float nqb = -(pq * rS) * rS;  // -qbar / S
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const float th = p[j] * fmaf(q[j], rS, nqb);  // a_j (q_j - qbar)
                if (DIST == DIST_SQL2) {
                    acc[j] = fmaf(th, t[j], acc[j]);  // times 2/s in finish()
                } else {
                    // sign(t_j), zero at t_j = 0: the median of (t_j 2^126, -1, 1) (an infinite product is fine)
                    const float sg = __builtin_amdgcn_fmed3f(t[j] * 8.5070592e37f, -1.f, 1.f);
                    acc[j] = fmaf(th, sg, acc[j]);
                }
            }
            return;
        }
        if (PASS == PASS_FWD && D == 1) {
            // Scalar weights, forward loop: work in scaled coordinates t_j = s w - s c_j with
            // s = sqrt(log2(e)/tau) (squared energy) or log2(e)/tau (plain norm), so that
            // exp(-e_j/tau) = exp2(-t_j^2) resp. exp2(-|t_j|), and the normalisation is folded into the
            // M-step FMAs: 10 K + 4 issue slots per vector instead of 13 K + 2.
            const float sc = a.escale;
            const float ws = w[0] * sc;
            float t[K];
#pragma unroll
            for (int j = 0; j < K; ++j) t[j] = ws - c[j][0] * sc;  // s c_j is loop-invariant
            // The row shift of the softmax is the smallest |t_j| (absolute values are free source modifiers).
            // A branch that skips it when the row cannot underflow was measured slower here: with one wavefront
            // per SIMD the straight-line form lets two vectors interleave.
            float tmin = fabsf(t[0]);
#pragma unroll
            for (int j = 1; j < K; ++j) tmin = fminf(tmin, fabsf(t[j]));
            const float qmin = tmin * tmin;
            float p[K], S = 0.f;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                p[j] = (DIST == DIST_SQL2) ? fast_exp2(fmaf(-t[j], t[j], qmin)) : fast_exp2(tmin - fabsf(t[j]));
                S = (j == 0) ? p[0] : S + p[j];
            }
            const float rS = fast_rcp(S);
            const float rw = rS * w[0];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                acc[j * ACCW] = fmaf(p[j], rS, acc[j * ACCW]);
                acc[j * ACCW + 1] = fmaf(p[j], rw, acc[j * ACCW + 1]);
            }
            return;
        }
        if constexpr (FWD_DOT) {
            float wm[D];
#pragma unroll
            for (int r = 0; r < D; ++r) wm[r] = w[r] - ff[r][1];
            float l[K];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                float x = fmaf(wm[0], hs[j][0], ff[j][0]);
#pragma unroll
                for (int r = 1; r < D; ++r) x = fmaf(wm[r], hs[j][r], x);
                l[j] = x;
            }
            float lmax = l[0];
#pragma unroll
            for (int j = 1; j < K; ++j) lmax = fmaxf(lmax, l[j]);
            float p[K], S = 0.f;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                p[j] = fast_exp2(l[j] - lmax);
                S = (j == 0) ? p[0] : S + p[j];
            }
            const float rS = fast_rcp(S);
            float rw[D];
#pragma unroll
            for (int r = 0; r < D; ++r) rw[r] = rS * w[r];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                acc[j * ACCW] = fmaf(p[j], rS, acc[j * ACCW]);
#pragma unroll
                for (int r = 0; r < D; ++r) acc[j * ACCW + 1 + r] = fmaf(p[j], rw[r], acc[j * ACCW + 1 + r]);
            }
            return;
        }
        float gs[D];
#pragma unroll
        for (int r = 0; r < D; ++r) gs[r] = USE_G ? g[r] * a.inv_tau : 0.f;
        float at[K], df[K][D], ri[K];
        estep_small<K, D, DIST, BACK>(w, c, a.nscale, a.escale, at, df, ri);

        if (STATS) {
#pragma unroll
            for (int j = 0; j < K; ++j) {
                acc[j * ACCW] += at[j];
#pragma unroll
                for (int r = 0; r < D; ++r) acc[j * ACCW + 1 + r] = fmaf(at[j], w[r], acc[j * ACCW + 1 + r]);
            }
        }
        if (PASS == PASS_FIN) {
            if (a.Wq_out) {
                float wq[D];
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    float s = 0.f;
#pragma unroll
                    for (int j = 0; j < K; ++j) s = fmaf(at[j], c[j][r], s);
                    wq[r] = s;
                }
                VecLoad<D>::store(a.Wq_out, i, wq);
            }
            if (a.A_out) {
#pragma unroll
                for (int j = 0; j < K; ++j) a.A_out[i * K + j] = at[j];
            }
            if (a.assign_out) {
                // closest codeword decided on a float32 key with separately rounded operations
                int best = 0;
                float bk = 0.f;
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    float key;
                    if (D == 1) {
                        key = fabsf(df[j][0]);
                    } else {
                        key = sum_sq_unfused<D>(df[j]);
                    }
                    if (j == 0 || key < bk) {
                        bk = key;
                        best = j;
                    }
                }
                a.assign_out[i] = best;
            }
        }
        if (BACK) {
            // q_j = (G_i . c_j)/tau [loss through A C]  +  (h_j/tau) . (w_i - F_j) [through F]
            float q[K], qbar = 0.f;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                float s = 0.f;
                if constexpr (FOLD_HF) {
                    s = -ff[j][0];
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        if (USE_G) s = fmaf(gs[r], c[j][r], s);
                        s = fmaf(hs[j][r], w[r] - ff[r][1], s);  // (w - mu: the same for every j, formed once)
                    }
                    q[j] = s;
                    qbar = fmaf(at[j], s, qbar);
                    continue;
                }
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    if (USE_G) s = fmaf(gs[r], c[j][r], s);
                    if (USE_H) s = fmaf(hs[j][r], w[r] - ff[j][r], s);
                }
                q[j] = s;
                qbar = fmaf(at[j], s, qbar);
            }
            if (PASS == PASS_BJ) {
                // explicit Jacobian terms: x_ls = a_l delta_l,s ; y_jr = (w_r - F_jr) a_j
                float x[K][D], wf[K][D];
#pragma unroll
                for (int j = 0; j < K; ++j)
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        x[j][r] = at[j] * delta_small<K, D, DIST>(df, ri, j, r);
                        wf[j][r] = w[r] - ff[j][r];
                    }
#pragma unroll
                for (int j = 0; j < K; ++j)
#pragma unroll
                    for (int r = 0; r < D; ++r) {
                        const float y = wf[j][r] * at[j];
                        const int row = j * D + r;
#pragma unroll
                        for (int l = 0; l < K; ++l)
#pragma unroll
                            for (int s2 = 0; s2 < D; ++s2)
                                acc[row * KD + l * D + s2] = fmaf(y, x[l][s2], acc[row * KD + l * D + s2]);
#pragma unroll
                        for (int s2 = 0; s2 < D; ++s2)
                            acc[KD * KD + row * D + s2] = fmaf(wf[j][r], x[j][s2], acc[KD * KD + row * D + s2]);
                    }
            }
            constexpr int VOFF = (PASS == PASS_BJ) ? KD * KD + KD * D : 0;
            float out[D];
#pragma unroll
            for (int r = 0; r < D; ++r) out[r] = 0.f;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const float th = at[j] * (q[j] - qbar);
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    const float dl = delta_small<K, D, DIST>(df, ri, j, r);
                    if (PASS == PASS_B3) {
                        // sum_j a_j h_j  -  (1/tau) sum_j theta_j delta_j   (theta already carries 1/tau)
                        out[r] = fmaf(at[j], hs[j][r] * a.tau, out[r]);
                        out[r] = fmaf(-th, dl, out[r]);
                    } else {
                        float t = acc[VOFF + j * ACCW + r];
                        if (PASS == PASS_B1 || PASS == PASS_BJ) t = fmaf(at[j], g[r], t);
                        acc[VOFF + j * ACCW + r] = fmaf(th, dl, t);
                    }
                }
            }
            if (PASS == PASS_B3) VecLoad<D>::store(a.dW_out, i, out);
        }
    }
};

template <int K, int D, int DIST, int PASS>
__global__ __launch_bounds__(WG) void small_pass(const Args a) {
    using Item = SmallItem<K, D, DIST, PASS>;
    constexpr int NACC = Item::NACC;

    if (PASS == PASS_FWD && a.ctrl->done) return;
    if (PASS == PASS_B2 && a.ctrl->b_done) return;
    const unsigned int seq = a.ctrl->launch_seq + 1u;  // stamp of this launch's partial sums

    float c[K][D], hs[K][D], ff[K][D + 1];
#pragma unroll
    for (int j = 0; j < K; ++j)
#pragma unroll
        for (int r = 0; r < D; ++r) {
            c[j][r] = a.Cf[j * D + r];
            hs[j][r] = Item::USE_H ? a.Hs[j * D + r] : 0.f;
            ff[j][r] = Item::USE_F ? a.Ff[j * D + r] : 0.f;
        }
    Item::prepare(a, c, hs, ff);

    float acc[Item::NREG];
#pragma unroll
    for (int q = 0; q < Item::NREG; ++q) acc[q] = 0.f;

    const int64_t base = (int64_t)blockIdx.x * a.vec_per_wg;
    int64_t end = base + a.vec_per_wg;
    if (end > a.m) end = a.m;

#pragma unroll 2
    for (int64_t i = base + threadIdx.x; i < end; i += WG) {
        float w[D], g[D];
        VecLoad<D>::load(a.W, i, w);
        if (Item::USE_G) {
            VecLoad<D>::load(a.G, i, g);
        } else {
#pragma unroll
            for (int r = 0; r < D; ++r) g[r] = 0.f;
        }
        Item::run(a, i, w, g, c, hs, ff, acc);
    }
    Item::finish(a, c, acc);

    if (PASS == PASS_B3) return;

    // workgroup partial, fixed order: the 16 lanes of a row (float32, 16 accumulators at a time), then the 16 rows
    // of the workgroup in float64
    __shared__ float s_part[WG / 16][NACC];
    const int lane = threadIdx.x & 63;
    constexpr int CH = 16;
#pragma unroll
    for (int q0 = 0; q0 < NACC; q0 += CH) {
        float v[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) v[u] = (q0 + u < NACC) ? acc[q0 + u] : 0.f;
        row_sums<CH>(v, lane);
        const int q = q0 + row_sum_index<CH>(lane & 15, 0);
        if (q < NACC) s_part[threadIdx.x >> 4][q] = v[0];
    }
    __syncthreads();
    for (int q = threadIdx.x; q < NACC; q += WG) {
        double s = 0.0;
#pragma unroll
        for (int r = 0; r < WG / 16; ++r) s += (double)s_part[r][q];
        // row = accumulator, column = workgroup: the reducing workgroup reads 64 consecutive words per load
        st_word(reinterpret_cast<unsigned long long*>(a.partials) + (size_t)q * gridDim.x + blockIdx.x, pack_f(seq, (float)s));
    }
    grid_tail<PASS, NACC>(a, seq);
}

}  // namespace idkm
