// Matrix-core form of the forward loop for d = 4 (lane<->codeword family, k <= 256), written for the squared energy;
// the plain norm takes the square root of the same product.
//
// In scaled coordinates t = s (w - c), s^2 = log2(e)/tau, the exponent of a weight of the row softmax
// (Eq. "aterms") is  x_ij = -|t_ij|^2 = -s^2|w_i|^2 + 2 s^2 w_i.c_j - s^2|c_j|^2 :  a 16 x 16 tile of it is one
// v_mfma_f32_16x16x4_f32 (the inner dimension is d = 4), with the vectors' squared norms as its additive operand and
// the codewords' added to the result.  The three terms cancel, so w and c are first moved by a common reference
// point mu inside the data (the mean of the initial codewords; the energy does not change): the rounding error of
// x is then a few float32 ulps of s^2 times the squared spread of the data, not of its distance from the origin.
// The first-moment sums of the M-step (Eq. "centers"),  s_j = sum_i a_ij w_i,  are outer products a_i (x) w_i:
// v_mfma_f32_4x4x1 takes sixteen of them (4 codewords x 4 coordinates each) per instruction.  What stays on the
// vector ALU per (vector, codeword) pair is the additive operand, exp2, the row sum and the mass n_j: 5 issue
// slots instead of about 19.
//
// Operand layouts (lane l of the wavefront, q = l / 16):
//   16x16x4:  A[i][kk] in lane i + 16 kk,  B[kk][j] in lane j + 16 kk,  D[i][j] in lane j + 16 (i / 4), register i % 4
//   4x4x1  :  block = l / 4:  A[i] in lane 4 block + i,  B[j] in lane 4 block + j,  D[i][j] in lane 4 block + j, register i
// so a lane that holds the weights of codeword 16 b + l % 16 for vectors 4 q + r (register r of the first product)
// feeds register r straight into the second as the A operand of block l / 4, whose B operand is coordinate l % 4 of
// vector 4 q + r.
#pragma once
#include "common.hpp"

namespace idkm {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_f<0xB1, 0xf>(0.f, x);   // quad_perm [1,0,3,2]
    x += dpp_f<0x4E, 0xf>(0.f, x);   // quad_perm [2,3,0,1]
    x += dpp_f<0x141, 0xf>(0.f, x);  // row_half_mirror
    x += dpp_f<0x140, 0xf>(0.f, x);  // row_mirror
    return x;                        // every lane of the row holds the row's total
}
__device__ __forceinline__ float row16_min(float x) {
    const float pinf = __builtin_inff();
    x = fminf(x, dpp_f<0xB1, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x4E, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x141, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x140, 0xf>(pinf, x));
    return x;
}
__device__ __forceinline__ float row16_max(float x) {
    const float ninf = -__builtin_inff();
    x = fmaxf(x, dpp_f<0xB1, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x4E, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x141, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x140, 0xf>(ninf, x));
    return x;
}

// Per-wavefront state of one forward pass: NB = 4 KPL blocks of 16 codewords.
//
// FOLD (chosen per pass, when s^2 |c_j - mu|^2 <= 100 for every codeword): the codeword's norm is not added to the
// exponent; the loop works with p'_ij = exp2(x_ij + s^2|c_j - mu|^2) <= 2^100 and the factor 2^(-s^2|c_j - mu|^2)
// of codeword j multiplies its term of the row sum (an FMA in place of the add) and, once per pass, its accumulators.
template <int KPL>
struct MfmaFwd {
    static constexpr int NB = 4 * KPL;
    static constexpr int TAB_STRIDE = 16 * NB + 16;  // entries per coordinate; the pad of 128 bytes spreads the four
                                                     // lane groups of a wavefront over different LDS banks
    static constexpr float FOLD_LIMIT = 100.f;
    f32x4 sacc[NB];  // first moments: register i = codeword 16 b + 4 ((l / 4) % 4) + i, coordinate l % 4, partial over q
    float nacc[NB];  // masses: codeword 16 b + l % 16, partial over q
    // codeword operands of the energy product, in LDS (they are the same for every step, and 32 registers more per
    // lane would not fit): entry 16 b of `tab` = {2 s (c_j - mu)[l / 16], -s^2 |c_j - mu|^2}, j = 16 b + l % 16;
    // entry 16 b of `fac` = 2^(-s^2 |c_j - mu|^2)
    const float2* tab;
    const float* fac;
    float mu_q;  // coordinate l / 16 of the reference point

    __device__ __forceinline__ void init(const float2* s_tab, const float* s_fac, const float* s_mu) {
        const int lane = threadIdx.x & 63;
        tab = s_tab + (lane >> 4) * TAB_STRIDE + (lane & 15);
        fac = s_fac + (lane & 15);
        mu_q = s_mu[lane >> 4];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            nacc[b] = 0.f;
            sacc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // The tables for init(): s_tab[kk][j], s_fac[j] for the 16 NB (padded) codewords; a padding codeword sits at
    // -1e30, so its weight is exactly zero.  Called by the whole workgroup (NT threads), with a barrier inside;
    // returns whether the pass may fold the codewords' norms.
    template <int NT>
    static __device__ __forceinline__ bool fill_table(float2* s_tab, float* s_fac, int k, const float* Cf,
                                                      const float* s_mu, float escale) {
        int too_far = 0;
        for (int idx = threadIdx.x; idx < 4 * TAB_STRIDE; idx += NT) {
            const int kk = idx / TAB_STRIDE, j = idx - kk * TAB_STRIDE;
            float2 e = {0.f, -1e30f};
            if (j < k) {
                float n2 = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float c = (Cf[j * 4 + r] - s_mu[r]) * escale;
                    n2 = fmaf(c, c, n2);
                }
                e.x = 2.f * escale * (Cf[j * 4 + kk] - s_mu[kk]);
                e.y = -n2;
                if (!(n2 <= FOLD_LIMIT)) too_far = 1;
            }
            s_tab[idx] = e;
            if (kk == 0) s_fac[j] = fast_exp2(e.y);
        }
        return __syncthreads_or(too_far) == 0;
    }

    // Vectors v0 .. v0+15 of the tile (s_w: [.][4] float32, s_wn: -s^2|w - mu|^2 per vector); those at or beyond vend
    // contribute nothing.  Both arrays are readable (finite values) up to index v0 + 15.
    // DIST_L2 (s = log2(e)/tau): the energy is the square root of the same product, exp(-e/tau) = exp2(-|t|); rows
    // underflow routinely there (|t| is large at small tau), so the row is always shifted by its minimum.
    //
    // WQ (the evaluation at C*): the step also writes the soft-quantised vectors of Eq. "softquant",
    // Wq_i = sum_j a_ij c_j = mu + (1/S_i) sum_j p'_ij f_j (c_j - mu)  (ctab: entry 16 b = f_j (c_j - mu), f_j the fold
    // factor or 1; smu: mu): the sum over codewords runs over the lane's registers and then over the 16 lanes of its
    // DPP row, and lane l % 16 = 4 r + c stores coordinate c of vector v0 + 4 (l / 16) + r (wq: the tile's share of
    // the output, [.][4] in memory).
    template <int DIST, bool FOLD, bool WQ = false>
    __device__ __forceinline__ void step(const float* s_w, const float* s_wn, int v0, int vend, float escale,
                                         const f32x4* ctab = nullptr, const float* smu = nullptr, float* wq = nullptr) {
        static_assert(DIST == DIST_SQL2 || !FOLD, "the fold factors belong to the squared energy");
        const int lane = threadIdx.x & 63, j0 = lane & 15, q = lane >> 4;
        // the table entries are read anew in every step (kept in registers across steps they would spill)
        asm volatile("" ::: "memory");
        const float aw = (s_w[(v0 + j0) * 4 + q] - mu_q) * escale;
        const f32x4 wn = *reinterpret_cast<const f32x4*>(&s_wn[v0 + 4 * q]);
        // the vectors' norms enter as the additive operand (one register quad for all blocks); the products are
        // issued back to back (see the note on the M-step below)
        // All operands of a group are fetched from LDS before the group starts (the scheduling barriers keep the
        // loads from sinking between the matrix instructions, where each would stall the pipeline for its latency):
        // first the codeword coordinates, then -- in flight while the products run -- the per-codeword term of the
        // next group (the fold factor, or the norm).
        float x[NB][4], cterm[NB];
        auto products = [&](bool want_norms) {
            float cbv[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) cbv[b] = tab[16 * b].x;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) cterm[b] = want_norms ? tab[16 * b].y : fac[16 * b];
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, cbv[b], wn, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] = e[b][r];
            }
        };
        auto add_norms = [&]() {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] += cterm[b];
            }
        };
        // weights (up to the fold factor, in cterm) from exponents in x, and their row sums
        float S[4];
        auto weights = [&](const float (&shift)[4]) {
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    x[b][r] = fast_exp2(x[b][r] - shift[r]);
                    S[r] = FOLD ? fmaf(x[b][r], cterm[b], S[r]) : S[r] + x[b][r];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = row16_sum(S[r]);
        };
        // exp2 of a non-positive number cannot overflow (folded: of a number <= FOLD_LIMIT); the row shift of the
        // softmax is only needed when the whole row underflows (a vector many kernel widths from every codeword),
        // which the unshifted row sum shows
        products(!FOLD);
        if (!FOLD) add_norms();
        if (DIST == DIST_L2) {
            // x = -|t|^2 up to rounding (it may come out slightly positive next to a codeword: |.| is a free source
            // modifier); a padding codeword is 1e15 away
            float mn[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) mn[r] = __builtin_inff();
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    x[b][r] = fast_sqrt(fabsf(x[b][r]));
                    mn[r] = fminf(mn[r], x[b][r]);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                mn[r] = row16_min(mn[r]);
                S[r] = 0.f;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    x[b][r] = fast_exp2(mn[r] - x[b][r]);
                    S[r] += x[b][r];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = row16_sum(S[r]);
        }
        const float zero[4] = {0.f, 0.f, 0.f, 0.f};
        if (DIST == DIST_SQL2) weights(zero);
        bool under = false;
#pragma unroll
        for (int r = 0; r < 4; ++r) under = under || (S[r] < 7.9e-31f);  // below 2^-100
        if (DIST == DIST_SQL2 && __builtin_amdgcn_ballot_w64(under) != 0ull) {
            // the row maximum of the full exponent; folded, the shifted exponent again stays below FOLD_LIMIT
            products(true);
            add_norms();
            float mx[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                mx[r] = x[0][r];
#pragma unroll
                for (int b = 1; b < NB; ++b) mx[r] = fmaxf(mx[r], x[b][r]);
                mx[r] = row16_max(mx[r]);
            }
            if (FOLD) products(false);
            weights(mx);
        }
        // the normalisation 1/S_i joins the vector (first moments) and the mass FMA
        float rinv[4], bw[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = v0 + 4 * q + r;
            rinv[r] = (v < vend) ? fast_rcp(S[r]) : 0.f;
            bw[r] = s_w[v * 4 + (lane & 3)] * rinv[r];
        }
        if constexpr (WQ) {
            float out[4][4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) out[r][c] = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const f32x4 cj = ctab[16 * b];
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) out[r][c] = fmaf(x[b][r], cj[c], out[r][c]);
            }
            float mine = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float t = fmaf(row16_sum(out[r][c]), rinv[r], smu[c]);
                    if (j0 == 4 * r + c) mine = t;
                }
            }
            const int v = v0 + 4 * q + (j0 >> 2);
            if (v < vend) wq[(size_t)v * 4 + (j0 & 3)] = mine;
        }
        // Matrix and vector instructions do not overlap on this part, and every change from one kind to the other
        // costs a few cycles more: the mass FMAs run as one group, the outer products back to back as another.
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int b = 0; b < NB; ++b) nacc[b] = fmaf(x[b][r], rinv[r], nacc[b]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int b = 0; b < NB; ++b) sacc[b] = __builtin_amdgcn_mfma_f32_4x4x1f32(x[b][r], bw[r], sacc[b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // The table of the WQ step: s_ctab[j] = f_j (c_j - mu).  Whole workgroup; the caller synchronises.
    template <int NT>
    static __device__ __forceinline__ void fill_codeword_table(f32x4* s_ctab, int k, const float* Cf, const float* s_mu,
                                                               const float* s_fac, bool fold) {
        for (int j = threadIdx.x; j < TAB_STRIDE; j += NT) {
            f32x4 c = {0.f, 0.f, 0.f, 0.f};
            if (j < k) {
                const float f = fold ? s_fac[j] : 1.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) c[r] = f * (Cf[j * 4 + r] - s_mu[r]);
            }
            s_ctab[j] = c;
        }
    }
};

// Per-wavefront state of one (dF/dC)^T pass (Eq. "backiter") on the matrix cores; written out for the squared energy.
//
// With h_j = g_j / (tau n_j) (the pass's input, `Hs`), u_ij = h_j.(w_i - F_j), a_ij the row softmax and
// ubar_i = sum_j a_ij u_ij, the pass returns  out_j = sum_i 2 a_ij (u_ij - ubar_i) (w_i - c_j)  (the caller divides by
// tau n_j where needed, as for the vector-ALU pass).  u is a second 16x16x4 product (A: the scaled vectors again,
// B: h_j / s, additive operand -h_j.(F_j - mu) from an LDS table of quads); the sum over i is the same pair of
// accumulations as in the forward loop -- outer products th'_ij (x) (w_i - mu) 2/S_i and a scalar sum th'_ij 2/S_i per
// codeword, th'_ij = p'_ij (u_ij - ubar_i) -- and  out_j = fac_j (sum th' (w - mu) - (c_j - mu) sum th').
template <int KPL>
struct MfmaB2 {
    static constexpr int NB = 4 * KPL;
    static constexpr int TAB_STRIDE = MfmaFwd<KPL>::TAB_STRIDE;
    f32x4 sacc[NB];  // sum th' (w - mu) 2/S: layout as MfmaFwd::sacc
    float tacc[NB];  // sum th' 2/S: layout as MfmaFwd::nacc
    const float2* tab;   // as MfmaFwd::tab
    const float* fac;    // as MfmaFwd::fac
    const float* hsb;    // entry 16 b: h_j[l / 16] / s, j = 16 b + l % 16
    const f32x4* hq;     // entry 16 b: four copies of -h_j.(F_j - mu)
    float mu_q, mu_c;    // coordinates l / 16 and l % 4 of the reference point

    __device__ __forceinline__ void init(const float2* s_tab, const float* s_fac, const float* s_hsb, const f32x4* s_hq,
                                         const float* s_mu) {
        const int lane = threadIdx.x & 63;
        tab = s_tab + (lane >> 4) * TAB_STRIDE + (lane & 15);
        fac = s_fac + (lane & 15);
        hsb = s_hsb + (lane >> 4) * TAB_STRIDE + (lane & 15);
        hq = s_hq + (lane & 15);
        mu_q = s_mu[lane >> 4];
        mu_c = s_mu[lane & 3];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            tacc[b] = 0.f;
            sacc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // Per-pass tables of the cotangent: s_hsb[kk][j] = h_j[kk] / s, s_hq[j] = -h_j.(F_j - mu) four times.  Whole
    // workgroup; the caller synchronises.
    template <int NT>
    static __device__ __forceinline__ void fill_cotangent(float* s_hsb, f32x4* s_hq, int k, const float* Hs,
                                                          const float* Ff, const float* s_mu, float escale) {
        const float inv = 1.0f / escale;
        for (int idx = threadIdx.x; idx < 4 * TAB_STRIDE; idx += NT) {
            const int kk = idx / TAB_STRIDE, j = idx - kk * TAB_STRIDE;
            s_hsb[idx] = (j < k) ? Hs[j * 4 + kk] * inv : 0.f;
            if (kk == 0) {
                float hf = 0.f;
                if (j < k) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) hf = fmaf(Hs[j * 4 + r], Ff[j * 4 + r] - s_mu[r], hf);
                }
                s_hq[j] = f32x4{-hf, -hf, -hf, -hf};
            }
        }
    }

    // DIST_L2 (s = log2(e)/tau): e_ij = sqrt(|x_ij|) in scaled units, the row is shifted by its minimum, and the
    // derivative of the energy is the unit vector (w - c) s / e:  out_j = sum_i a_ij (u_ij - ubar_i) (w_i - c_j) s / e_ij,
    // i.e. th'_ij = p_ij (u_ij - ubar_i) / e_ij with the per-vector factor s / S_i (zero where e_ij = 0 exactly).
    //
    // B1 (first pass of the backward): the same sums with u_ij = (G_i / tau).c_j -- the second product
    // takes A = ag (coordinate l / 16 of G_i / (2 s tau) for vector v0 + l % 16) and the codeword operand of the first
    // -- plus the term sum_i a_ij G_i, a second set of outer products p'_ij (x) G_i / S_i (gb[r]: coordinate l % 4 of
    // G for vector v0 + 4 (l / 16) + r) into the same accumulators:  v_j = fac_j (sacc_j - (c_j - mu) tacc_j).
    template <int DIST, bool FOLD, bool B1 = false>
    __device__ __forceinline__ void step(const float* s_w, const float* s_wn, int v0, int vend, float escale,
                                         float ag = 0.f, const float* gb = nullptr) {
        static_assert(DIST == DIST_SQL2 || !FOLD, "the fold factors belong to the squared energy");
        const int lane = threadIdx.x & 63, j0 = lane & 15, q = lane >> 4;
        asm volatile("" ::: "memory");
        const float aw = (s_w[(v0 + j0) * 4 + q] - mu_q) * escale;
        const f32x4 wn = *reinterpret_cast<const f32x4*>(&s_wn[v0 + 4 * q]);
        float x[NB][4], cterm[NB];
        auto products = [&](bool want_norms) {
            float cbv[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) cbv[b] = tab[16 * b].x;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) cterm[b] = want_norms ? tab[16 * b].y : fac[16 * b];
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, cbv[b], wn, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] = e[b][r];
            }
        };
        auto add_norms = [&]() {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] += cterm[b];
            }
        };
        float S[4];
        auto weights = [&](const float (&shift)[4]) {
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    x[b][r] = fast_exp2(x[b][r] - shift[r]);
                    S[r] = FOLD ? fmaf(x[b][r], cterm[b], S[r]) : S[r] + x[b][r];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = row16_sum(S[r]);
        };
        // u_ij (second product) into u
        float u[NB][4];
        auto cotangent_product = [&]() {
            float hv[NB];
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                hv[b] = B1 ? tab[16 * b].x : hsb[16 * b];
                e[b] = B1 ? f32x4{0.f, 0.f, 0.f, 0.f} : hq[16 * b];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                if (FOLD) cterm[b] = fac[16 * b];  // again: the rare path may have left norms there
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(B1 ? ag : aw, hv[b], e[b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) u[b][r] = e[b][r];
            }
        };
        float Q[4] = {0.f, 0.f, 0.f, 0.f};
        float pwv[(B1 && DIST == DIST_L2) ? NB : 1][4];  // plain norm, first pass: the weights p
        products(!FOLD);
        if (!FOLD) add_norms();
        if constexpr (DIST == DIST_SQL2) {
            const float zero[4] = {0.f, 0.f, 0.f, 0.f};
            weights(zero);
            bool under = false;
#pragma unroll
            for (int r = 0; r < 4; ++r) under = under || (S[r] < 7.9e-31f);  // below 2^-100
            if (__builtin_amdgcn_ballot_w64(under) != 0ull) {
                products(true);
                add_norms();
                float mx[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    mx[r] = x[0][r];
#pragma unroll
                    for (int b = 1; b < NB; ++b) mx[r] = fmaxf(mx[r], x[b][r]);
                    mx[r] = row16_max(mx[r]);
                }
                if (FOLD) products(false);
                weights(mx);
            }
            cotangent_product();
            // p' u in place of u, and the row sums Q_i = sum_j fac_j p'_ij u_ij
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    u[b][r] *= x[b][r];
                    Q[r] = FOLD ? fmaf(u[b][r], cterm[b], Q[r]) : Q[r] + u[b][r];
                }
            }
        } else {
            // energies and the row minimum; a padding codeword is 1e15 away
            float mn[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) mn[r] = __builtin_inff();
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    x[b][r] = fast_sqrt(fabsf(x[b][r]));
                    mn[r] = fminf(mn[r], x[b][r]);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                mn[r] = row16_min(mn[r]);
                S[r] = 0.f;
            }
            cotangent_product();
            // weights p, row sums S and Q = sum p u; then p / e in place of the energy and p u / e in place of u
            // (the first pass needs the weights themselves as well, for sum_i a_ij G_i)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float e = x[b][r];
                    const float pw = fast_exp2(mn[r] - e);
                    const float ri = (e > 0.f) ? fast_rcp(e) : 0.f;
                    const float pu = pw * u[b][r];
                    S[r] += pw;
                    Q[r] += pu;
                    x[b][r] = pw * ri;
                    u[b][r] = pu * ri;
                    if (B1) pwv[b][r] = pw;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = row16_sum(S[r]);
        }
        float r2[4], nub[4], bw[4], gw[4];
        const float vfac = (DIST == DIST_SQL2) ? 2.f : escale;  // d e / d w = 2 (w - c), resp. (w - c) s / e_scaled
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = v0 + 4 * q + r;
            const float rS = (v < vend) ? fast_rcp(S[r]) : 0.f;
            nub[r] = -(row16_sum(Q[r]) * rS);  // -ubar_i
            r2[r] = vfac * rS;
            bw[r] = (s_w[v * 4 + (lane & 3)] - mu_c) * r2[r];
            gw[r] = B1 ? gb[r] * rS : 0.f;
        }
        if constexpr (B1) {
            // sum_i a_ij G_i: the weights are still untouched in x (plain norm: kept aside in pwv)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    sacc[b] = __builtin_amdgcn_mfma_f32_4x4x1f32(DIST == DIST_L2 ? pwv[b][r] : x[b][r], gw[r], sacc[b], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                u[b][r] = fmaf(nub[r], x[b][r], u[b][r]);  // th' = p' u - ubar p'  (plain norm: both over e)
                tacc[b] = fmaf(u[b][r], r2[r], tacc[b]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int b = 0; b < NB; ++b) sacc[b] = __builtin_amdgcn_mfma_f32_4x4x1f32(u[b][r], bw[r], sacc[b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
};

// The last pass of the backward on the matrix cores (written out for the squared energy; step_l2 is the plain norm):
//   dL/dW_i = sum_j a_ij h_j - (1/tau) sum_j (rho_ij + gamma_ij) delta_ij            (Eq. "grad", Alg. 2 backward step)
// With z_ij = (G_i/tau).c_j + (h_j/tau).(w_i - F_j) (two chained 16x16x4 products), kappa_ij = a_ij (z_ij - zbar_i),
// zbar_i = sum_j a_ij z_ij, and delta_ij = 2 (w_i - c_j), the second sum is -2 sum_j kappa_ij (c_j - mu) because
// sum_j kappa_ij = 0:   dL/dW_i = (1/S_i) sum_j fac_j [ p'_ij h_j + kappa'_ij 2 (c_j - mu) ],  kappa' = p' (z - zbar).
// The sum over codewords runs over the registers of a lane (16 blocks) and then over the 16 lanes of its DPP row;
// lane l % 16 = 4 r + c stores coordinate c of vector v0 + 4 (l / 16) + r: one coalesced 256-byte store per step.
template <int KPL>
struct MfmaB3 {
    static constexpr int NB = 4 * KPL;
    static constexpr int TAB_STRIDE = MfmaFwd<KPL>::TAB_STRIDE;
    const float2* tab;
    const float* fac;
    const float* hsb;
    const f32x4* hq;
    const f32x4* hc;  // entry 16 b: fac_j h_j (4 coordinates); entry TAB_STRIDE + 16 b: fac_j 2 (c_j - mu)
    float mu_q, mu_c;

    __device__ __forceinline__ void init(const float2* s_tab, const float* s_fac, const float* s_hsb, const f32x4* s_hq,
                                         const f32x4* s_hc, const float* s_mu) {
        const int lane = threadIdx.x & 63;
        tab = s_tab + (lane >> 4) * TAB_STRIDE + (lane & 15);
        fac = s_fac + (lane & 15);
        hsb = s_hsb + (lane >> 4) * TAB_STRIDE + (lane & 15);
        hq = s_hq + (lane & 15);
        hc = s_hc + (lane & 15);
        mu_q = s_mu[lane >> 4];
        mu_c = s_mu[lane & 3];
    }
    // s_hc[0][j] = f_j tau Hs_j, s_hc[1][j] = f_j cfac (c_j - mu), f_j the fold factor (1 if the pass does not fold);
    // cfac = 2 for the squared energy, s for the plain norm (d e / d w = 2 (w - c), resp. (w - c) s / e_scaled).
    // Hs = h / tau as everywhere.  Whole workgroup; the caller synchronises.
    template <int NT>
    static __device__ __forceinline__ void fill_output_tables(f32x4* s_hc, int k, const float* Hs, const float* Cf,
                                                              const float* s_mu, const float* s_fac, bool fold, float tau,
                                                              float cfac) {
        for (int j = threadIdx.x; j < TAB_STRIDE; j += NT) {
            f32x4 h = {0.f, 0.f, 0.f, 0.f}, c2 = {0.f, 0.f, 0.f, 0.f};
            if (j < k) {
                const float f = fold ? s_fac[j] : 1.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    h[r] = f * tau * Hs[j * 4 + r];
                    c2[r] = f * cfac * (Cf[j * 4 + r] - s_mu[r]);
                }
            }
            s_hc[j] = h;
            s_hc[TAB_STRIDE + j] = c2;
        }
    }

    // ag: coordinate l / 16 of G_i / (2 s tau) for vector v0 + l % 16 (as in the first pass); dW: the tile's share of
    // the output, [cnt][4] in memory.
    template <bool FOLD>
    __device__ __forceinline__ void step(const float* s_w, const float* s_wn, int v0, int vend, float escale, float ag,
                                         float* dW) {
        const int lane = threadIdx.x & 63, j0 = lane & 15, q = lane >> 4;
        asm volatile("" ::: "memory");
        const float aw = (s_w[(v0 + j0) * 4 + q] - mu_q) * escale;
        const f32x4 wn = *reinterpret_cast<const f32x4*>(&s_wn[v0 + 4 * q]);
        float x[NB][4], cterm[NB];
        auto products = [&](bool want_norms) {
            float cbv[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) cbv[b] = tab[16 * b].x;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) cterm[b] = want_norms ? tab[16 * b].y : fac[16 * b];
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, cbv[b], wn, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] = e[b][r];
            }
        };
        auto add_norms = [&]() {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] += cterm[b];
            }
        };
        float S[4];
        auto weights = [&](const float (&shift)[4]) {
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    x[b][r] = fast_exp2(x[b][r] - shift[r]);
                    S[r] = FOLD ? fmaf(x[b][r], cterm[b], S[r]) : S[r] + x[b][r];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) S[r] = row16_sum(S[r]);
        };
        products(!FOLD);
        if (!FOLD) add_norms();
        const float zero[4] = {0.f, 0.f, 0.f, 0.f};
        weights(zero);
        bool under = false;
#pragma unroll
        for (int r = 0; r < 4; ++r) under = under || (S[r] < 7.9e-31f);  // below 2^-100
        if (__builtin_amdgcn_ballot_w64(under) != 0ull) {
            products(true);
            add_norms();
            float mx[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                mx[r] = x[0][r];
#pragma unroll
                for (int b = 1; b < NB; ++b) mx[r] = fmaxf(mx[r], x[b][r]);
                mx[r] = row16_max(mx[r]);
            }
            if (FOLD) products(false);
            weights(mx);
        }
        // z_ij: h.(w - F) first, (G/tau).(c - mu) accumulated onto it
        float z[NB][4];
        {
            float hv[NB], cbv[NB];
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                hv[b] = hsb[16 * b];
                cbv[b] = tab[16 * b].x;
                e[b] = hq[16 * b];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                if (FOLD) cterm[b] = fac[16 * b];  // again: the rare path may have left norms there
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, hv[b], e[b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(ag, cbv[b], e[b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) z[b][r] = e[b][r];
            }
        }
        float Z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                z[b][r] *= x[b][r];
                Z[r] = FOLD ? fmaf(z[b][r], cterm[b], Z[r]) : Z[r] + z[b][r];
            }
        }
        float rS[4], nzb[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            rS[r] = fast_rcp(S[r]);
            nzb[r] = -(row16_sum(Z[r]) * rS[r]);  // -zbar_i
        }
        float out[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) out[r][c] = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const f32x4 hj = hc[16 * b], cj = hc[TAB_STRIDE + 16 * b];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float kap = fmaf(nzb[r], x[b][r], z[b][r]);  // kappa' = p' z - zbar p'
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    out[r][c] = fmaf(x[b][r], hj[c], out[r][c]);
                    out[r][c] = fmaf(kap, cj[c], out[r][c]);
                }
            }
        }
        // over the 16 lanes of the row, then lane 4 r + c keeps (r, c)
        float mine = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float t = row16_sum(out[r][c]) * rS[r];
                if (j0 == 4 * r + c) mine = t;
            }
        }
        const int v = v0 + 4 * q + (j0 >> 2);
        if (v < vend) dW[(size_t)v * 4 + (j0 & 3)] = mine;
    }

    // The same pass for the plain norm (s = log2(e)/tau): e_ij = sqrt(|x_ij|) in scaled units, the row is shifted by
    // its minimum, delta_ij = (w_i - c_j) s / e_ij (zero where e_ij = 0 exactly), and sum_j kappa_ij / e_ij does not
    // vanish, so the term in (w_i - mu) stays:
    //   dL/dW_i = (1/S_i) [ sum_j p_ij h_j + s sum_j k_ij (c_j - mu) - s (w_i - mu) sum_j k_ij ],
    //   k_ij = p_ij (z_ij - zbar_i) / e_ij.
    __device__ __forceinline__ void step_l2(const float* s_w, const float* s_wn, int v0, int vend, float escale, float ag,
                                            float* dW) {
        const int lane = threadIdx.x & 63, j0 = lane & 15, q = lane >> 4;
        asm volatile("" ::: "memory");
        const float aw = (s_w[(v0 + j0) * 4 + q] - mu_q) * escale;
        const f32x4 wn = *reinterpret_cast<const f32x4*>(&s_wn[v0 + 4 * q]);
        float x[NB][4];
        {
            float cbv[NB], cn[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) cbv[b] = tab[16 * b].x;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) cn[b] = tab[16 * b].y;
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, cbv[b], wn, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            // energies; a padding codeword is 1e15 away
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) x[b][r] = fast_sqrt(fabsf(e[b][r] + cn[b]));
            }
        }
        float mn[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            mn[r] = x[0][r];
#pragma unroll
            for (int b = 1; b < NB; ++b) mn[r] = fminf(mn[r], x[b][r]);
            mn[r] = row16_min(mn[r]);
        }
        // z_ij: h.(w - F) first, (G/tau).(c - mu) accumulated onto it
        float z[NB][4];
        {
            float hv[NB], cbv[NB];
            f32x4 e[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                hv[b] = hsb[16 * b];
                cbv[b] = tab[16 * b].x;
                e[b] = hq[16 * b];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, hv[b], e[b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NB; ++b) e[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(ag, cbv[b], e[b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int r = 0; r < 4; ++r) z[b][r] = e[b][r];
            }
        }
        float out[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) out[r][c] = 0.f;
        // weights p, row sums S and Z = sum p z, the term sum_j p h_j; then p / e in place of the energy and p z / e
        // in place of z
        float S[4] = {0.f, 0.f, 0.f, 0.f}, Z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const f32x4 hj = hc[16 * b];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float e = x[b][r];
                const float pw = fast_exp2(mn[r] - e);
                const float ri = (e > 0.f) ? fast_rcp(e) : 0.f;
                const float pz = pw * z[b][r];
                S[r] += pw;
                Z[r] += pz;
#pragma unroll
                for (int c = 0; c < 4; ++c) out[r][c] = fmaf(pw, hj[c], out[r][c]);
                x[b][r] = pw * ri;
                z[b][r] = pz * ri;
            }
        }
        float rS[4], nzb[4], K[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            rS[r] = fast_rcp(row16_sum(S[r]));
            nzb[r] = -(row16_sum(Z[r]) * rS[r]);  // -zbar_i
            K[r] = 0.f;
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const f32x4 cj = hc[TAB_STRIDE + 16 * b];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float kap = fmaf(nzb[r], x[b][r], z[b][r]);  // k S = (p z - zbar p) / e
                K[r] += kap;
#pragma unroll
                for (int c = 0; c < 4; ++c) out[r][c] = fmaf(kap, cj[c], out[r][c]);
            }
        }
        // over the 16 lanes of the row, then lane 4 r + c keeps (r, c)
        float mine = 0.f, Kmine = 0.f, rSmine = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float Ks = row16_sum(K[r]);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float t = row16_sum(out[r][c]);
                if (j0 == 4 * r + c) {
                    mine = t;
                    Kmine = Ks;
                    rSmine = rS[r];
                }
            }
        }
        const int v = v0 + 4 * q + (j0 >> 2);
        if (v < vend) {
            const float wc = (s_w[v * 4 + (j0 & 3)] - mu_c) * escale;
            dW[(size_t)v * 4 + (j0 & 3)] = fmaf(-wc, Kmine, mine) * rSmine;
        }
    }
};

template <int KPL, int DIST, int NT>
__device__ __forceinline__ void mfma_b3_tile_pass(MfmaB3<KPL>& st, const float* s_w, const float* s_wn, const float* gG,
                                                  float* dW, int cnt, float escale, float inv_tau, bool fold) {
    constexpr int NW = NT / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = lane & 15, q = lane >> 4;
    int share = (cnt + NW - 1) / NW;
    share = (share + 15) & ~15;
    const int w0 = wave * share;
    const int w1 = (w0 + share < cnt) ? w0 + share : cnt;
    const float gscale = inv_tau / (2.f * escale);
    auto fetch = [&](int v) { return (v + j0 < cnt) ? gG[(size_t)(v + j0) * 4 + q] * gscale : 0.f; };
    float ag = (w0 < w1) ? fetch(w0) : 0.f;
    for (int v = w0; v < w1; v += 16) {
        const float ag_n = (v + 16 < w1) ? fetch(v + 16) : 0.f;
        if constexpr (DIST == DIST_L2)
            st.step_l2(s_w, s_wn, v, w1, escale, ag, dW);
        else if (fold)
            st.template step<true>(s_w, s_wn, v, w1, escale, ag, dW);
        else
            st.template step<false>(s_w, s_wn, v, w1, escale, ag, dW);
        ag = ag_n;
    }
}

template <int KPL, int DIST, int NT>
__device__ __forceinline__ void mfma_b2_tile_pass(MfmaB2<KPL>& st, const float* s_w, const float* s_wn, int cnt,
                                                  float escale, bool fold) {
    constexpr int NW = NT / 64;
    const int wave = threadIdx.x >> 6;
    int share = (cnt + NW - 1) / NW;
    share = (share + 15) & ~15;
    const int w0 = wave * share;
    const int w1 = (w0 + share < cnt) ? w0 + share : cnt;
    if (DIST == DIST_SQL2 && fold) {
        for (int v = w0; v < w1; v += 16) st.template step<DIST_SQL2, true>(s_w, s_wn, v, w1, escale);
    } else {
        for (int v = w0; v < w1; v += 16) st.template step<DIST, false>(s_w, s_wn, v, w1, escale);
    }
}

// The first pass of the backward: G (the workgroup's share of dL/dWq, [cnt][4] in memory) is read
// one step ahead, so that its latency is hidden behind the current step.
template <int KPL, int DIST, int NT>
__device__ __forceinline__ void mfma_b1_tile_pass(MfmaB2<KPL>& st, const float* s_w, const float* s_wn, const float* gG,
                                                  int cnt, float escale, float inv_tau, bool fold) {
    constexpr int NW = NT / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = lane & 15, q = lane >> 4, col = lane & 3;
    int share = (cnt + NW - 1) / NW;
    share = (share + 15) & ~15;
    const int w0 = wave * share;
    const int w1 = (w0 + share < cnt) ? w0 + share : cnt;
    const float gscale = inv_tau / (2.f * escale);
    auto fetch = [&](int v, float& ag, float (&gb)[4]) {
        ag = (v + j0 < cnt) ? gG[(size_t)(v + j0) * 4 + q] * gscale : 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) gb[r] = (v + 4 * q + r < cnt) ? gG[(size_t)(v + 4 * q + r) * 4 + col] : 0.f;
    };
    float ag = 0.f, gb[4] = {0.f, 0.f, 0.f, 0.f}, ag_n = 0.f, gb_n[4] = {0.f, 0.f, 0.f, 0.f};
    if (w0 < w1) fetch(w0, ag, gb);
    for (int v = w0; v < w1; v += 16) {
        if (v + 16 < w1) fetch(v + 16, ag_n, gb_n);
        if (DIST == DIST_SQL2 && fold)
            st.template step<DIST_SQL2, true, true>(s_w, s_wn, v, w1, escale, ag, gb);
        else
            st.template step<DIST, false, true>(s_w, s_wn, v, w1, escale, ag, gb);
        ag = ag_n;
#pragma unroll
        for (int r = 0; r < 4; ++r) gb[r] = gb_n[r];
    }
}

// Wavefront totals of the accumulators as float32 in s_part[NT / 64][64 KPL 5], word (codeword, sum th' | sum th' (w - mu)_r),
// without the fold factor (the caller applies it together with the codeword term).
template <int KPL, int NT>
__device__ __forceinline__ void mfma_b2_collect(const MfmaB2<KPL>& st, float* s_part) {
    constexpr int NB = 4 * KPL, ROW = 64 * KPL * 5;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, j0 = lane & 15, t = (lane >> 2) & 3, col = lane & 3;
    float* out = s_part + wave * ROW;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        float n = st.tacc[b];
        n += __shfl_xor(n, 16);
        n += __shfl_xor(n, 32);
        float s[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[i] = st.sacc[b][i];
            s[i] += __shfl_xor(s[i], 16);
            s[i] += __shfl_xor(s[i], 32);
        }
        if (q == 0) {
            out[(16 * b + j0) * 5] = n;
#pragma unroll
            for (int i = 0; i < 4; ++i) out[(16 * b + 4 * t + i) * 5 + 1 + col] = s[i];
        }
    }
}

// One forward pass over the workgroup's tile: every wavefront takes an equal share of whole 16-vector steps.
template <int KPL, int DIST, int NT, bool WQ = false>
__device__ __forceinline__ void mfma_tile_pass(MfmaFwd<KPL>& st, const float* s_w, const float* s_wn, int cnt,
                                               float escale, bool fold, const f32x4* s_ctab = nullptr,
                                               const float* s_mu = nullptr, float* wq = nullptr) {
    constexpr int NW = NT / 64;
    const int wave = threadIdx.x >> 6;
    int share = (cnt + NW - 1) / NW;
    share = (share + 15) & ~15;
    const int w0 = wave * share;
    const int w1 = (w0 + share < cnt) ? w0 + share : cnt;
    const f32x4* ctab = WQ ? s_ctab + (threadIdx.x & 15) : nullptr;
    if (DIST == DIST_SQL2 && fold) {
        for (int v = w0; v < w1; v += 16) st.template step<DIST_SQL2, true, WQ>(s_w, s_wn, v, w1, escale, ctab, s_mu, wq);
    } else {
        for (int v = w0; v < w1; v += 16) st.template step<DIST, false, WQ>(s_w, s_wn, v, w1, escale, ctab, s_mu, wq);
    }
}

// Workgroup totals of the accumulators as float32 per wavefront in s_part[NT / 64][64 KPL 5], word (codeword, n | s_r).
// fold: the accumulators still lack the factor of their codeword (s_fac).
template <int KPL, int NT>
__device__ __forceinline__ void mfma_collect(const MfmaFwd<KPL>& st, float* s_part, bool fold, const float* s_fac) {
    constexpr int NB = 4 * KPL, ROW = 64 * KPL * 5;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, j0 = lane & 15, t = (lane >> 2) & 3, col = lane & 3;
    float* out = s_part + wave * ROW;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        // the four lane groups q hold partial sums over different vectors: fixed order (q, q^1), then (., q^2)
        float n = st.nacc[b];
        n += __shfl_xor(n, 16);
        n += __shfl_xor(n, 32);
        float s[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[i] = st.sacc[b][i];
            s[i] += __shfl_xor(s[i], 16);
            s[i] += __shfl_xor(s[i], 32);
        }
        if (q == 0) {
            out[(16 * b + j0) * 5] = fold ? n * s_fac[16 * b + j0] : n;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = 16 * b + 4 * t + i;
                out[j * 5 + 1 + col] = fold ? s[i] * s_fac[j] : s[i];
            }
        }
    }
}

}  // namespace idkm
