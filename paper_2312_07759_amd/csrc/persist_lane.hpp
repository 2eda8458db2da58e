// Persistent kernels for the lane<->codeword family (k up to 512): one launch per
// solve, the workgroup's tile of W (and dL/dWq) resident in LDS, the same two-hop
// stamped exchange as the small-codebook kernels, with one reducer per codeword:
//   hop 1  workgroup g stores its k (d+1) partial sums contiguously at buf1[parity][g][.];
//          the reducer of codeword r (workgroup r mod G) reads that codeword's d+1
//          words from every workgroup, adds them in float64 in a fixed order and
//          updates its codeword;
//   hop 2  reducers store the float32 codeword (or h/tau) and a partial squared
//          norm into buf2; every workgroup reads the k d + k words.
// Waits are bounded exactly as in persist_small.hpp.
#pragma once
#include "common.hpp"
#include "lane_k.hpp"
#include "mfma_lane.hpp"
#include "persist_small.hpp"

namespace idkm {

constexpr int LT = 1024;          // threads per workgroup (16 wavefronts, 4 per SIMD)
constexpr int LWAVES = LT / 64;
constexpr int MT = 512;           // threads per workgroup of the matrix-core forward kernel (2 wavefronts per SIMD:
                                  // its accumulators and one 16 x 256 tile of weights need ~200 registers per lane)

struct LShared {
    float red[8][PT];     // reducer: one codeword's words of every workgroup (at most PT workgroups)
    double tot[8];
    double wsum[LWAVES];
    double scalar;        // result of block_sum
    int abort;
};

// Waits for `n` stamped words starting at src (strided by `stride` words, one per thread) -- helper for both hops.
__device__ __forceinline__ bool poll_word(const PArgs& pa, const unsigned long long* src, unsigned int seq,
                                          unsigned int* payload) {
    unsigned int spins = 0;
    for (;;) {
        const unsigned long long w = ld_word(src);
        if ((unsigned int)(w >> 32) == seq) {
            *payload = (unsigned int)w;
            return true;
        }
        ++spins;
        if (spins > pa.spin_limit ||
            ((spins & 31u) == 0u &&
             __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u))
            return false;
    }
}

__device__ __forceinline__ void raise_abort(const PArgs& pa, LShared& ls) {
    ls.abort = 1;
    __hip_atomic_store(pa.abort_word, pa.seq_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sum of one float64 per thread over the workgroup, fixed order, returned to every thread.
template <int NT = LT>
__device__ __forceinline__ double block_sum_fixed(double x, LShared& ls) {
    x = wave_sum_d_dpp(x);
    if ((threadIdx.x & 63) == 0) ls.wsum[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) s += ls.wsum[w];
        ls.scalar = s;
    }
    __syncthreads();
    return ls.scalar;
}

// Workgroup partial of the lane accumulators (wavefronts add one after the other, float64) and hop-1 store.
template <int NA, int ACCW, int NT = LT>
__device__ __forceinline__ void publish_lane(const PArgs& pa, unsigned int seq, const float (&acc)[NA], int k,
                                             double (*s_acc)[NA]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int wv = 0; wv < NT / 64; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int q = 0; q < NA; ++q) {
                if (wv == 0)
                    s_acc[lane][q] = (double)acc[q];
                else
                    s_acc[lane][q] += (double)acc[q];
            }
        }
        __syncthreads();
    }
    const int nacc = k * ACCW;
    unsigned long long* dst = pa.buf1 + ((size_t)(seq & 1u) * pa.G + pa.wg) * nacc;
    for (int idx = tid; idx < nacc; idx += NT) {
        const int j = idx / ACCW, comp = idx - j * ACCW;
        st_word(&dst[idx], pack_f(seq, (float)s_acc[j & 63][(j >> 6) * ACCW + comp]));
    }
}

// Totals over all workgroups of words [first, first+WPR) of every workgroup's hop-1 block into ls.tot.
template <int WPR>
__device__ __forceinline__ bool reduce_lane(const PArgs& pa, unsigned int seq, int nacc, int first, LShared& ls) {
    static_assert(WPR <= 8, "a reducer handles at most 8 words per workgroup");
    const int tid = threadIdx.x;
    const int G = pa.G;
    if (tid < PT) {
        float f[WPR];
#pragma unroll
        for (int q = 0; q < WPR; ++q) f[q] = 0.f;
        if (tid < G) {
            const unsigned long long* src = pa.buf1 + ((size_t)(seq & 1u) * G + tid) * nacc + first;
            unsigned int spins = 0;
            for (;;) {
                unsigned long long w[WPR];
#pragma unroll
                for (int q = 0; q < WPR; ++q) w[q] = ld_word(src + q);
                bool ok = true;
#pragma unroll
                for (int q = 0; q < WPR; ++q) ok = ok && ((unsigned int)(w[q] >> 32) == seq);
                if (ok) {
#pragma unroll
                    for (int q = 0; q < WPR; ++q) f[q] = __uint_as_float((unsigned int)w[q]);
                    break;
                }
                ++spins;
                if (spins > pa.spin_limit ||
                    ((spins & 31u) == 0u &&
                     __hip_atomic_load(pa.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pa.seq_base + 1u)) {
                    raise_abort(pa, ls);
                    break;
                }
            }
        }
#pragma unroll
        for (int q = 0; q < WPR; ++q) ls.red[q][tid] = f[q];
    }
    __syncthreads();
    if (ls.abort) return false;
    if (tid < PT) {
        const int q = tid >> 5, part = tid & 31;
        double s = 0.0;
        if (q < WPR) {
#pragma unroll
            for (int u = 0; u < 8; ++u) s += (double)ls.red[q][part * 8 + u];
        }
        s = half_sum_d_dpp(s);
        if (q < WPR && part == 31) ls.tot[q] = s;
    }
    __syncthreads();
    return true;
}

// hop 2: every thread polls words tid, tid+LT, ... < nwords of buf2 into dst (LDS).
template <int NT = LT>
__device__ __forceinline__ bool gather_lane(const PArgs& pa, unsigned int seq, int nwords, int stride2,
                                            unsigned int* dst, LShared& ls) {
    const unsigned long long* src = pa.buf2 + (size_t)(seq & 1u) * stride2;
    bool ok = true;
    for (int i = threadIdx.x; i < nwords; i += NT) {
        unsigned int p = 0;
        ok = ok && poll_word(pa, src + i, seq, &p);
        dst[i] = p;
    }
    if (!ok) raise_abort(pa, ls);
    __syncthreads();
    return ls.abort == 0;
}

template <int KPL, int D, int DIST, int PASS, int NT = LT>
__device__ __forceinline__ void lane_tile_pass(const Args& a, LaneWave<KPL, D, DIST, PASS>& st, const float* s_w,
                                               const float* s_g, int64_t base, int cnt) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // every wavefront takes an equal contiguous share of the tile
    const int share = (cnt + NT / 64 - 1) / (NT / 64);
    const int w0 = wave * share;
    const int w1 = (w0 + share < cnt) ? w0 + share : cnt;
    for (int b = w0; b < w1; b += 64) {
        float wv[D], gv[D];
        const int i = b + lane;
#pragma unroll
        for (int r = 0; r < D; ++r) {
            wv[r] = (i < w1) ? s_w[i * D + r] : 0.f;
            gv[r] = (LaneWave<KPL, D, DIST, PASS>::USE_G && i < w1) ? s_g[i * D + r] : 0.f;
        }
        st.batch(a, base + b, (w1 - b < 64) ? (w1 - b) : 64, wv, gv);
    }
}

#ifdef IDKM_TRACE
#define IDKM_LSTAMP(slot)                                                                        \
    do {                                                                                         \
        if (pa.trace && threadIdx.x == 0 && s_iters == 20 && pa.wg < 256)                        \
            pa.trace[2 * 64 * 8 + pa.wg * 8 + (slot)] = (long long)wall_clock64();               \
    } while (0)
#else
#define IDKM_LSTAMP(slot)
#endif

// Forward solve (Alg. 1) and the evaluation at C*.  MFMA: the loop's passes run on the matrix cores (mfma_lane.hpp;
// d = 4), with NT = MT threads; the dynamic LDS then holds the tile padded by 16 zero vectors and,
// behind it, -s^2 |w|^2 of every vector.
template <int KPL, int D, int DIST, int NT = LT, bool MFMA = false>
__device__ __forceinline__ void persist_lane_fwd_body(const Args& a, const PArgs& pa) {
    static_assert(!MFMA || (D == 4 && KPL <= 4), "matrix-core loop: d = 4, k <= 256");
    constexpr int ACCW = D + 1;
    constexpr int NA = KPL * ACCW;
    constexpr int KDP = 64 * KPL * D;  // padded codebook size
    extern __shared__ float s_tile[];
    __shared__ double s_acc[64][NA];
    __shared__ LShared ls;
    __shared__ double s_Cd[KDP];  // float64 master copy; the reducer's own codewords are the live ones
    __shared__ float s_Cf[KDP];
    __shared__ unsigned int s_new[KDP + 64 * KPL];
    __shared__ int s_done, s_iters, s_conv, s_bad;
    __shared__ double s_res;

    const int tid = threadIdx.x, wg = pa.wg, G = pa.G;
    const int k = a.k, kd = k * D, nacc = k * ACCW;
    const int stride2 = kd + k;
    const int64_t base = (int64_t)wg * pa.per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < pa.per) ? (int)(a.m - base) : pa.per;
    load_tile<NT>(s_tile, a.W + base * D, cnt * D);
    for (int i = tid; i < kd; i += NT) {
        const float c0 = pa.C0[i];
        s_Cd[i] = (double)c0;
        s_Cf[i] = c0;
    }
    if (tid == 0) {
        ls.abort = 0;
        s_done = 0;
        s_iters = 0;
        s_conv = 0;
        s_bad = 0;
        s_res = 0.0;
    }
    __syncthreads();
    const float* s_wn = s_tile + (size_t)(pa.per + 16) * D;
    __shared__ float s_mu[4];
    if constexpr (MFMA) {
        // reference point of the centred coordinates: the mean of the initial codewords
        if (tid < D) {
            float sm = 0.f;
            for (int j = 0; j < k; ++j) sm += s_Cf[j * D + tid];
            s_mu[tid] = sm / (float)k;
        }
        float* wn = s_tile + (size_t)(pa.per + 16) * D;
        for (int i = cnt * D + tid; i < (pa.per + 16) * D; i += NT) s_tile[i] = 0.f;
        __syncthreads();
        for (int i = tid; i < pa.per + 16; i += NT) {
            float n2 = 0.f;
#pragma unroll
            for (int r = 0; r < D; ++r) {
                const float t = (s_tile[i * D + r] - s_mu[r]) * a.escale;
                n2 = fmaf(t, t, n2);
            }
            wn[i] = -n2;
        }
        __syncthreads();
    }
    const double tol = pa.tol;
    const int max_iter = pa.max_iter;
    unsigned int seq = pa.seq_base;

    // matrix-core passes: per-wavefront partial sums, the codeword tables of the step, the table of the evaluation at C*
    constexpr int TS = MfmaFwd<(KPL <= 4 ? KPL : 4)>::TAB_STRIDE;
    __shared__ __align__(16) float s_part[MFMA ? NT / 64 : 1][MFMA ? 64 * KPL * ACCW : 1];
    __shared__ float2 s_tab[MFMA ? 4 * TS : 1];
    __shared__ float s_fac[MFMA ? TS : 1];
    __shared__ f32x4 s_ctab[MFMA ? TS : 1];
    // hop-1 store of a matrix-core pass: wavefront totals add up in wavefront order, float64, as in publish_lane
    auto publish_matrix = [&]() {
        if constexpr (MFMA) {
            unsigned long long* dst = pa.buf1 + ((size_t)(seq & 1u) * pa.G + pa.wg) * nacc;
            for (int idx = tid; idx < nacc; idx += NT) {
                double t = 0.0;
#pragma unroll
                for (int w = 0; w < NT / 64; ++w) t += (double)s_part[w][idx];
                st_word(&dst[idx], pack_f(seq, (float)t));
            }
        }
    };

    while (!s_done) {
        ++seq;
        IDKM_LSTAMP(0);
        if constexpr (MFMA) {
            const bool fold = MfmaFwd<KPL>::template fill_table<NT>(s_tab, s_fac, k, s_Cf, s_mu, a.escale) &&
                              DIST == DIST_SQL2;
            {
                MfmaFwd<KPL> st;
                st.init(s_tab, s_fac, s_mu);
                mfma_tile_pass<KPL, DIST, NT>(st, s_tile, s_wn, cnt, a.escale, fold);
                IDKM_LSTAMP(1);
                mfma_collect<KPL, NT>(st, &s_part[0][0], fold, s_fac);
            }
            __syncthreads();
            IDKM_LSTAMP(5);
            publish_matrix();
        } else {
            LaneWave<KPL, D, DIST, PASS_FWD> st;
            st.init(k, s_Cf, nullptr, nullptr, a.escale);
            lane_tile_pass<KPL, D, DIST, PASS_FWD, NT>(a, st, s_tile, nullptr, base, cnt);
            IDKM_LSTAMP(1);
            publish_lane<NA, ACCW, NT>(pa, seq, st.acc, k, s_acc);
        }
        IDKM_LSTAMP(2);
        for (int r = wg; r < k; r += G) {
            if (!reduce_lane<ACCW>(pa, seq, nacc, r * ACCW, ls)) return;
            if (tid < D) {
                const int idx = r * D + tid;
                const double n = ls.tot[0], s = ls.tot[1 + tid];
                const double cold = s_Cd[idx];
                double cnew = (n > 0.0) ? fast_div_d(s, n) : cold;
                if (!(n >= 0.0) || !(fabs(s) <= 1.7e308) || !(fabs(cnew) <= 1.7e308)) cnew = __builtin_nan("");
                s_Cd[idx] = cnew;
                st_word(&pa.buf2[(size_t)(seq & 1u) * stride2 + idx], pack_f(seq, (float)cnew));
            }
        }
        IDKM_LSTAMP(3);
        if (!gather_lane<NT>(pa, seq, kd, stride2, s_new, ls)) return;
        IDKM_LSTAMP(4);
        double r2 = 0.0;
        for (int i = tid; i < kd; i += NT) {
            const double df = (double)__uint_as_float(s_new[i]) - (double)s_Cf[i];
            r2 += df * df;
        }
        r2 = block_sum_fixed<NT>(r2, ls);
        for (int i = tid; i < kd; i += NT) s_Cf[i] = __uint_as_float(s_new[i]);
        IDKM_LSTAMP(6);
        if (tid == 0) {
            s_iters += 1;
            s_res = r2;
            const bool bad = !(r2 <= 1.7e308);
            if (bad) s_bad = 1;
            const bool conv = r2 < tol * tol;
            s_conv = conv ? 1 : 0;
            if (conv || bad || s_iters >= max_iter) s_done = 1;
        }
        __syncthreads();
    }

    // evaluation at C*
    {
        ++seq;
        bool done_here = false;
        if constexpr (MFMA) {
            // n*, F* and Wq on the matrix cores; the assignment (its float32 key has a prescribed form) and the
            // matrix A are outputs of the vector-ALU pass
            if (!a.assign_out && !a.A_out) {
                const bool fold = MfmaFwd<KPL>::template fill_table<NT>(s_tab, s_fac, k, s_Cf, s_mu, a.escale) &&
                                  DIST == DIST_SQL2;
                MfmaFwd<KPL>::template fill_codeword_table<NT>(s_ctab, k, s_Cf, s_mu, s_fac, fold);
                __syncthreads();
                {
                    MfmaFwd<KPL> st;
                    st.init(s_tab, s_fac, s_mu);
                    if (a.Wq_out)
                        mfma_tile_pass<KPL, DIST, NT, true>(st, s_tile, s_wn, cnt, a.escale, fold, s_ctab, s_mu,
                                                            a.Wq_out + base * D);
                    else
                        mfma_tile_pass<KPL, DIST, NT>(st, s_tile, s_wn, cnt, a.escale, fold);
                    mfma_collect<KPL, NT>(st, &s_part[0][0], fold, s_fac);
                }
                __syncthreads();
                publish_matrix();
                done_here = true;
            }
        }
        if (!done_here) {
            LaneWave<KPL, D, DIST, PASS_FIN> st;
            st.init(k, s_Cf, nullptr, nullptr);
            lane_tile_pass<KPL, D, DIST, PASS_FIN, NT>(a, st, s_tile, nullptr, base, cnt);
            publish_lane<NA, ACCW, NT>(pa, seq, st.acc, k, s_acc);
        }
        for (int r = wg; r < k; r += G) {
            if (!reduce_lane<ACCW>(pa, seq, nacc, r * ACCW, ls)) return;
            if (tid < D) {
                const int idx = r * D + tid;
                const double n = ls.tot[0], s = ls.tot[1 + tid];
                const double cst = (double)s_Cf[idx];
                const double f = (n > 0.0) ? fast_div_d(s, n) : cst;
                a.Cd[idx] = cst;
                a.Cf[idx] = s_Cf[idx];
                a.Fd[idx] = f;
                a.Ff[idx] = (float)f;
                if (a.C_out) a.C_out[idx] = s_Cf[idx];
            }
            if (tid == 0) {
                double n = ls.tot[0];
                a.nd[r] = n;
                bool bad = !(n >= 0.0);
                for (int rr = 0; rr < D; ++rr)
                    if (!(fabs(ls.tot[1 + rr]) <= 1.7e308)) bad = true;
                // the mass of codeword r travels to the last workgroup, which counts empty / non-finite clusters
                st_word(&pa.buf2[(size_t)(seq & 1u) * stride2 + kd + r], pack_f(seq, bad ? __builtin_nanf("") : (float)n));
            }
            __syncthreads();
        }
    }
    if (wg == G - 1) {
        // the masses of all codewords: count empty and non-finite clusters, then report
        {
            const unsigned long long* src = pa.buf2 + (size_t)(seq & 1u) * stride2 + kd;
            bool ok = true;
            for (int i = tid; i < k; i += NT) {
                unsigned int p = 0;
                ok = ok && poll_word(pa, src + i, seq, &p);
                s_new[i] = p;
            }
            if (!ok) raise_abort(pa, ls);
            __syncthreads();
            if (ls.abort) return;
        }
        double empty = 0.0, bad = 0.0;
        for (int i = tid; i < k; i += NT) {
            const float n = __uint_as_float(s_new[i]);
            if (!(n >= 0.f)) bad += 1.0;
            else if (!(n > 0.f)) empty += 1.0;
        }
        empty = block_sum_fixed<NT>(empty, ls);
        bad = block_sum_fixed<NT>(bad, ls);
        if (tid == 0) {
            PResult* o = pa.out;
            o->iters = s_iters;
            o->residual = sqrt(s_res);
            o->converged = s_conv;
            o->nonfinite = (s_bad || bad > 0.0) ? 1 : 0;
            o->empty[0] = (int)(empty + 0.5);
            o->done = pa.seq_base + 1u;
        }
    }
}

// Backward: v, the averaged iteration of Sec. 4.2 (skipped for JFB), and dW.  MFMA: the (dF/dC)^T passes run on the
// matrix cores (MfmaB2; d = 4), with NT = MT threads; the dynamic LDS then holds the tile of W padded
// by 16 zero vectors and -s^2 |w - mu|^2 of every vector, and dL/dWq -- needed by the first and the last pass only --
// is read from memory.
template <int KPL, int D, int DIST, int NT = LT, bool MFMA = false>
__device__ __forceinline__ void persist_lane_bwd_body(const Args& a, const PArgs& pa) {
    static_assert(!MFMA || (D == 4 && KPL <= 4), "matrix-core pass: d = 4, k <= 256");
    constexpr int NA = KPL * D;
    constexpr int KDP = 64 * KPL * D;
    extern __shared__ float s_tile[];
    __shared__ double s_acc[64][NA];
    __shared__ LShared ls;
    __shared__ double s_v[KDP], s_g[KDP];  // the reducer's own codewords are the live ones
    __shared__ double s_rn[64 * KPL];      // 1/(tau n_j), zero for an empty cluster
    __shared__ float s_Cf[KDP], s_Hs[KDP], s_Hv[KDP], s_Ff[KDP];
    __shared__ unsigned int s_new[KDP + 64 * KPL];
    __shared__ int s_done, s_iters, s_conv, s_attempt, s_grow, s_halv, s_bad, s_restart;
    __shared__ double s_alpha, s_prev, s_vnorm, s_res;

    const int tid = threadIdx.x, wg = pa.wg, G = pa.G;
    const int k = a.k, kd = k * D;
    const int stride2 = kd + k;
    const int64_t base = (int64_t)wg * pa.per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < pa.per) ? (int)(a.m - base) : pa.per;
    float* s_w = s_tile;
    const float* s_gt = MFMA ? a.G + base * D : s_tile + (size_t)pa.per * D;
    load_tile<NT>(s_w, a.W + base * D, cnt * D);
    if (!MFMA) load_tile<NT>(s_tile + (size_t)pa.per * D, a.G + base * D, cnt * D);
    for (int i = tid; i < kd; i += NT) {
        s_Cf[i] = a.Cf[i];
        s_Ff[i] = a.Ff[i];
        s_Hs[i] = 0.f;
        s_Hv[i] = 0.f;
    }
    for (int j = tid; j < k; j += NT) {
        const double n = a.nd[j];
        s_rn[j] = (n > 0.0) ? (double)a.inv_tau / n : 0.0;
    }
    const int mode = pa.mode;
    const double tol = pa.tol;
    const int max_iter = pa.max_iter;
    if (tid == 0) {
        ls.abort = 0;
        s_done = (mode == BWD_JFB) ? 1 : 0;
        s_iters = 0;
        s_conv = (mode == BWD_JFB) ? 1 : 0;
        s_attempt = 0;
        s_grow = 0;
        s_halv = 0;
        s_bad = 0;
        s_restart = 0;
        s_alpha = pa.alpha;
        s_prev = __builtin_inf();
        s_vnorm = 0.0;
        s_res = 0.0;
    }
    __syncthreads();
    unsigned int seq = pa.seq_base;
    // matrix-core passes: reference point, vector norms and the codeword tables (C* does not change in the backward)
    constexpr int TS = MfmaFwd<(KPL <= 4 ? KPL : 4)>::TAB_STRIDE;
    __shared__ float2 s_tab0[MFMA ? 4 * TS : 1];
    __shared__ float s_fac0[MFMA ? TS : 1];
    __shared__ float s_hsb[MFMA ? 4 * TS : 1];
    __shared__ f32x4 s_hq[MFMA ? TS : 1];
    __shared__ __align__(16) float s_part[MFMA ? NT / 64 : 1][MFMA ? 64 * KPL * 5 : 1];
    const float* s_wn = s_tile + (size_t)(pa.per + 16) * D;
    __shared__ float s_mu[4];
    bool fold = false;
    if constexpr (MFMA) {
        if (tid < D) {
            float sm = 0.f;
            for (int j = 0; j < k; ++j) sm += s_Cf[j * D + tid];
            s_mu[tid] = sm / (float)k;
        }
        float* wn = s_tile + (size_t)(pa.per + 16) * D;
        for (int i = cnt * D + tid; i < (pa.per + 16) * D; i += NT) s_tile[i] = 0.f;
        __syncthreads();
        for (int i = tid; i < pa.per + 16; i += NT) {
            float n2 = 0.f;
#pragma unroll
            for (int r = 0; r < D; ++r) {
                const float t = (s_tile[i * D + r] - s_mu[r]) * a.escale;
                n2 = fmaf(t, t, n2);
            }
            wn[i] = -n2;
        }
    }

    if constexpr (MFMA)
        fold = MfmaFwd<KPL>::template fill_table<NT>(s_tab0, s_fac0, k, s_Cf, s_mu, a.escale) && DIST == DIST_SQL2;
    // Hop-1 store of a matrix-core pass: wavefront totals add up in wavefront order (float64), then the codeword
    // term and the fold factor (see MfmaB2).
    auto publish_matrix = [&]() {
        if constexpr (MFMA) {
            unsigned long long* dst = pa.buf1 + ((size_t)(seq & 1u) * pa.G + pa.wg) * kd;
            for (int idx = tid; idx < kd; idx += NT) {
                const int j = idx >> 2, r = idx & 3;
                double sw = 0.0, st1 = 0.0;
#pragma unroll
                for (int w = 0; w < NT / 64; ++w) {
                    sw += (double)s_part[w][j * 5 + 1 + r];
                    st1 += (double)s_part[w][j * 5];
                }
                const double o = sw - (double)(s_Cf[idx] - s_mu[r]) * st1;
                st_word(&dst[idx], pack_f(seq, (float)(fold ? o * (double)s_fac0[j] : o)));
            }
        }
    };

    // B1
    {
        ++seq;
        if constexpr (MFMA) {
            {
                MfmaB2<KPL> st;
                st.init(s_tab0, s_fac0, s_hsb, s_hq, s_mu);
                mfma_b1_tile_pass<KPL, DIST, NT>(st, s_tile, s_wn, s_gt, cnt, a.escale, a.inv_tau, fold);
                mfma_b2_collect<KPL, NT>(st, &s_part[0][0]);
            }
            __syncthreads();
            publish_matrix();
        } else {
            LaneWave<KPL, D, DIST, PASS_B1> st;
            st.init(k, s_Cf, s_Hs, s_Ff, a.escale);
            lane_tile_pass<KPL, D, DIST, PASS_B1, NT>(a, st, s_w, s_gt, base, cnt);
            publish_lane<NA, D, NT>(pa, seq, st.acc, k, s_acc);
        }
        for (int r = wg; r < k; r += G) {
            if (!reduce_lane<D>(pa, seq, kd, r * D, ls)) return;
            if (tid < 64) {
                double v2 = 0.0;
                if (tid < D) {
                    const int idx = r * D + tid;
                    const double v = ls.tot[tid];
                    s_v[idx] = v;
                    s_g[idx] = v;
                    v2 = v * v;
                    st_word(&pa.buf2[(size_t)(seq & 1u) * stride2 + idx], pack_f(seq, (float)(v * s_rn[r])));
                }
                v2 = wave_sum_d_dpp(v2);
                if (tid == 0) st_word(&pa.buf2[(size_t)(seq & 1u) * stride2 + kd + r], pack_f(seq, (float)v2));
            }
        }
        if (!gather_lane<NT>(pa, seq, kd + k, stride2, s_new, ls)) return;
        double v2 = 0.0;
        for (int i = tid; i < k; i += NT) v2 += (double)__uint_as_float(s_new[kd + i]);
        v2 = block_sum_fixed<NT>(v2, ls);
        for (int i = tid; i < kd; i += NT) {
            s_Hs[i] = __uint_as_float(s_new[i]);
            s_Hv[i] = s_Hs[i];
        }
        if (tid == 0) {
            s_vnorm = v2;  // squared norms throughout
            if (!(v2 <= 1.7e308)) {
                s_bad = 1;
                s_done = 1;
            }
        }
        __syncthreads();
    }

    while (!s_done) {
        ++seq;
        if constexpr (MFMA) {
            MfmaB2<KPL>::template fill_cotangent<NT>(s_hsb, s_hq, k, s_Hs, s_Ff, s_mu, a.escale);
            __syncthreads();
            {
                MfmaB2<KPL> st;
                st.init(s_tab0, s_fac0, s_hsb, s_hq, s_mu);
                mfma_b2_tile_pass<KPL, DIST, NT>(st, s_tile, s_wn, cnt, a.escale, fold);
                mfma_b2_collect<KPL, NT>(st, &s_part[0][0]);
            }
            __syncthreads();
            publish_matrix();
        } else {
            LaneWave<KPL, D, DIST, PASS_B2> st;
            st.init(k, s_Cf, s_Hs, s_Ff, a.escale);
            lane_tile_pass<KPL, D, DIST, PASS_B2, NT>(a, st, s_w, s_gt, base, cnt);
            publish_lane<NA, D, NT>(pa, seq, st.acc, k, s_acc);
        }
        const double alpha = s_alpha;
        for (int r = wg; r < k; r += G) {
            if (!reduce_lane<D>(pa, seq, kd, r * D, ls)) return;
            if (tid < 64) {
                double d2 = 0.0;
                if (tid < D) {
                    const int idx = r * D + tid;
                    const double g = s_g[idx];
                    const double gn = alpha * (s_v[idx] + ls.tot[tid]) + (1.0 - alpha) * g;
                    const double df = gn - g;
                    d2 = df * df;
                    s_g[idx] = gn;
                    st_word(&pa.buf2[(size_t)(seq & 1u) * stride2 + idx], pack_f(seq, (float)(gn * s_rn[r])));
                }
                d2 = wave_sum_d_dpp(d2);
                if (tid == 0) st_word(&pa.buf2[(size_t)(seq & 1u) * stride2 + kd + r], pack_f(seq, (float)d2));
            }
        }
        if (!gather_lane<NT>(pa, seq, kd + k, stride2, s_new, ls)) return;
        double d2 = 0.0;
        for (int i = tid; i < k; i += NT) d2 += (double)__uint_as_float(s_new[kd + i]);
        d2 = block_sum_fixed<NT>(d2, ls);
        if (tid == 0) {
            const double dn = d2;  // squared step norm: every comparison below is between squares
            bool restart = false, done = false, conv = false, diverged = false;
            int grow = s_grow;
            const int attempt = s_attempt + 1;
            if (!(dn <= 1.7e308)) {
                diverged = true;
            } else if (dn <= tol * tol * s_vnorm) {
                conv = true;
                done = true;
            } else {
                grow = (dn > s_prev) ? grow + 1 : 0;
                if (grow >= 5) diverged = true;
            }
            if (!done && !diverged && attempt >= max_iter) done = true;
            if (diverged) {
                if (s_halv < 6) {
                    restart = true;
                } else {
                    done = true;
                    if (!(dn <= 1.7e308)) s_bad = 1;  // every damping factor tried ended in a non-finite step
                }
            }
            s_iters += 1;
            s_res = dn;
            if (conv) s_conv = 1;
            if (restart) {
                s_alpha = alpha * 0.5;
                s_halv += 1;
                s_attempt = 0;
                s_grow = 0;
                s_prev = __builtin_inf();
            } else {
                s_attempt = attempt;
                s_grow = grow;
                if (!diverged && !conv) s_prev = dn;
            }
            s_restart = restart ? 1 : 0;
            if (done) s_done = 1;
        }
        __syncthreads();
        if (s_restart) {
            for (int i = tid; i < kd; i += NT) {
                s_Hs[i] = s_Hv[i];
                s_g[i] = s_v[i];
            }
        } else {
            for (int i = tid; i < kd; i += NT) s_Hs[i] = __uint_as_float(s_new[i]);
        }
        __syncthreads();
    }

    // B3
    if constexpr (MFMA) {
        // the output tables take the place of the per-wavefront partial sums, which no later pass needs
        f32x4* s_hc = reinterpret_cast<f32x4*>(&s_part[0][0]);
        static_assert(sizeof(s_part) >= 2 * TS * sizeof(f32x4), "output tables do not fit");
        MfmaB2<KPL>::template fill_cotangent<NT>(s_hsb, s_hq, k, s_Hs, s_Ff, s_mu, a.escale);
        MfmaB3<KPL>::template fill_output_tables<NT>(s_hc, k, s_Hs, s_Cf, s_mu, s_fac0, fold, a.tau,
                                                     DIST == DIST_SQL2 ? 2.f : a.escale);
        __syncthreads();
        MfmaB3<KPL> st;
        st.init(s_tab0, s_fac0, s_hsb, s_hq, s_hc, s_mu);
        mfma_b3_tile_pass<KPL, DIST, NT>(st, s_tile, s_wn, s_gt, a.dW_out + base * D, cnt, a.escale, a.inv_tau, fold);
    } else {
        LaneWave<KPL, D, DIST, PASS_B3> st;
        st.init(k, s_Cf, s_Hs, s_Ff, a.escale);
        lane_tile_pass<KPL, D, DIST, PASS_B3, NT>(a, st, s_w, s_gt, base, cnt);
    }
    for (int r = wg; r < k; r += G) {
        if (tid < D) {
            a.gd[r * D + tid] = s_g[r * D + tid];
            a.vd[r * D + tid] = s_v[r * D + tid];
        }
    }
    if (wg == 0)
        for (int i = tid; i < kd; i += NT) a.Hs[i] = s_Hs[i];
    if (wg == G - 1 && tid == 0) {
        PResult* o = pa.out;
        o->iters = s_iters;
        o->converged = s_conv;
        o->residual = sqrt(s_res);
        o->alpha = s_alpha;
        o->vnorm = sqrt(s_vnorm);
        o->halvings = s_halv;
        o->nonfinite = s_bad;
        o->done = pa.seq_base + 1u;
    }
}

// Launch forms: one team per grid, or one team per batched problem (see persist_small.hpp).
template <int KPL, int D, int DIST>
__global__ __launch_bounds__(LT) void persist_lane_fwd(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_lane_fwd_body<KPL, D, DIST>(a, pa);
}
template <int KPL, int D, int DIST>
__global__ __launch_bounds__(LT) void persist_lane_fwd_batch(const BatchItem* items, const unsigned short* item_of_wg) {
    const BatchItem& it = items[item_of_wg[blockIdx.x]];
    const Args a = it.a;
    PArgs pa = it.p;
    pa.wg = (int)blockIdx.x - it.wg_begin;
    pa.G = it.wg_count;
    persist_lane_fwd_body<KPL, D, DIST>(a, pa);
}
// Forward solve with the loop on the matrix cores (d = 4): MT threads, see persist_lane_fwd_body.
template <int KPL, int DIST>
__global__ __launch_bounds__(MT) void persist_mfma_fwd(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_lane_fwd_body<KPL, 4, DIST, MT, true>(a, pa);
}
template <int KPL, int DIST>
__global__ __launch_bounds__(MT) void persist_mfma_fwd_batch(const BatchItem* items, const unsigned short* item_of_wg) {
    const BatchItem& it = items[item_of_wg[blockIdx.x]];
    const Args a = it.a;
    PArgs pa = it.p;
    pa.wg = (int)blockIdx.x - it.wg_begin;
    pa.G = it.wg_count;
    persist_lane_fwd_body<KPL, 4, DIST, MT, true>(a, pa);
}
// Backward with the (dF/dC)^T passes on the matrix cores (d = 4), see persist_lane_bwd_body.  The plain norm's pass
// keeps more per lane than 256 registers hold at k = 256 (energies and u for 16 x 256 pairs, the accumulators, the
// row minima): that kernel runs one wavefront per SIMD, which may use the whole register file.
template <int KPL, int DIST>
constexpr int mfma_bwd_threads() {
    return (DIST == DIST_L2 && KPL == 4) ? 256 : MT;
}
template <int KPL, int DIST>
__global__ __launch_bounds__((mfma_bwd_threads<KPL, DIST>())) void persist_mfma_bwd(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_lane_bwd_body<KPL, 4, DIST, mfma_bwd_threads<KPL, DIST>(), true>(a, pa);
}
template <int KPL, int DIST>
__global__ __launch_bounds__((mfma_bwd_threads<KPL, DIST>())) void persist_mfma_bwd_batch(const BatchItem* items, const unsigned short* item_of_wg) {
    const BatchItem& it = items[item_of_wg[blockIdx.x]];
    const Args a = it.a;
    PArgs pa = it.p;
    pa.wg = (int)blockIdx.x - it.wg_begin;
    pa.G = it.wg_count;
    persist_lane_bwd_body<KPL, 4, DIST, mfma_bwd_threads<KPL, DIST>(), true>(a, pa);
}
template <int KPL, int D, int DIST>
__global__ __launch_bounds__(LT) void persist_lane_bwd(const Args a, const PArgs pa_in) {
    PArgs pa = pa_in;
    pa.wg = blockIdx.x;
    pa.G = gridDim.x;
    persist_lane_bwd_body<KPL, D, DIST>(a, pa);
}
template <int KPL, int D, int DIST>
__global__ __launch_bounds__(LT) void persist_lane_bwd_batch(const BatchItem* items, const unsigned short* item_of_wg) {
    const BatchItem& it = items[item_of_wg[blockIdx.x]];
    const Args a = it.a;
    PArgs pa = it.p;
    pa.wg = (int)blockIdx.x - it.wg_begin;
    pa.G = it.wg_count;
    persist_lane_bwd_body<KPL, D, DIST>(a, pa);
}

}  // namespace idkm
