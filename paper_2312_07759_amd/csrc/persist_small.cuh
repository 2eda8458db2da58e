// Persistent kernels for small codebooks: one launch per solve.  Each workgroup
// keeps its tile of W (and of dL/dWq in the backward) in LDS for the whole solve,
// so after the first read no pass touches HBM for its inputs; the only grid-wide
// traffic per pass is one exchange of K (D+1) partial sums per workgroup.
//
// Exchange: every workgroup publishes its partial sums as 64-bit words
// {sequence number, float32 value} with device-scope stores, then reads all
// workgroups' words until every sequence number matches.  Value and stamp travel
// in one atomic word, so no fence and no counter round trip is needed; two
// buffers alternate by sequence parity.  All workgroups add the same words in
// the same order, hence take bit-identical decisions.  Waits are bounded: after
// spin_limit polls a workgroup raises Ctrl::abort_flag and leaves; the others
// see the flag and leave too.  The grid must be co-resident (cooperative launch).
#pragma once
#include "common.cuh"
#include "small_k.cuh"

namespace idkm {

constexpr int PT = 256;  // threads per workgroup of the persistent kernels

struct PArgs {
    unsigned long long* xbuf;  // [2][NP][gridDim.x] stamped words
    unsigned int seq_base;     // sequence numbers seq_base+1 ... are used by this launch
    unsigned int spin_limit;   // polls before a wait gives up
    int per;                   // vectors per workgroup tile
};

constexpr int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}
// Rows of the exchange buffer for NACC accumulators: a power of two, and at least
// PT/64 so that the threads sharing one row sit inside one wavefront.
constexpr int xchg_rows(int nacc) { return next_pow2(nacc) < PT / 64 ? PT / 64 : next_pow2(nacc); }

__device__ __forceinline__ unsigned long long ld_word(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_word(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sums acc[q] over the whole grid into s_tot[q] (float64, fixed order).  Returns
// false in every thread of the workgroup if the wait was abandoned.
template <int NACC>
__device__ __forceinline__ bool grid_exchange(const PArgs& pa, Ctrl* ctrl, unsigned int seq, const float (&acc)[NACC],
                                              double* s_wpart, double* s_tot, int* s_abort) {
    constexpr int NP = xchg_rows(NACC);
    constexpr int TPA = PT / NP;  // threads that share the words of one accumulator
    static_assert(NP <= PT && TPA <= 64, "accumulator count does not fit the exchange layout");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = gridDim.x;
#pragma unroll
    for (int q = 0; q < NACC; ++q) {
        const float v = wave_sum(acc[q]);
        if (lane == 0) s_wpart[wave * NACC + q] = (double)v;
    }
    __syncthreads();
    unsigned long long* buf = pa.xbuf + (size_t)(seq & 1u) * NP * G;
    if (tid < NACC) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < PT / 64; ++w) s += s_wpart[w * NACC + tid];
        const unsigned long long word = ((unsigned long long)seq << 32) | (unsigned long long)__float_as_uint((float)s);
        st_word(&buf[(size_t)tid * G + blockIdx.x], word);
    }
    const int ai = tid / TPA, sub = tid % TPA;
    const int wpt = (G + TPA - 1) / TPA;
    const int first = sub * wpt;
    int cnt = G - first;
    if (cnt > wpt) cnt = wpt;
    double sum = 0.0;
    bool aborted = false;
    if (ai < NACC && cnt > 0) {
        const unsigned long long* src = buf + (size_t)ai * G + first;
        unsigned int spins = 0;
        for (;;) {
            bool ok = true;
            sum = 0.0;
            for (int q = 0; q < cnt; q += 4) {
                unsigned long long w0 = ld_word(src + q);
                unsigned long long w1 = (q + 1 < cnt) ? ld_word(src + q + 1) : w0;
                unsigned long long w2 = (q + 2 < cnt) ? ld_word(src + q + 2) : w0;
                unsigned long long w3 = (q + 3 < cnt) ? ld_word(src + q + 3) : w0;
                ok = ok && ((unsigned int)(w0 >> 32) == seq) && ((unsigned int)(w1 >> 32) == seq) &&
                     ((unsigned int)(w2 >> 32) == seq) && ((unsigned int)(w3 >> 32) == seq);
                sum += (double)__uint_as_float((unsigned int)w0);
                if (q + 1 < cnt) sum += (double)__uint_as_float((unsigned int)w1);
                if (q + 2 < cnt) sum += (double)__uint_as_float((unsigned int)w2);
                if (q + 3 < cnt) sum += (double)__uint_as_float((unsigned int)w3);
            }
            if (ok) break;
            ++spins;
            if (spins > pa.spin_limit ||
                ((spins & 31u) == 0u && __hip_atomic_load(&ctrl->abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                aborted = true;
                break;
            }
        }
    }
#pragma unroll
    for (int o = 1; o < TPA; o <<= 1) sum += __shfl_xor(sum, o, 64);
    if (ai < NACC && sub == 0) s_tot[ai] = sum;
    if (aborted) {
        *s_abort = 1;
        __hip_atomic_store(&ctrl->abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return *s_abort == 0;
}

// One pass over the workgroup's LDS tile.
template <int K, int D, int DIST, int PASS>
__device__ __forceinline__ void tile_pass(const Args& a, const float* s_w, const float* s_g, int64_t base, int cnt,
                                          const float* s_Cf, const float* s_Hs, const float* s_Ff,
                                          float (&acc)[SmallItem<K, D, DIST, PASS>::NACC]) {
    using Item = SmallItem<K, D, DIST, PASS>;
    float c[K][D], hs[K][D], ff[K][D];
#pragma unroll
    for (int j = 0; j < K; ++j)
#pragma unroll
        for (int r = 0; r < D; ++r) {
            c[j][r] = s_Cf[j * D + r];
            hs[j][r] = Item::USE_H ? s_Hs[j * D + r] : 0.f;
            ff[j][r] = Item::USE_H ? s_Ff[j * D + r] : 0.f;
        }
#pragma unroll
    for (int q = 0; q < Item::NACC; ++q) acc[q] = 0.f;
#pragma unroll 2
    for (int it = threadIdx.x; it < cnt; it += PT) {
        float w[D], g[D];
#pragma unroll
        for (int r = 0; r < D; ++r) {
            w[r] = s_w[it * D + r];
            g[r] = Item::USE_G ? s_g[it * D + r] : 0.f;
        }
        Item::run(a, base + it, w, g, c, hs, ff, acc);
    }
}

// Forward solve (Alg. 1) and the evaluation at C*, in one launch.
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_fwd(const Args a, const PArgs pa) {
    constexpr int KD = K * D;
    constexpr int NACC = K * (D + 1);
    static_assert(KD <= 64, "codebook must fit one wavefront");
    extern __shared__ float s_tile[];
    __shared__ double s_wpart[(PT / 64) * NACC];
    __shared__ double s_tot[xchg_rows(NACC)];
    __shared__ double s_Cd[KD];
    __shared__ float s_Cf[KD];
    __shared__ int s_abort, s_done, s_iters, s_conv, s_bad, s_empty;
    __shared__ double s_res;

    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * pa.per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < pa.per) ? (int)(a.m - base) : pa.per;
    for (int i = tid; i < cnt * D; i += PT) s_tile[i] = a.W[base * D + i];
    if (tid < KD) {
        s_Cd[tid] = a.Cd[tid];
        s_Cf[tid] = a.Cf[tid];
    }
    if (tid == 0) {
        s_abort = 0;
        s_done = 0;
        s_iters = 0;
        s_conv = 0;
        s_bad = 0;
        s_empty = 0;
        s_res = 0.0;
    }
    __syncthreads();
    const double tol = a.ctrl->tol;
    const int max_iter = a.ctrl->max_iter;
    unsigned int seq = pa.seq_base;

    float acc[NACC];
    while (!s_done) {
        tile_pass<K, D, DIST, PASS_FWD>(a, s_tile, nullptr, base, cnt, s_Cf, nullptr, nullptr, acc);
        ++seq;
        if (!grid_exchange<NACC>(pa, a.ctrl, seq, acc, s_wpart, s_tot, &s_abort)) return;
        // centre update and stop test (Alg. 1), identically in every workgroup
        if (tid < 64) {
            double r2 = 0.0, bad = 0.0, empty = 0.0;
            if (tid < KD) {
                const int j = tid / D, r = tid - j * D;
                const double n = s_tot[j * (D + 1)], s = s_tot[j * (D + 1) + 1 + r];
                const double cold = s_Cd[tid];
                const double cnew = (n > 0.0) ? s / n : cold;
                if (!(n > 0.0) && r == 0) empty = 1.0;
                if (!(n >= 0.0) || !(fabs(s) <= 1.7e308) || !(fabs(cnew) <= 1.7e308)) bad = 1.0;
                const double df = cnew - cold;
                r2 = df * df;
                s_Cd[tid] = cnew;
                s_Cf[tid] = (float)cnew;
            }
            r2 = wave_sum_d(r2);
            bad = wave_sum_d(bad);
            empty = wave_sum_d(empty);
            if (tid == 0) {
                const double res = sqrt(r2);
                s_iters += 1;
                s_res = res;
                s_empty = (int)(empty + 0.5);
                if (bad > 0.0) s_bad = 1;
                const bool conv = res < tol;
                s_conv = conv ? 1 : 0;
                if (conv || bad > 0.0 || s_iters >= max_iter) s_done = 1;
            }
        }
        __syncthreads();
    }

    // evaluation at C*: outputs, and n*, F* for the backward
    tile_pass<K, D, DIST, PASS_FIN>(a, s_tile, nullptr, base, cnt, s_Cf, nullptr, nullptr, acc);
    ++seq;
    if (!grid_exchange<NACC>(pa, a.ctrl, seq, acc, s_wpart, s_tot, &s_abort)) return;
    if (blockIdx.x == 0 && tid < 64) {
        double bad = 0.0, empty = 0.0;
        if (tid < KD) {
            const int j = tid / D, r = tid - j * D;
            const double n = s_tot[j * (D + 1)], s = s_tot[j * (D + 1) + 1 + r];
            const double f = (n > 0.0) ? s / n : s_Cd[tid];
            if (!(n > 0.0) && r == 0) empty = 1.0;
            if (!(n >= 0.0) || !(fabs(s) <= 1.7e308)) bad = 1.0;
            a.Cd[tid] = s_Cd[tid];
            a.Cf[tid] = s_Cf[tid];
            a.Fd[tid] = f;
            a.Ff[tid] = (float)f;
            if (r == 0) a.nd[j] = n;
            if (a.C_out) a.C_out[tid] = s_Cf[tid];
        }
        bad = wave_sum_d(bad);
        empty = wave_sum_d(empty);
        if (tid == 0) {
            Ctrl* c = a.ctrl;
            c->iters = s_iters;
            c->residual = s_res;
            c->converged = s_conv;
            c->empty = (int)(empty + 0.5);
            c->nonfinite = (s_bad || bad > 0.0) ? 1 : 0;
            c->done = 1;
        }
    }
}

// Backward (Alg. 2 per-layer steps): v, the averaged fixed-point iteration of
// Sec. 4.2 for g (skipped for JFB), and dW, in one launch.
template <int K, int D, int DIST>
__global__ __launch_bounds__(PT) void persist_bwd(const Args a, const PArgs pa) {
    constexpr int KD = K * D;
    static_assert(KD <= 64, "codebook must fit one wavefront");
    extern __shared__ float s_tile[];
    __shared__ double s_wpart[(PT / 64) * KD];
    __shared__ double s_tot[xchg_rows(KD)];
    __shared__ double s_v[KD], s_g[KD], s_n[K];
    __shared__ float s_Cf[KD], s_Hs[KD], s_Ff[KD];
    __shared__ int s_abort, s_done, s_iters, s_conv, s_attempt, s_grow, s_halv, s_bad;
    __shared__ double s_alpha, s_prev, s_vnorm, s_res;

    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * pa.per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < pa.per) ? (int)(a.m - base) : pa.per;
    float* s_w = s_tile;
    float* s_gt = s_tile + (size_t)pa.per * D;
    for (int i = tid; i < cnt * D; i += PT) {
        s_w[i] = a.W[base * D + i];
        s_gt[i] = a.G[base * D + i];
    }
    if (tid < KD) {
        s_Cf[tid] = a.Cf[tid];
        s_Ff[tid] = a.Ff[tid];
        s_Hs[tid] = 0.f;
    }
    if (tid < K) s_n[tid] = a.nd[tid];
    const int mode = a.ctrl->b_mode;
    const double tol = a.ctrl->b_tol;
    const int max_iter = a.ctrl->b_max_iter;
    if (tid == 0) {
        s_abort = 0;
        s_done = (mode == BWD_JFB) ? 1 : 0;
        s_iters = 0;
        s_conv = (mode == BWD_JFB) ? 1 : 0;
        s_attempt = 0;
        s_grow = 0;
        s_halv = 0;
        s_bad = 0;
        s_alpha = a.ctrl->b_alpha;
        s_prev = __builtin_inf();
        s_vnorm = 0.0;
        s_res = 0.0;
    }
    __syncthreads();
    unsigned int seq = pa.seq_base;
    const double inv_tau = (double)a.inv_tau;

    float acc[KD];
    // B1: v = dL/dC* with W fixed; the solve starts at g = v
    tile_pass<K, D, DIST, PASS_B1>(a, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, acc);
    ++seq;
    if (!grid_exchange<KD>(pa, a.ctrl, seq, acc, s_wpart, s_tot, &s_abort)) return;
    if (tid < 64) {
        double v2 = 0.0;
        if (tid < KD) {
            const double v = s_tot[tid];
            const double n = s_n[tid / D];
            s_v[tid] = v;
            s_g[tid] = v;
            s_Hs[tid] = (n > 0.0) ? (float)(v / n * inv_tau) : 0.f;
            v2 = v * v;
        }
        v2 = wave_sum_d(v2);
        if (tid == 0) {
            s_vnorm = sqrt(v2);
            if (!(v2 <= 1.7e308)) {
                s_bad = 1;
                s_done = 1;
            }
        }
    }
    __syncthreads();

    while (!s_done) {
        tile_pass<K, D, DIST, PASS_B2>(a, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, acc);
        ++seq;
        if (!grid_exchange<KD>(pa, a.ctrl, seq, acc, s_wpart, s_tot, &s_abort)) return;
        if (tid < 64) {
            const double alpha = s_alpha;
            double d2 = 0.0, gn = 0.0;
            if (tid < KD) {
                const double g = s_g[tid];
                gn = alpha * (s_v[tid] + s_tot[tid]) + (1.0 - alpha) * g;
                const double df = gn - g;
                d2 = df * df;
            }
            d2 = wave_sum_d(d2);
            // the same decision in every lane and every workgroup (cf. tail_b2)
            const double dn = sqrt(d2);
            bool restart = false, done = false, conv = false, diverged = false;
            int grow = s_grow;
            const int attempt = s_attempt + 1;
            if (!(dn <= 1.7e308)) {
                diverged = true;
            } else if (dn <= tol * s_vnorm) {
                conv = true;
                done = true;
            } else {
                grow = (dn > s_prev) ? grow + 1 : 0;
                if (grow >= 5) diverged = true;
            }
            if (!done && !diverged && attempt >= max_iter) done = true;
            if (diverged) {
                if (s_halv < 6)
                    restart = true;
                else
                    done = true;
            }
            const double gnext = restart ? ((tid < KD) ? s_v[tid] : 0.0) : gn;
            __builtin_amdgcn_wave_barrier();
            if (tid < KD) {
                const double n = s_n[tid / D];
                s_g[tid] = gnext;
                s_Hs[tid] = (n > 0.0) ? (float)(gnext / n * inv_tau) : 0.f;
            }
            if (tid == 0) {
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
                if (done) s_done = 1;
            }
        }
        __syncthreads();
    }

    // B3: dW = direct + (dF/dW)^T g
    tile_pass<K, D, DIST, PASS_B3>(a, s_w, s_gt, base, cnt, s_Cf, s_Hs, s_Ff, reinterpret_cast<float(&)[1]>(acc[0]));
    if (blockIdx.x == 0 && tid == 0) {
        Ctrl* c = a.ctrl;
        c->b_iters = s_iters;
        c->b_converged = s_conv;
        c->b_residual = s_res;
        c->b_alpha = s_alpha;
        c->b_vnorm = s_vnorm;
        c->b_halvings = s_halv;
        c->b_done = 1;
        if (s_bad) c->nonfinite = 1;
    }
    if (blockIdx.x == 0 && tid < KD) {
        a.gd[tid] = s_g[tid];
        a.vd[tid] = s_v[tid];
        a.Hs[tid] = s_Hs[tid];
    }
}

}  // namespace idkm
