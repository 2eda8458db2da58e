// Stream-path form of the matrix-core passes (d = 4, 17 <= k <= 256): one launch per pass, every workgroup copies its
// chunk of W into LDS, runs the 16-vector steps of mfma_lane.hpp over it and leaves its partial sums in
// a.partials[workgroup][.] (float64), which reduce_rows and the one-workgroup tail of the lane<->codeword family
// then take as from lane_pass.  PASS_FWD and PASS_B2.
#pragma once
#include "common.hpp"
#include "lane_k.hpp"
#include "mfma_lane.hpp"

namespace idkm {

// Threads per workgroup: 2 wavefronts per SIMD, as in the persistent kernels; one for the plain norm's (dF/dC)^T pass
// at k = 256, whose state does not fit 256 registers per lane.
template <int KPL, int DIST, int PASS>
constexpr int mfma_stream_threads() {
    return (KPL == 4 && DIST == DIST_L2 && PASS == PASS_B2) ? 256 : 512;
}

// Dynamic LDS: (a.vec_per_wg + 16) vectors of 4 floats, then one float per vector.
template <int KPL, int DIST, int PASS>
__global__ __launch_bounds__((mfma_stream_threads<KPL, DIST, PASS>())) void mfma_pass(const Args a) {
    constexpr int MST = mfma_stream_threads<KPL, DIST, PASS>();
    static_assert(PASS == PASS_FWD || PASS == PASS_B2, "forward loop or (dF/dC)^T pass");
    constexpr int TS = MfmaFwd<KPL>::TAB_STRIDE;
    constexpr bool B2 = (PASS == PASS_B2);
    if (PASS == PASS_FWD && a.ctrl->done) return;
    if (PASS == PASS_B2 && a.ctrl->b_done) return;
    extern __shared__ float s_tile[];
    __shared__ float2 s_tab[4 * TS];
    __shared__ float s_fac[TS];
    __shared__ float s_hsb[B2 ? 4 * TS : 1];
    __shared__ f32x4 s_hq[B2 ? TS : 1];
    __shared__ float s_part[MST / 64][64 * KPL * 5];
    __shared__ float s_mu[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k = a.k, per = (int)a.vec_per_wg;
    const int64_t base = (int64_t)blockIdx.x * per;
    int cnt = 0;
    if (base < a.m) cnt = (a.m - base < per) ? (int)(a.m - base) : per;
    float* s_wn = s_tile + (size_t)(per + 16) * 4;
    for (int i = tid; i < cnt * 4; i += MST) s_tile[i] = a.W[base * 4 + i];
    for (int i = cnt * 4 + tid; i < (per + 16) * 4; i += MST) s_tile[i] = 0.f;
    // reference point of the centred coordinates: the mean of the current codewords (wavefront w: coordinate w)
    if (wave < 4) {
        float sm = 0.f;
        for (int j = lane; j < k; j += 64) sm += a.Cf[j * 4 + wave];
        sm = wave_sum(sm);
        if (lane == 0) s_mu[wave] = sm / (float)k;
    }
    __syncthreads();
    for (int i = tid; i < per + 16; i += MST) {
        float n2 = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float t = (s_tile[i * 4 + r] - s_mu[r]) * a.escale;
            n2 = fmaf(t, t, n2);
        }
        s_wn[i] = -n2;
    }
    const bool fold = MfmaFwd<KPL>::template fill_table<MST>(s_tab, s_fac, k, a.Cf, s_mu, a.escale) && DIST == DIST_SQL2;
    if constexpr (B2) {
        MfmaB2<KPL>::template fill_cotangent<MST>(s_hsb, s_hq, k, a.Hs, a.Ff, s_mu, a.escale);
        __syncthreads();
        {
            MfmaB2<KPL> st;
            st.init(s_tab, s_fac, s_hsb, s_hq, s_mu);
            mfma_b2_tile_pass<KPL, DIST, MST>(st, s_tile, s_wn, cnt, a.escale, fold);
            mfma_b2_collect<KPL, MST>(st, &s_part[0][0]);
        }
        __syncthreads();
        const int kd = k * 4;
        for (int idx = tid; idx < kd; idx += MST) {
            const int j = idx >> 2, r = idx & 3;
            double sw = 0.0, st1 = 0.0;
#pragma unroll
            for (int w = 0; w < MST / 64; ++w) {
                sw += (double)s_part[w][j * 5 + 1 + r];
                st1 += (double)s_part[w][j * 5];
            }
            const double o = sw - (double)(a.Cf[idx] - s_mu[r]) * st1;
            a.partials[(size_t)blockIdx.x * kd + idx] = fold ? o * (double)s_fac[j] : o;
        }
    } else {
        {
            MfmaFwd<KPL> st;
            st.init(s_tab, s_fac, s_mu);
            mfma_tile_pass<KPL, DIST, MST>(st, s_tile, s_wn, cnt, a.escale, fold);
            mfma_collect<KPL, MST>(st, &s_part[0][0], fold, s_fac);
        }
        __syncthreads();
        const int nacc = k * 5;
        for (int idx = tid; idx < nacc; idx += MST) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < MST / 64; ++w) t += (double)s_part[w][idx];
            a.partials[(size_t)blockIdx.x * nacc + idx] = t;
        }
    }
}

}  // namespace idkm
