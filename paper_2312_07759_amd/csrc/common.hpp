// Shared device-side definitions for the IDKM kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace idkm {

// Passes over the m weight vectors.  Every pass recomputes the attention row
// a_i. = softmax_tau(-e_i.) (Eq. "aterms") of each vector on the fly.
constexpr int PASS_FWD = 0;  // one evaluation of F inside the forward loop (Alg. 1 body)
constexpr int PASS_FIN = 1;  // evaluation at C*: Wq, A, assignments, and n*, F* kept for the backward
constexpr int PASS_B1 = 2;   // v = dL/dC* with W fixed
constexpr int PASS_B2 = 3;   // u = (dF/dC)^T g
constexpr int PASS_B3 = 4;   // dW = direct + (dF/dW)^T g
constexpr int PASS_BJ = 5;   // v and the explicit Jacobian dF/dC* in one pass, then a direct solve (k d <= 16)

constexpr int DIST_L2 = 0;
constexpr int DIST_SQL2 = 1;

constexpr int BWD_IMPLICIT = 0;
constexpr int BWD_JFB = 1;
constexpr int BWD_DENSE = 2;
constexpr int BWD_GMRES = 3;
constexpr int GM_RMAX = 256;  // longest Krylov basis the workspace layout allows
constexpr int DENSE_MAX_KD = 16;

constexpr int WG = 256;  // threads per workgroup of the streaming kernels (4 wavefronts)

// Device-resident control block of one context.
struct Ctrl {
    unsigned int launch_seq;  // stamp of the last stream-path launch that published partial sums
    int abort_flag;           // a bounded device-side wait expired
    // forward (Alg. 1)
    int done, iters, converged, empty, nonfinite, max_iter;
    double residual, tol;
    // backward (Sec. 4.2 averaged iteration)
    int b_done, b_iters, b_converged, b_attempt, b_grow, b_halvings, b_max_iter, b_mode;
    double b_alpha, b_prev, b_vnorm, b_residual, b_tol;
    // backward, minimal-residual solve of (I - dF/dC)^T g = v
    int k_phase;   // what the next pass applies (dF/dC)^T to: 0 a basis vector, 1 the iterate g
    int k_j;       // basis vectors orthogonalised in this cycle
    int k_R;       // basis length at which a cycle ends: min(k d, GM_RMAX)
    int k_stall;   // consecutive cycles that did not halve the residual
    double k_beta; // residual norm at the start of the cycle
};

// Kernel argument block.
struct Args {
    const float* W;  // [m,d]
    const float* G;  // [m,d] upstream gradient dL/dWq (backward passes)
    int64_t m;
    int k, d;
    float nscale;   // -log2(e)/tau: exp(-e/tau) = exp2(e*nscale)
    float escale;   // sqrt(log2(e)/tau) for the squared energy, log2(e)/tau for the plain norm
    float inv_tau;  // 1/tau
    float tau;
    int64_t vec_per_wg;  // vectors handled by one workgroup
    Ctrl* ctrl;
    unsigned int* tickets;  // [TICKET_WORDS] arrival counters of the stream path (see arrive_last)
    // O(k d) solver state
    double* Cd;  // [k,d] current codebook, float64 master copy
    float* Cf;   // [k,d] float32 copy used by the E-step
    double* nd;  // [k]   masses n = A^T 1 of the last evaluation
    double* Fd;  // [k,d] F(C*, W)
    float* Ff;   // [k,d]
    double* gd;  // [k,d] current iterate of the backward solve
    double* vd;  // [k,d] v = dL/dC*
    double* ud;  // [k,d] last (dF/dC)^T g
    float* Hs;   // [k,d] h/tau with h_j = g_j / n_j
    double* partials;  // [gridDim.x][nacc]
    double* kry;       // Krylov workspace of the minimal-residual solve (see gm_layout), or null
    double* stage;     // [<=256 + nacc] staging for the final reduction
    double* tot;       // [nacc] reduced totals
    // outputs
    float* C_out;         // [k,d]
    float* A_out;         // [m,k] or null
    float* Wq_out;        // [m,d] or null
    int32_t* assign_out;  // [m] or null
    float* dW_out;        // [m,d]
};

// ---------------------------------------------------------------- wavefront (64-lane) reductions via DPP

template <int CTRL, int ROWMASK>
__device__ __forceinline__ float dpp_f(float identity, float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity), __builtin_bit_cast(int, x), CTRL,
                                           ROWMASK, 0xf, false));
}
template <int CTRL, int ROWMASK>
__device__ __forceinline__ int dpp_i(int identity, int x) {
    return __builtin_amdgcn_update_dpp(identity, x, CTRL, ROWMASK, 0xf, false);
}
__device__ __forceinline__ float bcast_lane63(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// Fixed-order butterfly inside rows of 16 lanes, then row broadcasts; the total
// ends in lane 63 and is returned to every lane.  The order of additions is the
// same on every call, so results are reproducible bit for bit.
__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_f<0xB1, 0xf>(0.f, x);   // quad_perm [1,0,3,2]
    x += dpp_f<0x4E, 0xf>(0.f, x);   // quad_perm [2,3,0,1]
    x += dpp_f<0x141, 0xf>(0.f, x);  // row_half_mirror
    x += dpp_f<0x140, 0xf>(0.f, x);  // row_mirror
    x += dpp_f<0x142, 0xa>(0.f, x);  // row_bcast15 into rows 1,3
    x += dpp_f<0x143, 0xc>(0.f, x);  // row_bcast31 into rows 2,3
    return bcast_lane63(x);
}
// Sums of N per-lane values (N a power of two) over the 16 lanes of every DPP row, with the number of live values
// halved at each of the four exchange steps (lane bit s decides which half a lane keeps and which it hands to its
// partner), so the whole reduction costs about 2 N exchange-adds instead of 4 N, and the chains of different values
// run side by side.  On return a lane holds row totals in x[0 .. row_sum_live(N)): value i of row lane l is the
// total of accumulator row_sum_index<N>(l, i); lanes for which row_sum_owner<N>(l) is false hold duplicates.
// The order of additions is fixed.
__host__ __device__ constexpr int row_sum_live(int n) { return n >= 16 ? n / 16 : 1; }
template <int N>
__device__ __forceinline__ int row_sum_index(int l, int i) {
    int idx = i, half = N / 2;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (half >= 1) idx += ((l >> s) & 1) * half;
        half /= 2;
    }
    return idx;
}
template <int N>
__device__ __forceinline__ bool row_sum_owner(int l) {
    // steps that no longer halve (one value left) are plain butterflies: both partners end with the same total
    bool own = true;
    int half = N / 2;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (half < 1) own = own && (((l >> s) & 1) == 0);
        half /= 2;
    }
    return own;
}
template <int S>
__device__ __forceinline__ float row_xchg(float x) {
    // value of the lane whose index differs in bit S (within a row of 16 lanes)
    if (S == 0) return dpp_f<0xB1, 0xf>(0.f, x);                              // quad_perm [1,0,3,2]
    if (S == 1) return dpp_f<0x4E, 0xf>(0.f, x);                              // quad_perm [2,3,0,1]
    if (S == 2) return dpp_f<0x1B, 0xf>(0.f, dpp_f<0x141, 0xf>(0.f, x));      // 7-i, then i^3: together i^4
    return dpp_f<0x128, 0xf>(0.f, x);                                         // row_ror:8 = i^8
}
template <int N, int S, int CUR>
__device__ __forceinline__ void row_sum_step(float (&x)[N], int l) {
    if constexpr (CUR >= 2) {
        constexpr int HALF = CUR / 2;
        const bool up = ((l >> S) & 1) != 0;
#pragma unroll
        for (int i = 0; i < HALF; ++i) {
            const float keep = up ? x[i + HALF] : x[i];
            const float send = up ? x[i] : x[i + HALF];
            x[i] = keep + row_xchg<S>(send);
        }
    } else {
        x[0] += row_xchg<S>(x[0]);
    }
}
template <int N>
__device__ __forceinline__ void row_sums(float (&x)[N], int lane) {
    static_assert(N >= 2 && (N & (N - 1)) == 0, "N must be a power of two");
    const int l = lane & 15;
    row_sum_step<N, 0, N>(x, l);
    row_sum_step<N, 1, (N >= 2 ? N / 2 : 1)>(x, l);
    row_sum_step<N, 2, (N >= 4 ? N / 4 : 1)>(x, l);
    row_sum_step<N, 3, (N >= 8 ? N / 8 : 1)>(x, l);
}
constexpr int pow2_at_least(int n) {
    int p = 2;
    while (p < n) p *= 2;
    return p;
}
__device__ __forceinline__ float wave_max(float x) {
    const float ninf = -__builtin_inff();
    x = fmaxf(x, dpp_f<0xB1, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x4E, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x141, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x140, 0xf>(ninf, x));
    x = fmaxf(x, dpp_f<0x142, 0xa>(ninf, x));
    x = fmaxf(x, dpp_f<0x143, 0xc>(ninf, x));
    return bcast_lane63(x);
}
__device__ __forceinline__ float wave_min(float x) {
    const float pinf = __builtin_inff();
    x = fminf(x, dpp_f<0xB1, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x4E, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x141, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x140, 0xf>(pinf, x));
    x = fminf(x, dpp_f<0x142, 0xa>(pinf, x));
    x = fminf(x, dpp_f<0x143, 0xc>(pinf, x));
    return bcast_lane63(x);
}
// Minimum over the wavefront of NON-NEGATIVE floats (energies), compared as unsigned integers: the ordering of
// non-negative IEEE floats is that of their bit patterns, +inf included, and no canonicalisation is needed.  The
// lane's own value is passed as the "old" operand, so lanes without a DPP source take min(x, x).
template <int CTRL, int ROWMASK>
__device__ __forceinline__ unsigned int dpp_self_u(unsigned int x) {
    return (unsigned int)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, ROWMASK, 0xf, false);
}
__device__ __forceinline__ float wave_min_nonneg(float xf) {
    unsigned int x = __float_as_uint(xf);
    x = min(x, dpp_self_u<0xB1, 0xf>(x));
    x = min(x, dpp_self_u<0x4E, 0xf>(x));
    x = min(x, dpp_self_u<0x141, 0xf>(x));
    x = min(x, dpp_self_u<0x140, 0xf>(x));
    x = min(x, dpp_self_u<0x142, 0xa>(x));
    x = min(x, dpp_self_u<0x143, 0xc>(x));
    return __uint_as_float((unsigned int)__builtin_amdgcn_readlane((int)x, 63));
}
__device__ __forceinline__ int wave_min_i(int x) {
    const int big = 0x7fffffff;
    x = min(x, dpp_i<0xB1, 0xf>(big, x));
    x = min(x, dpp_i<0x4E, 0xf>(big, x));
    x = min(x, dpp_i<0x141, 0xf>(big, x));
    x = min(x, dpp_i<0x140, 0xf>(big, x));
    x = min(x, dpp_i<0x142, 0xa>(big, x));
    x = min(x, dpp_i<0x143, 0xc>(big, x));
    return __builtin_amdgcn_readlane(x, 63);
}
__device__ __forceinline__ double wave_sum_d(double x) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) x += __shfl_xor(x, o, 64);
    return x;
}
// The same fixed-order DPP network as wave_sum, on float64 (moves the two 32-bit halves).
template <int CTRL, int ROWMASK>
__device__ __forceinline__ double dpp_d(double x) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, ROWMASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, ROWMASK, 0xf, false);
    return __hiloint2double(hi, lo);
}
// Sums of lanes 0..31 and of lanes 32..63; valid in lane 31 and lane 63 respectively.
__device__ __forceinline__ double half_sum_d_dpp(double x) {
    x += dpp_d<0xB1, 0xf>(x);
    x += dpp_d<0x4E, 0xf>(x);
    x += dpp_d<0x141, 0xf>(x);
    x += dpp_d<0x140, 0xf>(x);
    x += dpp_d<0x142, 0xa>(x);
    return x;
}
// Sum of all 64 lanes, returned to every lane.
__device__ __forceinline__ double wave_sum_d_dpp(double x) {
    x = half_sum_d_dpp(x);
    x += dpp_d<0x143, 0xc>(x);
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), 63);
    return __hiloint2double(hi, lo);
}
// Sum of lanes 0 .. N-1 (the other lanes must hold zero), valid in lane 0: only as many butterfly steps as N needs.
template <int N>
__device__ __forceinline__ double first_lanes_sum_d_dpp(double x) {
    if (N > 16) return wave_sum_d_dpp(x);
    if (N > 1) x += dpp_d<0xB1, 0xf>(x);
    if (N > 2) x += dpp_d<0x4E, 0xf>(x);
    if (N > 4) x += dpp_d<0x141, 0xf>(x);
    if (N > 8) x += dpp_d<0x140, 0xf>(x);
    return x;
}
// s / n for n > 0 without the IEEE division sequence: float32 reciprocal refined by two Newton steps in float64
// (the error of the reciprocal squares with each step), then one multiply.
__device__ __forceinline__ double fast_div_d(double s, double n) {
    double r = (double)__builtin_amdgcn_rcpf((float)n);  // relative error ~1e-7
    r = r * (2.0 - n * r);                               // ~1e-14
    r = r * (2.0 - n * r);                               // below float64 rounding
    return s * r;
}

// sqrt(x) and 1/x for the O(k d) float64 steps that sit on the critical path of a pass (one lane, every workgroup
// waiting): float32 seed refined by Newton steps in float64 instead of the IEEE sequences (several hundred cycles each).
// Outside the range a float32 seed covers they fall back to the exact routines.  Relative error below 1e-15.
__device__ __forceinline__ double fast_sqrt_d(double x) {
    if (!(x > 1e-30 && x < 1e30)) return sqrt(x);
    double r = (double)__builtin_amdgcn_rsqf((float)x);  // ~1e-7
    r = r * (1.5 - 0.5 * x * r * r);                     // ~1e-14
    r = r * (1.5 - 0.5 * x * r * r);
    const double s = x * r;
    return s + 0.5 * r * (x - s * s);                    // one correction of the root itself
}
__device__ __forceinline__ double fast_rcp_d(double x) {
    const double ax = fabs(x);
    if (!(ax > 1e-30 && ax < 1e30)) return 1.0 / x;
    double r = (double)__builtin_amdgcn_rcpf((float)x);
    r = r * (2.0 - x * r);
    r = r * (2.0 - x * r);
    return r;
}

// Sum of squares with every multiplication and addition rounded on its own, in index order.  This is the float32 key
// of the hard assignment for d > 1 and has to be the same number in every kernel and in a checker that emulates it;
// the compiler's default would fuse the additions into multiply-adds (and the rounded-operation intrinsics are plain
// operators in this toolchain), so contraction is switched off for these statements.
template <int D>
__device__ __forceinline__ float sum_sq_unfused(const float (&x)[D]) {
#pragma clang fp contract(off)
    float key = x[0] * x[0];
#pragma unroll
    for (int r = 1; r < D; ++r) {
        const float sq = x[r] * x[r];
        key = key + sq;
    }
    return key;
}
// x s - y with the product rounded on its own: when x s was rounded into y the result is exactly zero (a fused
// multiply-add would leave the product's rounding residual, with a sign).
__device__ __forceinline__ float scaled_minus_unfused(float x, float s, float y) {
#pragma clang fp contract(off)
    const float xs = x * s;
    return xs - y;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
__device__ __forceinline__ float fast_rsq(float x) { return __builtin_amdgcn_rsqf(x); }

// ---------------------------------------------------------------- stamped words

// Values that cross workgroups travel as 64-bit words {sequence number, 32-bit payload} written and read with
// relaxed device-scope atomics: a reader that finds the expected stamp has the value that belongs to it, so no
// fence (on this part: no write-back and invalidation of a whole L2) is needed on either side.
__device__ __forceinline__ unsigned long long ld_word(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_word(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long pack_f(unsigned int seq, float v) {
    return ((unsigned long long)seq << 32) | (unsigned long long)__float_as_uint(v);
}
__device__ __forceinline__ unsigned long long pack_u(unsigned int seq, unsigned int v) {
    return ((unsigned long long)seq << 32) | (unsigned long long)v;
}

// ---------------------------------------------------------------- grid-level tail: last workgroup reduces

// Called by all threads of a workgroup after its partials are stored.  Returns
// true in every thread of the one workgroup that arrives last.
// Arrival is counted in two levels: workgroup b adds to counter b mod TSHARDS, and the workgroup that completes a
// counter adds to the top one.  A thousand workgroups adding to ONE word from eight dies are served one after the
// other by the memory side (tens of microseconds); 32 words in separate cache lines are served side by side.
// The counters are zero between launches: the last workgroup clears them (grid_tail).
constexpr int TSHARDS = 32;
constexpr int TSTRIDE = 32;  // 32-bit words between counters: one 128-byte line each
constexpr int TICKET_WORDS = (TSHARDS + 1) * TSTRIDE;
__device__ __forceinline__ bool arrive_last(unsigned int* tickets) {
    __shared__ int s_last;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int nwg = gridDim.x, ns = nwg < (unsigned)TSHARDS ? nwg : (unsigned)TSHARDS;
        const unsigned int sh = blockIdx.x % ns, members = (nwg - sh + ns - 1) / ns;
        int last = 0;
        if (__hip_atomic_fetch_add(&tickets[sh * TSTRIDE], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == members - 1u)
            last = (__hip_atomic_fetch_add(&tickets[TSHARDS * TSTRIDE], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ns - 1u) ? 1 : 0;
        s_last = last;
    }
    __syncthreads();
    return s_last != 0;
}

// (tot_out: LDS of the caller.)
// Sum over all workgroups of the stamped float32 partials xp[acc][wg] (written by every workgroup of this launch
// before it took its ticket) into tot[acc], float64, in a fixed order.  The counters say that every workgroup has
// issued its stores; the stamps say that a word has arrived, so a word that is still on its way is simply read
// again (bounded).  Returns false in every thread if a word never arrived.
__device__ __forceinline__ bool reduce_stamped(const Args& a, int nacc, unsigned int seq, double* tot_out) {
    __shared__ double s_red[8][WG];
    __shared__ int s_fail;
    const int tid = threadIdx.x, nwg = gridDim.x;
    const unsigned long long* xp = reinterpret_cast<const unsigned long long*>(a.partials);
    if (tid == 0) s_fail = 0;
    __syncthreads();
    for (int acc0 = 0; acc0 < nacc; acc0 += 8) {
        double s[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) s[u] = 0.0;
        for (int wg = tid; wg < nwg; wg += WG) {
            unsigned int spins = 0;
            for (;;) {
                unsigned long long w[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) w[u] = (acc0 + u < nacc) ? ld_word(xp + (size_t)(acc0 + u) * nwg + wg) : pack_f(seq, 0.f);
                bool ok = true;
#pragma unroll
                for (int u = 0; u < 8; ++u) ok = ok && ((unsigned int)(w[u] >> 32) == seq);
                if (ok) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) s[u] += (double)__uint_as_float((unsigned int)w[u]);
                    break;
                }
                if (++spins > (1u << 20)) {
                    s_fail = 1;
                    break;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s_red[u][tid] = s[u];
        __syncthreads();
        // thread (q, part) adds 8 consecutive entries of accumulator q, then a fixed 32-lane DPP network
        const int q = tid >> 5, part = tid & 31;
        double t = 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) t += s_red[q][part * 8 + u];
        t = half_sum_d_dpp(t);
        if (part == 31 && acc0 + q < nacc) tot_out[acc0 + q] = t;
        __syncthreads();
    }
    return s_fail == 0;
}

// Block-wide sum of one double per thread (fixed order); result to all threads.
__device__ __forceinline__ double block_sum_d(double x) {
    __shared__ double s_w[16];
    __shared__ double s_r;
    x = wave_sum_d_dpp(x);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += s_w[w];
        s_r = s;
    }
    __syncthreads();
    return s_r;
}
__device__ __forceinline__ int block_sum_i(int x) { return (int)(block_sum_d((double)x) + 0.5); }
// Three block-wide sums for the price of one (two barriers): x[0..2] are replaced by their totals in every thread.
__device__ __forceinline__ void block_sum_d3(double (&x)[3]) {
    __shared__ double s_w[16][3];
    __shared__ double s_r[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) x[q] = wave_sum_d_dpp(x[q]);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int q = 0; q < 3; ++q) s_w[threadIdx.x >> 6][q] = x[q];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        double t = 0.0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += s_w[w][threadIdx.x];
        s_r[threadIdx.x] = t;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 3; ++q) x[q] = s_r[q];
}

// Tail of a forward evaluation (Alg. 1: centre update and stop test).  tot holds
// [k][d+1] = (n_j, s_j).  A cluster with zero mass keeps its centre.
__device__ __forceinline__ void tail_forward(const Args& a, const double* tot) {
    const int k = a.k, d = a.d, kd = k * d;
    Ctrl* c = a.ctrl;
    // the control words are requested first, so that their way from memory overlaps the update below
    int iters0 = 0, max_iter = 0;
    double tol = 0.0;
    if (threadIdx.x == 0) {
        iters0 = c->iters;
        max_iter = c->max_iter;
        tol = c->tol;
    }
    double x[3] = {0.0, 0.0, 0.0};  // squared step, non-finite flag, empty clusters
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        int j = idx / d, r = idx - j * d;
        double n = tot[j * (d + 1)], s = tot[j * (d + 1) + 1 + r];
        double cold = a.Cd[idx];
        double cnew = (n > 0.0) ? fast_div_d(s, n) : cold;
        if (!(n > 0.0) && r == 0) x[2] += 1.0;
        if (!(n >= 0.0) || !(fabs(s) <= 1.7e308) || !(fabs(cnew) <= 1.7e308)) x[1] = 1.0;  // NaN or Inf anywhere
        double df = cnew - cold;
        x[0] += df * df;
        a.Cd[idx] = cnew;
        a.Cf[idx] = (float)cnew;
        if (r == 0) a.nd[j] = n;
    }
    block_sum_d3(x);
    if (threadIdx.x == 0) {
        const double res = sqrt(x[0]);
        const bool bad = x[1] > 0.0;
        const int iters = iters0 + 1;
        c->iters = iters;
        c->residual = res;
        c->empty = (int)(x[2] + 0.5);
        if (bad) c->nonfinite = 1;
        const bool conv = res < tol;
        c->converged = conv ? 1 : 0;
        if (conv || bad || iters >= max_iter) c->done = 1;
    }
}

// Tail of the evaluation at C* (Sec. 4.2 "plug it into F one time"): keeps n*, F*.
__device__ __forceinline__ void tail_final(const Args& a, const double* tot) {
    const int k = a.k, d = a.d, kd = k * d;
    Ctrl* c = a.ctrl;
    int empty = 0, bad = 0;
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        int j = idx / d, r = idx - j * d;
        double n = tot[j * (d + 1)], s = tot[j * (d + 1) + 1 + r];
        double f = (n > 0.0) ? s / n : a.Cd[idx];
        if (!(n > 0.0) && r == 0) empty++;
        if (!(n >= 0.0) || !(fabs(s) <= 1.7e308)) bad = 1;
        a.Fd[idx] = f;
        a.Ff[idx] = (float)f;
        if (r == 0) a.nd[j] = n;
        if (a.C_out) a.C_out[idx] = a.Cf[idx];
    }
    empty = block_sum_i(empty);
    bad = block_sum_i(bad);
    if (threadIdx.x == 0) {
        c->empty = empty;
        if (bad) c->nonfinite = 1;
        
    }
}

// Hs_j = (g_j / n_j) / tau as float32; zero for an empty cluster.
__device__ __forceinline__ void store_h(const Args& a, int idx, double g) {
    int j = idx / a.d;
    double n = a.nd[j];
    a.Hs[idx] = (n > 0.0) ? (float)(g / n * (double)a.inv_tau) : 0.f;
}

// Tail of B1: tot = v.  Starts the backward solve at g = v.
__device__ __forceinline__ void tail_b1(const Args& a, const double* tot) {
    const int kd = a.k * a.d;
    Ctrl* c = a.ctrl;
    double v2 = 0.0;
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        double v = tot[idx];
        a.vd[idx] = v;
        a.gd[idx] = v;
        store_h(a, idx, v);
        v2 += v * v;
    }
    v2 = block_sum_d(v2);
    if (c->b_mode == BWD_GMRES) {
        // minimal-residual solve from g = 0: the first residual is v itself, the first basis vector v/||v||
        const double inv = (v2 > 0.0 && v2 <= 1.7e308) ? 1.0 / sqrt(v2) : 0.0;
        for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
            const double q = a.vd[idx] * inv;
            a.gd[idx] = 0.0;
            a.kry[idx] = q;
            store_h(a, idx, q);
        }
    }
    if (threadIdx.x == 0) {
        c->k_phase = 0;
        c->k_j = 0;
        c->k_stall = 0;
        c->k_beta = sqrt(v2);
        if (c->b_mode == BWD_GMRES) {
            const int R = c->k_R;
            a.kry[(size_t)(R + 1) * kd + (size_t)R * (R + 1) + 2 * (size_t)R] = sqrt(v2);  // sv[0] = ||r_0||
        }
        c->b_vnorm = sqrt(v2);
        c->b_iters = 0;
        c->b_attempt = 0;
        c->b_grow = 0;
        c->b_halvings = 0;
        c->b_prev = __builtin_inf();
        c->b_residual = 0.0;
        c->b_converged = (c->b_mode == BWD_JFB) ? 1 : 0;
        c->b_done = (c->b_mode == BWD_JFB) ? 1 : 0;
        if (c->b_mode == BWD_GMRES && v2 == 0.0) {  // v = 0: g = 0 is the solution
            c->b_converged = 1;
            c->b_done = 1;
        }
        if (!(v2 <= 1.7e308)) {  // non-finite cotangent: nothing to iterate on
            c->nonfinite = 1;
            c->b_done = 1;
        }
        
    }
}

// Layout of the Krylov workspace for basis length R and n = k d unknowns (doubles):
//   Q  [(R+1)][n]   orthonormal basis          Hm [R][(R+1)]  Hessenberg columns, rotated in place to triangular
//   cs, sn [R]      Givens rotations           sv [R+1]       rotated right-hand side       y [R]  coefficients
__host__ __device__ inline size_t gm_doubles(int R, int n) {
    return (size_t)(R + 1) * n + (size_t)R * (R + 1) + 2 * (size_t)R + (size_t)(R + 1) + (size_t)R;
}

// Tail of one pass of the minimal-residual solve of (I - dF/dC*)^T g = v, the linear system whose solution the
// averaged iteration of Sec. 4.2 converges to (Eq. "grad", "inv").  Restarted GMRES from g = 0:
//   phase 0  tot = (dF/dC)^T q_j.  w = q_j - tot, orthogonalised twice against q_0..q_j (classical Gram-Schmidt,
//            one wavefront per inner product), Givens update of the least-squares problem; the cycle ends when the
//            estimated residual is below tol ||v||, after R vectors, or when w vanishes; then g += Q y.
//   phase 1  tot = (dF/dC)^T g.  True residual r = v + tot - g; ||r|| <= tol ||v|| is the stop test (the step
//            g+ - g of the undamped iteration IS r, so this is the same test); otherwise r/||r|| starts a new cycle.
// Every pass counts in b_iters.  Two consecutive cycles that leave more than 95 % of the residual end the solve
// unconverged (restarted GMRES can stagnate when I - dF/dC is far from definite).
__device__ __forceinline__ void tail_gmres(const Args& a, const double* tot) {
    const int n = a.k * a.d;
    Ctrl* c = a.ctrl;
    const int R = c->k_R;
    double* Q = a.kry;
    double* Hm = Q + (size_t)(R + 1) * n;
    double* cs = Hm + (size_t)R * (R + 1);
    double* sn = cs + R;
    double* sv = sn + R;
    double* y = sv + (R + 1);
    __shared__ double s_h[GM_RMAX + 1];
    __shared__ int s_next;  // 0 next basis vector, 1 cycle over: apply to g, 2 new cycle from the residual, 3 done
    __shared__ double s_scale;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;

    if (c->k_phase == 0) {
        const int j = c->k_j;
        const double* qj = Q + (size_t)j * n;
        double* w = Q + (size_t)(j + 1) * n;
        double* hcol = Hm + (size_t)j * (R + 1);
        for (int idx = tid; idx < n; idx += blockDim.x) w[idx] = qj[idx] - tot[idx];
        for (int round = 0; round < 2; ++round) {
            __syncthreads();
            for (int i = wave; i <= j; i += nw) {
                const double* qi = Q + (size_t)i * n;
                double p = 0.0;
                for (int idx = lane; idx < n; idx += 64) p += qi[idx] * w[idx];
                p = wave_sum_d_dpp(p);
                if (lane == 0) {
                    s_h[i] = p;
                    hcol[i] = round ? hcol[i] + p : p;
                }
            }
            __syncthreads();
            for (int idx = tid; idx < n; idx += blockDim.x) {
                double x = w[idx];
                for (int i = 0; i <= j; ++i) x -= s_h[i] * Q[(size_t)i * n + idx];
                w[idx] = x;
            }
        }
        __syncthreads();
        double w2 = 0.0;
        for (int idx = tid; idx < n; idx += blockDim.x) w2 += w[idx] * w[idx];
        w2 = block_sum_d(w2);
        if (tid == 0) {
            const double hn = sqrt(w2);
            // earlier rotations on the new column, then the rotation that removes hn
            for (int i = 0; i < j; ++i) {
                const double t0 = cs[i] * hcol[i] + sn[i] * hcol[i + 1];
                hcol[i + 1] = -sn[i] * hcol[i] + cs[i] * hcol[i + 1];
                hcol[i] = t0;
            }
            const double hj = hcol[j];
            const double rr = sqrt(hj * hj + hn * hn);
            const double cj = rr > 0.0 ? hj / rr : 1.0, sj = rr > 0.0 ? hn / rr : 0.0;
            cs[j] = cj;
            sn[j] = sj;
            hcol[j] = rr;
            sv[j + 1] = -sj * sv[j];
            sv[j] = cj * sv[j];
            const double est = fabs(sv[j + 1]);
            c->b_iters += 1;
            c->b_residual = est;
            const bool finite = (w2 <= 1.7e308) && (rr <= 1.7e308);
            const bool vanished = !(hn > 1e-14 * rr);  // the Krylov space is exhausted: the solution lies in it
            const bool last = (j + 1 >= R) || (c->b_iters + 1 >= c->b_max_iter);
            int next = 0;
            if (!finite) {
                c->nonfinite = 1;
                c->b_done = 1;
                next = 3;
            } else if (vanished || last || est <= 0.5 * c->b_tol * c->b_vnorm) {
                // back substitution of the (j+1) x (j+1) triangular system
                const int nj = (rr > 0.0) ? j + 1 : j;
                for (int i = nj - 1; i >= 0; --i) {
                    double t0 = sv[i];
                    for (int l = i + 1; l < nj; ++l) t0 -= Hm[(size_t)l * (R + 1) + i] * y[l];
                    y[i] = t0 / Hm[(size_t)i * (R + 1) + i];
                }
                c->k_j = nj;
                next = 1;
            } else {
                c->k_j = j + 1;
                s_scale = 1.0 / hn;
            }
            s_next = next;
            
        }
        __syncthreads();
        if (s_next == 0) {
            const double inv = s_scale;
            for (int idx = tid; idx < n; idx += blockDim.x) {
                const double q = w[idx] * inv;
                w[idx] = q;
                store_h(a, idx, q);
            }
        } else if (s_next == 1) {
            const int nj = c->k_j;
            for (int idx = tid; idx < n; idx += blockDim.x) {
                double g = a.gd[idx];
                for (int i = 0; i < nj; ++i) g += y[i] * Q[(size_t)i * n + idx];
                a.gd[idx] = g;
                store_h(a, idx, g);
            }
            if (tid == 0) c->k_phase = 1;
        }
        return;
    }

    // phase 1: true residual at g
    double r2 = 0.0;
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const double u = tot[idx];
        a.ud[idx] = u;
        const double r = a.vd[idx] + u - a.gd[idx];
        Q[idx] = r;
        r2 += r * r;
    }
    r2 = block_sum_d(r2);
    if (tid == 0) {
        const double beta = sqrt(r2);
        c->b_iters += 1;
        c->b_residual = beta;
        int next = 2;
        if (!(r2 <= 1.7e308)) {
            c->nonfinite = 1;
            c->b_done = 1;
            next = 3;
        } else if (beta <= c->b_tol * c->b_vnorm) {
            c->b_converged = 1;
            c->b_done = 1;
            next = 3;
        } else {
            c->k_stall = (beta > 0.95 * c->k_beta) ? c->k_stall + 1 : 0;
            if (c->k_stall >= 2 || c->b_iters + 2 > c->b_max_iter) {
                c->b_done = 1;
                next = 3;
            }
        }
        if (next == 2) {
            c->k_beta = beta;
            c->k_phase = 0;
            c->k_j = 0;
            sv[0] = beta;
            s_scale = 1.0 / beta;
        }
        s_next = next;
        
    }
    __syncthreads();
    if (s_next == 2) {
        const double inv = s_scale;
        for (int idx = tid; idx < n; idx += blockDim.x) {
            const double q = Q[idx] * inv;
            Q[idx] = q;
            store_h(a, idx, q);
        }
    }
    // when done, Hs already holds h(g)/tau from the end of the cycle: the final pass uses it as it is
}

// Tail of one pass of the averaged iteration (Sec. 4.2): tot = u = (dF/dC)^T g.
//   g+ = alpha (v + u) + (1 - alpha) g ; stop when ||g+ - g|| <= tol ||v||.
// A non-finite step or 5 consecutive growing steps restart from g = v with alpha/2.
__device__ __forceinline__ void tail_b2(const Args& a, const double* tot) {
    const int kd = a.k * a.d;
    Ctrl* c = a.ctrl;
    if (c->b_mode == BWD_GMRES) {
        tail_gmres(a, tot);
        return;
    }
    const double alpha = c->b_alpha;
    double d2 = 0.0;
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        double u = tot[idx];
        a.ud[idx] = u;
        double g = a.gd[idx];
        double gn = alpha * (a.vd[idx] + u) + (1.0 - alpha) * g;
        double df = gn - g;
        d2 += df * df;
        a.gd[idx] = gn;
    }
    d2 = block_sum_d(d2);
    __shared__ int s_restart;
    if (threadIdx.x == 0) {
        double dn = sqrt(d2);
        int restart = 0;
        c->b_iters += 1;
        c->b_attempt += 1;
        c->b_residual = dn;
        bool finite = (dn <= 1.7e308);
        bool diverged = false;
        if (!finite) {
            diverged = true;
        } else if (dn <= c->b_tol * c->b_vnorm) {
            c->b_converged = 1;
            c->b_done = 1;
        } else {
            c->b_grow = (dn > c->b_prev) ? c->b_grow + 1 : 0;
            if (c->b_grow >= 5) diverged = true;
            c->b_prev = dn;
        }
        if (!c->b_done && !diverged && c->b_attempt >= c->b_max_iter) c->b_done = 1;
        if (diverged) {
            if (c->b_halvings < 6) {
                c->b_alpha = alpha * 0.5;
                c->b_halvings += 1;
                c->b_attempt = 0;
                c->b_grow = 0;
                c->b_prev = __builtin_inf();
                restart = 1;
            } else {
                c->b_done = 1;
                if (!finite) c->nonfinite = 1;  // every damping factor tried ended in a non-finite step
            }
        }
        s_restart = restart;
        
    }
    __syncthreads();
    const int restart = s_restart;
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        double g = restart ? a.vd[idx] : a.gd[idx];
        if (restart) a.gd[idx] = g;
        store_h(a, idx, g);
    }
}

// Tail of the dense backward (Sec. 4.2, Eq. "grad"/"inv" taken literally): tot holds, for n = k d,
//   T[n][n]  T[(j,r)][(l,s)] = sum_i (w_ir - F_jr) a_ij a_il delta_il,s
//   U[n][d]  U[(j,r)][s]     = sum_i (w_ir - F_jr) a_ij delta_ij,s
//   V[n]     v = dL/dC*
// so that dF_jr/dc_ls = ([l == j] U[(j,r)][s] - T[(j,r)][(l,s)]) / (tau n_j).  Solves (I - dF/dC)^T g = v by
// Gauss-Jordan elimination with partial pivoting in float64 (the workgroup's threads update the augmented
// matrix in parallel) and leaves g, v and h/tau for the final pass.
__device__ __forceinline__ void tail_bj(const Args& a, const double* tot) {
    const int k = a.k, d = a.d, n = k * d, n1 = n + 1;
    Ctrl* c = a.ctrl;
    __shared__ double s_M[DENSE_MAX_KD * (DENSE_MAX_KD + 1)];
    __shared__ int s_piv, s_sing;
    const double* T = tot;
    const double* U = tot + n * n;
    const double* V = tot + n * n + n * d;
    // augmented matrix [I - J^T | v]: row (l,s), column (j,r)
    for (int t = threadIdx.x; t < n * n1; t += blockDim.x) {
        const int row = t / n1, col = t - row * n1;
        double val;
        if (col == n) {
            val = V[row];
        } else {
            const int l = row / d, s = row - l * d, j = col / d;
            const double nj = a.nd[j];
            double J = 0.0;
            if (nj > 0.0) J = ((l == j ? U[col * d + s] : 0.0) - T[col * n + row]) * ((double)a.inv_tau / nj);
            val = (row == col ? 1.0 : 0.0) - J;
        }
        s_M[t] = val;
    }
    if (threadIdx.x == 0) s_sing = 0;
    __syncthreads();
    for (int p = 0; p < n; ++p) {
        if (threadIdx.x == 0) {
            int best = p;
            double bv = fabs(s_M[p * n1 + p]);
            for (int i = p + 1; i < n; ++i) {
                const double x = fabs(s_M[i * n1 + p]);
                if (x > bv) {
                    bv = x;
                    best = i;
                }
            }
            s_piv = best;
            if (!(bv > 1e-300) || !(bv <= 1.7e308)) s_sing = 1;
        }
        __syncthreads();
        const int piv = s_piv;
        if (piv != p) {
            for (int j = threadIdx.x; j < n1; j += blockDim.x) {
                const double x = s_M[p * n1 + j];
                s_M[p * n1 + j] = s_M[piv * n1 + j];
                s_M[piv * n1 + j] = x;
            }
        }
        __syncthreads();
        // every thread owns at most two entries (n (n+1) <= 272 <= 2 blockDim); new values are formed before any is stored
        double nv[2];
        for (int u = 0; u < 2; ++u) {
            const int t = threadIdx.x + u * blockDim.x;
            nv[u] = 0.0;
            if (t < n * n1) {
                const int i = t / n1, j = t - i * n1;
                const double pp = s_M[p * n1 + p];
                nv[u] = (i == p) ? s_M[t] : s_M[t] - (s_M[i * n1 + p] / pp) * s_M[p * n1 + j];
            }
        }
        __syncthreads();
        for (int u = 0; u < 2; ++u) {
            const int t = threadIdx.x + u * blockDim.x;
            if (t < n * n1) s_M[t] = nv[u];
        }
        __syncthreads();
    }
    double v2 = 0.0;
    int bad = 0;
    for (int idx = threadIdx.x; idx < n; idx += blockDim.x) {
        const double g = s_M[idx * n1 + n] / s_M[idx * n1 + idx];
        const double v = V[idx];
        if (!(fabs(g) <= 1.7e308)) bad = 1;
        a.gd[idx] = g;
        a.vd[idx] = v;
        store_h(a, idx, g);
        v2 += v * v;
    }
    v2 = block_sum_d(v2);
    bad = block_sum_i(bad);
    if (threadIdx.x == 0) {
        const bool ok = !bad && !s_sing;
        c->b_vnorm = sqrt(v2);
        c->b_iters = 0;
        c->b_residual = 0.0;
        c->b_converged = ok ? 1 : 0;
        c->b_done = 1;
        if (!ok) c->nonfinite = 1;
        
    }
}

template <int PASS, int NACC>
__device__ __forceinline__ void grid_tail(const Args& a, unsigned int seq) {
    constexpr int nacc = NACC;
    if (!arrive_last(a.tickets)) return;
    if (threadIdx.x <= TSHARDS) a.tickets[threadIdx.x * TSTRIDE] = 0u;  // every workgroup has arrived
    if (threadIdx.x == 0) a.ctrl->launch_seq = seq;
    // the totals stay in LDS: the tail that follows reads them without a trip through memory
    __shared__ double s_tot[NACC];
    if (!reduce_stamped(a, nacc, seq, s_tot)) {
        if (threadIdx.x == 0) {  // ends the host's loops; the call reports a device error
            a.ctrl->abort_flag = 1;
            a.ctrl->done = 1;
            a.ctrl->b_done = 1;
        }
        return;
    }
    if (PASS == PASS_FWD) tail_forward(a, s_tot);
    if (PASS == PASS_FIN) tail_final(a, s_tot);
    if (PASS == PASS_B1) tail_b1(a, s_tot);
    if (PASS == PASS_B2) tail_b2(a, s_tot);
    if (PASS == PASS_BJ) tail_bj(a, s_tot);
}

// Copy of n floats from memory into LDS by a workgroup of NT threads, with up to eight loads of a thread in flight (16-byte
// loads where the source allows): a loop that waits for each load before it issues the next is bound by the memory
// latency -- 36 round trips for the 36 KB tile of a 2.4 M-weight layer, 9 us of a 184 us solve.
template <int NT>
__device__ __forceinline__ void load_tile(float* dst, const float* __restrict__ src, int n) {
    const int tid = threadIdx.x;
    typedef float f4 __attribute__((ext_vector_type(4)));
    if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        const int n4 = n >> 2;
        const f4* s4 = reinterpret_cast<const f4*>(src);
        int i = tid;
        for (; i + 7 * NT < n4; i += 8 * NT) {
            f4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = s4[i + u * NT];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[4 * (i + u * NT) + e] = v[u][e];
            }
        }
        for (; i + NT < n4; i += 2 * NT) {
            const f4 v0 = s4[i], v1 = s4[i + NT];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[4 * i + e] = v0[e];
                dst[4 * (i + NT) + e] = v1[e];
            }
        }
        for (; i < n4; i += NT) {
            const f4 v0 = s4[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[4 * i + e] = v0[e];
        }
        for (int k = (n4 << 2) + tid; k < n; k += NT) dst[k] = src[k];
        return;
    }
    int i = tid;
    for (; i + 7 * NT < n; i += 8 * NT) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * NT];
#pragma unroll
        for (int u = 0; u < 8; ++u) dst[i + u * NT] = v[u];
    }
    for (; i < n; i += NT) dst[i] = src[i];
}

}  // namespace idkm
