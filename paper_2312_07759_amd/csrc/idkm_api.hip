// C ABI of the IDKM library: argument validation, scratch management and the
// scheduling of passes over W.  All arithmetic of the method runs in the kernels.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <algorithm>
#include <string>
#include <vector>

#include "../../include/idkm.h"
#include "common.hpp"
#include "dispatch.h"
#include "persist_small.hpp"
#include "persist_lane.hpp"

namespace idkm {
KernelFn small_kernel_0(int, int, int);
KernelFn small_kernel_1(int, int, int);
KernelFn lane_kernel_0(int, int, int);
KernelFn lane_kernel_1(int, int, int);

KernelFn small_kernel(int K, int D, int dist, int pass) {
    return dist == DIST_L2 ? small_kernel_0(K, D, pass) : small_kernel_1(K, D, pass);
}
PersistFns persist_lane_kernel_0(int, int, bool, bool);
PersistFns persist_lane_kernel_1(int, int, bool, bool);
PersistFns persist_lane_kernel(int KPL, int D, int dist, bool bwd, bool matrix) {
    return dist == DIST_L2 ? persist_lane_kernel_0(KPL, D, bwd, matrix) : persist_lane_kernel_1(KPL, D, bwd, matrix);
}
KernelFn lane_kernel(int KPL, int D, int dist, int pass) {
    return dist == DIST_L2 ? lane_kernel_0(KPL, D, pass) : lane_kernel_1(KPL, D, pass);
}

constexpr int MAX_K = 1024, MAX_D = 8, MAX_KD = 4096;
constexpr int MAX_NACC = MAX_K * 5 > MAX_KD + MAX_K ? MAX_K * 5 : MAX_KD + MAX_K;  // k (d+1) <= kd + k

// ---------------------------------------------------------------- small utility kernels

__global__ void k_init_forward(Args a, const float* C0, double tol, int max_iter) {
    const int kd = a.k * a.d;
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        float c = C0[idx];
        a.Cd[idx] = (double)c;
        a.Cf[idx] = c;
    }
    if (threadIdx.x == 0) {
        Ctrl* c = a.ctrl;
        c->abort_flag = 0;
        c->done = 0;
        c->iters = 0;
        c->converged = 0;
        c->empty = 0;
        c->nonfinite = 0;
        c->max_iter = max_iter;
        c->residual = 0.0;
        c->tol = tol;
        c->b_done = 1;
    }
}

__global__ void k_init_backward(Args a, int mode, double tol, int max_iter, double alpha, int basis) {
    Ctrl* c = a.ctrl;
    c->abort_flag = 0;
    c->nonfinite = 0;  // (a forward on the persistent path does not pass through k_init_forward)
    c->b_done = 0;
    c->b_iters = 0;
    c->b_converged = 0;
    c->b_attempt = 0;
    c->b_grow = 0;
    c->b_halvings = 0;
    c->b_max_iter = max_iter;
    c->b_mode = mode;
    c->b_alpha = alpha;
    c->b_prev = __builtin_inf();
    c->b_vnorm = 0.0;
    c->b_residual = 0.0;
    c->b_tol = tol;
    const int kd = a.k * a.d;
    c->k_R = kd < basis ? kd : basis;
    c->k_phase = 0;
    c->k_j = 0;
    c->k_stall = 0;
    c->k_beta = 0.0;
}

__global__ void k_reset_launch_seq(Ctrl* c) { c->launch_seq = 0; }
__global__ void k_add_launch_seq(Ctrl* c, unsigned int n) { c->launch_seq += n; }

// Hs = (g / n) / tau from a caller-supplied float32 cotangent; arms one raw (dF/dC)^T pass.
__global__ void k_set_g(Args a, const float* g) {
    const int kd = a.k * a.d;
    for (int idx = threadIdx.x; idx < kd; idx += blockDim.x) {
        double gv = (double)g[idx];
        a.gd[idx] = gv;
        a.vd[idx] = 0.0;
        store_h(a, idx, gv);
    }
    if (threadIdx.x == 0) {
        Ctrl* c = a.ctrl;
        c->b_done = 0;
        c->b_iters = 0;
        c->b_attempt = 0;
        c->b_grow = 0;
        c->b_halvings = 0;
        c->b_max_iter = 1;
        c->b_alpha = 1.0;
        c->b_prev = __builtin_inf();
        c->b_vnorm = 0.0;
        c->b_tol = 0.0;
    }
}

__global__ void k_fill_u64(unsigned long long* p, size_t n, unsigned long long v) {
    for (size_t i = threadIdx.x + (size_t)blockIdx.x * blockDim.x; i < n; i += (size_t)blockDim.x * gridDim.x) p[i] = v;
}

__global__ void k_f64_to_f32(const double* src, float* dst, int n) {
    for (int i = threadIdx.x + blockIdx.x * blockDim.x; i < n; i += blockDim.x * gridDim.x) dst[i] = (float)src[i];
}

}  // namespace idkm

using namespace idkm;

namespace {
struct Deferred;
}

struct idkm_ctx {
    int device = 0;
    std::string err;
    idkm_path path = IDKM_PATH_AUTO;
    // device scratch
    Ctrl* ctrl = nullptr;
    Ctrl* h_ctrl = nullptr;  // pinned host mirror
    unsigned int* tickets = nullptr;  // arrival counters of the stream path, zero between launches
    unsigned int stream_launches = 0; // upper bound of Ctrl::launch_seq
    bool wide_tail = false;           // lane family, GMRES with k d >= 512: the pass tail runs with 1024 threads
    int gmres_basis = 64;             // basis length of IDKM_BWD_GMRES before a restart (idkm_set_gmres_basis, <= GM_RMAX)
    double *Cd = nullptr, *nd = nullptr, *Fd = nullptr, *gd = nullptr, *vd = nullptr, *ud = nullptr;
    float *Cf = nullptr, *Ff = nullptr, *Hs = nullptr;
    double *stage = nullptr, *tot = nullptr;
    double* partials = nullptr;
    size_t partials_cap = 0;  // in doubles
    double* kry = nullptr;    // Krylov workspace of IDKM_BWD_GMRES (allocated on first use)
    size_t kry_cap = 0;       // in doubles
    // persistent path
    int num_cu = 0;
    bool coop = false;
    bool coop_launch = false;  // IDKM_COOPERATIVE=1 launches the persistent kernels cooperatively
    int min_vec_per_thread = 4;  // vectors per thread before another workgroup is added (IDKM_MIN_VPT)
    bool tree_exchange = true;   // two-level (die-local, then cross-die) exchange for full-device teams (IDKM_TREE=0: off)
    bool tree_remote = false;    // IDKM_TREE=2: hop 1 with device-scope stores, as for workgroups that are not on their leader's die
    // idkm_set_kernel_timing: events recorded on the caller's stream right before and after a persistent launch
    bool timing = false;
    bool timed = false;          // ev0 / ev1 bracket the last persistent launch
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    unsigned long long* xbuf = nullptr;  // exchange words: buf1 [2][PT][XLINE], then buf2 [2][XBCAST]
    size_t xbuf_words = 0;
    unsigned int seq_base = 0;
    unsigned long long* lane_xbuf = nullptr;  // exchange words of the lane<->codeword persistent kernels (lazy)
    unsigned int* abort_word = nullptr;  // device
    PResult* h_res = nullptr;            // pinned host; device memory when res_on_device
    bool res_on_device = false;          // the context of idkm_forward_noalloc: the kernel reports into device memory
    PResult res_copy;                    // ... and the host reads this copy of it
    int last_empty = 0;                  // empty clusters seen by the last forward
    // a persistent launch whose result has not been collected yet (batched calls defer the wait)
    bool defer_wait = false;
    int pending_kind = 0;  // 0 none, 1 forward, 2 backward
    unsigned int pending_id = 0;
    hipStream_t pending_stream = nullptr;
    std::vector<Deferred>* sink = nullptr;  // set by a batched call: persistent launches are handed over, not issued
    std::map<const void*, std::pair<size_t, int>> checked;  // kernel -> (largest LDS size set, blocks per CU at that size)
    std::map<const void*, size_t> static_lds;               // bytes of static LDS of the kernels whose dynamic LDS is sized against it
    unsigned int spin_limit = 1u << 20;
    bool use_matrix = true;           // d = 4, 17 <= k <= 256: matrix-core kernels where they exist
    size_t tile_limit = 144 * 1024;   // largest tile of W (and dL/dWq) a persistent workgroup of the lane<->vector family keeps in LDS
#ifdef IDKM_TRACE
    long long* trace = nullptr;
#endif
    // forward state
    bool has_forward = false;
    bool has_backward = false;  // a backward has been issued since the last forward: vd, gd hold its v and g
    const float* W = nullptr;
    int64_t m = 0;
    int d = 0, k = 0, dist = 0;
    float tau = 0.f;
};

namespace {

idkm_status fail(idkm_ctx* ctx, idkm_status s, const std::string& msg) {
    if (ctx) ctx->err = msg;
    return s;
}

#define HIP_TRY(ctx, expr)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return fail(ctx, IDKM_ERR_DEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

struct Geometry {
    bool small;    // lane<->vector family
    int kpl;       // lane<->codeword family: codewords per lane
    int nwg;       // workgroups per pass
    int64_t vec_per_wg;
    // d = 4, 17 <= k <= 256: the forward loop and the squared energy's (dF/dC)^T pass have a matrix-core form
    bool matrix = false;
    int nwg_m = 0;
    int64_t vec_per_wg_m = 0;
};

bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// Which kernel family serves (k, d), and how a pass is cut into workgroups.
idkm_status plan(idkm_ctx* ctx, int64_t m, int k, int d, Geometry* g) {
    if (k > MAX_K || d > MAX_D || (int64_t)k * d > MAX_KD)
        return fail(ctx, IDKM_ERR_UNSUPPORTED, "shape exceeds idkm_limits (k<=1024, d<=8, k*d<=4096)");
    if (!(d == 1 || d == 2 || d == 4 || d == 8)) return fail(ctx, IDKM_ERR_UNSUPPORTED, "d must be 1, 2, 4 or 8");
    g->small = (k >= 2 && k <= 16 && pow2(k) && d <= 4);
    if (g->small) {
        int64_t vpt = (m + (int64_t)WG * 1024 - 1) / ((int64_t)WG * 1024);
        if (vpt < 1) vpt = 1;
        if (vpt > 32) vpt = 32;
        g->vec_per_wg = (int64_t)WG * vpt;
        g->kpl = 0;
    } else {
        int kpl = (k + 63) / 64, p = 1;
        while (p < kpl) p <<= 1;
        g->kpl = p;
        if (p * (d + 1) > 80) return fail(ctx, IDKM_ERR_UNSUPPORTED, "ceil(k/64)*(d+1) must be <= 80");
        // about 1024 workgroups for mid-sized layers, never more than 2048 (their partials are reduced afterwards)
        int64_t vpw = (m + 4095) / 4096;
        if (vpw < 1) vpw = 1;
        if (vpw > 512) vpw = (m + 8191) / 8192 > 512 ? (m + 8191) / 8192 : 512;
        g->vec_per_wg = vpw * (WG / 64);
    }
    int64_t nwg = (m + g->vec_per_wg - 1) / g->vec_per_wg;
    if (nwg > 0x3fffffff) return fail(ctx, IDKM_ERR_UNSUPPORTED, "m too large");
    g->nwg = (int)nwg;
    g->matrix = false;
    if (!g->small && d == 4 && g->kpl <= 4 && ctx->use_matrix) {
        // one workgroup of 512 threads per compute unit and round where the layer allows it; a chunk is a whole
        // number of 16-vector steps for each of the 8 wavefronts and at most 46 KB of LDS
        int64_t v = (m + ctx->num_cu - 1) / (ctx->num_cu > 0 ? ctx->num_cu : 1);
        v = (v + 127) / 128 * 128;
        if (v > 2304) v = 2304;
        const int64_t n = (m + v - 1) / v;
        if (n <= nwg) {  // the partial-sum buffer is sized for nwg workgroups
            g->matrix = true;
            g->vec_per_wg_m = v;
            g->nwg_m = (int)n;
        }
    }
    return IDKM_OK;
}

idkm_status ensure_partials(idkm_ctx* ctx, size_t need) {
    if (need <= ctx->partials_cap) return IDKM_OK;
    if (ctx->partials) {
        (void)hipDeviceSynchronize();  // earlier launches may still read the old buffer
        (void)hipFree(ctx->partials);
        ctx->partials = nullptr;
        ctx->partials_cap = 0;
    }
    if (hipMalloc(&ctx->partials, need * sizeof(double)) != hipSuccess)
        return fail(ctx, IDKM_ERR_ALLOC, "hipMalloc of the partial-sum buffer failed");
    // stamped words: sequence number 0 is never used, so a cleared buffer holds no valid word
    HIP_TRY(ctx, hipMemset(ctx->partials, 0, need * sizeof(double)));
    ctx->partials_cap = need;
    return IDKM_OK;
}

Args base_args(idkm_ctx* ctx) {
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.W = ctx->W;
    a.m = ctx->m;
    a.k = ctx->k;
    a.d = ctx->d;
    a.tau = ctx->tau;
    a.inv_tau = 1.0f / ctx->tau;
    a.nscale = (float)(-1.4426950408889634 / (double)ctx->tau);
    a.escale = (ctx->dist == DIST_SQL2) ? (float)std::sqrt(1.4426950408889634 / (double)ctx->tau)
                                        : (float)(1.4426950408889634 / (double)ctx->tau);
    a.ctrl = ctx->ctrl;
    a.tickets = ctx->tickets;
    a.Cd = ctx->Cd;
    a.Cf = ctx->Cf;
    a.nd = ctx->nd;
    a.Fd = ctx->Fd;
    a.Ff = ctx->Ff;
    a.gd = ctx->gd;
    a.vd = ctx->vd;
    a.ud = ctx->ud;
    a.Hs = ctx->Hs;
    a.partials = ctx->partials;
    a.kry = ctx->kry;
    a.stage = ctx->stage;
    a.tot = ctx->tot;
    return a;
}

idkm_status launch_pass(idkm_ctx* ctx, const Geometry& g, int pass, Args& a, hipStream_t s) {
    KernelFn fn = g.small ? small_kernel(ctx->k, ctx->d, ctx->dist, pass) : lane_kernel(g.kpl, ctx->d, ctx->dist, pass);
    KernelFn fn_m = g.matrix ? mfma_lane_kernel(g.kpl, ctx->dist, pass) : nullptr;
    if (!fn && !fn_m) return fail(ctx, IDKM_ERR_UNSUPPORTED, "no kernel for this (k, d)");
    const int nwg = fn_m ? g.nwg_m : g.nwg;
    a.vec_per_wg = fn_m ? g.vec_per_wg_m : g.vec_per_wg;
    if (++ctx->stream_launches > 0x7fff0000u) {
        // the sequence numbers that stamp the partial sums would wrap: start over from a cleared buffer
        hipLaunchKernelGGL(k_fill_u64, dim3(256), dim3(256), 0, s, reinterpret_cast<unsigned long long*>(ctx->partials),
                           ctx->partials_cap, 0ull);
        hipLaunchKernelGGL(k_reset_launch_seq, dim3(1), dim3(1), 0, s, ctx->ctrl);
        HIP_TRY(ctx, hipGetLastError());
        ctx->stream_launches = 1;
    }
    if (fn_m)
        hipLaunchKernelGGL(fn_m, dim3(nwg), dim3(mfma_lane_threads(g.kpl, ctx->dist, pass)), (size_t)(a.vec_per_wg + 16) * 20, s, a);
    else
        hipLaunchKernelGGL(fn, dim3(nwg), dim3(WG), 0, s, a);
    HIP_TRY(ctx, hipGetLastError());
    if (!g.small && pass != PASS_B3) {
        // this family carries k (d+1) sums per workgroup: a many-workgroup reduction, then a one-workgroup tail
        const int nacc = ctx->k * ((pass == PASS_FWD || pass == PASS_FIN) ? ctx->d + 1 : ctx->d);
        launch_reduce_rows(a, nacc, nwg, pass, s);
        HIP_TRY(ctx, hipGetLastError());
        if (pass == PASS_B2 && ctx->wide_tail)
            hipLaunchKernelGGL(lane_tail_wide_kernel(), dim3(1), dim3(1024), 0, s, a);
        else
            hipLaunchKernelGGL(lane_tail_kernel(pass), dim3(1), dim3(WG), 0, s, a);
        HIP_TRY(ctx, hipGetLastError());
    }
    return IDKM_OK;
}

constexpr size_t XBUF1_WORDS = (size_t)2 * PT * XLINE;
constexpr size_t XBUF3_WORDS = (size_t)2 * DIES * XLINE;  // two-level exchange: totals of the dies
constexpr size_t XBUF_WORDS = XBUF1_WORDS + (size_t)2 * XBCAST + XBUF3_WORDS + DIES;
constexpr size_t LDS_TILE_MAX = 144 * 1024;  // bytes of LDS a persistent workgroup may use for its tile

struct PersistPlan {
    PersistFn fn;
    PersistBatchFn fn_batch;
    int grid, per, threads;
    bool lane;  // lane<->codeword family: own exchange buffers
    size_t lds;
};
// A persistent solve that a batched call will launch together with others.
struct Deferred {
    idkm_ctx* ctx;
    PersistPlan pp;
    Args a;
    PArgs pa;
};
constexpr size_t LDS_PER_CU = 160 * 1024;
constexpr size_t LANE_TILE_MAX = 94 * 1024;                       // the lane kernels keep ~55 KB of static LDS
constexpr size_t LANE_BUF1_WORDS = (size_t)2 * PT * 1536;          // k (d+1) <= 1536
constexpr size_t LANE_BUF2_WORDS = (size_t)2 * (1024 + 512);       // k d + k


// Can (m, k, d) run as one persistent launch with `tiles` resident tensors (1: W; 2: W and dL/dWq)?
// matrix_ok: the matrix-core kernels may serve the call (every pass of both energies has a matrix-core form).
// dwq: the backward's upstream gradient (a layer too large for LDS is streamed from memory with 16-byte loads, which
// W and dL/dWq must allow).
bool plan_persistent(idkm_ctx* ctx, bool bwd, PersistPlan* pp, bool matrix_ok = true, const void* dwq = nullptr) {
    if (!ctx->coop || ctx->num_cu < 1) return false;
    const int k = ctx->k, d = ctx->d;
    const int64_t m = ctx->m;
    if (!(k >= 2 && k <= 16 && pow2(k) && d <= 4)) {
        // lane<->codeword family
        int kpl = (k + 63) / 64, p = 1;
        while (p < kpl) p <<= 1;
        if (d > 4 || p * d > 16 || p * (d + 1) > 24) return false;
        int64_t g = (m + 255) / 256;  // at least 16 vectors per wavefront before adding workgroups
        if (g < 1) g = 1;
        if (g > ctx->num_cu) g = ctx->num_cu;
        if (g > PT) g = PT;
        int64_t per = (m + g - 1) / g;
        per = (per + 3) / 4 * 4;
        PersistFns fl = persist_lane_kernel(p, d, ctx->dist, bwd, matrix_ok && ctx->use_matrix);
        size_t lds = (size_t)per * d * sizeof(float) * (bwd ? 2 : 1);
        if (fl.matrix) {
            // tile padded by 16 vectors, then one float per vector (dL/dWq is not kept); these kernels hold more
            // static LDS than the vector-ALU ones.  A tile too large for what is left goes to the vector-ALU kernel.
            const size_t lds_m = (size_t)(per + 16) * (d + 1) * sizeof(float);
            size_t& fixed = ctx->static_lds[(const void*)fl.one];
            if (fixed == 0) {
                hipFuncAttributes at;
                fixed = (hipFuncGetAttributes(&at, (const void*)fl.one) == hipSuccess) ? at.sharedSizeBytes : LDS_PER_CU;
                (void)hipGetLastError();
            }
            if (fixed + lds_m <= LDS_PER_CU) {
                pp->fn = fl.one;
                pp->fn_batch = fl.batch;
                pp->grid = (int)((m + per - 1) / per);
                pp->per = (int)per;
                pp->lds = lds_m;
                pp->threads = fl.threads;
                pp->lane = true;
                return true;
            }
            fl = persist_lane_kernel(p, d, ctx->dist, bwd, false);
        }
        pp->fn = fl.one;
        pp->fn_batch = fl.batch;
        if (!pp->fn) return false;
        if (lds > LANE_TILE_MAX) return false;
        pp->grid = (int)((m + per - 1) / per);
        pp->per = (int)per;
        pp->lds = lds;
        pp->threads = LT;
        pp->lane = true;
        return true;
    }
    if (k * (d + 1) > XLINE) return false;
    const PersistFns fs = persist_kernel(k, d, ctx->dist, bwd);
    pp->fn = fs.one;
    pp->fn_batch = fs.batch;
    if (!pp->fn) return false;
    pp->threads = PT;
    pp->lane = false;
    const int64_t chunk = (int64_t)ctx->min_vec_per_thread * PT;
    int64_t g = (m + chunk - 1) / chunk;  // a few vectors per thread before adding workgroups
    // up to 16 vectors per thread one workgroup alone is faster (measured: 2.7 us per pass at m = 4096 against 3.7):
    // it needs no exchange through memory
    if (m <= (int64_t)16 * PT) g = 1;
    if (g < 1) g = 1;
    // (a team of 2 to 7 workgroups would take the one-level exchange; 8 smaller workgroups take the two-level one)
    if (ctx->tree_exchange && g > 1 && g < DIES) g = DIES;
    if (g > ctx->num_cu) g = ctx->num_cu;
    if (g > PT) g = PT;  // a reducer reads one workgroup per thread
    int64_t per = (m + g - 1) / g;
    per = (per + 3) / 4 * 4;
    const size_t lds = (size_t)per * d * sizeof(float) * (bwd ? 2 : 1);
    pp->grid = (int)((m + per - 1) / per);
    pp->per = (int)per;
    pp->lds = lds;
    if (lds > ctx->tile_limit) {
        // the layer does not fit on chip: the same solve with W (and dL/dWq) read from memory in every pass.  Not
        // inside a batched launch (such a layer fills the device on its own), and only from 16-byte aligned tensors.
        const PersistFns fg = persist_kernel_global(k, d, ctx->dist, bwd);
        const bool aligned = (reinterpret_cast<uintptr_t>(ctx->W) & 15u) == 0 &&
                             (!bwd || (dwq && (reinterpret_cast<uintptr_t>(dwq) & 15u) == 0));
        // Measured on a 16.8 M-weight layer this form is within 5 % of the stream path (forward 28.3 against 29.9 us
        // per evaluation, (dF/dC)^T pass 41.3 against 39.7): both are bound by the same arithmetic, so the default
        // keeps the stream path and this one serves callers that ask for the persistent path (one launch per solve).
        if (!fg.one || ctx->sink || !aligned || ctx->path != IDKM_PATH_PERSISTENT) return false;
        pp->fn = fg.one;
        pp->fn_batch = nullptr;
        pp->lds = 0;
    }
    return true;
}

idkm_status launch_persistent(idkm_ctx* ctx, const PersistPlan& pp, Args& a, PArgs pa, unsigned int exchanges,
                              hipStream_t s) {
    if (pp.grid > PT || ctx->xbuf_words < XBUF_WORDS) return fail(ctx, IDKM_ERR_DEVICE, "exchange buffer too small");
    if (ctx->seq_base > 0xffffffffu - exchanges - 2u) {  // stamps would wrap: start over from clean buffers
        hipLaunchKernelGGL(k_fill_u64, dim3(64), dim3(256), 0, s, ctx->xbuf, ctx->xbuf_words, 0ull);
        HIP_TRY(ctx, hipGetLastError());
        if (ctx->lane_xbuf) {
            hipLaunchKernelGGL(k_fill_u64, dim3(256), dim3(256), 0, s, ctx->lane_xbuf, LANE_BUF1_WORDS + LANE_BUF2_WORDS, 0ull);
            HIP_TRY(ctx, hipGetLastError());
        }
        ctx->seq_base = 0;
    }
    if (pp.lane) {
        if (!ctx->lane_xbuf) {
            const size_t bytes = (LANE_BUF1_WORDS + LANE_BUF2_WORDS) * sizeof(unsigned long long);
            if (hipMalloc(&ctx->lane_xbuf, bytes) != hipSuccess)
                return fail(ctx, IDKM_ERR_ALLOC, "hipMalloc of the exchange buffer failed");
            hipLaunchKernelGGL(k_fill_u64, dim3(256), dim3(256), 0, s, ctx->lane_xbuf, LANE_BUF1_WORDS + LANE_BUF2_WORDS, 0ull);
            HIP_TRY(ctx, hipGetLastError());
        }
        pa.buf1 = ctx->lane_xbuf;
        pa.buf2 = ctx->lane_xbuf + LANE_BUF1_WORDS;
    } else {
        pa.buf1 = ctx->xbuf;
        pa.buf2 = ctx->xbuf + XBUF1_WORDS;
        pa.buf3 = pa.buf2 + (size_t)2 * XBCAST;
        pa.tab = pa.buf3 + XBUF3_WORDS;
        // teams of DIES workgroups or more: hop 1 stays inside each die (the explicit-Jacobian mode keeps the plain
        // exchange, its one reduction ends in workgroup 0).  Also inside a batched launch: a team's workgroups are
        // consecutive in the grid, so its first DIES lie on DIES different dies and member i shares its die with member
        // i mod DIES wherever the team starts (checked by every workgroup at the start of the launch, as always)
        pa.tree = (ctx->tree_exchange && pp.grid >= TREE_MIN_G && pa.mode != BWD_DENSE) ? (ctx->tree_remote ? 2 : 1) : 0;
    }
    pa.seq_base = ctx->seq_base;
    pa.spin_limit = ctx->spin_limit;
    pa.per = pp.per;
    pa.abort_word = ctx->abort_word;
    pa.out = ctx->h_res;
    if (ctx->res_on_device) {
        static_assert(sizeof(PResult) % sizeof(unsigned long long) == 0, "PResult is cleared in 64-bit words");
        hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(64), 0, s, reinterpret_cast<unsigned long long*>(ctx->h_res),
                           sizeof(PResult) / sizeof(unsigned long long), 0ull);
        HIP_TRY(ctx, hipGetLastError());
    } else {
        std::memset(ctx->h_res, 0, sizeof(PResult));
    }
#ifdef IDKM_TRACE
    pa.trace = ctx->trace;
#endif
    if (ctx->sink) {
        // part of a batched call: the batch launches this solve together with others of its shape
        ctx->sink->push_back(Deferred{ctx, pp, a, pa});
        ctx->pending_id = ctx->seq_base + 1u;
        ctx->pending_stream = s;
        ctx->seq_base += exchanges;
        return IDKM_OK;
    }
    // attribute and occupancy are queried once per (kernel, LDS size); later launches reuse the answer
    auto& checked = ctx->checked[(const void*)pp.fn];
    if (checked.second == 0 || checked.first < pp.lds) {
        HIP_TRY(ctx, hipFuncSetAttribute((const void*)pp.fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pp.lds));
        int nb = 0;
        HIP_TRY(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)pp.fn, pp.threads, pp.lds));
        if (nb < 1) return fail(ctx, IDKM_ERR_DEVICE, "persistent workgroup does not fit a compute unit");
        checked.first = pp.lds;
        checked.second = nb;
    }
    if ((int64_t)checked.second * ctx->num_cu < pp.grid)
        return fail(ctx, IDKM_ERR_DEVICE, "persistent grid would not be co-resident");
    if (ctx->timing) HIP_TRY(ctx, hipEventRecord(ctx->ev0, s));
    if (ctx->coop_launch) {
        void* args[] = {(void*)&a, (void*)&pa};
        HIP_TRY(ctx, hipLaunchCooperativeKernel((const void*)pp.fn, dim3(pp.grid), dim3(pp.threads), args, pp.lds, s));
    } else {
        // plain launch: the grid fits the device (checked above), every wait in the kernel is bounded
        hipLaunchKernelGGL(pp.fn, dim3(pp.grid), dim3(pp.threads), pp.lds, s, a, pa);
        HIP_TRY(ctx, hipGetLastError());
    }
    if (ctx->timing) {
        HIP_TRY(ctx, hipEventRecord(ctx->ev1, s));
        ctx->timed = true;
    }
    ctx->pending_id = ctx->seq_base + 1u;
    ctx->pending_stream = s;
    ctx->seq_base += exchanges;
    return IDKM_OK;
}

// Waits for the persistent launch recorded in ctx->pending_* and turns what the kernel reported (pinned host
// memory: one wait, no copy) into a status and an idkm_info.
idkm_status finish_persistent(idkm_ctx* ctx, idkm_info* info) {
    const int kind = ctx->pending_kind;
    if (!kind) return IDKM_OK;
    ctx->pending_kind = 0;
    if (ctx->res_on_device)
        HIP_TRY(ctx, hipMemcpyAsync(&ctx->res_copy, ctx->h_res, sizeof(PResult), hipMemcpyDeviceToHost, ctx->pending_stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->pending_stream));
    const PResult& c = ctx->res_on_device ? ctx->res_copy : *ctx->h_res;
    if (c.done != ctx->pending_id) return fail(ctx, IDKM_ERR_DEVICE, "a grid-wide wait hit its limit");
    if (kind == 1) {
        for (int r = 0; r < c.nred && r < 16; ++r)
            if (c.fin[r] != ctx->pending_id) return fail(ctx, IDKM_ERR_DEVICE, "a grid-wide wait hit its limit");
        int empty = 0, bad = c.nonfinite;
        for (int r = 0; r < 16; ++r) {
            empty += c.empty[r];
            bad |= c.bad[r];
        }
        if (bad) return fail(ctx, IDKM_ERR_NONFINITE, "the codebook became non-finite");
        ctx->has_forward = true;
        ctx->last_empty = empty;
        if (info) {
            info->iters = c.iters;
            info->converged = c.converged;
            info->residual = c.residual;
            info->empty_clusters = empty;
            info->path = IDKM_PATH_PERSISTENT;
            info->alpha = 0.0;
        }
    } else {
        if (c.nonfinite) return fail(ctx, IDKM_ERR_NONFINITE, "the cotangent became non-finite");
        if (info) {
            info->iters = c.iters;
            info->converged = c.converged;
            info->residual = c.residual;
            info->empty_clusters = ctx->last_empty;
            info->path = IDKM_PATH_PERSISTENT;
            info->alpha = c.alpha;
        }
    }
    return IDKM_OK;
}

idkm_status read_ctrl(idkm_ctx* ctx, hipStream_t s) {
    HIP_TRY(ctx, hipMemcpyAsync(ctx->h_ctrl, ctx->ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    if (ctx->h_ctrl->abort_flag) return fail(ctx, IDKM_ERR_DEVICE, "partial sums of a pass did not arrive");
    return IDKM_OK;
}

idkm_status finish_persistent(idkm_ctx* ctx, idkm_info* info);

idkm_status check_common(idkm_ctx* ctx) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    ctx->err.clear();
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    if (ctx->pending_kind) (void)finish_persistent(ctx, nullptr);  // never leave an earlier launch uncollected
    ctx->err.clear();
    return IDKM_OK;
}

idkm_status validate_problem(idkm_ctx* ctx, const float* W, int64_t m, int d, const float* C, int k, float tau) {
    if (!W || !C) return fail(ctx, IDKM_ERR_INVALID_ARG, "W and the codebook must be non-NULL");
    if (m < 1 || d < 1 || k < 1) return fail(ctx, IDKM_ERR_INVALID_ARG, "m, d, k must be >= 1");
    if ((int64_t)k > m) return fail(ctx, IDKM_ERR_INVALID_ARG, "k must be <= m");
    if (!(tau > 0.f) || !std::isfinite(tau)) return fail(ctx, IDKM_ERR_INVALID_ARG, "tau must be finite and > 0");
    return IDKM_OK;
}

// Runs `pass` repeatedly in growing chunks until the device-side flag says the solve is over.
template <class DoneFn>
idkm_status run_until_done(idkm_ctx* ctx, const Geometry& g, int pass, Args& a, hipStream_t s, int64_t budget,
                           DoneFn done) {
    int chunk = 8;
    int64_t launched = 0;
    while (launched < budget) {
        int n = (int)((budget - launched < chunk) ? (budget - launched) : chunk);
        for (int t = 0; t < n; ++t) {
            idkm_status st = launch_pass(ctx, g, pass, a, s);
            if (st != IDKM_OK) return st;
        }
        launched += n;
        idkm_status st = read_ctrl(ctx, s);
        if (st != IDKM_OK) return st;
        if (done(*ctx->h_ctrl)) break;
        if (chunk < 64) chunk *= 2;
    }
    return IDKM_OK;
}

}  // namespace

extern "C" {

int32_t idkm_version(void) { return 200; }

void idkm_limits(idkm_limits_t* out) {
    if (!out) return;
    out->max_k = MAX_K;
    out->max_d = MAX_D;
    out->max_kd = MAX_KD;
}

const char* idkm_status_string(idkm_status s) {
    switch (s) {
        case IDKM_OK: return "ok";
        case IDKM_ERR_INVALID_ARG: return "invalid argument";
        case IDKM_ERR_ALLOC: return "allocation failed";
        case IDKM_ERR_DEVICE: return "device error";
        case IDKM_ERR_NONFINITE: return "non-finite result";
        case IDKM_ERR_NO_FORWARD: return "no forward state";
        case IDKM_ERR_UNSUPPORTED: return "unsupported shape";
    }
    return "unknown";
}

idkm_status idkm_create(idkm_ctx** out, int device_id) {
    if (!out) return IDKM_ERR_INVALID_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return IDKM_ERR_DEVICE;
    if (device_id < 0 || device_id >= ndev) return IDKM_ERR_INVALID_ARG;
    if (hipSetDevice(device_id) != hipSuccess) return IDKM_ERR_DEVICE;
    idkm_ctx* c = new (std::nothrow) idkm_ctx();
    if (!c) return IDKM_ERR_ALLOC;
    c->device = device_id;
    bool ok = true;
    ok &= hipMalloc(&c->ctrl, sizeof(Ctrl)) == hipSuccess;
    if (ok) ok &= hipMemset(c->ctrl, 0, sizeof(Ctrl)) == hipSuccess;
    ok &= hipHostMalloc(&c->h_ctrl, sizeof(Ctrl)) == hipSuccess;
    ok &= hipMalloc(&c->Cd, MAX_KD * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->Fd, MAX_KD * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->gd, MAX_KD * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->vd, MAX_KD * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->ud, MAX_KD * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->nd, MAX_K * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->Cf, MAX_KD * sizeof(float)) == hipSuccess;
    ok &= hipMalloc(&c->Ff, MAX_KD * sizeof(float)) == hipSuccess;
    ok &= hipMalloc(&c->Hs, MAX_KD * sizeof(float)) == hipSuccess;
    ok &= hipMalloc(&c->stage, (MAX_NACC + 2 * WG) * sizeof(double)) == hipSuccess;
    ok &= hipMalloc(&c->tot, MAX_NACC * sizeof(double)) == hipSuccess;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device_id) == hipSuccess) {
        c->num_cu = prop.multiProcessorCount;
        c->coop = prop.cooperativeLaunch != 0;
    }
    if (const char* e = std::getenv("IDKM_COOPERATIVE")) c->coop_launch = (e[0] == '1');
    if (const char* e = std::getenv("IDKM_TREE")) {
        c->tree_exchange = (e[0] != '0');
        c->tree_remote = (e[0] == '2');
    }
    if (const char* e = std::getenv("IDKM_MIN_VPT")) {
        int v = std::atoi(e);
        if (v >= 1 && v <= 1024) c->min_vec_per_thread = v;
    }
    ok &= hipMalloc(&c->tickets, TICKET_WORDS * sizeof(unsigned int)) == hipSuccess;
    if (ok) ok &= hipMemset(c->tickets, 0, TICKET_WORDS * sizeof(unsigned int)) == hipSuccess;
    ok &= hipMalloc(&c->abort_word, sizeof(unsigned int)) == hipSuccess;
    if (ok) ok &= hipMemset(c->abort_word, 0, sizeof(unsigned int)) == hipSuccess;
    ok &= hipHostMalloc(&c->h_res, sizeof(PResult)) == hipSuccess;
    if (ok) std::memset(c->h_res, 0, sizeof(PResult));
    c->xbuf_words = XBUF_WORDS;
    ok &= hipMalloc(&c->xbuf, c->xbuf_words * sizeof(unsigned long long)) == hipSuccess;
    if (ok) ok &= hipMemset(c->xbuf, 0, c->xbuf_words * sizeof(unsigned long long)) == hipSuccess;
    if (ok) ok &= hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        idkm_destroy(c);
        return IDKM_ERR_ALLOC;
    }
    *out = c;
    return IDKM_OK;
}

idkm_status idkm_destroy(idkm_ctx* c) {
    if (!c) return IDKM_ERR_INVALID_ARG;
    (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    void* dev[] = {c->ctrl, c->Cd, c->Fd, c->gd, c->vd, c->ud, c->nd, c->Cf, c->Ff, c->Hs, c->stage, c->tot, c->partials, c->kry, c->tickets, c->xbuf, c->lane_xbuf, c->abort_word};
    for (void* p : dev)
        if (p) (void)hipFree(p);
    if (c->ev0) (void)hipEventDestroy(c->ev0);
    if (c->ev1) (void)hipEventDestroy(c->ev1);
    if (c->h_ctrl) (void)hipHostFree(c->h_ctrl);
    if (c->h_res) (void)hipHostFree(c->h_res);
    delete c;
    return IDKM_OK;
}

const char* idkm_last_error(const idkm_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

idkm_status idkm_set_path(idkm_ctx* ctx, idkm_path path) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    if (path != IDKM_PATH_AUTO && path != IDKM_PATH_STREAM && path != IDKM_PATH_PERSISTENT)
        return fail(ctx, IDKM_ERR_INVALID_ARG, "unknown path");
    ctx->path = path;
    return IDKM_OK;
}

idkm_status idkm_set_tile_limit(idkm_ctx* ctx, int64_t bytes) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    if (bytes < 0 || (size_t)bytes > LDS_TILE_MAX) return fail(ctx, IDKM_ERR_INVALID_ARG, "tile limit must be in [0, 147456]");
    ctx->tile_limit = (size_t)bytes;
    return IDKM_OK;
}

idkm_status idkm_set_matrix_cores(idkm_ctx* ctx, int32_t enable) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    ctx->use_matrix = enable != 0;
    return IDKM_OK;
}

idkm_status idkm_set_gmres_basis(idkm_ctx* ctx, int32_t basis) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    if (basis < 1 || basis > GM_RMAX) return fail(ctx, IDKM_ERR_INVALID_ARG, "basis must be in [1, 256]");
    ctx->gmres_basis = basis;
    return IDKM_OK;
}

idkm_status idkm_advance_sequence(idkm_ctx* ctx, uint32_t n, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    // as if n more exchanges (persistent path) and n more launches (stream path) had been made
    const uint64_t sb = (uint64_t)ctx->seq_base + n;
    ctx->seq_base = sb > 0xfffffff0ull ? 0xfffffff0u : (unsigned int)sb;
    const uint64_t sl = (uint64_t)ctx->stream_launches + n;
    const unsigned int capped = sl > 0x7ffeff00ull ? 0x7ffeff00u : (unsigned int)sl;
    hipLaunchKernelGGL(k_add_launch_seq, dim3(1), dim3(1), 0, (hipStream_t)hip_stream, ctx->ctrl, capped - ctx->stream_launches);
    HIP_TRY(ctx, hipGetLastError());
    ctx->stream_launches = capped;
    return IDKM_OK;
}

idkm_status idkm_set_kernel_timing(idkm_ctx* ctx, int32_t enable) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (enable && !ctx->ev0) {
        HIP_TRY(ctx, hipEventCreate(&ctx->ev0));
        HIP_TRY(ctx, hipEventCreate(&ctx->ev1));
    }
    ctx->timing = enable != 0;
    ctx->timed = false;
    return IDKM_OK;
}

idkm_status idkm_last_kernel_ms(idkm_ctx* ctx, float* ms_out) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (!ms_out) return fail(ctx, IDKM_ERR_INVALID_ARG, "ms_out must be non-NULL");
    if (!ctx->timing || !ctx->timed)
        return fail(ctx, IDKM_ERR_INVALID_ARG, "no timed persistent launch: enable idkm_set_kernel_timing and make a call on the persistent path first");
    HIP_TRY(ctx, hipEventSynchronize(ctx->ev1));
    HIP_TRY(ctx, hipEventElapsedTime(ms_out, ctx->ev0, ctx->ev1));
    return IDKM_OK;
}

idkm_status idkm_set_spin_limit(idkm_ctx* ctx, uint32_t polls) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    ctx->spin_limit = polls;
    return IDKM_OK;
}

idkm_status idkm_forward(idkm_ctx* ctx, const float* W, int64_t m, int32_t d, const float* C0, int32_t k, float tau,
                         float tol, int32_t max_iter, idkm_dist dist, float* C_out, float* A_out, float* Wq_out,
                         int32_t* assign_out, idkm_info* info, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    ctx->has_forward = false;
    ctx->has_backward = false;
    ctx->timed = false;
    st = validate_problem(ctx, W, m, d, C0, k, tau);
    if (st != IDKM_OK) return st;
    if (!C_out) return fail(ctx, IDKM_ERR_INVALID_ARG, "C_out must be non-NULL");
    if (!(tol >= 0.f)) return fail(ctx, IDKM_ERR_INVALID_ARG, "tol must be >= 0");
    if (max_iter < 1) return fail(ctx, IDKM_ERR_INVALID_ARG, "max_iter must be >= 1");
    if (dist != IDKM_DIST_L2 && dist != IDKM_DIST_SQL2) return fail(ctx, IDKM_ERR_INVALID_ARG, "unknown dist");
    Geometry g;
    st = plan(ctx, m, k, d, &g);
    if (st != IDKM_OK) return st;
    st = ensure_partials(ctx, (size_t)g.nwg * (size_t)k * (d + 1));
    if (st != IDKM_OK) return st;
    hipStream_t s = (hipStream_t)hip_stream;

    ctx->W = W;
    ctx->m = m;
    ctx->d = d;
    ctx->k = k;
    ctx->dist = (int)dist;
    ctx->tau = tau;
    Args a = base_args(ctx);

    PersistPlan pp;
    const bool persistent = ctx->path != IDKM_PATH_STREAM && plan_persistent(ctx, false, &pp);
    if (ctx->path == IDKM_PATH_PERSISTENT && !persistent)
        return fail(ctx, IDKM_ERR_UNSUPPORTED, "the persistent path needs k <= 512, d <= 4 and, for k > 16, the tile of W to fit in LDS");
    if (persistent) {
        a.C_out = C_out;
        a.A_out = A_out;
        a.Wq_out = Wq_out;
        a.assign_out = assign_out;
        PArgs pa;
        std::memset(&pa, 0, sizeof(pa));
        pa.C0 = C0;
        pa.tol = (double)tol;
        pa.max_iter = (int)max_iter;
        st = launch_persistent(ctx, pp, a, pa, (unsigned int)max_iter + 1u, s);
        if (st == IDKM_OK) {
            ctx->pending_kind = 1;
            if (ctx->defer_wait) return IDKM_OK;
            st = finish_persistent(ctx, info);
        }
        // Under IDKM_PATH_AUTO a persistent attempt that could not run to its end -- the grid was not co-resident
        // (other work occupies compute units) or a bounded wait expired -- is answered by the stream path, which
        // depends on nothing but its own launches; an explicit IDKM_PATH_PERSISTENT reports the error.
        if (st != IDKM_ERR_DEVICE || ctx->path != IDKM_PATH_AUTO) return st;
        ctx->err.clear();
        a.C_out = nullptr;
        a.A_out = nullptr;
        a.Wq_out = nullptr;
        a.assign_out = nullptr;
    }

    hipLaunchKernelGGL(k_init_forward, dim3(1), dim3(WG), 0, s, a, C0, (double)tol, (int)max_iter);
    HIP_TRY(ctx, hipGetLastError());

    st = run_until_done(ctx, g, PASS_FWD, a, s, max_iter, [](const Ctrl& c) { return c.done != 0; });
    if (st != IDKM_OK) return st;
    if (ctx->h_ctrl->nonfinite) return fail(ctx, IDKM_ERR_NONFINITE, "the codebook became non-finite");

    a.C_out = C_out;
    a.A_out = A_out;
    a.Wq_out = Wq_out;
    a.assign_out = assign_out;
    st = launch_pass(ctx, g, PASS_FIN, a, s);
    if (st != IDKM_OK) return st;
    ctx->has_forward = true;
    if (info) {
        int iters = ctx->h_ctrl->iters, conv = ctx->h_ctrl->converged;
        double res = ctx->h_ctrl->residual;
        st = read_ctrl(ctx, s);
        if (st != IDKM_OK) return st;
        info->iters = iters;
        info->converged = conv;
        info->residual = res;
        info->empty_clusters = ctx->h_ctrl->empty;
        ctx->last_empty = ctx->h_ctrl->empty;
        info->path = IDKM_PATH_STREAM;
        info->alpha = 0.0;
        if (ctx->h_ctrl->nonfinite) {
            ctx->has_forward = false;
            return fail(ctx, IDKM_ERR_NONFINITE, "non-finite masses in the evaluation at C*");
        }
    }
    return IDKM_OK;
}

idkm_status idkm_backward(idkm_ctx* ctx, const float* dWq, idkm_bwd_mode mode, float tol, int32_t max_iter,
                          float alpha, float* dW_out, idkm_info* info, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    ctx->timed = false;
    if (!ctx->has_forward) return fail(ctx, IDKM_ERR_NO_FORWARD, "idkm_backward needs a successful idkm_forward first");
    if (!dWq || !dW_out) return fail(ctx, IDKM_ERR_INVALID_ARG, "dWq and dW_out must be non-NULL");
    if (mode != IDKM_BWD_IMPLICIT && mode != IDKM_BWD_JFB && mode != IDKM_BWD_DENSE && mode != IDKM_BWD_GMRES)
        return fail(ctx, IDKM_ERR_INVALID_ARG, "unknown mode");
    if (!(tol >= 0.f)) return fail(ctx, IDKM_ERR_INVALID_ARG, "tol must be >= 0");
    if (max_iter < 1) return fail(ctx, IDKM_ERR_INVALID_ARG, "max_iter must be >= 1");
    if (!(alpha > 0.f && alpha <= 1.f)) return fail(ctx, IDKM_ERR_INVALID_ARG, "alpha must be in (0,1]");
    Geometry g;
    st = plan(ctx, ctx->m, ctx->k, ctx->d, &g);
    if (st != IDKM_OK) return st;
    st = ensure_partials(ctx, (size_t)g.nwg * (size_t)ctx->k * (ctx->d + 1));
    if (st != IDKM_OK) return st;
    hipStream_t s = (hipStream_t)hip_stream;
    if (mode == IDKM_BWD_GMRES) {
        const int kd = ctx->k * ctx->d;
        const size_t need = gm_doubles(kd < ctx->gmres_basis ? kd : ctx->gmres_basis, kd);
        if (ctx->kry_cap < need) {
            if (ctx->kry) {
                HIP_TRY(ctx, hipStreamSynchronize(s));
                (void)hipFree(ctx->kry);
                ctx->kry = nullptr;
                ctx->kry_cap = 0;
            }
            if (hipMalloc((void**)&ctx->kry, need * sizeof(double)) != hipSuccess) {
                (void)hipGetLastError();
                return fail(ctx, IDKM_ERR_ALLOC, "hipMalloc of the Krylov workspace failed");
            }
            ctx->kry_cap = need;
        }
    }
    Args a = base_args(ctx);
    a.G = dWq;
    a.dW_out = dW_out;
    ctx->has_backward = true;

    if (mode == IDKM_BWD_DENSE) {
        if (!g.small || ctx->k * ctx->d > DENSE_MAX_KD)
            return fail(ctx, IDKM_ERR_UNSUPPORTED, "the dense backward needs k in {2,4,8,16} and k*d <= 16");
        const int kd = ctx->k * ctx->d;
        // when the K D (K D + D + 1) sums fit one exchange line the persistent kernel does it in one launch
        // (and batched calls can share that launch between layers)
        PersistPlan ppd;
        if (kd * kd + kd * ctx->d + kd <= XDENSE && ctx->path != IDKM_PATH_STREAM && plan_persistent(ctx, true, &ppd, true, dWq)) {
            PArgs pa;
            std::memset(&pa, 0, sizeof(pa));
            pa.tol = 0.0;
            pa.max_iter = 1;
            pa.mode = (int)mode;
            pa.alpha = 1.0;
            st = launch_persistent(ctx, ppd, a, pa, 1u, s);
            if (st == IDKM_OK) {
                ctx->pending_kind = 2;
                if (ctx->defer_wait) return IDKM_OK;
                st = finish_persistent(ctx, info);
            }
            if (st != IDKM_ERR_DEVICE || ctx->path != IDKM_PATH_AUTO) return st;
            ctx->err.clear();  // as in idkm_forward: the stream path answers instead
        }
        // otherwise two launches whatever the path: (v, dF/dC*) + direct solve, then the final pass
        const size_t nacc = (size_t)kd * kd + (size_t)kd * ctx->d + kd;
        Geometry gj = g;
        int64_t vpt = (ctx->m + (int64_t)WG * 256 - 1) / ((int64_t)WG * 256);  // about one workgroup per CU
        if (vpt < 1) vpt = 1;
        if (vpt > 64) vpt = 64;
        gj.vec_per_wg = (int64_t)WG * vpt;
        gj.nwg = (int)((ctx->m + gj.vec_per_wg - 1) / gj.vec_per_wg);
        st = ensure_partials(ctx, (size_t)gj.nwg * nacc);
        if (st != IDKM_OK) return st;
        a.partials = ctx->partials;
        hipLaunchKernelGGL(k_init_backward, dim3(1), dim3(1), 0, s, a, (int)mode, 0.0, 1, 1.0, 1);
        HIP_TRY(ctx, hipGetLastError());
        st = launch_pass(ctx, gj, PASS_BJ, a, s);
        if (st != IDKM_OK) return st;
        st = launch_pass(ctx, g, PASS_B3, a, s);
        if (st != IDKM_OK) return st;
        if (info) {
            st = read_ctrl(ctx, s);
            if (st != IDKM_OK) return st;
            const Ctrl& c = *ctx->h_ctrl;
            info->iters = 0;
            info->converged = c.b_converged;
            info->residual = 0.0;
            info->empty_clusters = ctx->last_empty;
            info->path = IDKM_PATH_STREAM;
            info->alpha = 1.0;
            if (c.nonfinite) return fail(ctx, IDKM_ERR_NONFINITE, "I - dF/dC* is singular or non-finite");
        }
        return IDKM_OK;
    }

    PersistPlan pp;
    bool persistent = ctx->path != IDKM_PATH_STREAM && plan_persistent(ctx, true, &pp, true, dWq);
    // The minimal-residual solve keeps O(k d R) state.  Inside the persistent kernel every workgroup holds all of it
    // (in LDS, behind its tiles), which takes a team where every workgroup receives the grid totals (one workgroup, or
    // the two-level exchange of a full-device team), k d <= 64 and room for the state beside the tiles; everything
    // else runs it in the pass tail of the stream path.
    unsigned int gm_off = 0;
    if (persistent && mode == IDKM_BWD_GMRES) {
        const int kd = ctx->k * ctx->d;
        persistent = !pp.lane && kd <= 64 &&
                     (pp.grid == 1 || (ctx->tree_exchange && !ctx->sink && pp.grid >= TREE_MIN_G));
        if (persistent) {
            size_t& fixed = ctx->static_lds[(const void*)pp.fn];
            if (fixed == 0) {
                hipFuncAttributes at;
                fixed = (hipFuncGetAttributes(&at, (const void*)pp.fn) == hipSuccess) ? at.sharedSizeBytes : LDS_PER_CU;
                (void)hipGetLastError();
            }
            gm_off = (unsigned int)((pp.lds + 15) / 16 * 16);
            const size_t lds = gm_off + gm_state_bytes(kd, gm_basis_length(ctx->gmres_basis, kd));
            if (fixed + lds <= LDS_PER_CU)
                pp.lds = lds;
            else
                persistent = false;
        }
    }
    if (ctx->path == IDKM_PATH_PERSISTENT && !persistent)
        return fail(ctx, IDKM_ERR_UNSUPPORTED, mode == IDKM_BWD_GMRES
                        ? "IDKM_BWD_GMRES on the persistent path needs k in {2,4,8,16}, k*d <= 64, a team of one or of at least 8 workgroups and room in LDS for its basis beside the tiles"
                        : "the persistent path needs k <= 512, d <= 4 and the tiles of W and dWq to fit in LDS");
    if (persistent) {
        const uint64_t ex = 1ull + (mode == IDKM_BWD_IMPLICIT ? (uint64_t)max_iter * 7ull
                                                               : (mode == IDKM_BWD_GMRES ? (uint64_t)max_iter + 3ull : 0ull));
        if (ex < 0x7fffffffull) {
            PArgs pa;
            std::memset(&pa, 0, sizeof(pa));
            pa.tol = (double)tol;
            pa.max_iter = (int)max_iter;
            pa.mode = (int)mode;
            pa.alpha = (double)alpha;
            pa.gm_basis = ctx->gmres_basis;
            pa.gm_off = gm_off;
            st = launch_persistent(ctx, pp, a, pa, (unsigned int)ex, s);
            if (st == IDKM_OK) {
                ctx->pending_kind = 2;
                if (ctx->defer_wait) return IDKM_OK;
                st = finish_persistent(ctx, info);
            }
            if (st != IDKM_ERR_DEVICE || ctx->path != IDKM_PATH_AUTO) return st;
            ctx->err.clear();  // as in idkm_forward: the stream path answers instead
        }
    }
    hipLaunchKernelGGL(k_init_backward, dim3(1), dim3(1), 0, s, a, (int)mode, (double)tol, (int)max_iter, (double)alpha,
                       ctx->gmres_basis);
    HIP_TRY(ctx, hipGetLastError());
    st = launch_pass(ctx, g, PASS_B1, a, s);
    if (st != IDKM_OK) return st;
    if (mode == IDKM_BWD_IMPLICIT) {
        // every attempt (alpha, alpha/2, ...) may use max_iter passes; at most 7 attempts
        st = run_until_done(ctx, g, PASS_B2, a, s, (int64_t)max_iter * 7, [](const Ctrl& c) { return c.b_done != 0; });
        if (st != IDKM_OK) return st;
    } else if (mode == IDKM_BWD_GMRES) {
        ctx->wide_tail = !g.small && ctx->k * ctx->d >= 512;
        st = run_until_done(ctx, g, PASS_B2, a, s, (int64_t)max_iter + 2, [](const Ctrl& c) { return c.b_done != 0; });
        ctx->wide_tail = false;
        if (st != IDKM_OK) return st;
    }
    st = launch_pass(ctx, g, PASS_B3, a, s);
    if (st != IDKM_OK) return st;
    if (info) {
        st = read_ctrl(ctx, s);
        if (st != IDKM_OK) return st;
        const Ctrl& c = *ctx->h_ctrl;
        info->iters = c.b_iters;
        info->converged = c.b_converged;
        info->residual = c.b_residual;
        info->empty_clusters = ctx->last_empty;
        info->path = IDKM_PATH_STREAM;
        info->alpha = c.b_alpha;
        if (c.nonfinite) return fail(ctx, IDKM_ERR_NONFINITE, "the cotangent became non-finite");
    }
    return IDKM_OK;
}

idkm_status idkm_get_cotangents(idkm_ctx* ctx, double* v_out, double* g_out, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (!ctx->has_forward || !ctx->has_backward)
        return fail(ctx, IDKM_ERR_NO_FORWARD, "idkm_get_cotangents needs an idkm_backward after the last idkm_forward");
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t bytes = (size_t)ctx->k * ctx->d * sizeof(double);
    if (v_out) HIP_TRY(ctx, hipMemcpyAsync(v_out, ctx->vd, bytes, hipMemcpyDeviceToHost, s));
    if (g_out) HIP_TRY(ctx, hipMemcpyAsync(g_out, ctx->gd, bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    return IDKM_OK;
}

idkm_status idkm_calibrate(idkm_ctx* ctx, int32_t kind, const float* buf, int64_t n_floats, double* result,
                           void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (!result || kind < 0 || kind > 11) return fail(ctx, IDKM_ERR_INVALID_ARG, "kind must be 0 .. 11 and result non-NULL");
    if (kind == 2 && (!buf || n_floats < 4 || (reinterpret_cast<uintptr_t>(buf) & 15u) != 0))
        return fail(ctx, IDKM_ERR_INVALID_ARG, "the streaming read needs a 16-byte aligned buffer");
    hipStream_t s = (hipStream_t)hip_stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(ctx, hipEventCreate(&e0));
    HIP_TRY(ctx, hipEventCreate(&e1));
    const int grid = ctx->num_cu * 8;  // eight wavefronts per SIMD
    const int iters = 4096;
    float* sink = reinterpret_cast<float*>(ctx->tot);
    double work = 0.0;
    for (int rep = 0; rep < 2; ++rep) {  // the first repetition warms up
        HIP_TRY(ctx, hipEventRecord(e0, s));
        if (kind == 0) {
            launch_cal_fma(sink, grid, iters, s);
            work = (double)grid * 256.0 * iters * 16.0;  // lane operations
        } else if (kind >= 9) {
            // the matrix / vector mix (and the matrix instruction alone) with more wavefronts per SIMD: can the vector
            // work of other wavefronts run while a matrix instruction holds the pipeline?
            const int wgs = ctx->num_cu * (kind == 10 ? 4 : 2);  // 512 threads each: 4 or 8 wavefronts per SIMD
            launch_cal_mfma(sink, wgs, iters, kind == 11 ? 0 : 1, s);
            work = (double)wgs * 8.0 * iters * 8.0 * 1024.0;  // multiply-adds
        } else if (kind >= 6) {
            // one workgroup of 512 threads per compute unit: two wavefronts per SIMD, as in the kernel that uses them
            launch_cal_mfma(sink, ctx->num_cu, iters, kind - 6, s);
            work = (double)ctx->num_cu * 8.0 * iters * 8.0 * (kind == 8 ? 256.0 : 1024.0);  // multiply-adds
        } else if (kind == 1 || kind >= 3) {
            const int fmas = kind == 1 ? 0 : (kind == 3 ? 1 : (kind == 4 ? 2 : 4));
            launch_cal_exp(sink, grid, iters, fmas, s);
            work = (double)grid * 256.0 * iters * 8.0;  // exponentials
        } else {
            launch_cal_read(buf, (size_t)n_floats, grid * 2, sink, s);
            work = (double)(n_floats / 4 * 4) * 4.0;     // bytes
        }
        HIP_TRY(ctx, hipGetLastError());
        HIP_TRY(ctx, hipEventRecord(e1, s));
        HIP_TRY(ctx, hipEventSynchronize(e1));
    }
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *result = work / ((double)ms * 1e-3);
    return IDKM_OK;
}

int32_t idkm_code_bits(int32_t k) {
    if (k < 1) return 0;
    int b = 1;
    while ((1 << b) < k) ++b;
    return b;
}

int64_t idkm_code_words(int64_t m, int32_t k) {
    if (m < 0 || k < 1 || k > 1024) return -1;
    return (m * idkm_code_bits(k) + 31) / 32;
}

idkm_status idkm_pack_codes(idkm_ctx* ctx, const int32_t* assign, int64_t m, int32_t k, uint32_t* words_out,
                            void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (m < 0 || k < 1 || k > 1024) return fail(ctx, IDKM_ERR_INVALID_ARG, "need m >= 0 and 1 <= k <= 1024");
    if (m == 0) return IDKM_OK;
    if (!assign || !words_out) return fail(ctx, IDKM_ERR_INVALID_ARG, "assign and words_out must be non-NULL");
    if ((reinterpret_cast<uintptr_t>(assign) & 15u) != 0) return fail(ctx, IDKM_ERR_INVALID_ARG, "assign must be 16-byte aligned");
    if (m > ((int64_t)1 << 36)) return fail(ctx, IDKM_ERR_INVALID_ARG, "m too large");
    launch_pack_codes(assign, m, idkm_code_bits(k), words_out, idkm_code_words(m, k), (hipStream_t)hip_stream);
    HIP_TRY(ctx, hipGetLastError());
    return IDKM_OK;
}

idkm_status idkm_unpack_quantize(idkm_ctx* ctx, const uint32_t* words, int64_t m, const float* C, int32_t k, int32_t d,
                                 float* Wh_out, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (m < 0 || k < 1 || k > 1024 || d < 1 || d > 64) return fail(ctx, IDKM_ERR_INVALID_ARG, "need m >= 0, 1 <= k <= 1024, 1 <= d <= 64");
    if (m == 0) return IDKM_OK;
    if (!words || !C || !Wh_out) return fail(ctx, IDKM_ERR_INVALID_ARG, "words, C and Wh_out must be non-NULL");
    if (m > ((int64_t)1 << 36)) return fail(ctx, IDKM_ERR_INVALID_ARG, "m too large");
    launch_unpack_quantize(words, idkm_code_words(m, k), m, idkm_code_bits(k), C, k, d, Wh_out, (hipStream_t)hip_stream);
    HIP_TRY(ctx, hipGetLastError());
    return IDKM_OK;
}

#ifdef IDKM_TRACE
// development builds only: device buffer of 2*64*8 int64 clock stamps filled by the persistent forward kernel
idkm_status idkm_debug_trace(idkm_ctx* ctx, long long* dev_buf) {
    if (!ctx) return IDKM_ERR_INVALID_ARG;
    ctx->trace = dev_buf;
    return IDKM_OK;
}
#endif

}  // extern "C"

struct idkm_batch {
    int device = 0;
    int num_cu = 0;
    std::vector<idkm_ctx*> ctx;
    std::vector<Deferred> deferred;
    // launch tables: pinned host staging and their device copies
    BatchItem *h_items = nullptr, *d_items = nullptr;
    unsigned short *h_map = nullptr, *d_map = nullptr;
    size_t map_cap = 0;
    std::map<std::pair<const void*, size_t>, int> blocks_per_cu;  // (kernel, LDS rounded up to 1 KiB) -> occupancy
    std::map<const void*, size_t> lds_attr;                       // kernel -> dynamic LDS limit set so far
    int launches = 0;                                             // of the last batched call
    std::string err;
};

namespace {

idkm_status batch_fail(idkm_batch* b, idkm_status st, const std::string& msg) {
    b->err = msg;
    return st;
}

// Workgroups of `fn` with `lds` bytes of dynamic LDS that the device holds at once (0 on error).
int64_t batch_capacity(idkm_batch* b, const void* fn, int threads, size_t lds) {
    const size_t rounded = (lds + 1023) / 1024 * 1024;
    auto key = std::make_pair(fn, rounded);
    auto it = b->blocks_per_cu.find(key);
    if (it == b->blocks_per_cu.end()) {
        size_t& attr = b->lds_attr[fn];
        if (attr < rounded) {
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)rounded) != hipSuccess) {
                (void)hipGetLastError();
                return 0;
            }
            attr = rounded;
        }
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, threads, rounded) != hipSuccess) {
            (void)hipGetLastError();
            return 0;
        }
        it = b->blocks_per_cu.emplace(key, nb).first;
    }
    return (int64_t)it->second * b->num_cu;
}

// Launches the deferred solves: solves of one kernel shape share launches, each launch as large as the device
// can hold at once (every team's workgroups must be resident together, since they wait for one another).
idkm_status batch_launch(idkm_batch* b, hipStream_t s) {
    std::vector<Deferred>& q = b->deferred;
    b->launches = 0;
    if (q.empty()) return IDKM_OK;
    std::vector<char> taken(q.size(), 0);
    size_t item_off = 0, map_off = 0;
    for (size_t first = 0; first < q.size(); ++first) {
        if (taken[first]) continue;
        const void* fn = (const void*)q[first].pp.fn_batch;
        const int threads = q[first].pp.threads;
        size_t i = first;
        while (i < q.size()) {
            // one launch: members i.. of this shape while the grid stays co-resident
            const size_t item_begin = item_off, map_begin = map_off;
            size_t lds = 0;
            int64_t total = 0;
            for (; i < q.size(); ++i) {
                if (taken[i] || (const void*)q[i].pp.fn_batch != fn) continue;
                const size_t lds_new = std::max(lds, q[i].pp.lds);
                const int64_t cap = batch_capacity(b, fn, threads, lds_new);
                if (cap < q[i].pp.grid) return batch_fail(b, IDKM_ERR_DEVICE, "persistent grid would not be co-resident");
                if (total + q[i].pp.grid > cap || total + q[i].pp.grid > 65535) break;  // full: next launch
                if (map_off + (size_t)q[i].pp.grid > b->map_cap) return batch_fail(b, IDKM_ERR_DEVICE, "launch table overflow");
                BatchItem& it = b->h_items[item_off];
                it.a = q[i].a;
                it.p = q[i].pa;
                it.wg_begin = (int)total;
                it.wg_count = q[i].pp.grid;
                for (int w = 0; w < q[i].pp.grid; ++w) b->h_map[map_off + w] = (unsigned short)(item_off - item_begin);
                map_off += (size_t)q[i].pp.grid;
                item_off += 1;
                total += q[i].pp.grid;
                lds = lds_new;
                taken[i] = 1;
            }
            if (total == 0) break;
            if (hipMemcpyAsync(b->d_items + item_begin, b->h_items + item_begin, (item_off - item_begin) * sizeof(BatchItem),
                               hipMemcpyHostToDevice, s) != hipSuccess ||
                hipMemcpyAsync(b->d_map + map_begin, b->h_map + map_begin, (map_off - map_begin) * sizeof(unsigned short),
                               hipMemcpyHostToDevice, s) != hipSuccess)
                return batch_fail(b, IDKM_ERR_DEVICE, "copy of the launch tables failed");
            hipLaunchKernelGGL(q[first].pp.fn_batch, dim3((unsigned)total), dim3(threads), lds, s,
                               (const BatchItem*)(b->d_items + item_begin), (const unsigned short*)(b->d_map + map_begin));
            if (hipGetLastError() != hipSuccess) return batch_fail(b, IDKM_ERR_DEVICE, "batched launch failed");
            b->launches += 1;
        }
    }
    return IDKM_OK;
}

// Collects the deferred solves after batch_launch (or abandons them if the launch failed).
idkm_status batch_collect(idkm_batch* b, idkm_status launched, int32_t n, idkm_info* infos, idkm_status* statuses) {
    idkm_status first = launched;
    for (int i = 0; i < n; ++i) {
        idkm_ctx* c = b->ctx[i];
        if (statuses[i] == IDKM_OK && c->pending_kind) {
            if (launched == IDKM_OK) {
                statuses[i] = finish_persistent(c, &infos[i]);
            } else {
                c->pending_kind = 0;
                statuses[i] = launched;
                c->err = b->err;
            }
        }
        if (statuses[i] != IDKM_OK && first == IDKM_OK) {
            first = statuses[i];
            b->err = "layer " + std::to_string(i) + ": " + c->err;
        }
    }
    b->deferred.clear();
    return first;
}

}  // namespace

extern "C" {

idkm_status idkm_batch_create(idkm_batch** out, int device_id, int32_t n_layers) {
    if (!out) return IDKM_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_layers < 1 || n_layers > 1024) return IDKM_ERR_INVALID_ARG;
    idkm_batch* b = new (std::nothrow) idkm_batch();
    if (!b) return IDKM_ERR_ALLOC;
    b->device = device_id;
    for (int i = 0; i < n_layers; ++i) {
        idkm_ctx* c = nullptr;
        idkm_status st = idkm_create(&c, device_id);
        if (st != IDKM_OK) {
            idkm_batch_destroy(b);
            return st;
        }
        b->ctx.push_back(c);
    }
    b->num_cu = b->ctx[0]->num_cu;
    b->map_cap = (size_t)n_layers * PT;  // a team has at most PT workgroups
    const bool ok = hipHostMalloc((void**)&b->h_items, (size_t)n_layers * sizeof(BatchItem), hipHostMallocDefault) == hipSuccess &&
                    hipHostMalloc((void**)&b->h_map, b->map_cap * sizeof(unsigned short), hipHostMallocDefault) == hipSuccess &&
                    hipMalloc((void**)&b->d_items, (size_t)n_layers * sizeof(BatchItem)) == hipSuccess &&
                    hipMalloc((void**)&b->d_map, b->map_cap * sizeof(unsigned short)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        idkm_batch_destroy(b);
        return IDKM_ERR_ALLOC;
    }
    *out = b;
    return IDKM_OK;
}

idkm_status idkm_batch_destroy(idkm_batch* b) {
    if (!b) return IDKM_ERR_INVALID_ARG;
    (void)hipSetDevice(b->device);
    (void)hipDeviceSynchronize();
    for (idkm_ctx* c : b->ctx) (void)idkm_destroy(c);
    if (b->h_items) (void)hipHostFree(b->h_items);
    if (b->h_map) (void)hipHostFree(b->h_map);
    if (b->d_items) (void)hipFree(b->d_items);
    if (b->d_map) (void)hipFree(b->d_map);
    delete b;
    return IDKM_OK;
}

const char* idkm_batch_last_error(const idkm_batch* b) { return b ? b->err.c_str() : "null batch"; }

int32_t idkm_batch_launches(const idkm_batch* b) { return b ? b->launches : -1; }

idkm_ctx* idkm_batch_context(idkm_batch* b, int32_t i) {
    return (b && i >= 0 && i < (int32_t)b->ctx.size()) ? b->ctx[i] : nullptr;
}

idkm_status idkm_batch_forward(idkm_batch* b, const idkm_fwd_desc* layers, int32_t n, idkm_info* infos,
                               idkm_status* statuses, void* hip_stream) {
    if (!b || !layers || !infos || !statuses || n < 1 || n > (int32_t)b->ctx.size()) return IDKM_ERR_INVALID_ARG;
    b->err.clear();
    b->deferred.clear();
    if (hipSetDevice(b->device) != hipSuccess) return IDKM_ERR_DEVICE;
    for (int i = 0; i < n; ++i) {
        idkm_ctx* c = b->ctx[i];
        const idkm_fwd_desc& L = layers[i];
        std::memset(&infos[i], 0, sizeof(idkm_info));
        c->defer_wait = true;
        c->sink = &b->deferred;
        statuses[i] = idkm_forward(c, L.W, L.m, L.d, L.C0, L.k, L.tau, L.tol, L.max_iter, (idkm_dist)L.dist, L.C_out,
                                   L.A_out, L.Wq_out, L.assign_out, &infos[i], hip_stream);
        c->defer_wait = false;
        c->sink = nullptr;
    }
    const idkm_status launched = batch_launch(b, (hipStream_t)hip_stream);
    idkm_status first = batch_collect(b, launched, n, infos, statuses);
    if (first != IDKM_OK) {
        // layers whose persistent solve could not run to its end are solved again, one by one, on the stream path
        // (contexts left at IDKM_PATH_AUTO only)
        first = IDKM_OK;
        for (int i = 0; i < n; ++i) {
            idkm_ctx* c = b->ctx[i];
            const idkm_fwd_desc& L = layers[i];
            if (statuses[i] == IDKM_ERR_DEVICE && c->path == IDKM_PATH_AUTO) {
                c->path = IDKM_PATH_STREAM;
                statuses[i] = idkm_forward(c, L.W, L.m, L.d, L.C0, L.k, L.tau, L.tol, L.max_iter, (idkm_dist)L.dist, L.C_out,
                                           L.A_out, L.Wq_out, L.assign_out, &infos[i], hip_stream);
                c->path = IDKM_PATH_AUTO;
            }
            if (statuses[i] != IDKM_OK && first == IDKM_OK) {
                first = statuses[i];
                b->err = "layer " + std::to_string(i) + ": " + c->err;
            }
        }
        if (first == IDKM_OK) b->err.clear();
    }
    return first;
}

idkm_status idkm_batch_backward(idkm_batch* b, const idkm_bwd_desc* layers, int32_t n, idkm_info* infos,
                                idkm_status* statuses, void* hip_stream) {
    if (!b || !layers || !infos || !statuses || n < 1 || n > (int32_t)b->ctx.size()) return IDKM_ERR_INVALID_ARG;
    b->err.clear();
    b->deferred.clear();
    if (hipSetDevice(b->device) != hipSuccess) return IDKM_ERR_DEVICE;
    for (int i = 0; i < n; ++i) {
        idkm_ctx* c = b->ctx[i];
        const idkm_bwd_desc& L = layers[i];
        std::memset(&infos[i], 0, sizeof(idkm_info));
        c->defer_wait = true;
        c->sink = &b->deferred;
        statuses[i] = idkm_backward(c, L.dWq, (idkm_bwd_mode)L.mode, L.tol, L.max_iter, L.alpha, L.dW_out, &infos[i],
                                    hip_stream);
        c->defer_wait = false;
        c->sink = nullptr;
    }
    const idkm_status launched = batch_launch(b, (hipStream_t)hip_stream);
    idkm_status first = batch_collect(b, launched, n, infos, statuses);
    if (first != IDKM_OK) {
        first = IDKM_OK;  // as in idkm_batch_forward
        for (int i = 0; i < n; ++i) {
            idkm_ctx* c = b->ctx[i];
            const idkm_bwd_desc& L = layers[i];
            if (statuses[i] == IDKM_ERR_DEVICE && c->path == IDKM_PATH_AUTO) {
                c->path = IDKM_PATH_STREAM;
                statuses[i] = idkm_backward(c, L.dWq, (idkm_bwd_mode)L.mode, L.tol, L.max_iter, L.alpha, L.dW_out, &infos[i],
                                            hip_stream);
                c->path = IDKM_PATH_AUTO;
            }
            if (statuses[i] != IDKM_OK && first == IDKM_OK) {
                first = statuses[i];
                b->err = "layer " + std::to_string(i) + ": " + c->err;
            }
        }
        if (first == IDKM_OK) b->err.clear();
    }
    return first;
}

idkm_status idkm_step_F(idkm_ctx* ctx, const float* W, int64_t m, int32_t d, const float* C, int32_t k, float tau,
                        idkm_dist dist, float* Cplus_out, float* n_out, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    ctx->has_forward = false;
    ctx->has_backward = false;
    st = validate_problem(ctx, W, m, d, C, k, tau);
    if (st != IDKM_OK) return st;
    if (!Cplus_out) return fail(ctx, IDKM_ERR_INVALID_ARG, "Cplus_out must be non-NULL");
    if (dist != IDKM_DIST_L2 && dist != IDKM_DIST_SQL2) return fail(ctx, IDKM_ERR_INVALID_ARG, "unknown dist");
    Geometry g;
    st = plan(ctx, m, k, d, &g);
    if (st != IDKM_OK) return st;
    st = ensure_partials(ctx, (size_t)g.nwg * (size_t)k * (d + 1));
    if (st != IDKM_OK) return st;
    hipStream_t s = (hipStream_t)hip_stream;
    ctx->W = W;
    ctx->m = m;
    ctx->d = d;
    ctx->k = k;
    ctx->dist = (int)dist;
    ctx->tau = tau;
    Args a = base_args(ctx);
    hipLaunchKernelGGL(k_init_forward, dim3(1), dim3(WG), 0, s, a, C, 0.0, 1);
    HIP_TRY(ctx, hipGetLastError());
    st = launch_pass(ctx, g, PASS_FIN, a, s);
    if (st != IDKM_OK) return st;
    HIP_TRY(ctx, hipMemcpyAsync(Cplus_out, ctx->Ff, sizeof(float) * k * d, hipMemcpyDeviceToDevice, s));
    if (n_out) {
        hipLaunchKernelGGL(k_f64_to_f32, dim3(1), dim3(WG), 0, s, ctx->nd, n_out, (int)k);
        HIP_TRY(ctx, hipGetLastError());
    }
    ctx->has_forward = true;
    return IDKM_OK;
}

idkm_status idkm_step_JCT(idkm_ctx* ctx, const float* gvec, float* out, void* hip_stream) {
    idkm_status st = check_common(ctx);
    if (st != IDKM_OK) return st;
    if (!ctx->has_forward) return fail(ctx, IDKM_ERR_NO_FORWARD, "idkm_step_JCT needs idkm_step_F or idkm_forward first");
    if (!gvec || !out) return fail(ctx, IDKM_ERR_INVALID_ARG, "g and out must be non-NULL");
    Geometry g;
    st = plan(ctx, ctx->m, ctx->k, ctx->d, &g);
    if (st != IDKM_OK) return st;
    st = ensure_partials(ctx, (size_t)g.nwg * (size_t)ctx->k * (ctx->d + 1));
    if (st != IDKM_OK) return st;
    hipStream_t s = (hipStream_t)hip_stream;
    Args a = base_args(ctx);
    hipLaunchKernelGGL(k_set_g, dim3(1), dim3(WG), 0, s, a, gvec);
    HIP_TRY(ctx, hipGetLastError());
    st = launch_pass(ctx, g, PASS_B2, a, s);
    if (st != IDKM_OK) return st;
    hipLaunchKernelGGL(k_f64_to_f32, dim3(1), dim3(WG), 0, s, ctx->ud, out, ctx->k * ctx->d);
    HIP_TRY(ctx, hipGetLastError());
    return IDKM_OK;
}

}  // extern "C"

// ---------------------------------------------------------------- the entry point that allocates nothing

namespace {

// Everything the persistent forward kernel needs beyond the caller's tensors: the exchange words of the grid-wide
// sums, the O(k d) solver state it leaves behind, the abort word and the block it reports into.
struct StaticScratch {
    unsigned long long xbuf[XBUF_WORDS];
    double Cd[64], Fd[64], nd[16];
    float Cf[64], Ff[64];
    unsigned int abort_word;
    unsigned int pad_;
    PResult res;
};
constexpr size_t STATIC_SCRATCH_BYTES = (sizeof(StaticScratch) + 255) / 256 * 256;
constexpr int STATIC_MAX_DEVICES = 64;

}  // namespace

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the address the kernels get is the one that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

struct StaticDevice {
    bool ready = false;
    idkm_ctx ctx;  // a host-side context whose device pointers all point into this device's copy of `scratch`
};
StaticDevice g_static[STATIC_MAX_DEVICES];
std::mutex g_static_mutex;
std::string g_static_err;

}  // namespace

extern "C" {

const char* idkm_noalloc_last_error(void) { return g_static_err.c_str(); }

idkm_status idkm_forward_noalloc(int device_id, const float* W, int64_t m, int32_t d, const float* C0, int32_t k,
                                 float tau, float tol, int32_t max_iter, idkm_dist dist, float* C_out, float* A_out,
                                 float* Wq_out, int32_t* assign_out, idkm_info* info, void* hip_stream) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    g_static_err.clear();
    auto bad = [&](idkm_status st, const std::string& msg) {
        g_static_err = msg;
        return st;
    };
    if (device_id < 0 || device_id >= STATIC_MAX_DEVICES) return bad(IDKM_ERR_INVALID_ARG, "device_id out of range");
    if (hipSetDevice(device_id) != hipSuccess) {
        (void)hipGetLastError();
        return bad(IDKM_ERR_DEVICE, "hipSetDevice failed");
    }
    hipStream_t s = (hipStream_t)hip_stream;
    StaticDevice& sd = g_static[device_id];
    idkm_ctx* ctx = &sd.ctx;
    if (!sd.ready) {
        // once per device, with that device current: the address of this device's copy of the array
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return bad(IDKM_ERR_DEVICE, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        }
        StaticScratch* sc = reinterpret_cast<StaticScratch*>(ptr);
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device_id) != hipSuccess || cus < 1) {
            (void)hipGetLastError();
            return bad(IDKM_ERR_DEVICE, "hipDeviceGetAttribute failed");
        }
        ctx->device = device_id;
        ctx->num_cu = cus;
        ctx->coop = true;  // plain launches of a grid that the occupancy query shows to be co-resident
        ctx->xbuf = sc->xbuf;
        ctx->xbuf_words = XBUF_WORDS;
        ctx->Cd = sc->Cd;
        ctx->Fd = sc->Fd;
        ctx->nd = sc->nd;
        ctx->Cf = sc->Cf;
        ctx->Ff = sc->Ff;
        ctx->abort_word = &sc->abort_word;
        ctx->h_res = &sc->res;
        ctx->res_on_device = true;
        ctx->seq_base = 0;
        // the stamps start from a cleared array (sequence number 0 is never used); a fill kernel, not a memset
        hipLaunchKernelGGL(k_fill_u64, dim3(64), dim3(256), 0, s, reinterpret_cast<unsigned long long*>(ptr),
                           STATIC_SCRATCH_BYTES / sizeof(unsigned long long), 0ull);
        if (hipGetLastError() != hipSuccess) return bad(IDKM_ERR_DEVICE, "clearing the scratch array failed");
        sd.ready = true;
    }
    ctx->err.clear();
    ctx->pending_kind = 0;
    idkm_status st = validate_problem(ctx, W, m, d, C0, k, tau);
    if (st == IDKM_OK && !C_out) st = fail(ctx, IDKM_ERR_INVALID_ARG, "C_out must be non-NULL");
    if (st == IDKM_OK && !(tol >= 0.f)) st = fail(ctx, IDKM_ERR_INVALID_ARG, "tol must be >= 0");
    if (st == IDKM_OK && max_iter < 1) st = fail(ctx, IDKM_ERR_INVALID_ARG, "max_iter must be >= 1");
    if (st == IDKM_OK && dist != IDKM_DIST_L2 && dist != IDKM_DIST_SQL2) st = fail(ctx, IDKM_ERR_INVALID_ARG, "unknown dist");
    if (st != IDKM_OK) return bad(st, ctx->err);
    const bool shape_ok = k >= 2 && k <= 16 && pow2(k) && (d == 1 || d == 2 || d == 4);
    if (!shape_ok || m * d > IDKM_NOALLOC_MAX_WEIGHTS)
        return bad(IDKM_ERR_UNSUPPORTED, "idkm_forward_noalloc serves k in {2,4,8,16}, d in {1,2,4} and m*d <= " +
                                             std::to_string((long long)IDKM_NOALLOC_MAX_WEIGHTS) +
                                             " (the layer is held in LDS)");
    ctx->W = W;
    ctx->m = m;
    ctx->d = d;
    ctx->k = k;
    ctx->dist = (int)dist;
    ctx->tau = tau;
    ctx->path = IDKM_PATH_AUTO;
    Args a = base_args(ctx);
    a.C_out = C_out;
    a.A_out = A_out;
    a.Wq_out = Wq_out;
    a.assign_out = assign_out;
    PersistPlan pp;
    if (!plan_persistent(ctx, false, &pp) || pp.lane || pp.lds == 0 || pp.lds > LDS_TILE_MAX)
        return bad(IDKM_ERR_UNSUPPORTED, "idkm_forward_noalloc: the layer does not fit this device's LDS");
    PArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    pa.C0 = C0;
    pa.tol = (double)tol;
    pa.max_iter = (int)max_iter;
    st = launch_persistent(ctx, pp, a, pa, (unsigned int)max_iter + 1u, s);
    if (st != IDKM_OK) return bad(st, ctx->err);
    if (!info) return IDKM_OK;  // enqueued; nothing waits
    ctx->pending_kind = 1;
    st = finish_persistent(ctx, info);
    if (st != IDKM_OK) return bad(st, ctx->err);
    return IDKM_OK;
}

}  // extern "C"
