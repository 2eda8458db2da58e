/*
 * idkm.h -- C ABI of the MI355X (gfx950) implementation of implicit differentiable soft k-means
 * (IDKM, arXiv 2312.07759): the soft-k-means fixed-point solve of one layer and its
 * implicit-differentiation / Jacobian-free backward.
 *
 * Shapes, all row-major, all float32 in DEVICE memory unless a parameter says "host":
 *   W [m,d]  the layer's m weight sub-vectors of dimension d   (Sec. 3, product-quantisation set-up)
 *   C [k,d]  codebook of k codewords                           (Sec. 3)
 *   A [m,k]  attention matrix, rows sum to one                 (Eq. "aterms", Eq. "arow")
 *   Wq[m,d]  soft-quantised weights  Wq = A C                  (Eq. "softquant", "softquantmatrix")
 *
 * Ownership: every tensor pointer is caller-owned device memory; the library never frees or
 * reallocates it.  A context owns only its scratch memory and O(k d) solver state.
 * Threading: one context must not be used from two host threads at once.
 * Errors: functions return an idkm_status; on any error nothing the caller can rely on has been
 * written to the outputs.  Non-convergence and empty clusters are reported in idkm_info, not as
 * errors.  Nothing is printed and the process is never terminated.
 */
#ifndef IDKM_H
#define IDKM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct idkm_ctx idkm_ctx; /* opaque */

typedef enum {
    IDKM_OK = 0,
    IDKM_ERR_INVALID_ARG = 1, /* bad shape / NULL / out-of-range parameter; see idkm_last_error */
    IDKM_ERR_ALLOC = 2,       /* device or host allocation failed */
    IDKM_ERR_DEVICE = 3,      /* a HIP call failed, or a device-side wait hit its time limit */
    IDKM_ERR_NONFINITE = 4,   /* the solve produced a non-finite codebook (non-finite input) */
    IDKM_ERR_NO_FORWARD = 5,  /* idkm_backward without a preceding successful idkm_forward */
    IDKM_ERR_UNSUPPORTED = 6  /* shape outside the limits reported by idkm_limits */
} idkm_status;

/* Energy between a weight vector and a codeword inside the softmax of Eq. "aterms". */
typedef enum {
    IDKM_DIST_L2 = 0,  /* ||w - c||   : the paper's distance matrix (Alg. 1, distance step) */
    IDKM_DIST_SQL2 = 1 /* ||w - c||^2 : squared variant (fixed-variance spherical mixture EM) */
} idkm_dist;

typedef enum {
    IDKM_BWD_IMPLICIT = 0, /* solve the fixed point of Sec. 4.2 (Eq. "grad", "inv", "backiter") */
    IDKM_BWD_JFB = 1,      /* Jacobian-free: M* = I (Sec. 4.3, Eq. "jfbgrad") */
    IDKM_BWD_DENSE = 2,    /* explicit k d x k d Jacobian dF/dC* accumulated in one pass over W, then a direct
                              solve with (I - dF/dC*) (Eq. "grad", "inv"); offered for k d <= 16, k a power of two */
    IDKM_BWD_GMRES = 3     /* the same linear system (I - dF/dC*)^T g = v (Eq. "grad", "inv") by a restarted
                              minimal-residual Krylov solve; one pass over W per basis vector, any shape */
} idkm_bwd_mode;

/* How the device work is scheduled.  Results are identical up to rounding order. */
typedef enum {
    IDKM_PATH_AUTO = 0,      /* persistent when the problem fits on chip, else stream; also stream when a persistent
                                attempt could not run to its end (see idkm_set_spin_limit) */
    IDKM_PATH_STREAM = 1,    /* one kernel launch per pass over W */
    IDKM_PATH_PERSISTENT = 2 /* one launch per solve, W held in LDS, one grid-wide exchange per pass */
} idkm_path;

typedef struct {
    int32_t iters;          /* forward: evaluations of F; backward: passes of (dF/dC)^T, all attempts */
    int32_t converged;      /* 1 if the stop rule was met before max_iter */
    double residual;        /* forward: last ||C+ - C||_F; backward: last ||g+ - g||_F */
    int32_t empty_clusters; /* clusters whose mass was exactly zero in the last evaluation */
    int32_t path;           /* idkm_path actually used (never AUTO) */
    double alpha;           /* backward: damping factor in use when the solve ended */
} idkm_info;

/* Largest shapes accepted: k <= max_k, d <= max_d, k*d <= max_kd. */
typedef struct {
    int32_t max_k, max_d, max_kd;
} idkm_limits_t;

/* Library version (major*10000 + minor*100 + patch). */
int32_t idkm_version(void);
void idkm_limits(idkm_limits_t* out);
const char* idkm_status_string(idkm_status s);

/* Create / destroy a context bound to HIP device `device_id`.  Allocates the scratch buffers. */
idkm_status idkm_create(idkm_ctx** out, int device_id);
idkm_status idkm_destroy(idkm_ctx* ctx);
/* Human-readable detail of the last error on this context (owned by the context; "" if none). */
const char* idkm_last_error(const idkm_ctx* ctx);
/* Select the scheduling path for subsequent calls (default IDKM_PATH_AUTO). */
idkm_status idkm_set_path(idkm_ctx* ctx, idkm_path path);
/* Shapes with d = 4 and 17 <= k <= 256 run the forward loop (Alg. 1) and every pass of the backward (the pass for
 * v, the (dF/dC)^T passes of Eq. "backiter", the last pass for dL/dW) on the matrix cores, for both energies.
 * enable = 0 sends them to the vector-ALU kernels that serve every other shape instead (diagnostics, comparisons);
 * the default is 1.  Takes effect from the next idkm_forward; a backward follows the setting in force at its call. */
idkm_status idkm_set_matrix_cores(idkm_ctx* ctx, int32_t enable);
/* Persistent path, k in {2,4,8,16}: a workgroup keeps its share of W (and of dL/dWq in the backward) in LDS when it
 * is at most `bytes` (default and maximum 147456).  A layer with larger shares (more than about 9.4 M weights) is
 * served by the stream path under IDKM_PATH_AUTO; under IDKM_PATH_PERSISTENT the same one-launch solve reads W and
 * dL/dWq from memory in every pass (needs both 16-byte aligned, else IDKM_ERR_UNSUPPORTED).  Smaller values of
 * `bytes` send smaller layers that way (test support, comparisons). */
idkm_status idkm_set_tile_limit(idkm_ctx* ctx, int64_t bytes);
/* Bound of every device-side wait of the persistent kernels, in polls (default 2^20, about a second).  When a
 * wait expires all workgroups leave the kernel.  Under IDKM_PATH_AUTO the call is then answered by the stream path
 * (a new launch from the host; idkm_info.path says IDKM_PATH_STREAM), and so is a call whose persistent grid would
 * not be resident at once; under an explicit IDKM_PATH_PERSISTENT the call returns IDKM_ERR_DEVICE.  The context
 * stays usable either way.  A limit of 0 makes the first unsuccessful poll give up (used to exercise that path). */
idkm_status idkm_set_spin_limit(idkm_ctx* ctx, uint32_t polls);
/* Measurement support.  With enable != 0 the library records a HIP event on the caller's stream immediately before
 * and immediately after every launch of a persistent kernel (one launch = one whole solve); idkm_last_kernel_ms then
 * waits for the second event and gives the time between the two -- the duration of that launch as the stream saw it,
 * without the host-side work of the call around it.  IDKM_ERR_INVALID_ARG if timing is off or the last call did not
 * launch a persistent kernel (stream path, batched calls).  ms_out: host. */
idkm_status idkm_set_kernel_timing(idkm_ctx* ctx, int32_t enable);
idkm_status idkm_last_kernel_ms(idkm_ctx* ctx, float* ms_out);
/* Test support.  The words that cross workgroups are stamped with 32-bit sequence numbers that the context counts up
 * over its lifetime (one per exchange of the persistent kernels, one per launch of the stream path); shortly before
 * they would wrap the library clears its exchange buffers and starts over.  This call advances both counters by n
 * (saturating just below the wrap), so that a test can cross that point without billions of calls. */
idkm_status idkm_advance_sequence(idkm_ctx* ctx, uint32_t n, void* hip_stream);
/* Longest Krylov basis IDKM_BWD_GMRES keeps before it restarts from the current residual: 1 .. 256, default 64
 * (the basis never exceeds k d).  The workspace holds (basis + 1) k d doubles. */
idkm_status idkm_set_gmres_basis(idkm_ctx* ctx, int32_t basis);

/*
 * Algorithm 1 (soft k-means) followed by one evaluation at the solution.
 *
 *   C <- C0;  repeat  C+ = F(C, W)  until ||C+ - C||_F < tol  or max_iter evaluations   (Eq. "deepeqc")
 *   F(C, W) = diag(A^T 1)^-1 A^T W,  A = rowsoftmax_tau(-D(W, C))                        (Eq. "centers")
 * then, at the returned C* (the last C+):  A = A(W, C*), Wq = A C*, and the masses n* = A^T 1 and
 * F* = F(C*, W) are kept in the context for idkm_backward ("plug it into F one time", Sec. 4.2).
 *
 *   W       device [m,d]; borrowed by the context until the next idkm_forward or idkm_destroy: it must
 *           stay alive and unchanged through idkm_backward (Alg. 2: solve, loss, backward).
 *   C0      device [k,d] initial codebook (Alg. 1 leaves it open; it is an input here).
 *   tau>0   temperature; tol>=0 absolute Frobenius tolerance; max_iter>=1.
 *   C_out   device [k,d], required.
 *   A_out   device [m,k] or NULL (NULL: the attention matrix is never materialised).
 *   Wq_out  device [m,d] or NULL.
 *   assign_out device int32 [m] or NULL: index of the closest codeword q(w_i, C*) (Sec. 3), decided in
 *           float32 on the key |w-c| (d==1) or sum_r (w_r-c_r)^2 with separately rounded multiply and add
 *           in index order (d>1); ties go to the lowest index.
 *   info    host pointer or NULL.  If non-NULL the call waits for the stream before returning.
 *   hip_stream  a hipStream_t (NULL = default stream).  All work is enqueued on it.
 * A cluster with zero mass keeps its previous centre.  Requires 1<=k<=m.
 */
idkm_status idkm_forward(idkm_ctx* ctx, const float* W, int64_t m, int32_t d, const float* C0, int32_t k,
                         float tau, float tol, int32_t max_iter, idkm_dist dist, float* C_out, float* A_out,
                         float* Wq_out, int32_t* assign_out, idkm_info* info, void* hip_stream);

/*
 * Backward of the layer W -> Wq = A(W, C*(W)) C*(W) for the last idkm_forward on this context
 * (Alg. 2, per-layer backward steps): total derivative, including the direct dependence of A on W.
 *
 *   v = dL/dC* with W fixed;  g solves (I - dF/dC*)^T g = v  by the averaged iteration of Sec. 4.2
 *       g <- alpha (v + (dF/dC*)^T g) + (1-alpha) g,  g_0 = v,
 *   stopped when ||g+ - g||_F <= tol ||v||_F or after max_iter passes; a non-finite step or a step norm
 *   that grows on 5 consecutive passes restarts from g = v with alpha halved (at most 6 times).
 *   IDKM_BWD_JFB sets g = v (no pass).  IDKM_BWD_DENSE forms dF/dC* explicitly (the k x k matrix of Sec. 4.2,
 *   k d x k d in general) in the same pass that computes v and solves (I - dF/dC*)^T g = v by Gaussian
 *   elimination in float64: two passes over W in total, tol / max_iter / alpha are ignored, info.iters = 0 and
 *   info.converged = 0 only if the matrix is singular.  When the k d (k d + d + 1) sums fit one exchange line
 *   (k = 2 with d <= 2, k = 4 with d = 1) and the tiles fit in LDS, the persistent kernel does all of it in one
 *   launch (info.path says which form ran), and batched calls share that launch between layers.
 *   IDKM_BWD_GMRES solves the same system from g = 0 by restarted GMRES (basis length min(k d, 64) unless idkm_set_gmres_basis changed it, float64
 *   orthogonalisation): every pass applies (dF/dC*)^T to one basis vector; when the estimated residual falls
 *   below tol ||v||_F (or the basis is full) the iterate is updated and one more pass measures the true residual
 *   ||v + (dF/dC*)^T g - g||_F, which is the step norm of the undamped iteration at g and is held to the same
 *   test <= tol ||v||_F; otherwise a new cycle starts from that residual.  info.iters counts all these passes
 *   (at most max_iter + 1), info.residual is the last true residual, alpha is ignored; two cycles in a row that
 *   leave more than 95 % of the residual end the solve with converged = 0.  With k d <= 64 the first cycle is exact up to
 *   rounding.  With k in {2,4,8,16}, k d <= 64 and a layer whose tiles leave
 *   room on chip for the Krylov state (about 8 (R + 1)(k d + R + 1) bytes for a basis of R = min(k d, basis) vectors: 67 KB
 *   at k d = 64) the whole solve runs inside the persistent kernel (every workgroup keeps that state and takes the
 *   same steps); otherwise one launch per pass on the stream path (there IDKM_PATH_PERSISTENT gives
 *   IDKM_ERR_UNSUPPORTED).
 *   dL/dW = (direct term through A) + (dF/dW)^T g.
 * The attention weights are recomputed on the fly in every pass; nothing of size m*k is stored.
 *
 *   dWq     device [m,d], upstream gradient dL/dWq.
 *   alpha   in (0,1]; 1 = undamped, 0.25 = the paper's setting.
 *   dW_out  device [m,d], required.
 *   info    host or NULL (as in idkm_forward).
 */
idkm_status idkm_backward(idkm_ctx* ctx, const float* dWq, idkm_bwd_mode mode, float tol, int32_t max_iter,
                          float alpha, float* dW_out, idkm_info* info, void* hip_stream);

/*
 * The two O(k d) vectors of the last idkm_backward on this context (Eq. "grad"): v = dL/dC* with W fixed, and the
 * g with which the call formed dL/dW -- the solution of (I - dF/dC*)^T g = v as far as the chosen mode took it
 * (the iterate after the last pass of the averaged iteration of Sec. 4.2, the direct or Krylov solution, or v itself
 * for IDKM_BWD_JFB).  v_out, g_out: HOST pointers to k d doubles each (row-major [k,d]), either may be NULL.
 * Waits for hip_stream.  IDKM_ERR_NO_FORWARD if no backward has completed since the last forward.
 */
idkm_status idkm_get_cotangents(idkm_ctx* ctx, double* v_out, double* g_out, void* hip_stream);

/*
 * Diagnostic: measures one of the ceilings a roofline of this path is drawn against, on the context's device.
 *   kind 0  full-rate lane operations per second (dependent-free v_fma_f32 chains, 8 wavefronts per SIMD)
 *   kind 1  exponentials per second (v_exp_f32 alone)
 *   kind 2  bytes per second of a streaming read of buf (device, 16-byte aligned, n_floats floats)
 *   kind 3, 4, 5  exponentials per second with 1, 2, 4 independent v_fma_f32 issued beside each of them
 *           (shows how transcendental and full-rate operations share the issue slots)
 *   kind 6  float32 multiply-adds per second of the matrix cores (v_mfma_f32_16x16x4_f32 alone, 2 wavefronts per SIMD)
 *   kind 7  the same count with 8 independent v_fma_f32 issued after every matrix instruction (equal to kind 6 if
 *           matrix and vector instructions overlapped; they do not on gfx950: about half)
 *   kind 8  float32 multiply-adds per second of v_mfma_f32_4x4x1_f32 (16 blocks per instruction)
 *   kind 9, 10  kind 7 with 4 and with 8 wavefronts per SIMD (does vector work of OTHER wavefronts fill the cycles a
 *           matrix instruction holds the pipeline?); kind 11  kind 6 with 4 wavefronts per SIMD
 * Waits for completion; *result (host) receives the rate.  Nothing on the method's path calls this.
 */
idkm_status idkm_calibrate(idkm_ctx* ctx, int32_t kind, const float* buf, int64_t n_floats, double* result,
                           void* hip_stream);

/*
 * The stored form of a quantised layer (Sec. 3, product-quantisation set-up: every sub-vector w_i is replaced by
 * its closest codeword q(w_i, C), one of k = 2^b, so a layer is kept as m codes of b bits plus the codebook).
 *
 *   idkm_code_bits     b = the smallest b >= 1 with 2^b >= k (0 if k < 1)
 *   idkm_code_words    number of 32-bit words of the stream: ceil(m b / 32) (-1 for invalid m, k)
 *   idkm_pack_codes    assign (device int32 [m], 16-byte aligned, values in [0, k); idkm_forward's assign_out)
 *                      -> words_out (device uint32 [idkm_code_words(m, k)]).  Code i occupies bits [i b, (i+1) b) of
 *                      one little-endian bit stream (stream bit t = bit t mod 32 of word t div 32); the unused high
 *                      bits of the last word are zero.  Only the low b bits of each value are used.
 *   idkm_unpack_quantize  words + codebook C (device [k,d]) -> Wh_out (device [m,d]) = q(W, C): row i is a bitwise
 *                      copy of codeword row code_i.  A code >= k (possible only in a stream that idkm_pack_codes did
 *                      not write when k is not a power of two) gives a row of NaN.
 * Both enqueue one kernel on hip_stream and do not wait.  1 <= k <= 1024, 1 <= d <= 64; m = 0 is a no-op.
 */
int32_t idkm_code_bits(int32_t k);
int64_t idkm_code_words(int64_t m, int32_t k);
idkm_status idkm_pack_codes(idkm_ctx* ctx, const int32_t* assign, int64_t m, int32_t k, uint32_t* words_out,
                            void* hip_stream);
idkm_status idkm_unpack_quantize(idkm_ctx* ctx, const uint32_t* words, int64_t m, const float* C, int32_t k, int32_t d,
                                 float* Wh_out, void* hip_stream);

/*
 * Batched calls for the per-layer loops of Algorithm 2 ("for all layers: find C*(W)" and the matching backward
 * loop).  The layers are independent problems.  A batch owns one context per layer; layers that the persistent
 * path serves and that share a kernel shape (k, d, dist) are solved by ONE launch in which every layer has its own
 * team of workgroups, as many layers per launch as the device can hold resident at once.  Small layers are bound
 * by the latency of the grid-wide exchange of every pass; teams that share compute units hide each other's
 * waiting, and the launch and wait costs are paid once per batch instead of once per layer.  A layer that needs
 * the stream path is solved synchronously in its turn.
 *
 *   idkm_batch_create   n_layers in [1, 1024] contexts
 *   idkm_batch_forward  layers[i] is solved with the batch's i-th context, with the results idkm_forward gives;
 *                       infos (host, [n]) and statuses (host, [n]) receive the per-layer results.  Work is issued
 *                       on hip_stream; the call returns when every layer is complete.
 *   idkm_batch_backward layer i must have had a successful idkm_batch_forward with the same index.
 *   idkm_batch_launches number of batched kernel launches the last call needed (diagnostic)
 *   idkm_batch_context  the i-th layer's context, owned by the batch (for idkm_set_path, idkm_set_spin_limit,
 *                       idkm_last_error, idkm_step_JCT ...); NULL if i is out of range
 * Return value: IDKM_OK if every layer succeeded, otherwise the status of the first layer that failed
 * (idkm_batch_last_error gives its message); the other layers are still attempted.
 */
typedef struct idkm_batch idkm_batch; /* opaque */
typedef struct {
    const float* W;  /* device [m,d] */
    int64_t m;
    int32_t d;
    const float* C0; /* device [k,d] */
    int32_t k;
    float tau, tol;
    int32_t max_iter;
    int32_t dist;        /* idkm_dist */
    float* C_out;        /* device [k,d], required */
    float* A_out;        /* device [m,k] or NULL */
    float* Wq_out;       /* device [m,d] or NULL */
    int32_t* assign_out; /* device [m] or NULL */
} idkm_fwd_desc;
typedef struct {
    const float* dWq; /* device [m,d] */
    int32_t mode;     /* idkm_bwd_mode */
    float tol;
    int32_t max_iter;
    float alpha;
    float* dW_out; /* device [m,d], required */
} idkm_bwd_desc;
idkm_status idkm_batch_create(idkm_batch** out, int device_id, int32_t n_layers);
idkm_status idkm_batch_destroy(idkm_batch* b);
const char* idkm_batch_last_error(const idkm_batch* b);
int32_t idkm_batch_launches(const idkm_batch* b);
idkm_ctx* idkm_batch_context(idkm_batch* b, int32_t i);
idkm_status idkm_batch_forward(idkm_batch* b, const idkm_fwd_desc* layers, int32_t n, idkm_info* infos,
                               idkm_status* statuses, void* hip_stream);
idkm_status idkm_batch_backward(idkm_batch* b, const idkm_bwd_desc* layers, int32_t n, idkm_info* infos,
                                idkm_status* statuses, void* hip_stream);

/*
 * idkm_forward for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and error behaviour as idkm_forward, but there is no context: every
 * byte the kernels need beyond the caller's tensors (the exchange words of the grid-wide sums, the O(k d) solver
 * state, the block the kernel reports into -- about 545 KB) lies in one array in the library's device image, one
 * copy per GPU, held until the process ends.  The call makes no hipMalloc / hipFree and no other allocating call.
 *   device_id   the HIP device (0 .. 63) whose copy of the array is used; made current by the call.
 *   Limits      k in {2, 4, 8, 16}, d in {1, 2, 4}, m d <= IDKM_NOALLOC_MAX_WEIGHTS (the whole layer is held in LDS, one
 *               launch per solve); anything else returns IDKM_ERR_UNSUPPORTED and touches nothing.
 *   info        host or NULL.  With NULL the solve is only enqueued on hip_stream and nothing waits; otherwise the
 *               call copies the kernel's report back and waits for the stream.
 * No state for idkm_backward is kept.  All calls on one GPU share that GPU's array, which keeps the previous call's
 * contents (its words carry sequence numbers, so stale ones are never taken for new): calls that overlap on one GPU
 * -- from several threads or on several streams -- race; the library serialises only its own host-side bookkeeping.
 * idkm_noalloc_last_error gives the detail of the last failed call (process-wide; "" if none).
 */
#define IDKM_NOALLOC_MAX_WEIGHTS 9400000
idkm_status idkm_forward_noalloc(int device_id, const float* W, int64_t m, int32_t d, const float* C0, int32_t k,
                                 float tau, float tol, int32_t max_iter, idkm_dist dist, float* C_out, float* A_out,
                                 float* Wq_out, int32_t* assign_out, idkm_info* info, void* hip_stream);
const char* idkm_noalloc_last_error(void);

/*
 * Single evaluations at a caller-supplied codebook C (device [k,d]), for testing one step in
 * isolation.  They overwrite the forward state of the context with (W, C, n = A^T 1, F(C, W)).
 *   idkm_step_F:   Cplus_out[k,d] = F(C, W)                         (Eq. "deepeqc"); n_out device [k] or NULL
 *   idkm_step_JCT: out[k,d] = (dF/dC)^T g at the state left by idkm_step_F / idkm_forward, g device [k,d]
 */
idkm_status idkm_step_F(idkm_ctx* ctx, const float* W, int64_t m, int32_t d, const float* C, int32_t k,
                        float tau, idkm_dist dist, float* Cplus_out, float* n_out, void* hip_stream);
idkm_status idkm_step_JCT(idkm_ctx* ctx, const float* g, float* out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* IDKM_H */
