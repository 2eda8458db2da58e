// Host-side lookup of kernel instantiations.
#pragma once
#include "common.hpp"

namespace idkm {

typedef void (*KernelFn)(const Args);

// Lane<->vector family: K in {2,4,8,16}, D in {1,2,4}.  nullptr if not instantiated.
KernelFn small_kernel(int K, int D, int dist, int pass);
// Lane<->codeword family: KPL = ceil(k/64) rounded up to {1,2,4,8,16}, D in {1,2,4,8}, KPL*(D+1) <= 80.
KernelFn lane_kernel(int KPL, int D, int dist, int pass);

// Matrix-core form of a lane<->codeword pass for d = 4 (mfma_lane_threads threads, dynamic LDS = (vec_per_wg + 16) * 20 bytes);
// nullptr where there is none (KPL > 4; passes other than the forward loop and (dF/dC)^T).
KernelFn mfma_lane_kernel(int KPL, int dist, int pass);
int mfma_lane_threads(int KPL, int dist, int pass);  // workgroup size that kernel is launched with

// Lane<->codeword family, stream path: reduction of the per-workgroup partials and the O(k d) tail of a pass.
KernelFn lane_tail_kernel(int pass);
KernelFn lane_tail_wide_kernel();  // PASS_B2 tail for 1024 threads
void launch_reduce_rows(const Args& a, int nacc, int nwg, int pass, hipStream_t s);

struct PArgs;
struct BatchItem;
typedef void (*PersistFn)(const Args, const PArgs);
typedef void (*PersistBatchFn)(const BatchItem*, const unsigned short*);
// The two launch forms of one persistent solve: a single problem, or several problems of the same shape.
struct PersistFns {
    PersistFn one = nullptr;
    PersistBatchFn batch = nullptr;
    bool matrix = false;  // matrix-core kernel: tile padded by 16 vectors plus one float per vector, `threads` per workgroup
    int threads = 0;
};
// Persistent forward / backward solve for the lane<->vector family; empty if K (D+1) > 32.
PersistFns persist_kernel(int K, int D, int dist, bool bwd);
// The same for a layer that does not fit the chip's LDS: W (and dL/dWq) are read from memory in every pass, no
// dynamic LDS; single-problem launch form only.
PersistFns persist_kernel_global(int K, int D, int dist, bool bwd);
// Persistent solve for the lane<->codeword family (launch with 1024 threads); empty if not instantiated.
// matrix: prefer the matrix-core forward loop where one exists (d = 4, k <= 256).
PersistFns persist_lane_kernel(int KPL, int D, int dist, bool bwd, bool matrix);

// b-bit code stream of the hard assignments and the reconstruction q(W, C) from it (codes.hip).
void launch_pack_codes(const int32_t* assign, int64_t m, int bits, uint32_t* words, int64_t nwords, hipStream_t s);
void launch_unpack_quantize(const uint32_t* words, int64_t nwords, int64_t m, int bits, const float* C, int k, int d,
                            float* out, hipStream_t s);

// Micro-benchmarks of the roofline's ceilings (calibrate.hip).
void launch_cal_fma(float* out, int grid, int iters, hipStream_t s);
void launch_cal_exp(float* out, int grid, int iters, int fmas, hipStream_t s);  // fmas in {0, 1, 2, 4}
void launch_cal_mfma(float* out, int grid, int iters, int mode, hipStream_t s);  // mode 0: 16x16x4, 1: + 8 FMAs each, 2: 4x4x1
void launch_cal_read(const float* src, size_t n_floats, int grid, float* out, hipStream_t s);

}  // namespace idkm
