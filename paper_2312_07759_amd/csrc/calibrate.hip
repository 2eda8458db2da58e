// Micro-benchmarks of the ceilings the roofline uses: full-rate lane operations (v_fma_f32), transcendentals
// (v_exp_f32), float32 matrix instructions and a streaming read.  Diagnostic only; nothing on the method's path calls these.
#include "dispatch.h"

namespace idkm {

// 16 independent chains per lane keep the pipeline full; `iters` rounds of 16 operations each.
__global__ __launch_bounds__(256) void k_cal_fma(float* out, int iters, float a, float b) {
    float x[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) x[u] = (float)(threadIdx.x + u) * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) x[u] = fmaf(x[u], a, b);
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) s += x[u];
    if (s == 12345.678f) out[0] = s;  // keeps the chains alive without a store in the common case
}

// NF full-rate operations (FMAs on separate chains) issued beside every exponential: NF = 0 gives the rate of the
// transcendental alone (the negated absolute value is a free source modifier), NF > 0 shows how the two share the
// issue slots.
template <int NF>
__global__ __launch_bounds__(256) void k_cal_exp(float* out, int iters, float a, float b) {
    float x[8], y[8 * (NF > 0 ? NF : 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = (float)(threadIdx.x + u) * 1e-3f;
#pragma unroll
    for (int u = 0; u < 8 * (NF > 0 ? NF : 1); ++u) y[u] = (float)(threadIdx.x + u) * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            x[u] = __builtin_amdgcn_exp2f(-fabsf(x[u]));
#pragma unroll
            for (int f = 0; f < NF; ++f) y[u * NF + f] = fmaf(y[u * NF + f], a, b);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += x[u];
#pragma unroll
    for (int u = 0; u < 8 * (NF > 0 ? NF : 1); ++u) s += y[u];
    if (s == 12345.678f) out[0] = s;
}

// Float32 matrix instructions, eight independent accumulators per wavefront.  MODE 0: v_mfma_f32_16x16x4_f32 alone;
// MODE 1: the same with eight independent v_fma_f32 after each (do the two kinds overlap?); MODE 2: v_mfma_f32_4x4x1.
typedef float cal_f32x4 __attribute__((ext_vector_type(4)));
template <int MODE>
__global__ __launch_bounds__(512) void k_cal_mfma(float* out, int iters, float a, float b) {
    cal_f32x4 c[8];
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        c[u] = cal_f32x4{0.f, 0.f, 0.f, 0.f};
        v[u] = (float)(threadIdx.x + u) * 1e-3f;
    }
    const float x = a + (float)threadIdx.x * 1e-6f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (MODE == 2)
                c[u] = __builtin_amdgcn_mfma_f32_4x4x1f32(x, b, c[u], 0, 0, 0);
            else
                c[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(x, b, c[u], 0, 0, 0);
            if (MODE == 1) {
#pragma unroll
                for (int f = 0; f < 8; ++f) v[f] = fmaf(v[f], a, b);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (c[u][0] + c[u][1]) + (c[u][2] + c[u][3]) + v[u];
    if (s == 12345.678f) out[0] = s;
}

// Grid-stride read of n float4 values.
__global__ __launch_bounds__(256) void k_cal_read(const float4* __restrict__ src, size_t n, float* out) {
    float s = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float4 v = src[i];
        s += (v.x + v.y) + (v.z + v.w);
    }
    if (s == 12345.678f) out[0] = s;
}

void launch_cal_fma(float* out, int grid, int iters, hipStream_t s) {
    hipLaunchKernelGGL(k_cal_fma, dim3(grid), dim3(256), 0, s, out, iters, 0.999f, 1e-3f);
}
void launch_cal_exp(float* out, int grid, int iters, int fmas, hipStream_t s) {
    if (fmas == 0) hipLaunchKernelGGL(k_cal_exp<0>, dim3(grid), dim3(256), 0, s, out, iters, 0.999f, 1e-3f);
    if (fmas == 1) hipLaunchKernelGGL(k_cal_exp<1>, dim3(grid), dim3(256), 0, s, out, iters, 0.999f, 1e-3f);
    if (fmas == 2) hipLaunchKernelGGL(k_cal_exp<2>, dim3(grid), dim3(256), 0, s, out, iters, 0.999f, 1e-3f);
    if (fmas == 4) hipLaunchKernelGGL(k_cal_exp<4>, dim3(grid), dim3(256), 0, s, out, iters, 0.999f, 1e-3f);
}
void launch_cal_mfma(float* out, int grid, int iters, int mode, hipStream_t s) {
    if (mode == 0) hipLaunchKernelGGL(k_cal_mfma<0>, dim3(grid), dim3(512), 0, s, out, iters, 0.999f, 1e-3f);
    if (mode == 1) hipLaunchKernelGGL(k_cal_mfma<1>, dim3(grid), dim3(512), 0, s, out, iters, 0.999f, 1e-3f);
    if (mode == 2) hipLaunchKernelGGL(k_cal_mfma<2>, dim3(grid), dim3(512), 0, s, out, iters, 0.999f, 1e-3f);
}
void launch_cal_read(const float* src, size_t n_floats, int grid, float* out, hipStream_t s) {
    hipLaunchKernelGGL(k_cal_read, dim3(grid), dim3(256), 0, s, reinterpret_cast<const float4*>(src), n_floats / 4, out);
}

}  // namespace idkm
