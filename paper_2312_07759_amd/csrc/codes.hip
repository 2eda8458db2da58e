// The stored form of a quantised layer (Sec. 3: every sub-vector is replaced by one of k = 2^b codewords):
// b-bit codes in one little-endian bit stream, and the reconstruction q(W, C) from codes and codebook.
#include "dispatch.h"

namespace idkm {

// Thread t packs codes [32 t, 32 t + 32) into exactly `bits` words [bits t, bits t + bits).
__global__ __launch_bounds__(256) void k_pack_codes(const int32_t* __restrict__ assign, int64_t m, int bits,
                                                     uint32_t* __restrict__ words, int64_t nwords) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t first = t * 32;
    if (first >= m) return;
    int32_t c[32];
    if (first + 32 <= m) {
        const int4* src = reinterpret_cast<const int4*>(assign + first);  // 128-byte aligned: first is a multiple of 32
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int4 v = src[q];
            c[4 * q] = v.x;
            c[4 * q + 1] = v.y;
            c[4 * q + 2] = v.z;
            c[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) c[i] = (first + i < m) ? assign[first + i] : 0;
    }
    const uint32_t mask = (1u << bits) - 1u;
    unsigned long long buf = 0ull;
    int fill = 0;
    int64_t w = t * bits;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        buf |= (unsigned long long)((uint32_t)c[i] & mask) << fill;
        fill += bits;
        if (fill >= 32) {
            if (w < nwords) words[w] = (uint32_t)buf;
            ++w;
            buf >>= 32;
            fill -= 32;
        }
    }
}

// Thread i reads code i and copies codeword row C[code] to out[i]; a code >= k (not a valid stream) gives NaN.
__global__ __launch_bounds__(256) void k_unpack_quantize(const uint32_t* __restrict__ words, int64_t nwords, int64_t m,
                                                          int bits, const float* __restrict__ C, int k, int d,
                                                          float* __restrict__ out, int c_in_lds) {
    extern __shared__ float s_C[];
    if (c_in_lds) {
        for (int i = threadIdx.x; i < k * d; i += 256) s_C[i] = C[i];
        __syncthreads();
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= m) return;
    const int64_t off = i * bits;
    const int64_t w = off >> 5;
    const int sh = (int)(off & 31);
    unsigned long long win = words[w];
    if (sh + bits > 32 && w + 1 < nwords) win |= (unsigned long long)words[w + 1] << 32;
    const uint32_t code = (uint32_t)(win >> sh) & ((1u << bits) - 1u);
    const bool ok = code < (uint32_t)k;
    const float* row = (c_in_lds ? s_C : C) + (size_t)(ok ? code : 0u) * d;
    for (int r = 0; r < d; ++r) out[i * d + r] = ok ? row[r] : __builtin_nanf("");
}

void launch_pack_codes(const int32_t* assign, int64_t m, int bits, uint32_t* words, int64_t nwords, hipStream_t s) {
    const int64_t threads = (m + 31) / 32;
    const unsigned grid = (unsigned)((threads + 255) / 256);
    hipLaunchKernelGGL(k_pack_codes, dim3(grid), dim3(256), 0, s, assign, m, bits, words, nwords);
}

void launch_unpack_quantize(const uint32_t* words, int64_t nwords, int64_t m, int bits, const float* C, int k, int d,
                            float* out, hipStream_t s) {
    const unsigned grid = (unsigned)((m + 255) / 256);
    const size_t cbytes = (size_t)k * d * sizeof(float);
    const int in_lds = cbytes <= 32 * 1024 ? 1 : 0;
    hipLaunchKernelGGL(k_unpack_quantize, dim3(grid), dim3(256), in_lds ? cbytes : 0, s, words, nwords, m, bits, C, k, d,
                       out, in_lds);
}

}  // namespace idkm
