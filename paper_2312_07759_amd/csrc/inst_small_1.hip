// Instantiations of the lane<->vector kernels for energy variant 1.
#include "dispatch.h"
#include "small_k.hpp"

namespace idkm {

template <int K, int D, bool OK>
struct pick_bj {
    static KernelFn get() { return nullptr; }
};
template <int K, int D>
struct pick_bj<K, D, true> {
    static KernelFn get() { return small_pass<K, D, 1, PASS_BJ>; }
};

template <int K, int D>
static KernelFn pick(int pass) {
    switch (pass) {
        case PASS_FWD: return small_pass<K, D, 1, PASS_FWD>;
        case PASS_FIN: return small_pass<K, D, 1, PASS_FIN>;
        case PASS_B1: return small_pass<K, D, 1, PASS_B1>;
        case PASS_B2: return small_pass<K, D, 1, PASS_B2>;
        case PASS_B3: return small_pass<K, D, 1, PASS_B3>;
        case PASS_BJ: return pick_bj<K, D, (K * D <= DENSE_MAX_KD)>::get();
    }
    return nullptr;
}

template <int K>
static KernelFn pick_d(int D, int pass) {
    switch (D) {
        case 1: return pick<K, 1>(pass);
        case 2: return pick<K, 2>(pass);
        case 4: return pick<K, 4>(pass);
    }
    return nullptr;
}

KernelFn small_kernel_1(int K, int D, int pass) {
    switch (K) {
        case 2: return pick_d<2>(D, pass);
        case 4: return pick_d<4>(D, pass);
        case 8: return pick_d<8>(D, pass);
        case 16: return pick_d<16>(D, pass);
    }
    return nullptr;
}

}  // namespace idkm
