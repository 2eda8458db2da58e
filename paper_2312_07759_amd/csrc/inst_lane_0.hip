// Instantiations of the lane<->codeword kernels for energy variant 0.
#include "dispatch.h"
#include "lane_k.hpp"

namespace idkm {

template <int KPL, int D>
static KernelFn pick(int pass) {
    if (KPL * (D + 1) > 80) return nullptr;
    switch (pass) {
        case PASS_FWD: return lane_pass<KPL, D, 0, PASS_FWD>;
        case PASS_FIN: return lane_pass<KPL, D, 0, PASS_FIN>;
        case PASS_B1: return lane_pass<KPL, D, 0, PASS_B1>;
        case PASS_B2: return lane_pass<KPL, D, 0, PASS_B2>;
        case PASS_B3: return lane_pass<KPL, D, 0, PASS_B3>;
    }
    return nullptr;
}

template <int KPL>
static KernelFn pick_d(int D, int pass) {
    switch (D) {
        case 1: return pick<KPL, 1>(pass);
        case 2: return pick<KPL, 2>(pass);
        case 4: return pick<KPL, 4>(pass);
        case 8: return pick<(KPL > 8 ? 8 : KPL), 8>(pass);
    }
    return nullptr;
}

KernelFn lane_kernel_0(int KPL, int D, int pass) {
    if (D == 8 && KPL > 8) return nullptr;
    switch (KPL) {
        case 1: return pick_d<1>(D, pass);
        case 2: return pick_d<2>(D, pass);
        case 4: return pick_d<4>(D, pass);
        case 8: return pick_d<8>(D, pass);
        case 16: return pick_d<16>(D, pass);
    }
    return nullptr;
}

KernelFn lane_tail_kernel(int pass) {
    switch (pass) {
        case PASS_FWD: return lane_tail<PASS_FWD>;
        case PASS_FIN: return lane_tail<PASS_FIN>;
        case PASS_B1: return lane_tail<PASS_B1>;
        case PASS_B2: return lane_tail<PASS_B2>;
    }
    return nullptr;
}

KernelFn lane_tail_wide_kernel() { return lane_tail_b2_wide<0>; }

void launch_reduce_rows(const Args& a, int nacc, int nwg, int pass, hipStream_t s) {
    hipLaunchKernelGGL(reduce_rows<0>, dim3((nacc + 63) / 64), dim3(WG), 0, s, a, nacc, nwg, pass);
}

}  // namespace idkm
