// Instantiations of the persistent lane<->codeword kernels for energy variant 0.
#include "dispatch.h"
#include "persist_lane.hpp"

namespace idkm {

template <int KPL, int D>
static PersistFns pick(bool bwd) {
    return bwd ? PersistFns{persist_lane_bwd<KPL, D, 0>, persist_lane_bwd_batch<KPL, D, 0>}
               : PersistFns{persist_lane_fwd<KPL, D, 0>, persist_lane_fwd_batch<KPL, D, 0>};
}

// d = 4: the forward loop runs on the matrix cores (k <= 256).
template <int KPL>
static PersistFns pick4(bool bwd, bool matrix) {
    if (!matrix) return pick<KPL, 4>(bwd);
    if (bwd) return PersistFns{persist_mfma_bwd<KPL, 0>, persist_mfma_bwd_batch<KPL, 0>, true, mfma_bwd_threads<KPL, 0>()};
    return PersistFns{persist_mfma_fwd<KPL, 0>, persist_mfma_fwd_batch<KPL, 0>, true, MT};
}

// Offered for KPL*D <= 16 and KPL*(D+1) <= 24 (k <= 512), d <= 4.
PersistFns persist_lane_kernel_0(int KPL, int D, bool bwd, bool matrix) {
    switch (KPL * 16 + D) {
        case 1 * 16 + 1: return pick<1, 1>(bwd);
        case 1 * 16 + 2: return pick<1, 2>(bwd);
        case 1 * 16 + 4: return pick4<1>(bwd, matrix);
        case 2 * 16 + 1: return pick<2, 1>(bwd);
        case 2 * 16 + 2: return pick<2, 2>(bwd);
        case 2 * 16 + 4: return pick4<2>(bwd, matrix);
        case 4 * 16 + 1: return pick<4, 1>(bwd);
        case 4 * 16 + 2: return pick<4, 2>(bwd);
        case 4 * 16 + 4: return pick4<4>(bwd, matrix);
        case 8 * 16 + 1: return pick<8, 1>(bwd);
        case 8 * 16 + 2: return pick<8, 2>(bwd);
    }
    return PersistFns{};
}

}  // namespace idkm
