// Instantiations of the persistent kernels for layers larger than the chip's LDS (W streamed from memory).
#include "dispatch.h"
#include "persist_small.hpp"

namespace idkm {

template <int K, int D>
static PersistFns pick(int dist, bool bwd) {
    if (dist == DIST_L2)
        return bwd ? PersistFns{persist_bwd_global<K, D, DIST_L2>, nullptr} : PersistFns{persist_fwd_global<K, D, DIST_L2>, nullptr};
    return bwd ? PersistFns{persist_bwd_global<K, D, DIST_SQL2>, nullptr} : PersistFns{persist_fwd_global<K, D, DIST_SQL2>, nullptr};
}

PersistFns persist_kernel_global(int K, int D, int dist, bool bwd) {
    switch (K * 16 + D) {
        case 2 * 16 + 1: return pick<2, 1>(dist, bwd);
        case 4 * 16 + 1: return pick<4, 1>(dist, bwd);
        case 8 * 16 + 1: return pick<8, 1>(dist, bwd);
        case 16 * 16 + 1: return pick<16, 1>(dist, bwd);
        case 2 * 16 + 2: return pick<2, 2>(dist, bwd);
        case 4 * 16 + 2: return pick<4, 2>(dist, bwd);
        case 8 * 16 + 2: return pick<8, 2>(dist, bwd);
        case 2 * 16 + 4: return pick<2, 4>(dist, bwd);
        case 4 * 16 + 4: return pick<4, 4>(dist, bwd);
        case 16 * 16 + 2: return pick<16, 2>(dist, bwd);
        case 8 * 16 + 4: return pick<8, 4>(dist, bwd);
        case 16 * 16 + 4: return pick<16, 4>(dist, bwd);
    }
    return PersistFns{};
}

}  // namespace idkm
