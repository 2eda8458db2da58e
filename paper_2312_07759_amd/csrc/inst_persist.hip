// Instantiations of the persistent (one launch per solve) kernels.
#include "dispatch.h"
#include "persist_small.hpp"

namespace idkm {

template <int K, int D>
static PersistFns pick(int dist, bool bwd) {
    if (dist == DIST_L2)
        return bwd ? PersistFns{persist_bwd<K, D, DIST_L2>, persist_bwd_batch<K, D, DIST_L2>}
                   : PersistFns{persist_fwd<K, D, DIST_L2>, persist_fwd_batch<K, D, DIST_L2>};
    return bwd ? PersistFns{persist_bwd<K, D, DIST_SQL2>, persist_bwd_batch<K, D, DIST_SQL2>}
               : PersistFns{persist_fwd<K, D, DIST_SQL2>, persist_fwd_batch<K, D, DIST_SQL2>};
}

// Offered for every shape of the lane<->vector family: K (D+1) <= 80 sums per workgroup.
PersistFns persist_kernel(int K, int D, int dist, bool bwd) {
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
