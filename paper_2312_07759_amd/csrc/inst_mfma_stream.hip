// Instantiations of the stream-path matrix-core passes.
#include "dispatch.h"
#include "mfma_stream.cuh"

namespace idkm {

template <int KPL>
static KernelFn pick(int dist, int pass) {
    if (pass == PASS_FWD) return dist == DIST_L2 ? mfma_pass<KPL, DIST_L2, PASS_FWD> : mfma_pass<KPL, DIST_SQL2, PASS_FWD>;
    if (pass == PASS_B2 && dist == DIST_SQL2) return mfma_pass<KPL, DIST_SQL2, PASS_B2>;
    return nullptr;
}

KernelFn mfma_lane_kernel(int KPL, int dist, int pass) {
    switch (KPL) {
        case 1: return pick<1>(dist, pass);
        case 2: return pick<2>(dist, pass);
        case 4: return pick<4>(dist, pass);
    }
    return nullptr;
}

}  // namespace idkm
