// Instantiations of the stream-path matrix-core passes.
#include "dispatch.h"
#include "mfma_stream.hpp"

namespace idkm {

template <int KPL>
static KernelFn pick(int dist, int pass) {
    if (pass == PASS_FWD) return dist == DIST_L2 ? mfma_pass<KPL, DIST_L2, PASS_FWD> : mfma_pass<KPL, DIST_SQL2, PASS_FWD>;
    if (pass == PASS_B2) return dist == DIST_L2 ? mfma_pass<KPL, DIST_L2, PASS_B2> : mfma_pass<KPL, DIST_SQL2, PASS_B2>;
    return nullptr;
}

int mfma_lane_threads(int KPL, int dist, int pass) {
    return (KPL == 4 && dist == DIST_L2 && pass == PASS_B2) ? mfma_stream_threads<4, DIST_L2, PASS_B2>()
                                                             : mfma_stream_threads<1, DIST_SQL2, PASS_FWD>();
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
