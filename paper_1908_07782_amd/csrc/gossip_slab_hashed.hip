// Table-free instantiations of the LDS-slab aggregation kernel: peer selection
// (Sec. 4.1 step 2), the optional local steps (step 1) and the aggregation (Eq. 3 / 4) in
// ONE launch.  Every workgroup derives the peer lists of its strip from the counter-based
// hash while its slab loads are in flight, so no table is written to or read from memory
// and a round is a single kernel.  Results are identical to the table-driven path.
#include "gossip_slab_kernel.h"

namespace combo {
namespace {

template <int RT>
hipError_t launch_hashed_rt(const RoundArgs& a, int W, uint32_t grid, size_t lds, hipStream_t st) {
    const bool weighted = a.dsz != nullptr, fused = a.grad != nullptr;
    const bool small = slab_threads(a.N, W) == 256;
#define COMBO_HASHED_LAUNCH(WT, FU)                                                                \
    do {                                                                                           \
        if (small)                                                                                 \
            hipLaunchKernelGGL((gossip_slab_kernel<RT, WT, FU, false, 256, true>), dim3(grid),         \
                               dim3(256), lds, st, a, W);                                          \
        else                                                                                       \
            hipLaunchKernelGGL((gossip_slab_kernel<RT, WT, FU, false, 512, true>), dim3(grid),         \
                               dim3(512), lds, st, a, W);                                          \
    } while (0)
    if (weighted) {
        if (fused) COMBO_HASHED_LAUNCH(true, true);
        else COMBO_HASHED_LAUNCH(true, false);
    } else {
        if (fused) COMBO_HASHED_LAUNCH(false, true);
        else COMBO_HASHED_LAUNCH(false, false);
    }
#undef COMBO_HASHED_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_round_slab_hashed(const RoundArgs& a, int W, hipStream_t st) {
    const uint32_t grid = slab_grid(a, W);
    if (grid == 0) return hipErrorInvalidValue;
    const size_t lds = slab_lds_request(a, W, true);
    switch (a.R) {
        case 0: return launch_hashed_rt<0>(a, W, grid, lds, st);
        case 1: return launch_hashed_rt<1>(a, W, grid, lds, st);
        case 2: return launch_hashed_rt<2>(a, W, grid, lds, st);
        case 3: return launch_hashed_rt<3>(a, W, grid, lds, st);
        case 4: return launch_hashed_rt<4>(a, W, grid, lds, st);
        case 5: return launch_hashed_rt<5>(a, W, grid, lds, st);
        case 6: return launch_hashed_rt<6>(a, W, grid, lds, st);
        case 7: return launch_hashed_rt<7>(a, W, grid, lds, st);
        case 8: return launch_hashed_rt<8>(a, W, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace combo
