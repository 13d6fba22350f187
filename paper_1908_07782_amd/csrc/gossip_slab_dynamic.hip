// Dynamic-worker instantiations (Sec. 4.2 semantics) of the LDS-slab aggregation kernel.
#include "gossip_slab_kernel.h"

namespace combo {
namespace {

template <int RT>
hipError_t launch_dynamic_rt(const RoundArgs& a, int W, uint32_t grid, size_t lds, hipStream_t st) {
    const bool small = slab_threads(a.N, W) == 256;
    if (a.dsz != nullptr) {
        if (small)
            hipLaunchKernelGGL((gossip_slab_kernel<RT, true, false, true, 256>), dim3(grid), dim3(256),
                               lds, st, a, W);
        else
            hipLaunchKernelGGL((gossip_slab_kernel<RT, true, false, true, 512>), dim3(grid), dim3(512),
                               lds, st, a, W);
    } else {
        if (small)
            hipLaunchKernelGGL((gossip_slab_kernel<RT, false, false, true, 256>), dim3(grid), dim3(256),
                               lds, st, a, W);
        else
            hipLaunchKernelGGL((gossip_slab_kernel<RT, false, false, true, 512>), dim3(grid), dim3(512),
                               lds, st, a, W);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_round_slab_dynamic(const RoundArgs& a, int W, uint32_t grid, size_t lds,
                                     hipStream_t st) {
    switch (a.R) {
        case 0: return launch_dynamic_rt<0>(a, W, grid, lds, st);
        case 1: return launch_dynamic_rt<1>(a, W, grid, lds, st);
        case 2: return launch_dynamic_rt<2>(a, W, grid, lds, st);
        case 3: return launch_dynamic_rt<3>(a, W, grid, lds, st);
        case 4: return launch_dynamic_rt<4>(a, W, grid, lds, st);
        case 5: return launch_dynamic_rt<5>(a, W, grid, lds, st);
        case 6: return launch_dynamic_rt<6>(a, W, grid, lds, st);
        case 7: return launch_dynamic_rt<7>(a, W, grid, lds, st);
        case 8: return launch_dynamic_rt<8>(a, W, grid, lds, st);
        default: return launch_dynamic_rt<-1>(a, W, grid, lds, st);
    }
}

}  // namespace combo
