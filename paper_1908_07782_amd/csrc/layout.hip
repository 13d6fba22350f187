// Conversion between the two arena layouts.
//   row-major  [N][ld]      : worker w's parameter e at w*ld + e
//   tiled      [T][N][Wt]   : tile e / Wt holds Wt consecutive columns of all N workers,
//                             worker-major inside the tile; T = ceil(P / Wt)
// In the tiled layout the N x Wt slab a workgroup of the aggregation kernel needs is one
// contiguous block of memory, which HBM streams measurably faster than N separate row
// chunks.  Columns >= P of the last tile are padding: never read, never written.
#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

// one workgroup per tile; consecutive lanes walk along a row chunk, so both sides are
// coalesced (the tiled side fully, the row-major side in Wt-column chunks)
template <bool PACK>
__global__ __launch_bounds__(kThreads) void relayout_kernel(float* __restrict__ out,
                                                            const float* __restrict__ in, int64_t ld,
                                                            int32_t N, int64_t P, int Wt) {
    const int64_t col0 = (int64_t)blockIdx.x * Wt;
    const int width = (int)(col0 + Wt <= P ? Wt : P - col0);
    const size_t tile_base = (size_t)blockIdx.x * (size_t)N * (size_t)Wt;
    const int total = N * Wt;
    for (int idx = threadIdx.x; idx < total; idx += kThreads) {
        const int row = idx / Wt;
        const int c = idx - row * Wt;
        if (c >= width) continue;
        const size_t t = tile_base + (size_t)row * (size_t)Wt + (size_t)c;
        const size_t r = (size_t)row * (size_t)ld + (size_t)col0 + (size_t)c;
        if (PACK) out[t] = in[r];
        else out[r] = in[t];
    }
}

}  // namespace

hipError_t launch_pack_tiled(float* tiled, const float* rows, int64_t ld, int32_t N, int64_t P,
                             int Wt, hipStream_t st) {
    const uint64_t tiles = ((uint64_t)P + (uint64_t)Wt - 1) / (uint64_t)Wt;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(relayout_kernel<true>, dim3((uint32_t)tiles), dim3(kThreads), 0, st, tiled, rows,
                       ld, N, P, Wt);
    return hipGetLastError();
}

hipError_t launch_unpack_tiled(float* rows, int64_t ld, const float* tiled, int32_t N, int64_t P,
                               int Wt, hipStream_t st) {
    const uint64_t tiles = ((uint64_t)P + (uint64_t)Wt - 1) / (uint64_t)Wt;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(relayout_kernel<false>, dim3((uint32_t)tiles), dim3(kThreads), 0, st, rows, tiled,
                       ld, N, P, Wt);
    return hipGetLastError();
}

}  // namespace combo
