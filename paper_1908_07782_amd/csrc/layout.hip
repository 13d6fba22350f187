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
// coalesced (the tiled side fully, the row-major side in Wt-column chunks).  Scalar form:
// any alignment, any pitch.
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

// 128-bit form for 16-byte aligned buffers with ld % 4 == 0: streaming loads and stores,
// up to four words per thread in flight; the ragged columns of the last tile go one by one.
constexpr int kRelayoutBatch = 4;

template <bool PACK>
__global__ __launch_bounds__(kThreads) void relayout_vec_kernel(float* __restrict__ out,
                                                                const float* __restrict__ in,
                                                                int64_t ld, int32_t N, int64_t P,
                                                                int Wt, uint32_t ntiles, uint32_t run) {
    // which tile: workgroup i takes tile i, or the XCDs (i mod 8) take turns at runs of `run` tiles
    const uint32_t tile = xcd_run_block(blockIdx.x, run);
    if (tile >= ntiles) return;
    const int64_t col0 = (int64_t)tile * Wt;
    const int width = (int)(col0 + Wt <= P ? Wt : P - col0);
    const size_t tile_base = (size_t)tile * (size_t)N * (size_t)Wt;
    const int W4 = Wt >> 2;
    const int w4_shift = 31 - __clz(W4);
    const int total4 = N * W4;
    for (int base = 0; base < total4; base += kThreads * kRelayoutBatch) {
        v4f v[kRelayoutBatch];
        size_t dst[kRelayoutBatch];
        bool whole[kRelayoutBatch];
#pragma unroll
        for (int u = 0; u < kRelayoutBatch; ++u) {
            const int idx = base + u * kThreads + (int)threadIdx.x;
            whole[u] = false;
            if (idx < total4) {
                const int row = idx >> w4_shift;
                const int c = (idx & (W4 - 1)) * 4;
                const size_t t = tile_base + (size_t)row * (size_t)Wt + (size_t)c;
                const size_t r = (size_t)row * (size_t)ld + (size_t)col0 + (size_t)c;
                if (c + 4 <= width) {
                    whole[u] = true;
                    dst[u] = PACK ? t : r;
                    v[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(in + (PACK ? r : t)));
                } else {
                    for (int k = 0; c + k < width; ++k) {
                        if (PACK) out[t + k] = in[r + k];
                        else out[r + k] = in[t + k];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kRelayoutBatch; ++u)
            if (whole[u]) store4_stream(out + dst[u], v[u]);
        // every load of the pass has been consumed; stating it keeps the compiler from
        // putting a wait in front of each load of the next pass (see gossip_slab_kernel.h)
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
}

template <bool PACK>
hipError_t launch_relayout(float* out, const float* in, int64_t ld, int32_t N, int64_t P, int Wt,
                           uint32_t run, hipStream_t st) {
    const uint64_t tiles = ((uint64_t)P + (uint64_t)Wt - 1) / (uint64_t)Wt;
    uint64_t groups = tiles;
    if (run != 0) groups = (tiles + 8ull * run - 1) / (8ull * run) * (8ull * run);
    // a grid dimension holds fewer than 2^32 work-items
    if (tiles > 0x7FFFFFF0ull || groups * kThreads > 0xFFFFFFFFull) return hipErrorInvalidValue;
    const bool vec = (((uintptr_t)out | (uintptr_t)in) & 15u) == 0 && ld % 4 == 0 && Wt % 4 == 0 &&
                     (Wt & (Wt - 1)) == 0;
    if (vec)
        hipLaunchKernelGGL(relayout_vec_kernel<PACK>, dim3((uint32_t)groups), dim3(kThreads), 0, st, out,
                           in, ld, N, P, Wt, (uint32_t)tiles, run);
    else
        hipLaunchKernelGGL(relayout_kernel<PACK>, dim3((uint32_t)tiles), dim3(kThreads), 0, st, out, in,
                           ld, N, P, Wt);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pack_tiled(float* tiled, const float* rows, int64_t ld, int32_t N, int64_t P,
                             int Wt, uint32_t run, hipStream_t st) {
    return launch_relayout<true>(tiled, rows, ld, N, P, Wt, run, st);
}

hipError_t launch_unpack_tiled(float* rows, int64_t ld, const float* tiled, int32_t N, int64_t P,
                               int Wt, uint32_t run, hipStream_t st) {
    return launch_relayout<false>(rows, tiled, ld, N, P, Wt, run, st);
}

}  // namespace combo
