// Aggregation-divergence monitor (Sec. 4.3, Definition 2 of the segmented-gossip paper):
// squared L2 distance of every worker's parameter vector from the aggregate of all
// workers (the dataset-size weighted mean; the plain mean for equal sizes).
//
// Read-only streaming pass, HBM bound (4 bytes per element).  A persistent workgroup
// walks over column strips; for each strip it stages the N x W slab in LDS, forms the
// W column means in binary64 (one thread per column, workers in order), then every
// thread squares its differences in binary64, a wavefront (64 consecutive columns of
// one row) reduces them with a fixed shuffle tree, and one thread per row adds the
// strip's partial to its private accumulator.  Per-workgroup partials go to a caller-
// supplied workspace and a second tiny kernel adds them in workgroup order, so the
// result is reproducible bit for bit (no floating-point atomics).
#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

constexpr int kDivThreads = 512;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <bool WEIGHTED>
__global__ __launch_bounds__(kDivThreads) void divergence_partial_kernel(
    double* __restrict__ partial, const float* __restrict__ x, int64_t ld,
    const float* __restrict__ dsz, int32_t N, int64_t P, int W, uint32_t nstrips, int vec) {
    extern __shared__ double lds64[];
    const int w_shift = 31 - __clz(W);
    const int groups = W >> 6;                       // wavefronts per row of the strip
    const int total = N * W;
    float* slab = reinterpret_cast<float*>(lds64);   // [N][W], 16-byte aligned for 128-bit stores
    double* mean = lds64 + (total >> 1);             // [W]   (N*W*4 bytes is a multiple of 256)
    double* part = mean + W;                         // [N][groups]
    float* lds_d = reinterpret_cast<float*>(part + (size_t)N * groups);   // [N]
    const int t = (int)threadIdx.x;

    if (WEIGHTED)
        for (int i = t; i < N; i += kDivThreads) lds_d[i] = dsz[i];
    __syncthreads();
    double den = 0.0;
    if (WEIGHTED) { for (int w = 0; w < N; ++w) den += (double)lds_d[w]; }
    else den = (double)N;

    double acc = 0.0;                                // thread r < N: row r of this workgroup
    for (uint32_t strip = blockIdx.x; strip < nstrips; strip += gridDim.x) {
        const int64_t col0 = (int64_t)strip * W;
        const int width = (int)(col0 + W <= P ? W : P - col0);
        if (vec && width == W) {
            const int W4 = W >> 2;
            for (int idx = t; idx < N * W4; idx += kDivThreads) {
                const int row = idx >> (w_shift - 2);
                const int c4 = idx & (W4 - 1);
                const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(
                    x + (size_t)row * (size_t)ld + (size_t)col0 + (size_t)c4 * 4));
                reinterpret_cast<v4f*>(slab)[idx] = v;
            }
        } else {
            for (int idx = t; idx < total; idx += kDivThreads) {
                const int row = idx >> w_shift;
                const int c = idx & (W - 1);
                slab[idx] = c < width ? x[(size_t)row * (size_t)ld + (size_t)col0 + (size_t)c] : 0.0f;
            }
        }
        __syncthreads();
        if (t < W) {
            double num = 0.0;
            for (int w = 0; w < N; ++w)
                num += (WEIGHTED ? (double)lds_d[w] : 1.0) * (double)slab[w * W + t];
            mean[t] = num / den;
        }
        __syncthreads();
        for (int idx = t; idx < total; idx += kDivThreads) {
            const int row = idx >> w_shift;
            const int c = idx & (W - 1);
            const double diff = (double)slab[idx] - mean[c];
            const double s = wave_sum(diff * diff);
            if ((t & 63) == 0) part[row * groups + (c >> 6)] = s;
        }
        __syncthreads();
        if (t < N)
            for (int k = 0; k < groups; ++k) acc += part[t * groups + k];
    }
    if (t < N) partial[(size_t)blockIdx.x * (size_t)N + (size_t)t] = acc;
}

__global__ __launch_bounds__(256) void divergence_reduce_kernel(double* __restrict__ dist2,
                                                                const double* __restrict__ partial,
                                                                int32_t N, uint32_t nblocks) {
    const int r = (int)(blockIdx.x * 256 + threadIdx.x);
    if (r >= N) return;
    double s = 0.0;
    for (uint32_t b = 0; b < nblocks; ++b) s += partial[(size_t)b * (size_t)N + (size_t)r];
    dist2[r] = s;
}

size_t divergence_lds_bytes(int32_t N, int W) {
    return (size_t)W * 8 + (size_t)N * (size_t)(W / 64) * 8 + (size_t)N * (size_t)W * 4 + (size_t)N * 4;
}

}  // namespace

// strip width for the divergence pass, 0 if N rows of 64 columns do not fit in LDS
int divergence_strip_cols(int32_t N) {
    if (N > kDivThreads) return 0;                   // one accumulator thread per worker
    for (int W = 512; W >= 64; W >>= 1)
        if ((size_t)N * (size_t)W * 4 <= 16 * 1024 && divergence_lds_bytes(N, W) <= 64 * 1024) return W;
    return divergence_lds_bytes(N, 64) <= 64 * 1024 ? 64 : 0;
}

uint32_t divergence_grid(int64_t P, int W) {
    const uint64_t strips = ((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W;
    return (uint32_t)(strips < 2048 ? strips : 2048);
}

hipError_t launch_divergence(double* dist2, double* workspace, const float* x, int64_t ld,
                             const float* dsz, int32_t N, int64_t P, int W, bool vec,
                             hipStream_t st) {
    const uint64_t strips = ((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W;
    if (strips > 0xFFFFFFFFull) return hipErrorInvalidValue;
    const uint32_t grid = divergence_grid(P, W);
    const size_t lds = divergence_lds_bytes(N, W);
    if (dsz != nullptr)
        hipLaunchKernelGGL(divergence_partial_kernel<true>, dim3(grid), dim3(kDivThreads), lds, st,
                           workspace, x, ld, dsz, N, P, W, (uint32_t)strips, vec ? 1 : 0);
    else
        hipLaunchKernelGGL(divergence_partial_kernel<false>, dim3(grid), dim3(kDivThreads), lds, st,
                           workspace, x, ld, dsz, N, P, W, (uint32_t)strips, vec ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(divergence_reduce_kernel, dim3((uint32_t)((N + 255) / 256)), dim3(256), 0, st,
                       dist2, workspace, N, grid);
    return hipGetLastError();
}

}  // namespace combo
