// Aggregation-divergence monitor (Sec. 4.3, Definition 2 of the segmented-gossip paper):
// squared L2 distance of every worker's parameter vector from the aggregate of all
// workers (the dataset-size weighted mean; the plain mean for equal sizes).
//
// Read-only streaming pass, HBM bound (4 bytes per element).  A persistent workgroup
// walks over column strips.  For each strip every thread loads its 128-bit words of the
// N x W slab (the same (row, column-in-strip) slots for every strip), keeps them in
// registers and also parks them in LDS; the W column means are then formed in binary64
// from LDS (each of the 512/W thread groups sums a share of the workers, the shares are
// added in group order); finally every thread squares the differences of its own
// register values against the means and adds them to a private binary64 accumulator per
// slot.  A slot always belongs to the same worker row, so nothing is reduced per strip:
// only at the end of the kernel are the slots of a row added (in slot order) and the
// workgroup's N partial sums written to a caller-supplied workspace.  A second tiny
// kernel adds the partials of each row with a fixed tree.  No floating-point atomics, so the
// result is reproducible bit for bit.
#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

// Workgroup size: 256 threads (8 KiB slabs, eight workgroups per compute unit) measured
// 20-25 % faster than 512; 512 is kept for many workers, whose slab needs the extra
// register slots.
constexpr int kDivThreadsMax = 512;

constexpr int kDivSlots = 8;   // 128-bit words per thread: slabs up to 64 KiB

template <bool WEIGHTED, int kDivThreads>
__global__ __launch_bounds__(kDivThreads) void divergence_partial_kernel(
    double* __restrict__ partial, const float* __restrict__ x, int64_t ld,
    const float* __restrict__ dsz, int32_t N, int64_t P, int W, uint32_t nstrips, int vec) {
    extern __shared__ double lds64[];
    const int W4 = W >> 2;
    const int w4_shift = 31 - __clz(W4);
    const int total4 = N * W4;
    v4f* slab = reinterpret_cast<v4f*>(lds64);        // [N][W4]
    double* mean = lds64 + 2 * total4;                // [W]
    double* share = mean + W;                         // [kDivThreads]: partial column sums / fold
    float* lds_d = reinterpret_cast<float*>(share + kDivThreads);   // [N]
    const int t = (int)threadIdx.x;

    if (WEIGHTED)
        for (int i = t; i < N; i += kDivThreads) lds_d[i] = dsz[i];
    __syncthreads();
    double den = 0.0;
    if (WEIGHTED) { for (int w = 0; w < N; ++w) den += (double)lds_d[w]; }
    else den = (double)N;

    const int groups = kDivThreads / W;              // thread groups sharing the column sums
    const int my_group = t / W, my_col = t - my_group * W;
    const float* slab_f = reinterpret_cast<const float*>(slab);

    double acc[kDivSlots];
#pragma unroll
    for (int k = 0; k < kDivSlots; ++k) acc[k] = 0.0;

    // loads of one strip into registers (zero beyond the ragged end of the row)
    auto load_strip = [&](uint32_t strip, v4f (&dst)[kDivSlots]) {
        const int64_t col0 = (int64_t)strip * W;
        const int width = (int)(col0 + W <= P ? W : P - col0);
        const bool fast = vec && width == W;
#pragma unroll
        for (int k = 0; k < kDivSlots; ++k) {
            const int idx = k * kDivThreads + t;
            if (idx < total4) {
                const int row = idx >> w4_shift;
                const int c = (idx & (W4 - 1)) * 4;
                const float* p = x + (size_t)row * (size_t)ld + (size_t)col0 + (size_t)c;
                if (fast) {
                    dst[k] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
                } else {
                    dst[k].x = c + 0 < width ? p[0] : 0.0f;
                    dst[k].y = c + 1 < width ? p[1] : 0.0f;
                    dst[k].z = c + 2 < width ? p[2] : 0.0f;
                    dst[k].w = c + 3 < width ? p[3] : 0.0f;
                }
            }
        }
    };

    // (Prefetching the next strip into a second register set while this one is reduced was
    // measured slower than letting the four resident workgroups of a compute unit overlap.)
    for (uint32_t strip = blockIdx.x; strip < nstrips; strip += gridDim.x) {
        v4f v[kDivSlots];
        load_strip(strip, v);
#pragma unroll
        for (int k = 0; k < kDivSlots; ++k) {
            const int idx = k * kDivThreads + t;
            if (idx < total4) slab[idx] = v[k];
        }
        __syncthreads();
        {   // share of the column sum: workers my_group, my_group + groups, ...
            double num = 0.0;
            for (int w = my_group; w < N; w += groups)
                num += (WEIGHTED ? (double)lds_d[w] : 1.0) * (double)slab_f[w * W + my_col];
            share[t] = num;
        }
        __syncthreads();
        if (t < W) {
            double num = 0.0;
            for (int gidx = 0; gidx < groups; ++gidx) num += share[gidx * W + t];
            mean[t] = num / den;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kDivSlots; ++k) {
            const int idx = k * kDivThreads + t;
            if (idx < total4) {
                const int c = (idx & (W4 - 1)) * 4;
                const double d0 = (double)v[k].x - mean[c + 0];
                const double d1 = (double)v[k].y - mean[c + 1];
                const double d2 = (double)v[k].z - mean[c + 2];
                const double d3 = (double)v[k].w - mean[c + 3];
                acc[k] += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
            }
        }
        // no barrier needed here: the next strip writes slab (last read two barriers ago)
        // and share (last read one barrier ago); mean is rewritten three barriers later
    }

    // fold: slot k of thread t belongs to row (k*512 + t) >> w4_shift; add a row's slots in
    // slot order, one pass per k
    double row_sum = 0.0;
#pragma unroll
    for (int k = 0; k < kDivSlots; ++k) {
        if (k * kDivThreads < total4) {               // uniform
            __syncthreads();
            share[t] = acc[k];
            __syncthreads();
            if (t < N) {
                const int lo = t * W4 - k * kDivThreads;          // first slot of row t in this pass
                const int first = lo < 0 ? 0 : lo;
                const int last = lo + W4 < kDivThreads ? lo + W4 : kDivThreads;
                for (int i = first; i < last; ++i) row_sum += share[i];
            }
        }
    }
    if (t < N) partial[(size_t)t * (size_t)gridDim.x + (size_t)blockIdx.x] = row_sum;   // [N][grid]
}

// dist2[r] = sum over workgroups of partial[r][b]: one workgroup per worker row, each
// thread adds every 256th partial (coalesced), then a fixed binary tree in LDS.
__global__ __launch_bounds__(256) void divergence_reduce_kernel(double* __restrict__ dist2,
                                                                const double* __restrict__ partial,
                                                                uint32_t nblocks) {
    __shared__ double tree[256];
    const uint32_t r = blockIdx.x;
    const double* row = partial + (size_t)r * (size_t)nblocks;
    double s = 0.0;
    for (uint32_t b = threadIdx.x; b < nblocks; b += 256) s += row[b];
    tree[threadIdx.x] = s;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) tree[threadIdx.x] += tree[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) dist2[r] = tree[0];
}

size_t divergence_lds_bytes(int32_t N, int W, int threads) {
    // slab, column means, share/fold buffer, dataset sizes
    return (size_t)N * (size_t)W * 4 + (size_t)W * 8 + (size_t)threads * 8 + (size_t)N * 4;
}

// 256 threads when N rows of a 64-column strip fit in their register slots (N <= 128)
int divergence_threads(int32_t N) { return (int64_t)N * 16 <= 256 * kDivSlots ? 256 : 512; }

}  // namespace

// strip width for the divergence pass, 0 if N rows of 64 columns do not fit in LDS
int divergence_strip_cols(int32_t N) {
    if (N > kDivThreadsMax) return 0;                // one fold thread per worker
    const int threads = divergence_threads(N);
    for (int W = 512; W >= 64; W >>= 1)
        if ((size_t)N * (size_t)W * 4 <= (size_t)threads * 32 && W <= threads &&
            divergence_lds_bytes(N, W, threads) <= 64 * 1024)
            return W;
    return ((int64_t)N * 16 <= (int64_t)threads * kDivSlots &&
            divergence_lds_bytes(N, 64, threads) <= 64 * 1024) ? 64 : 0;
}

uint32_t divergence_grid(int32_t N, int64_t P, int W) {
    const uint64_t strips = ((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W;
    const uint64_t cap = divergence_threads(N) == 256 ? 4096 : 2048;   // resident workgroups x 2
    return (uint32_t)(strips < cap ? strips : cap);
}

hipError_t launch_divergence(double* dist2, double* workspace, const float* x, int64_t ld,
                             const float* dsz, int32_t N, int64_t P, int W, bool vec,
                             hipStream_t st) {
    const uint64_t strips = ((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W;
    if (strips > 0xFFFFFFFFull) return hipErrorInvalidValue;
    const uint32_t grid = divergence_grid(N, P, W);
    const int threads = divergence_threads(N);
    const size_t lds = divergence_lds_bytes(N, W, threads);
#define COMBO_DIV_LAUNCH(WT, TH)                                                                  \
    hipLaunchKernelGGL((divergence_partial_kernel<WT, TH>), dim3(grid), dim3(TH), lds, st, workspace, \
                       x, ld, dsz, N, P, W, (uint32_t)strips, vec ? 1 : 0)
    if (dsz != nullptr) {
        if (threads == 256) COMBO_DIV_LAUNCH(true, 256);
        else COMBO_DIV_LAUNCH(true, 512);
    } else {
        if (threads == 256) COMBO_DIV_LAUNCH(false, 256);
        else COMBO_DIV_LAUNCH(false, 512);
    }
#undef COMBO_DIV_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(divergence_reduce_kernel, dim3((uint32_t)N), dim3(256), 0, st, dist2, workspace,
                       grid);
    return hipGetLastError();
}

}  // namespace combo
