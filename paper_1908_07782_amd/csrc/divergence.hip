// Aggregation-divergence monitor (Sec. 4.3, Definition 2 of the segmented-gossip paper):
// squared L2 distance of every worker's parameter vector from the aggregate of all
// workers (the dataset-size weighted mean; the plain mean for equal sizes).
//
// Read-only streaming pass, HBM bound (4 bytes per element).  A persistent workgroup
// walks over column strips of W columns.  Every thread owns the same (row, 4-column group)
// slots in every strip: slot k of thread t is row k*(threads/W4) + t/W4, columns
// 4*(t mod W4)..+3 (W4 = W/4).  Per strip it loads its 128-bit words into registers, adds
// its own rows' (weighted) values in binary64, adds the lanes of its wavefront that hold
// the same column group with a fixed xor-shuffle tree, and the wavefronts exchange their
// four column sums through a small LDS buffer; after ONE barrier every thread adds the
// wavefronts' sums in wavefront order, divides, and squares the differences of its
// register values against the means into one binary64 accumulator per slot.  The LDS
// exchange buffer is double-buffered, so one barrier per strip suffices and no parameter
// data is ever staged in LDS.  A slot always
// belongs to the same worker row, so nothing is reduced per strip: at the end of the
// kernel the slots of a row are added in slot order and the workgroup's N partial sums
// go to a caller-supplied workspace; a second tiny kernel adds the partials of each row
// with a fixed tree.  No floating-point atomics: the result is reproducible bit for bit.
//
// Layouts: row-major [N][ld] and tiled [T][N][Wt] (a strip then spans W/Wt whole tiles).
//
// Tiled arenas whose tiles are small enough for the register slots of ONE wavefront
// (N * Wt/4 <= 512 words, Wt <= 256: every tile of at most 8 KiB) take a second kernel:
// a wavefront owns whole tiles, its 64 lanes cover 64/(Wt/4) adjacent rows of the tile per
// slot, so every load instruction reads one contiguous kilobyte, the column sums are
// complete after the xor-shuffle tree, and the strip loop needs neither LDS nor barriers.
#include <mutex>

#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

// Partial sums for callers that cannot bring a workspace (see divergence_static_workspace):
// one [rows][4096 workgroups] block of binary64 partials, 4 MiB, held by every GPU the
// library runs on until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and host calls use the address obtained from it.
static __device__ __align__(256) double scratch[(size_t)kDivPartialsPerRow * kDivStaticRows];

constexpr int kDivThreadsMax = 512;
constexpr int kDivFold = 2;    // worker rows folded per thread at the end: N <= 2 * threads
constexpr int kDivSlots = 8;   // 128-bit words per thread and strip; filling all eight
                               // (measured: 2 words 2.8, 4 words 4.7, 8 words 6.0 TB/s) keeps
                               // enough loads in flight for the persistent workgroups

struct DivArgs {
    double* partial;
    const float* x;
    const float* dsz;
    int64_t ld;
    int64_t P;
    int32_t N;
    int32_t W;            // strip width (power of two, 16..512)
    uint32_t nstrips;
    int32_t vec;          // 16-byte aligned with ld % 4 == 0: 128-bit loads allowed
    int32_t tile_shift;   // 0: row-major [N][ld]; else log2(Wt) of a tiled arena [T][N][Wt], W % Wt == 0
};

template <bool WEIGHTED, int kDivThreads>
__global__ __launch_bounds__(kDivThreads) void divergence_partial_kernel(const DivArgs a) {
    extern __shared__ double lds64[];
    const int N = a.N, W = a.W;
    const int W4 = W >> 2;
    const int w4_shift = 31 - __clz(W4);
    const int total4 = N * W4;
    const int groups = kDivThreads >> w4_shift;       // threads sharing one column group
    double* share = lds64;                            // [2][kDivThreads][4]
    double* fold = share + 2 * kDivThreads * 4;       // [kDivThreads] end-of-kernel fold
    float* lds_d = reinterpret_cast<float*>(fold + kDivThreads);   // [N]
    const int t = (int)threadIdx.x;
    const int my_c4 = t & (W4 - 1);
    const int my_row0 = t >> w4_shift;

    if (WEIGHTED)
        for (int i = t; i < N; i += kDivThreads) lds_d[i] = a.dsz[i];
    __syncthreads();
    double den = 0.0;
    if (WEIGHTED) { for (int w = 0; w < N; ++w) den += (double)lds_d[w]; }
    else den = (double)N;
    const double inv_den = 1.0 / den;                 // one division per thread, not four per strip

    double wt[kDivSlots];                             // dataset size of each slot's row
    // Where slot k's 128-bit word lives relative to the strip's base: the part of the address
    // that does not change from strip to strip (row-major: row*ld + c; tiled: a strip spans
    // W/Wt whole tiles, the word is in tile c/Wt of them).  Per strip only the base is added.
    size_t slot_off[kDivSlots];
#pragma unroll
    for (int k = 0; k < kDivSlots; ++k) {
        const int row = k * groups + my_row0;
        wt[k] = (WEIGHTED && row < N) ? (double)lds_d[row] : 1.0;
        const size_t c = (size_t)my_c4 * 4;
        if (a.tile_shift == 0)
            slot_off[k] = (size_t)row * (size_t)a.ld + c;
        else
            slot_off[k] = (((c >> a.tile_shift) * (size_t)N + (size_t)row) << a.tile_shift) +
                          (c & (((size_t)1 << a.tile_shift) - 1));
    }
    double acc[kDivSlots];
#pragma unroll
    for (int k = 0; k < kDivSlots; ++k) acc[k] = 0.0;
    const size_t strip_elems = a.tile_shift == 0 ? (size_t)W : (size_t)N * (size_t)W;

    int buf = 0;
    for (uint32_t strip = blockIdx.x; strip < a.nstrips; strip += gridDim.x) {
        const int64_t col0 = (int64_t)strip * W;
        const int width = (int)(col0 + W <= a.P ? W : a.P - col0);
        const bool fast = a.vec && width == W;
        const float* base = a.x + (size_t)strip * strip_elems;
        v4f v[kDivSlots];
#pragma unroll
        for (int k = 0; k < kDivSlots; ++k) {
            const int row = k * groups + my_row0;
            if (k * kDivThreads < total4 && row < N) {
                const int c = my_c4 * 4;
                const float* p = base + slot_off[k];
                if (fast) {
                    v[k] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
                } else {                              // ragged end or unaligned: zero beyond the row
                    v[k].x = c + 0 < width ? p[0] : 0.0f;
                    v[k].y = c + 1 < width ? p[1] : 0.0f;
                    v[k].z = c + 2 < width ? p[2] : 0.0f;
                    v[k].w = c + 3 < width ? p[3] : 0.0f;
                }
            }
        }
        // this thread's share of the four column sums
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
        for (int k = 0; k < kDivSlots; ++k) {
            const int row = k * groups + my_row0;
            if (k * kDivThreads < total4 && row < N) {
                s0 += wt[k] * (double)v[k].x;
                s1 += wt[k] * (double)v[k].y;
                s2 += wt[k] * (double)v[k].z;
                s3 += wt[k] * (double)v[k].w;
            }
        }
        // lanes of one wavefront that share a column group: fixed xor tree
        for (int off = W4; off < 64; off <<= 1) {
            s0 += __shfl_xor(s0, off, 64);
            s1 += __shfl_xor(s1, off, 64);
            s2 += __shfl_xor(s2, off, 64);
            s3 += __shfl_xor(s3, off, 64);
        }
        // wavefronts exchange their sums through LDS: share[buf][wave][lane][4]
        double* sh = share + (size_t)buf * kDivThreads * 4;
        const int lane = t & 63, wave = t >> 6;
        if (lane < W4) {
            double* q = sh + (size_t)(wave * 64 + lane) * 4;
            q[0] = s0;
            q[1] = s1;
            q[2] = s2;
            q[3] = s3;
        }
        __syncthreads();
        double m0 = 0.0, m1 = 0.0, m2 = 0.0, m3 = 0.0;
        {
            const int my_hi = my_c4 & ~63;            // which 64-group block of columns (W4 > 64)
#pragma unroll
            for (int wv = 0; wv < kDivThreads / 64; ++wv) {
                if (((wv << 6) & (W4 - 1)) == my_hi) {
                    const double* q = sh + (size_t)(wv * 64 + (my_c4 & 63)) * 4;
                    m0 += q[0];
                    m1 += q[1];
                    m2 += q[2];
                    m3 += q[3];
                }
            }
            m0 *= inv_den;
            m1 *= inv_den;
            m2 *= inv_den;
            m3 *= inv_den;
        }
#pragma unroll
        for (int k = 0; k < kDivSlots; ++k) {
            const int row = k * groups + my_row0;
            if (k * kDivThreads < total4 && row < N) {
                const int c = my_c4 * 4;
                // columns beyond the ragged end hold zeros and a zero mean: no contribution
                const double d0 = (double)v[k].x - m0;
                const double d1 = (double)v[k].y - m1;
                const double d2 = (double)v[k].z - m2;
                const double d3 = (double)v[k].w - m3;
                (void)c;
                acc[k] += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
            }
        }
        buf ^= 1;     // the other exchange buffer is free: its readers have passed this strip's barrier
    }

    // fold: slot k of thread t belongs to row k*groups + t/W4; add a row's threads in
    // thread order, slot by slot.  Thread t folds rows t and t + kDivThreads.
    double row_sum[kDivFold];
#pragma unroll
    for (int m = 0; m < kDivFold; ++m) row_sum[m] = 0.0;
#pragma unroll
    for (int k = 0; k < kDivSlots; ++k) {
        if (k * kDivThreads < total4) {               // uniform
            __syncthreads();
            fold[t] = acc[k];
            __syncthreads();
            // row r is served in this pass by threads [ (r - k*groups)*W4, +W4 ) if in range
#pragma unroll
            for (int m = 0; m < kDivFold; ++m) {
                const int r = t + m * kDivThreads;
                const int g = r - k * groups;
                if (r < N && g >= 0 && g < groups)
                    for (int i = 0; i < W4; ++i) row_sum[m] += fold[g * W4 + i];
            }
        }
    }
#pragma unroll
    for (int m = 0; m < kDivFold; ++m) {
        const int r = t + m * kDivThreads;
        if (r < N) a.partial[(size_t)r * (size_t)gridDim.x + (size_t)blockIdx.x] = row_sum[m];   // [N][grid]
    }
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

// ---- one wavefront per tile ------------------------------------------------------------

struct TileDivArgs {
    double* partial;
    const float* x;       // tiled arena [T][N][Wt], 16-byte aligned
    const float* dsz;
    int64_t P;
    int32_t N;
    int32_t Wt;           // tile width: 64, 128 or 256
    uint64_t ntiles;
    uint32_t run;         // the XCDs take turns at runs of `run` consecutive workgroup positions (0: none)
};

// U tiles per pass of a wavefront, kDivSlots / U register slots for the rows of each.
template <bool WEIGHTED, int U>
__global__ __launch_bounds__(256) void divergence_tile_kernel(const TileDivArgs a) {
    extern __shared__ double lds64[];
    constexpr int SPS = kDivSlots / U;
    const int N = a.N;
    const int W4 = a.Wt >> 2;
    const int w4_shift = 31 - __clz(W4);
    const int rpp = 64 >> w4_shift;                   // rows covered by one slot of the wavefront
    double* fold = lds64;                             // [256]
    float* lds_d = reinterpret_cast<float*>(fold + 256);   // [N]
    const int t = (int)threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int my_c4 = lane & (W4 - 1);
    const int my_row0 = lane >> w4_shift;

    if (WEIGHTED)
        for (int i = t; i < N; i += 256) lds_d[i] = a.dsz[i];
    __syncthreads();
    double den = 0.0;
    if (WEIGHTED) { for (int w = 0; w < N; ++w) den += (double)lds_d[w]; }
    else den = (double)N;
    const double inv_den = 1.0 / den;

    // slot kk (of every tile of a pass) holds row kk*rpp + my_row0
    double wt[SPS], acc[SPS];
#pragma unroll
    for (int kk = 0; kk < SPS; ++kk) {
        const int row = kk * rpp + my_row0;
        wt[kk] = (WEIGHTED && row < N) ? (double)lds_d[row] : 1.0;
        acc[kk] = 0.0;
    }

    const uint64_t nwaves = (uint64_t)gridDim.x * 4u;
    for (uint64_t first = ((uint64_t)xcd_run_block(blockIdx.x, a.run) * 4u + (uint64_t)wave) * U; first < a.ntiles;
         first += nwaves * U) {
        v4f v[kDivSlots];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t tile = first + (uint64_t)u;
            const int64_t left = tile < a.ntiles ? a.P - (int64_t)tile * a.Wt : 0;
            const int width = (int)(left >= a.Wt ? a.Wt : left);   // 0: no such tile
            const float* base = a.x + (size_t)tile * (size_t)N * (size_t)a.Wt + (size_t)(my_c4 * 4);
#pragma unroll
            for (int kk = 0; kk < SPS; ++kk) {
                const int k = u * SPS + kk;
                const int row = kk * rpp + my_row0;
                v[k] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
                if (row < N && width > 0) {
                    const float* p = base + (size_t)row * (size_t)a.Wt;
                    if (width == a.Wt) {
                        v[k] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
                    } else {                          // last tile: zero beyond column P
                        const int c = my_c4 * 4;
                        v[k].x = c + 0 < width ? p[0] : 0.0f;
                        v[k].y = c + 1 < width ? p[1] : 0.0f;
                        v[k].z = c + 2 < width ? p[2] : 0.0f;
                        v[k].w = c + 3 < width ? p[3] : 0.0f;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
            for (int kk = 0; kk < SPS; ++kk) {
                const int k = u * SPS + kk;
                if (kk * rpp + my_row0 < N) {
                    s0 += wt[kk] * (double)v[k].x;
                    s1 += wt[kk] * (double)v[k].y;
                    s2 += wt[kk] * (double)v[k].z;
                    s3 += wt[kk] * (double)v[k].w;
                }
            }
            // lanes that hold the same column group of other rows: fixed xor tree; afterwards
            // every lane has the complete column sums of its tile
            for (int off = W4; off < 64; off <<= 1) {
                s0 += __shfl_xor(s0, off, 64);
                s1 += __shfl_xor(s1, off, 64);
                s2 += __shfl_xor(s2, off, 64);
                s3 += __shfl_xor(s3, off, 64);
            }
            const double m0 = s0 * inv_den, m1 = s1 * inv_den, m2 = s2 * inv_den, m3 = s3 * inv_den;
#pragma unroll
            for (int kk = 0; kk < SPS; ++kk) {
                const int k = u * SPS + kk;
                if (kk * rpp + my_row0 < N) {
                    // columns beyond P hold zeros and a zero mean: no contribution
                    const double d0 = (double)v[k].x - m0;
                    const double d1 = (double)v[k].y - m1;
                    const double d2 = (double)v[k].z - m2;
                    const double d3 = (double)v[k].w - m3;
                    acc[kk] += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
                }
            }
        }
    }

    // fold: row r lives in slot r / rpp, lanes (r % rpp)*W4 .. +W4 of every wavefront; add
    // them in wavefront order, lane order
    double row_sum = 0.0;
#pragma unroll
    for (int kk = 0; kk < SPS; ++kk) {
        if (kk * rpp < N) {                           // uniform
            __syncthreads();
            fold[t] = acc[kk];
            __syncthreads();
            const int g = t - kk * rpp;               // candidate: thread t folds row t
            if (t < N && g >= 0 && g < rpp)
                for (int wv = 0; wv < 4; ++wv)
                    for (int i = 0; i < W4; ++i) row_sum += fold[wv * 64 + g * W4 + i];
        }
    }
    if (t < N) a.partial[(size_t)t * (size_t)gridDim.x + (size_t)blockIdx.x] = row_sum;   // [N][grid]
}

using TileDivKernel = void (*)(const TileDivArgs);

TileDivKernel tile_kernel_for(bool weighted, int U) {
    switch (U) {
        case 8: return weighted ? divergence_tile_kernel<true, 8> : divergence_tile_kernel<false, 8>;
        case 4: return weighted ? divergence_tile_kernel<true, 4> : divergence_tile_kernel<false, 4>;
        case 2: return weighted ? divergence_tile_kernel<true, 2> : divergence_tile_kernel<false, 2>;
        default: return weighted ? divergence_tile_kernel<true, 1> : divergence_tile_kernel<false, 1>;
    }
}

// tiles per wavefront pass: as many as the register slots hold
int tiles_per_pass(int32_t N, int tile_cols) {
    const int rpp = 64 / (tile_cols / 4);
    const int slots = (N + rpp - 1) / rpp;            // 1..8 by divergence_tile_fits
    int pow2 = 1;
    while (pow2 < slots) pow2 <<= 1;
    return kDivSlots / pow2;
}

size_t divergence_lds_bytes(int32_t N, int W, int threads) {
    // two exchange buffers, fold buffer, dataset sizes
    (void)W;
    return (size_t)2 * threads * 4 * 8 + (size_t)threads * 8 + (size_t)N * 4;
}

}  // namespace

// 256 threads while N rows of the strip fit in their register slots, else 512
int divergence_threads(int32_t N, int W) {
    return (int64_t)N * (W / 4) <= 256 * kDivSlots ? 256 : 512;
}

// strip width: the widest one whose N rows fill at most eight 128-bit words per thread of
// a 256-thread workgroup; for many workers narrower strips (down to 16 columns) with 512
// threads (0: more than 1024 workers)
int divergence_strip_cols(int32_t N) {
    if (N > kDivFold * kDivThreadsMax) return 0;     // fold capacity of the largest workgroup
    for (int W = 512; W >= 64; W >>= 1)
        if ((int64_t)N * (W / 4) <= kDivSlots * 256) return W;
    for (int W = 64; W >= 16; W >>= 1)
        if ((int64_t)N * (W / 4) <= (int64_t)kDivThreadsMax * kDivSlots) return W;
    return 0;
}

// can a strip of W columns (e.g. the tile width of a tiled arena) be handled at all
bool divergence_width_ok(int32_t N, int W) {
    return N <= kDivFold * divergence_threads(N, W) && W >= 16 && W <= 512 && (W & (W - 1)) == 0 &&
           (int64_t)N * (W / 4) <= (int64_t)divergence_threads(N, W) * kDivSlots;
}

hipError_t launch_divergence(double* dist2, double* workspace, const float* x, int64_t ld,
                             const float* dsz, int32_t N, int64_t P, int W, bool vec, int arena_tile,
                             hipStream_t st) {
    const uint64_t strips = ((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W;
    if (strips > 0xFFFFFFFFull) return hipErrorInvalidValue;
    const int threads = divergence_threads(N, W);
    const size_t lds = divergence_lds_bytes(N, W, threads);
    // persistent grid: workgroups that are resident at once (no tail round), but no more than
    // three per compute unit for 256-thread workgroups: each keeps 32 KiB of loads in flight, and
    // beyond about 96 KiB per compute unit the memory system delivers less, not more (MI355X,
    // row-major arenas: c2 6.37 against 6.15 TB/s with all five resident, c3 6.74 / 6.33,
    // c5 6.71 / 6.44, c4 5.5 / 5.1; two per compute unit are slower again)
    static int resident[2][2] = {{0, 0}, {0, 0}};   // [weighted][512 threads]
    int& res = resident[dsz != nullptr][threads == 512];
    if (res == 0) {
        int per_cu = 0, dev = 0, cus = 0;
        hipError_t qe;
        if (dsz != nullptr)
            qe = threads == 256
                     ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, divergence_partial_kernel<true, 256>, 256, lds)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, divergence_partial_kernel<true, 512>, 512, lds);
        else
            qe = threads == 256
                     ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, divergence_partial_kernel<false, 256>, 256, lds)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, divergence_partial_kernel<false, 512>, 512, lds);
        if (qe != hipSuccess || hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return hipErrorUnknown;
        if (threads == 256 && per_cu > 3) per_cu = 3;
        res = per_cu * cus;
        if (res < 1) res = 256;
        if (res > kDivPartialsPerRow) res = kDivPartialsPerRow;   // the workspace's partials per row
    }
    const uint32_t grid = (uint32_t)(strips < (uint64_t)res ? strips : (uint64_t)res);
    DivArgs a;
    a.partial = workspace;
    a.x = x;
    a.dsz = dsz;
    a.ld = ld;
    a.P = P;
    a.N = N;
    a.W = W;
    a.nstrips = (uint32_t)strips;
    a.vec = vec ? 1 : 0;
    a.tile_shift = 0;
    while (arena_tile && (1 << a.tile_shift) < arena_tile) ++a.tile_shift;
#define COMBO_DIV_LAUNCH(WT, TH) \
    hipLaunchKernelGGL((divergence_partial_kernel<WT, TH>), dim3(grid), dim3(TH), lds, st, a)
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

// Device address of the library-held workspace on the current device.  Every GPU has its
// own copy of the array at its own address, so the lookup is done once per device, with
// that device current, and remembered.
hipError_t divergence_static_workspace(double** workspace, int64_t* bytes) {
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static double* known[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(guard);
    if (known[dev] == nullptr) {
        double* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        known[dev] = p;
    }
    *workspace = known[dev];
    *bytes = (int64_t)sizeof(double) * kDivPartialsPerRow * kDivStaticRows;
    return hipSuccess;
}

bool divergence_tile_fits(int32_t N, int tile_cols) {
    return (tile_cols == 64 || tile_cols == 128 || tile_cols == 256) &&
           (int64_t)N * (tile_cols / 4) <= 64 * kDivSlots;
}

hipError_t launch_divergence_tiles(double* dist2, double* workspace, const float* x,
                                   const float* dsz, int32_t N, int64_t P, int tile_cols,
                                   hipStream_t st) {
    if (!divergence_tile_fits(N, tile_cols)) return hipErrorInvalidValue;
    const int U = tiles_per_pass(N, tile_cols);
    const TileDivKernel kernel = tile_kernel_for(dsz != nullptr, U);
    const size_t lds = (size_t)256 * 8 + (size_t)N * 4;
    // persistent grid: two workgroups per compute unit (eight wavefronts with 8 KiB of loads in
    // flight each; with all four that fit, the memory system delivers 3-4 % less: c5 6.79 against
    // 7.09 TB/s, c3 6.64 / 6.95, c2 6.45 / 6.70), the XCDs taking turns at runs of four
    // workgroup positions (128 KiB of consecutive tiles per pass; worth 1 % of that)
    static int resident[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};   // [weighted][log2 U]
    int& res = resident[dsz != nullptr][U == 8 ? 3 : U == 4 ? 2 : U == 2 ? 1 : 0];
    if (res == 0) {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, lds) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return hipErrorUnknown;
        if (per_cu > 2) per_cu = 2;
        res = per_cu * cus;
        if (res < 1) res = 256;
        if (res > kDivPartialsPerRow) res = kDivPartialsPerRow;   // the workspace's partials per row
    }
    TileDivArgs a;
    a.partial = workspace;
    a.x = x;
    a.dsz = dsz;
    a.P = P;
    a.N = N;
    a.Wt = tile_cols;
    a.ntiles = ((uint64_t)P + (uint64_t)tile_cols - 1) / (uint64_t)tile_cols;
    const uint64_t passes = (a.ntiles + (uint64_t)(4 * U) - 1) / (uint64_t)(4 * U);   // per workgroup of 4 wavefronts
    const uint32_t grid = (uint32_t)(passes < (uint64_t)res ? passes : (uint64_t)res);
    // the run order permutes the positions [0, grid) only if grid is a whole number of rounds of 8 runs
    a.run = grid % (kXcds * 4u) == 0 ? 4u : 0u;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(divergence_reduce_kernel, dim3((uint32_t)N), dim3(256), 0, st, dist2, workspace,
                       grid);
    return hipGetLastError();
}

}  // namespace combo
