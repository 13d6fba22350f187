// Gather-average round, LDS-slab form: Eq. (3) / Eq. (4) of the segmented-gossip paper
// with every front-buffer element fetched exactly once.
//
// One workgroup owns a strip of `W` consecutive columns of ALL N workers.  It first
// copies the N x W slab of the front buffer into LDS (each wave instruction moves whole
// 128-bit words of one row: fully coalesced), together with the strip's peer list
// peers[.][s][.] and, for weighted rounds, the dataset sizes.  After one barrier every
// output element is formed from LDS: own value, then the R providers in table order,
// then the scale - the same fixed order as the row-tile kernel - and streamed to the
// back buffer with non-temporal 128-bit stores.  HBM and L2 see one read and one write
// per element whatever R is; the R+1 reads per output are LDS reads.
//
// With the local update fused in, the slab is filled with the parameters after the tau
// SGD steps x <- x - lr*g_t (each gradient slice read once, product rounded before the
// difference, slices in order), so peers are served post-update values as Sec. 4.1
// requires, and the front buffer itself is left untouched.  (Callers pass tau >= 1.)
//
// A strip that contains a segment boundary or the ragged end of the row (at most S
// strips per round) falls back to per-element evaluation from global memory.
#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

constexpr int kBatch = 4;   // 128-bit loads kept in flight per thread while filling the slab

// Workgroup size of the slab kernel: 256 or 512 threads, chosen on the host so that a
// thread moves about two 128-bit words (measured on MI355X: 8 KiB slabs with 256 threads
// and 16 KiB slabs with 512 threads beat every other combination of 128..1024 threads
// and 4..64 KiB slabs).
constexpr int kSlabThreadsMax = 512;

// every front-buffer element is read once, so the slab fill uses streaming loads
__device__ __forceinline__ v4f load4_slab(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
}

// DYNAMIC: Sec. 4.2 semantics (offline rows copied, newcomers aggregated without their own
// value, unused table slots < 0 skipped, scale by the number of terms).
template <int RT, bool WEIGHTED, bool FUSED, bool DYNAMIC, int kSlabThreads>
__global__ __launch_bounds__(kSlabThreads) void gossip_slab_kernel(const RoundArgs a, const int W) {
    extern __shared__ v4f lds[];
    const int32_t R = RT >= 0 ? RT : a.R;
    const int32_t N = a.N;
    const int W4 = W >> 2;                       // 128-bit words per row of the strip
    const int w4_shift = 31 - __clz(W4);         // W4 is a power of two
    const int total4 = N * W4;

    v4f* slab = lds;                                                   // [N][W4]
    int32_t* lds_peers = reinterpret_cast<int32_t*>(lds + total4);     // [N][R]
    float* lds_d = reinterpret_cast<float*>(lds_peers + (size_t)N * (size_t)R);   // [N]
    int32_t* lds_status = reinterpret_cast<int32_t*>(lds_d + N);                  // [N]

    const int64_t col0 = (int64_t)blockIdx.x * W;
    const int64_t col_end = col0 + W < a.P ? col0 + W : a.P;
    // where the strip's row chunks live: row-major rows are ld apart and start at col0;
    // in the tiled layout (tile width == W) the whole slab is one contiguous block
    const size_t row_stride = a.tile_shift == 0 ? (size_t)a.ld : (size_t)W;
    const size_t strip_base = a.tile_shift == 0 ? (size_t)col0
                                                : (size_t)blockIdx.x * (size_t)N * (size_t)W;
    const int32_t s0 = segment_of(col0, a);
    const int64_t seg_end = (s0 == a.S - 1) ? a.P : (int64_t)(s0 + 1) * a.L;

    if (col_end - col0 == W && col_end <= seg_end) {
        // ---- fill: peer list, weights, then the slab --------------------------------
        for (int i = threadIdx.x; R > 0 && i < N * R; i += kSlabThreads) {
            const int w = i / (R > 0 ? R : 1);
            const int j = i - w * R;
            lds_peers[i] = a.peers[((size_t)w * (size_t)a.S + (size_t)s0) * (size_t)R + (size_t)j];
        }
        if (WEIGHTED)
            for (int i = threadIdx.x; i < N; i += kSlabThreads) lds_d[i] = a.dsz[i];
        if (DYNAMIC)
            for (int i = threadIdx.x; i < N; i += kSlabThreads) lds_status[i] = a.status[i];

        for (int base = 0; base < total4; base += kSlabThreads * kBatch) {
            v4f x[kBatch], g[kBatch];
            size_t off[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                if (idx < total4) {
                    const int row = idx >> w4_shift;
                    const int c4 = idx & (W4 - 1);
                    off[u] = (size_t)row * row_stride + strip_base + (size_t)c4 * 4;
                    x[u] = load4_slab(a.src + off[u]);
                    if (FUSED) g[u] = load4_slab(a.grad + off[u]);
                }
            }
            if (FUSED) {
                // local steps in slice order; the first slice's loads are already in flight
                for (int32_t t = 0; t < a.tau; ++t) {
                    if (t > 0) {
#pragma unroll
                        for (int u = 0; u < kBatch; ++u) {
                            const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                            if (idx < total4)
                                g[u] = load4_slab(a.grad + (size_t)t * (size_t)a.grad_slice + off[u]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                        if (idx < total4) x[u] = sgd_step4(x[u], a.lr, g[u]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                if (idx < total4) slab[idx] = x[u];
            }
        }
        __syncthreads();

        // ---- aggregate from LDS ---------------------------------------------------
        for (int idx = threadIdx.x; idx < total4; idx += kSlabThreads) {
            const int w = idx >> w4_shift;
            const int c4 = idx & (W4 - 1);
            const int32_t* pl = lds_peers + w * R;
            v4f acc = slab[idx];
            v4f y;
            if (DYNAMIC) {
                const v4f own = acc;
                const int st = lds_status[w];
                int cnt = 0;
                float den = 0.0f;
                if (st == 1) {
                    if (WEIGHTED) { den = lds_d[w]; acc = scale4(den, own); }
                    cnt = 1;
                }
                if (st != 0) {
                    for (int j = 0; j < R; ++j) {
                        const int p = pl[j];
                        if (p < 0) continue;
                        v4f v = slab[(p << w4_shift) + c4];
                        if (WEIGHTED) {
                            const float dp = lds_d[p];
                            v = scale4(dp, v);
                            den = cnt == 0 ? dp : __fadd_rn(den, dp);
                        }
                        acc = cnt == 0 ? v : add4(acc, v);
                        ++cnt;
                    }
                }
                if (cnt == 0) y = own;
                else y = WEIGHTED ? div4(acc, den) : scale4(__fdiv_rn(1.0f, (float)cnt), acc);
            } else if (!WEIGHTED) {
                if (RT >= 0) {
#pragma unroll
                    for (int j = 0; j < (RT >= 0 ? RT : 0); ++j)
                        acc = add4(acc, slab[(pl[j] << w4_shift) + c4]);
                } else {
                    for (int j = 0; j < R; ++j) acc = add4(acc, slab[(pl[j] << w4_shift) + c4]);
                }
                y = scale4(a.inv, acc);
            } else {
                float den = lds_d[w];
                acc = scale4(den, acc);
                for (int j = 0; j < R; ++j) {
                    const int p = pl[j];
                    const float dp = lds_d[p];
                    den = __fadd_rn(den, dp);
                    acc = add4(acc, scale4(dp, slab[(p << w4_shift) + c4]));
                }
                y = div4(acc, den);
            }
            store4_stream(a.dst + (size_t)w * row_stride + strip_base + (size_t)c4 * 4, y);
        }
    } else {
        // ---- boundary or ragged strip: element by element from global memory --------
        const int width = (int)(col_end - col0);
        const int total = N * width;
        for (int idx = threadIdx.x; idx < total; idx += kSlabThreads) {
            const int w = idx / width;
            const int64_t e = col0 + (idx - w * width);
            if (DYNAMIC) average_element_dynamic<WEIGHTED>(a, w, e);
            else average_element<WEIGHTED, FUSED>(a, w, e);
        }
    }
}

size_t slab_lds_bytes(int32_t N, int32_t R, int W) {
    // slab, peer list, dataset sizes, status
    return (size_t)N * (size_t)W * 4 + (size_t)N * (size_t)R * 4 + (size_t)N * 4 + (size_t)N * 4;
}

// 256 threads for slabs of up to 768 128-bit words (12 KiB), 512 beyond
int slab_threads(int32_t N, int W) { return (int64_t)N * (W / 4) <= 768 ? 256 : 512; }

template <int RT>
hipError_t launch_rt(const RoundArgs& a, int W, uint32_t grid, size_t lds, hipStream_t st) {
    const bool weighted = a.dsz != nullptr, fused = a.grad != nullptr;
    const bool small = slab_threads(a.N, W) == 256;
#define COMBO_SLAB_LAUNCH(WT, FU)                                                                  \
    do {                                                                                           \
        if (small)                                                                                 \
            hipLaunchKernelGGL((gossip_slab_kernel<RT, WT, FU, false, 256>), dim3(grid), dim3(256),    \
                               lds, st, a, W);                                                     \
        else                                                                                       \
            hipLaunchKernelGGL((gossip_slab_kernel<RT, WT, FU, false, 512>), dim3(grid), dim3(512),    \
                               lds, st, a, W);                                                     \
    } while (0)
    if (weighted) {
        if (fused) COMBO_SLAB_LAUNCH(true, true);
        else COMBO_SLAB_LAUNCH(true, false);
    } else {
        if (fused) COMBO_SLAB_LAUNCH(false, true);
        else COMBO_SLAB_LAUNCH(false, false);
    }
#undef COMBO_SLAB_LAUNCH
    return hipGetLastError();
}

}  // namespace

// Strip width: the widest power of two in [64, 1024] columns whose slab is at most
// 16 KiB (two 128-bit words per thread, four workgroups per compute unit); for many
// workers 64 columns as long as slab, peer list and weights fit in 64 KiB of LDS.
// `requested` != 0 forces a width if it fits.
int slab_strip_cols(int32_t N, int32_t R, int requested) {
    const size_t kLimit = 64 * 1024;
    if (requested) {
        const bool pow2 = (requested & (requested - 1)) == 0;
        if (pow2 && requested >= 64 && requested <= 1024 &&
            slab_lds_bytes(N, R, requested) <= kLimit)
            return requested;
    }
    for (int W = 1024; W >= 64; W >>= 1)
        if ((size_t)N * (size_t)W * 4 <= 16 * 1024 && slab_lds_bytes(N, R, W) <= kLimit) return W;
    return slab_lds_bytes(N, R, 64) <= kLimit ? 64 : 0;
}

hipError_t launch_round_slab(const RoundArgs& a, int W, hipStream_t st) {
    const uint64_t strips = ((uint64_t)a.P + (uint64_t)W - 1) / (uint64_t)W;
    if (strips > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const size_t lds = slab_lds_bytes(a.N, a.R, W);
    const uint32_t grid = (uint32_t)strips;
    if (a.status != nullptr) {
        // dynamic workers: run-time replica loop, no fused step
        const bool small = slab_threads(a.N, W) == 256;
        if (a.dsz != nullptr) {
            if (small)
                hipLaunchKernelGGL((gossip_slab_kernel<-1, true, false, true, 256>), dim3(grid),
                                   dim3(256), lds, st, a, W);
            else
                hipLaunchKernelGGL((gossip_slab_kernel<-1, true, false, true, 512>), dim3(grid),
                                   dim3(512), lds, st, a, W);
        } else {
            if (small)
                hipLaunchKernelGGL((gossip_slab_kernel<-1, false, false, true, 256>), dim3(grid),
                                   dim3(256), lds, st, a, W);
            else
                hipLaunchKernelGGL((gossip_slab_kernel<-1, false, false, true, 512>), dim3(grid),
                                   dim3(512), lds, st, a, W);
        }
        return hipGetLastError();
    }
    switch (a.R) {
        case 0: return launch_rt<0>(a, W, grid, lds, st);
        case 1: return launch_rt<1>(a, W, grid, lds, st);
        case 2: return launch_rt<2>(a, W, grid, lds, st);
        case 3: return launch_rt<3>(a, W, grid, lds, st);
        case 4: return launch_rt<4>(a, W, grid, lds, st);
        case 5: return launch_rt<5>(a, W, grid, lds, st);
        case 6: return launch_rt<6>(a, W, grid, lds, st);
        case 7: return launch_rt<7>(a, W, grid, lds, st);
        case 8: return launch_rt<8>(a, W, grid, lds, st);
        default: return launch_rt<-1>(a, W, grid, lds, st);
    }
}

}  // namespace combo
