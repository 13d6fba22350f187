// Gather-average kernels: Eq. (3) of the segmented-gossip paper applied to every
// segment of every worker, output concatenated in place in the back buffer (Eq. 4),
// all reads from the front buffer (the synchronous semantics of Sec. 4.1 / 5.1).
//
// Work decomposition.  The parameter matrix is [N][ld] float32.  A workgroup of 256
// threads owns one (column tile, worker): `tile_cols` consecutive, 16-byte aligned
// columns of one row.  Tiles are cut from the whole row, not from segment starts, so
// that a column has the same alignment in every row and 128-bit loads are legal for
// the worker's own row and all R provider rows alike.  A tile that lies inside one
// segment (all but at most S-1 per row) takes the fast path: the R provider ids are
// wave-uniform, every lane issues its R+1 128-bit loads back to back, adds them in
// the fixed order self, p_0, ..., p_{R-1}, scales and stores with a non-temporal
// 128-bit store.  A tile that contains a segment boundary, a ragged row end
// (P % 4 != 0) or unaligned buffers is handled element by element.
//
// Workgroup order.  Every element of the front buffer is wanted by about R+1 workers.
// Hardware hands consecutive workgroup ids to the 8 XCDs round-robin and each XCD has
// its own L2, so with the XCD-aware order the ids that land on one XCD enumerate
// (tile, worker) with the worker index fastest: the N workgroups that read the same
// column tile run back to back on the same L2, the tile is fetched from HBM once and
// the other R reads per element hit in L2.  HBM traffic then approaches the compulsory
// one read + one write per element instead of (R+1) reads + one write.
//
// This is a streaming gather, not a contraction: no MFMA.
#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

// RT >= 0: replica count known at compile time (loads fully unrolled); RT < 0: a.R.
// VPT: 128-bit vectors per thread; the tile is kThreads*VPT*4 columns.
// VEC: buffers are 16-byte aligned with ld % 4 == 0.
template <int RT, int VPT, bool WEIGHTED, bool VEC>
__global__ __launch_bounds__(kThreads) void gossip_round_kernel(const RoundArgs a) {
    constexpr int64_t kTile = (int64_t)kThreads * VPT * 4;
    const int32_t R = RT >= 0 ? RT : a.R;

    // ---- which (tile, worker) is this workgroup -------------------------------------
    const uint32_t b = blockIdx.x;
    uint32_t tile;
    int32_t w;
    if (a.swizzle) {
        const uint32_t xcd = b % (uint32_t)kXcds;     // the XCD this id is dispatched to
        const uint32_t k = b / (uint32_t)kXcds;       // k-th workgroup of that XCD
        const uint32_t t = k / (uint32_t)a.N;
        w = (int32_t)(k - t * (uint32_t)a.N);
        tile = t * (uint32_t)kXcds + xcd;
        if (tile >= a.tiles_per_row) return;
    } else {
        w = (int32_t)(b / a.tiles_per_row);
        tile = b - (uint32_t)w * a.tiles_per_row;
    }

    const int64_t col_begin = (int64_t)tile * kTile;
    const int64_t col_end = col_begin + kTile < a.P ? col_begin + kTile : a.P;
    const int32_t s0 = segment_of(col_begin, a);
    const int64_t seg_end = (s0 == a.S - 1) ? a.P : (int64_t)(s0 + 1) * a.L;
    const bool one_segment = col_end <= seg_end;

    if (VEC && one_segment) {
        // ---- fast path: wave-uniform providers, 128-bit traffic ---------------------
        const int32_t* pl = a.peers + ((size_t)w * (size_t)a.S + (size_t)s0) * (size_t)R;
        const float* own_row = a.src + (size_t)w * (size_t)a.ld;
        float* out_row = a.dst + (size_t)w * (size_t)a.ld;

        if constexpr (RT >= 0) {
            const float* rows[RT + 1];
            float wt[RT + 1];
            float den = 0.0f;
            rows[0] = own_row;
            if (WEIGHTED) { wt[0] = a.dsz[w]; den = wt[0]; }
#pragma unroll
            for (int j = 0; j < RT; ++j) {
                const int32_t p = pl[j];
                rows[j + 1] = a.src + (size_t)p * (size_t)a.ld;
                if (WEIGHTED) { wt[j + 1] = a.dsz[p]; den = __fadd_rn(den, wt[j + 1]); }
            }
            v4f x[VPT][RT + 1];
            bool full[VPT];
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                const int64_t col = col_begin + ((int64_t)v * kThreads + threadIdx.x) * 4;
                full[v] = col + 4 <= col_end;
                if (full[v]) {
#pragma unroll
                    for (int j = 0; j <= RT; ++j) x[v][j] = load4(rows[j] + col);
                }
            }
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                const int64_t col = col_begin + ((int64_t)v * kThreads + threadIdx.x) * 4;
                if (full[v]) {
                    v4f y;
                    if (!WEIGHTED) {
                        v4f acc = x[v][0];
#pragma unroll
                        for (int j = 1; j <= RT; ++j) {
                            acc.x = __fadd_rn(acc.x, x[v][j].x);
                            acc.y = __fadd_rn(acc.y, x[v][j].y);
                            acc.z = __fadd_rn(acc.z, x[v][j].z);
                            acc.w = __fadd_rn(acc.w, x[v][j].w);
                        }
                        y.x = __fmul_rn(acc.x, a.inv);
                        y.y = __fmul_rn(acc.y, a.inv);
                        y.z = __fmul_rn(acc.z, a.inv);
                        y.w = __fmul_rn(acc.w, a.inv);
                    } else {
                        v4f num;
                        num.x = __fmul_rn(wt[0], x[v][0].x);
                        num.y = __fmul_rn(wt[0], x[v][0].y);
                        num.z = __fmul_rn(wt[0], x[v][0].z);
                        num.w = __fmul_rn(wt[0], x[v][0].w);
#pragma unroll
                        for (int j = 1; j <= RT; ++j) {
                            num.x = __fadd_rn(num.x, __fmul_rn(wt[j], x[v][j].x));
                            num.y = __fadd_rn(num.y, __fmul_rn(wt[j], x[v][j].y));
                            num.z = __fadd_rn(num.z, __fmul_rn(wt[j], x[v][j].z));
                            num.w = __fadd_rn(num.w, __fmul_rn(wt[j], x[v][j].w));
                        }
                        y.x = __fdiv_rn(num.x, den);
                        y.y = __fdiv_rn(num.y, den);
                        y.z = __fdiv_rn(num.z, den);
                        y.w = __fdiv_rn(num.w, den);
                    }
                    store4_stream(out_row + col, y);
                } else {
                    for (int64_t e = col; e < col_end; ++e) average_element<WEIGHTED, false>(a, w, e);
                }
            }
        } else {
            // run-time replica count: same arithmetic, provider loop not unrolled
            float den = 0.0f, w0 = 0.0f;
            if (WEIGHTED) {
                w0 = a.dsz[w];
                den = w0;
                for (int32_t j = 0; j < R; ++j) den = __fadd_rn(den, a.dsz[pl[j]]);
            }
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                const int64_t col = col_begin + ((int64_t)v * kThreads + threadIdx.x) * 4;
                if (col + 4 <= col_end) {
                    v4f acc = load4(own_row + col);
                    if (WEIGHTED) {
                        acc.x = __fmul_rn(w0, acc.x);
                        acc.y = __fmul_rn(w0, acc.y);
                        acc.z = __fmul_rn(w0, acc.z);
                        acc.w = __fmul_rn(w0, acc.w);
                    }
                    for (int32_t j = 0; j < R; ++j) {
                        const int32_t p = pl[j];
                        const v4f t = load4(a.src + (size_t)p * (size_t)a.ld + col);
                        if (!WEIGHTED) {
                            acc.x = __fadd_rn(acc.x, t.x);
                            acc.y = __fadd_rn(acc.y, t.y);
                            acc.z = __fadd_rn(acc.z, t.z);
                            acc.w = __fadd_rn(acc.w, t.w);
                        } else {
                            const float dp = a.dsz[p];
                            acc.x = __fadd_rn(acc.x, __fmul_rn(dp, t.x));
                            acc.y = __fadd_rn(acc.y, __fmul_rn(dp, t.y));
                            acc.z = __fadd_rn(acc.z, __fmul_rn(dp, t.z));
                            acc.w = __fadd_rn(acc.w, __fmul_rn(dp, t.w));
                        }
                    }
                    v4f y;
                    if (!WEIGHTED) {
                        y.x = __fmul_rn(acc.x, a.inv);
                        y.y = __fmul_rn(acc.y, a.inv);
                        y.z = __fmul_rn(acc.z, a.inv);
                        y.w = __fmul_rn(acc.w, a.inv);
                    } else {
                        y.x = __fdiv_rn(acc.x, den);
                        y.y = __fdiv_rn(acc.y, den);
                        y.z = __fdiv_rn(acc.z, den);
                        y.w = __fdiv_rn(acc.w, den);
                    }
                    store4_stream(out_row + col, y);
                } else {
                    for (int64_t e = col; e < col_end; ++e) average_element<WEIGHTED, false>(a, w, e);
                }
            }
        }
    } else {
        // ---- boundary tile or unaligned buffers: one element per lane, coalesced ----
        for (int64_t e = col_begin + threadIdx.x; e < col_end; e += kThreads)
            average_element<WEIGHTED, false>(a, w, e);
    }
}

// x <- x - lr*g on every row (Sec. 4.1 step 1 with a given gradient), product rounded
// before the difference.  One workgroup per 4096-column tile of one row.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void sgd_step_kernel(float* __restrict__ x,
                                                            const float* __restrict__ g, float lr,
                                                            int64_t ld, int64_t P,
                                                            uint32_t tiles_per_row) {
    constexpr int kVpt = 4;
    constexpr int64_t kTile = (int64_t)kThreads * kVpt * 4;
    const uint32_t w = blockIdx.x / tiles_per_row;
    const uint32_t tile = blockIdx.x - w * tiles_per_row;
    const int64_t col_begin = (int64_t)tile * kTile;
    const int64_t col_end = col_begin + kTile < P ? col_begin + kTile : P;
    float* xr = x + (size_t)w * (size_t)ld;
    const float* gr = g + (size_t)w * (size_t)ld;
    if (VEC) {
#pragma unroll
        for (int v = 0; v < kVpt; ++v) {
            const int64_t col = col_begin + ((int64_t)v * kThreads + threadIdx.x) * 4;
            if (col + 4 <= col_end) {
                const v4f xv = load4(xr + col);
                const v4f gv = load4(gr + col);
                v4f y;
                y.x = __fsub_rn(xv.x, __fmul_rn(lr, gv.x));
                y.y = __fsub_rn(xv.y, __fmul_rn(lr, gv.y));
                y.z = __fsub_rn(xv.z, __fmul_rn(lr, gv.z));
                y.w = __fsub_rn(xv.w, __fmul_rn(lr, gv.w));
                *reinterpret_cast<v4f*>(xr + col) = y;
            } else {
                for (int64_t e = col; e < col_end; ++e)
                    xr[e] = __fsub_rn(xr[e], __fmul_rn(lr, gr[e]));
            }
        }
    } else {
        for (int64_t e = col_begin + threadIdx.x; e < col_end; e += kThreads)
            xr[e] = __fsub_rn(xr[e], __fmul_rn(lr, gr[e]));
    }
}

// Dynamic workers (Sec. 4.2) without the LDS slab: one element per lane, any alignment.
// Only used when the slab kernel cannot run (unaligned buffers or very many workers).
template <bool WEIGHTED>
__global__ __launch_bounds__(kThreads) void gossip_dynamic_elementwise_kernel(const RoundArgs a) {
    const uint32_t w = blockIdx.x / a.tiles_per_row;
    const uint32_t tile = blockIdx.x - w * a.tiles_per_row;
    const int64_t col_begin = (int64_t)tile * 1024;
    const int64_t col_end = col_begin + 1024 < a.P ? col_begin + 1024 : a.P;
    for (int64_t e = col_begin + threadIdx.x; e < col_end; e += kThreads)
        average_element_dynamic<WEIGHTED>(a, (int32_t)w, e);
}

template <int RT, int VPT>
hipError_t launch_rt_vpt(const RoundArgs& a, bool vec, uint32_t grid, hipStream_t st) {
    const bool weighted = a.dsz != nullptr;
    if (vec) {
        if (weighted)
            hipLaunchKernelGGL((gossip_round_kernel<RT, VPT, true, true>), dim3(grid),
                               dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((gossip_round_kernel<RT, VPT, false, true>), dim3(grid),
                               dim3(kThreads), 0, st, a);
    } else {
        // scalar fallback: only the run-time-R instantiation is needed, it never unrolls
        if (weighted)
            hipLaunchKernelGGL((gossip_round_kernel<-1, VPT, true, false>), dim3(grid),
                               dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((gossip_round_kernel<-1, VPT, false, false>), dim3(grid),
                               dim3(kThreads), 0, st, a);
    }
    return hipGetLastError();
}

template <int VPT>
hipError_t launch_vpt(const RoundArgs& a, bool vec, uint32_t grid, hipStream_t st) {
    switch (a.R) {
        case 0: return launch_rt_vpt<0, VPT>(a, vec, grid, st);
        case 1: return launch_rt_vpt<1, VPT>(a, vec, grid, st);
        case 2: return launch_rt_vpt<2, VPT>(a, vec, grid, st);
        case 3: return launch_rt_vpt<3, VPT>(a, vec, grid, st);
        case 4: return launch_rt_vpt<4, VPT>(a, vec, grid, st);
        case 5: return launch_rt_vpt<5, VPT>(a, vec, grid, st);
        case 6: return launch_rt_vpt<6, VPT>(a, vec, grid, st);
        case 7: return launch_rt_vpt<7, VPT>(a, vec, grid, st);
        case 8: return launch_rt_vpt<8, VPT>(a, vec, grid, st);
        default: return launch_rt_vpt<-1, VPT>(a, vec, grid, st);
    }
}

}  // namespace

uint64_t round_grid_size(int32_t N, int64_t P, int tile_cols, bool swizzle) {
    uint64_t tiles = ((uint64_t)P + (uint64_t)tile_cols - 1) / (uint64_t)tile_cols;
    if (swizzle) tiles = (tiles + kXcds - 1) / kXcds * kXcds;
    const uint64_t grid = tiles * (uint64_t)N;
    return grid > 0x7FFFFFFFull ? 0 : grid;
}

hipError_t launch_round(const RoundArgs& a, int tile_cols, bool vec, hipStream_t st) {
    const uint32_t grid = (uint32_t)round_grid_size(a.N, a.P, tile_cols, a.swizzle != 0);
    switch (tile_cols) {
        case 1024: return launch_vpt<1>(a, vec, grid, st);
        case 2048: return launch_vpt<2>(a, vec, grid, st);
        case 4096: return launch_vpt<4>(a, vec, grid, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_round_dynamic_elementwise(const RoundArgs& a_in, hipStream_t st) {
    RoundArgs a = a_in;
    const uint64_t tiles = ((uint64_t)a.P + 1023) / 1024;
    const uint64_t grid = tiles * (uint64_t)a.N;
    if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
    a.tiles_per_row = (uint32_t)tiles;
    if (a.dsz != nullptr)
        hipLaunchKernelGGL(gossip_dynamic_elementwise_kernel<true>, dim3((uint32_t)grid),
                           dim3(kThreads), 0, st, a);
    else
        hipLaunchKernelGGL(gossip_dynamic_elementwise_kernel<false>, dim3((uint32_t)grid),
                           dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_sgd_step(float* x, const float* g, float lr, int64_t ld, int32_t N, int64_t P,
                           bool vec, hipStream_t st) {
    const uint64_t tiles = ((uint64_t)P + 4095) / 4096;
    const uint64_t grid = tiles * (uint64_t)N;
    if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (vec)
        hipLaunchKernelGGL(sgd_step_kernel<true>, dim3((uint32_t)grid), dim3(kThreads), 0, st, x, g,
                           lr, ld, P, (uint32_t)tiles);
    else
        hipLaunchKernelGGL(sgd_step_kernel<false>, dim3((uint32_t)grid), dim3(kThreads), 0, st, x,
                           g, lr, ld, P, (uint32_t)tiles);
    return hipGetLastError();
}

}  // namespace combo
