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
// A full-width strip that contains segment boundaries is staged in LDS all the same; only
// its peer lists are looked up per 128-bit word (per element where a word straddles a
// boundary) from the table in global memory, so HBM still sees one read and one write per
// element however short the segments are (L < W: every strip holds boundaries).  The one
// strip with the ragged end of the row is evaluated element by element from global memory.
//
// The front buffer (with the gradients) and the back buffer may have different layouts
// (row-major or tiled): the slab is filled from the one and written to the other, which
// turns the conversion between the layouts into a by-product of a round.
//
// This header holds the kernel template; it is included by the translation units that
// instantiate it (the table-driven variants and the table-free ones).
#ifndef COMBO_GOSSIP_SLAB_KERNEL_H_
#define COMBO_GOSSIP_SLAB_KERNEL_H_

#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

constexpr int kBatch = 4;   // 128-bit loads kept in flight per thread while filling the slab

// Workgroup size of the slab kernel (template parameter): 256 or 512 threads, chosen on
// the host so that a thread moves about two 128-bit words (measured on MI355X: 8 KiB slabs
// with 256 threads and 16 KiB slabs with 512 threads beat every other combination of
// 128..1024 threads and 4..64 KiB slabs).

// every front-buffer element is read once, so the slab fill uses streaming loads
__device__ __forceinline__ v4f load4_slab(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
}

// acc + the K providers p[0..K) of one output word, in list order.  All K list entries are
// fetched first, then all K slab words, then the adds: the LDS reads of a chunk are in
// flight together instead of forming a chain of dependent round trips.
template <int K>
__device__ __forceinline__ v4f add_providers(v4f acc, const v4f* slab, const int32_t* pl, int w4_shift,
                                             int c4) {
    int32_t p[K];
    v4f v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) p[k] = pl[k];
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = slab[(p[k] << w4_shift) + c4];
#pragma unroll
    for (int k = 0; k < K; ++k) acc = add4(acc, v[k]);
    return acc;
}

// any number of providers: chunks of 8, then 4, 2, 1 (same order as one by one)
__device__ __forceinline__ v4f add_providers_any(v4f acc, const v4f* slab, const int32_t* pl, int32_t R,
                                                 int w4_shift, int c4) {
    int32_t j = 0;
    for (; j + 8 <= R; j += 8) acc = add_providers<8>(acc, slab, pl + j, w4_shift, c4);
    if (j + 4 <= R) { acc = add_providers<4>(acc, slab, pl + j, w4_shift, c4); j += 4; }
    if (j + 2 <= R) { acc = add_providers<2>(acc, slab, pl + j, w4_shift, c4); j += 2; }
    if (j < R) acc = add_providers<1>(acc, slab, pl + j, w4_shift, c4);
    return acc;
}

// One lane type for the strips that hold several segments: a whole 128-bit word (all four
// columns in one segment) or a single element of a word that straddles a boundary.
struct WordLane {
    typedef v4f T;
    int c4;
    __device__ __forceinline__ T get(const v4f* slab, int row, int w4_shift) const {
        return slab[(row << w4_shift) + c4];
    }
    static __device__ __forceinline__ T add(T a, T b) { return add4(a, b); }
    static __device__ __forceinline__ T scale(float s, T a) { return scale4(s, a); }
    static __device__ __forceinline__ T div(T a, float d) { return div4(a, d); }
};
struct ElemLane {
    typedef float T;
    int c;    // column inside the strip
    __device__ __forceinline__ T get(const v4f* slab, int row, int w4_shift) const {
        return reinterpret_cast<const float*>(slab)[((size_t)row << (w4_shift + 2)) + c];
    }
    static __device__ __forceinline__ T add(T a, T b) { return __fadd_rn(a, b); }
    static __device__ __forceinline__ T scale(float s, T a) { return __fmul_rn(s, a); }
    static __device__ __forceinline__ T div(T a, float d) { return __fdiv_rn(a, d); }
};

// Eq. (3) for one lane of worker w in segment s with the served values in the LDS slab
// (size * value for static weighted rounds) and the peer list taken from the table in
// global memory (or drawn from the hash).  Same terms, order and roundings as the
// single-segment path and as average_element / average_element_dynamic.
template <bool WEIGHTED, bool DYNAMIC, bool HASHED, class Lane>
__device__ __forceinline__ typename Lane::T aggregate_lane(const RoundArgs& a, const v4f* slab,
                                                           const float* lds_d, const int32_t* lds_status,
                                                           int w4_shift, int32_t w, int32_t s, Lane lane) {
    typedef typename Lane::T T;
    const int32_t R = a.R;
    int32_t drawn[kMaxHashedR];
    const int32_t* pl;
    if (HASHED) {
        draw_peers(a.hash_sr, w, s, a.N, R, drawn);
        pl = drawn;
    } else {
        pl = a.peers + ((size_t)w * (size_t)a.S + (size_t)s) * (size_t)R;
    }
    const T own = lane.get(slab, w, w4_shift);
    if (DYNAMIC) {
        const int st = lds_status[w];
        int cnt = 0;
        float den = 0.0f;
        T acc = own;
        if (st == 1) {
            if (WEIGHTED) { den = lds_d[w]; acc = Lane::scale(den, own); }
            cnt = 1;
        }
        if (st != 0) {
            for (int32_t j = 0; j < R; ++j) {
                const int32_t p = pl[j];
                if (p < 0) continue;
                T v = lane.get(slab, p, w4_shift);
                if (WEIGHTED) {
                    const float dp = lds_d[p];
                    v = Lane::scale(dp, v);
                    den = cnt == 0 ? dp : __fadd_rn(den, dp);
                }
                acc = cnt == 0 ? v : Lane::add(acc, v);
                ++cnt;
            }
        }
        if (cnt == 0) return own;
        return WEIGHTED ? Lane::div(acc, den) : Lane::scale(__fdiv_rn(1.0f, (float)cnt), acc);
    }
    T acc = own;
    if (!WEIGHTED) {
        for (int32_t j = 0; j < R; ++j) acc = Lane::add(acc, lane.get(slab, HASHED ? drawn[j] : pl[j], w4_shift));
        return Lane::scale(a.inv, acc);
    }
    float den = a.dsz[w];
    for (int32_t j = 0; j < R; ++j) {
        const int32_t p = HASHED ? drawn[j] : pl[j];
        den = __fadd_rn(den, a.dsz[p]);
        acc = Lane::add(acc, lane.get(slab, p, w4_shift));
    }
    return Lane::div(acc, den);
}

// DYNAMIC: Sec. 4.2 semantics (offline rows copied, newcomers aggregated without their own
// value, unused table slots < 0 skipped, scale by the number of terms).
// HASHED: no peer table; every workgroup draws the strip's peer lists itself from the
// counter-based hash while its slab loads are in flight (RT in 0..8).
template <int RT, bool WEIGHTED, bool FUSED, bool DYNAMIC, int kSlabThreads, bool HASHED = false>
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
    int32_t* lds_partner = lds_status + N;                                        // [N][R], HASHED
    // static weighted rounds keep each row's denominator (the sizes of the worker and its
    // peers added in list order) and its reciprocal; the slab then holds size * value
    float* lds_den = reinterpret_cast<float*>(lds_status);                        // [N] (no status then)
    float* lds_rcp = reinterpret_cast<float*>(lds_partner + (HASHED ? (size_t)N * (size_t)R : 0));   // [N]
    constexpr bool kPrescaled = WEIGHTED && !DYNAMIC;

    // which strip: workgroup i takes strip i, or - workgroup ids go round-robin over the 8
    // XCDs - the XCDs take turns at runs of strips_per_xcd consecutive strips (with
    // strips_per_xcd = ceil(nstrips / 8) every XCD works through its own contiguous eighth)
    const uint32_t strip = xcd_run_block(blockIdx.x, a.strips_per_xcd);
    if (strip >= a.nstrips) return;                 // surplus workgroup of the last round of runs; uniform
    const int64_t col0 = (int64_t)strip * W;
    const int64_t col_end = col0 + W < a.P ? col0 + W : a.P;
    // where the strip's row chunks live: row-major rows are ld apart and start at col0;
    // in the tiled layout (tile width == W) the whole slab is one contiguous block
    const size_t row_stride = a.tile_shift == 0 ? (size_t)a.ld : (size_t)W;
    const size_t strip_base = a.tile_shift == 0 ? (size_t)col0 : (size_t)strip * (size_t)N * (size_t)W;
    const size_t dst_row_stride = a.dst_tile_shift == 0 ? (size_t)a.dst_ld : (size_t)W;
    const size_t dst_strip_base = a.dst_tile_shift == 0 ? (size_t)col0 : (size_t)strip * (size_t)N * (size_t)W;
    const int32_t s0 = segment_of(col0, a);
    const int64_t seg_end = (s0 == a.S - 1) ? a.P : (int64_t)(s0 + 1) * a.L;
    const bool one_segment = col_end <= seg_end;    // else: peer lists are looked up per word

    if (col_end - col0 == W) {
        // ---- fill: peer list, weights, then the slab --------------------------------
        if (!HASHED && one_segment) {
            for (int i = threadIdx.x; R > 0 && i < N * R; i += kSlabThreads) {
                const int w = i / (R > 0 ? R : 1);
                const int j = i - w * R;
                lds_peers[i] = a.peers[((size_t)w * (size_t)a.S + (size_t)s0) * (size_t)R + (size_t)j];
            }
        }
        // prescaled rounds: thread w < N adds up row w's denominator; its picks are fetched
        // ahead of the slab loads so that the dependent size loads need not wait for those
        int32_t den_pick[RT > 0 ? RT : 1];
        if (kPrescaled && !HASHED && RT > 0 && one_segment && (int)threadIdx.x < N) {
#pragma unroll
            for (int j = 0; j < (RT > 0 ? RT : 0); ++j)
                den_pick[j] = a.peers[((size_t)threadIdx.x * (size_t)a.S + (size_t)s0) * (size_t)R + (size_t)j];
        }
        if (WEIGHTED && (!kPrescaled || HASHED))
            for (int i = threadIdx.x; i < N; i += kSlabThreads) lds_d[i] = a.dsz[i];
        if (DYNAMIC)
            for (int i = threadIdx.x; i < N; i += kSlabThreads) lds_status[i] = a.status[i];

        for (int base = 0; base < total4; base += kSlabThreads * kBatch) {
            v4f x[kBatch], g[kBatch];
            size_t off[kBatch];
            float d_row[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                if (idx < total4) {
                    const int row = idx >> w4_shift;
                    const int c4 = idx & (W4 - 1);
                    off[u] = (size_t)row * row_stride + strip_base + (size_t)c4 * 4;
                    x[u] = load4_slab(a.src + off[u]);
                    if (FUSED) g[u] = load4_slab(a.grad + off[u]);
                    if (kPrescaled) d_row[u] = a.dsz[row];
                }
            }
            if (HASHED && base == 0 && one_segment) {
                // the slab loads are in flight: draw the peer lists of this strip meanwhile.
                // One thread per (worker, step) evaluates the hash and the swap partner; after
                // a barrier one thread per worker turns its R partners into picks.
                for (int i = threadIdx.x; R > 0 && i < N * R; i += kSlabThreads) {
                    const int w = i / (R > 0 ? R : 1);
                    lds_partner[i] = shuffle_partner(a.hash_sr, w, s0, i - w * R, N);
                }
                __syncthreads();
                for (int w = threadIdx.x; w < N; w += kSlabThreads) {
                    int32_t drawn[kMaxHashedR];
                    picks_from_partners(lds_partner + w * R, w, R, drawn);
#pragma unroll
                    for (int j = 0; j < kMaxHashedR; ++j)
                        if (j < R) lds_peers[w * R + j] = drawn[j];
                    if (kPrescaled) {
                        float den = lds_d[w];
#pragma unroll
                        for (int j = 0; j < kMaxHashedR; ++j)
                            if (j < R) den = __fadd_rn(den, lds_d[drawn[j]]);
                        lds_den[w] = den;
                        lds_rcp[w] = shared_reciprocal(den);
                    }
                }
            }
            if (kPrescaled && !HASHED && base == 0 && one_segment) {
                // the slab loads are in flight; the picks fetched ahead have arrived before them
                for (int w = threadIdx.x; w < N; w += kSlabThreads) {
                    float den = a.dsz[w];
                    if (RT > 0 && w == (int)threadIdx.x) {
#pragma unroll
                        for (int j = 0; j < (RT > 0 ? RT : 0); ++j) den = __fadd_rn(den, a.dsz[den_pick[j]]);
                    } else {
                        const int32_t* pw = a.peers + ((size_t)w * (size_t)a.S + (size_t)s0) * (size_t)R;
                        for (int j = 0; j < R; ++j) den = __fadd_rn(den, a.dsz[pw[j]]);
                    }
                    lds_den[w] = den;
                    lds_rcp[w] = shared_reciprocal(den);
                }
            }
            if (FUSED) {
                // local steps in slice order; the first slice's loads are already in flight, and
                // the loads of slice t+1 are issued before slice t is applied
                for (int32_t t = 0; t < a.tau; ++t) {
                    v4f g_next[kBatch];
                    if (t + 1 < a.tau) {
#pragma unroll
                        for (int u = 0; u < kBatch; ++u) {
                            const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                            if (idx < total4)
                                g_next[u] = load4_slab(a.grad + (size_t)(t + 1) * (size_t)a.grad_slice + off[u]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                        if (idx < total4) x[u] = sgd_step4(x[u], a.lr, g[u]);
                    }
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) g[u] = g_next[u];
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int idx = base + u * kSlabThreads + (int)threadIdx.x;
                if (idx < total4) slab[idx] = kPrescaled ? scale4(d_row[u], x[u]) : x[u];
            }
            // All loads of this pass have been consumed.  Saying so explicitly (vmcnt(0); the
            // other counters at their maxima, i.e. not waited for) matters: the stores above
            // sit in per-thread conditionals, so without it the compiler must assume at the
            // loop's back edge that loads into the same registers may still be pending, and it
            // then puts a wait in front of every load of the pass, which serialises them.
            __builtin_amdgcn_s_waitcnt(0x0F70);
        }
        __syncthreads();

        // ---- aggregate from LDS ---------------------------------------------------
        if (!one_segment) {
            // several segments in the strip: the segment, and with it the peer list, is found
            // per 128-bit word, or per element where a word straddles a boundary
            for (int idx = threadIdx.x; idx < total4; idx += kSlabThreads) {
                const int w = idx >> w4_shift;
                const int c4 = idx & (W4 - 1);
                const int64_t e0 = col0 + (int64_t)c4 * 4;
                const int32_t sa = segment_of(e0, a), sb = segment_of(e0 + 3, a);
                v4f y;
                if (sa == sb) {
                    y = aggregate_lane<WEIGHTED, DYNAMIC, HASHED>(a, slab, lds_d, lds_status, w4_shift, w, sa,
                                                                  WordLane{c4});
                } else {
                    y.x = aggregate_lane<WEIGHTED, DYNAMIC, HASHED>(a, slab, lds_d, lds_status, w4_shift, w, sa,
                                                                    ElemLane{c4 * 4});
                    y.y = aggregate_lane<WEIGHTED, DYNAMIC, HASHED>(a, slab, lds_d, lds_status, w4_shift, w,
                                                                    segment_of(e0 + 1, a), ElemLane{c4 * 4 + 1});
                    y.z = aggregate_lane<WEIGHTED, DYNAMIC, HASHED>(a, slab, lds_d, lds_status, w4_shift, w,
                                                                    segment_of(e0 + 2, a), ElemLane{c4 * 4 + 2});
                    y.w = aggregate_lane<WEIGHTED, DYNAMIC, HASHED>(a, slab, lds_d, lds_status, w4_shift, w, sb,
                                                                    ElemLane{c4 * 4 + 3});
                }
                store4_stream(a.dst + (size_t)w * dst_row_stride + dst_strip_base + (size_t)c4 * 4, y);
            }
            return;
        }
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
#pragma unroll
                    for (int j = 0; j < (RT >= 0 ? RT : R); ++j) {
                        const int p = pl[j];
                        // read unconditionally (own row for an unused slot) so that the LDS
                        // reads of all slots can be issued together; use only valid ones
                        v4f v = slab[((p < 0 ? w : p) << w4_shift) + c4];
                        if (p < 0) continue;
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
                    acc = add_providers_any(acc, slab, pl, R, w4_shift, c4);
                }
                y = scale4(a.inv, acc);
            } else {
                // the slab holds size * value: add in list order, divide by the row's denominator
                if (RT >= 0) {
#pragma unroll
                    for (int j = 0; j < (RT >= 0 ? RT : 0); ++j)
                        acc = add4(acc, slab[(pl[j] << w4_shift) + c4]);
                } else {
                    acc = add_providers_any(acc, slab, pl, R, w4_shift, c4);
                }
                y = div4_shared(acc, lds_den[w], lds_rcp[w]);
            }
            store4_stream(a.dst + (size_t)w * dst_row_stride + dst_strip_base + (size_t)c4 * 4, y);
        }
    } else {
        // ---- the strip with the ragged end of the row: element by element from global memory
        const int width = (int)(col_end - col0);
        const int total = N * width;
        for (int idx = threadIdx.x; idx < total; idx += kSlabThreads) {
            const int w = idx / width;
            const int64_t e = col0 + (idx - w * width);
            if (DYNAMIC) average_element_dynamic<WEIGHTED>(a, w, e);
            else average_element<WEIGHTED, FUSED, HASHED>(a, w, e);
        }
    }
}

}  // namespace
}  // namespace combo
#endif
