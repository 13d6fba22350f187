// Device helpers shared by the aggregation kernels (HIP path only).
#ifndef COMBO_ROUND_DEVICE_H_
#define COMBO_ROUND_DEVICE_H_

#include "combo_internal.h"

namespace combo {

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v4f load4(const float* p) { return *reinterpret_cast<const v4f*>(p); }

__device__ __forceinline__ void store4_stream(float* p, v4f v) {
    __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
}

// x - lr*g with the product rounded before the difference (one SGD step, Sec. 4.1 step 1)
__device__ __forceinline__ float sgd_step(float x, float lr, float g) {
    return __fsub_rn(x, __fmul_rn(lr, g));
}

__device__ __forceinline__ v4f sgd_step4(v4f x, float lr, v4f g) {
    v4f y;
    y.x = sgd_step(x.x, lr, g.x);
    y.y = sgd_step(x.y, lr, g.y);
    y.z = sgd_step(x.z, lr, g.z);
    y.w = sgd_step(x.w, lr, g.w);
    return y;
}

__device__ __forceinline__ v4f add4(v4f a, v4f b) {
    v4f y;
    y.x = __fadd_rn(a.x, b.x);
    y.y = __fadd_rn(a.y, b.y);
    y.z = __fadd_rn(a.z, b.z);
    y.w = __fadd_rn(a.w, b.w);
    return y;
}

__device__ __forceinline__ v4f scale4(float s, v4f a) {
    v4f y;
    y.x = __fmul_rn(s, a.x);
    y.y = __fmul_rn(s, a.y);
    y.z = __fmul_rn(s, a.z);
    y.w = __fmul_rn(s, a.w);
    return y;
}

// Quotients by a shared denominator.  Given r = RN(1/d) (the correctly rounded reciprocal),
// a / d is obtained, correctly rounded, with one multiply and four fused multiply-adds
// instead of a division sequence per element:
//     q0 = RN(a*r)                        within 2 ulp of a/d (r and the product each
//                                         contribute a relative error of up to 2^-24); NOT
//                                         necessarily faithful, so its residual a - q0*d
//                                         need not be exact
//     q1 = RN(q0 + RN(a - q0*d)*r)        one correction: q1 = RN(a/d + e) with |e| far
//                                         below an ulp, hence faithful (one of the two
//                                         floats around a/d), though e could still tip a
//                                         quotient that lies very close to a midpoint
//     q2 = RN(q1 + (a - q1*d)*r)          the residual of a faithful quotient is exact in
//                                         one fma, and with r = RN(1/d) this last step
//                                         returns RN(a/d) (Markstein's theorem on the
//                                         final correction of a division)
// provided nothing under- or overflows on the way, which holds for d and |a| in
// [2^-60, 2^60] (the residuals are multiples of 2^-46*|a|).  A zero numerator gives a zero
// of the numerator's sign.  Everything else takes the division instruction sequence.
constexpr uint32_t kDivLoBits = 0x21800000u;   // 2^-60
constexpr uint32_t kDivHiBits = 0x5d800000u;   // 2^60

// fl(1/d) if d is in the range of the shortcut, else 0 ("use the division")
__device__ __forceinline__ float shared_reciprocal(float d) {
    return (d >= 0x1p-60f && d <= 0x1p60f) ? __fdiv_rn(1.0f, d) : 0.0f;
}

__device__ __forceinline__ float quotient_by_reciprocal(float a, float d, float r) {
    const float q0 = __fmul_rn(a, r);
    const float q1 = __fmaf_rn(__fmaf_rn(-q0, d, a), r, q0);
    const float q2 = __fmaf_rn(__fmaf_rn(-q1, d, a), r, q1);
    return __builtin_copysignf(q2, a);           // only matters for a == -0
}

// the four quotients of one 128-bit word by the same denominator; r = shared_reciprocal(d)
__device__ __forceinline__ v4f div4_shared(v4f a, float d, float r) {
    const uint32_t ux = __float_as_uint(a.x) & 0x7fffffffu, uy = __float_as_uint(a.y) & 0x7fffffffu;
    const uint32_t uz = __float_as_uint(a.z) & 0x7fffffffu, uw = __float_as_uint(a.w) & 0x7fffffffu;
    const uint32_t hi = max(max(ux, uy), max(uz, uw));                  // NaN and inf are the largest
    const uint32_t lo = min(min(ux - 1u, uy - 1u), min(uz - 1u, uw - 1u));   // zero wraps to the top
    v4f y;
    if (r != 0.0f && hi <= kDivHiBits && lo >= kDivLoBits - 1u) {
        y.x = quotient_by_reciprocal(a.x, d, r);
        y.y = quotient_by_reciprocal(a.y, d, r);
        y.z = quotient_by_reciprocal(a.z, d, r);
        y.w = quotient_by_reciprocal(a.w, d, r);
    } else {
        y.x = __fdiv_rn(a.x, d);
        y.y = __fdiv_rn(a.y, d);
        y.z = __fdiv_rn(a.z, d);
        y.w = __fdiv_rn(a.w, d);
    }
    return y;
}

__device__ __forceinline__ v4f div4(v4f a, float d) { return div4_shared(a, d, shared_reciprocal(d)); }

// ---- the counter-based peer hash (see combo_make_peer_table in the header) ------------
constexpr uint64_t kHashGamma = 0x9E3779B97F4A7C15ull;   // SplitMix64 increment

__host__ __device__ __forceinline__ uint64_t hash_finalise(uint64_t z) {
    // output function of SplitMix64: two xor-shift-multiply rounds and a last xor-shift
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__host__ __device__ __forceinline__ uint64_t hash_take_in(uint64_t h, uint64_t counter) {
    return hash_finalise((h ^ counter) + kHashGamma);
}

constexpr int kMaxHashedR = 8;   // replica counts the in-kernel peer draw supports

// The R providers of (worker w, segment s) without a table: the first R steps of the
// Fisher-Yates shuffle of the N-1 other workers, on a virtual array whose displaced
// slots (at most one per step) are kept in registers.  Same picks, same order as the
// peer-table kernel.  h_sr = hash state after seed and round.
//   shuffle_partner      swap partner of step j: j + reduce(hash(seed, round, w, s, j), N-1-j)
//   picks_from_partners  the picks given the R partners (pure integer bookkeeping)
//   draw_peers           both, for one (w, s)
__device__ __forceinline__ int32_t shuffle_partner(uint64_t h_sr, int32_t w, int32_t s, int32_t j,
                                                   int32_t N) {
    const uint64_t h = hash_take_in(hash_take_in(h_sr, (uint64_t)w), (uint64_t)s);
    const uint64_t word = hash_take_in(h, (uint64_t)j);
    return j + (int32_t)(((word >> 32) * (uint64_t)(uint32_t)(N - 1 - j)) >> 32);
}

__device__ __forceinline__ void picks_from_partners(const int32_t* partner, int32_t w, int32_t R,
                                                    int32_t (&out)[kMaxHashedR]) {
    int32_t pos[kMaxHashedR], val[kMaxHashedR];
#pragma unroll
    for (int j = 0; j < kMaxHashedR; ++j) {
        if (j < R) {
            const int32_t r = partner[j];
            int32_t at_r = r, at_j = j;              // current contents of slots r and j
#pragma unroll
            for (int k = 0; k < j; ++k) {            // the latest displacement of a slot wins
                if (pos[k] == r) at_r = val[k];
                if (pos[k] == j) at_j = val[k];
            }
            out[j] = at_r + (at_r >= w ? 1 : 0);     // skip over w itself
            pos[j] = r;                              // slot r now holds what slot j held
            val[j] = at_j;
        }
    }
}

__device__ __forceinline__ void draw_peers(uint64_t h_sr, int32_t w, int32_t s, int32_t N, int32_t R,
                                           int32_t (&out)[kMaxHashedR]) {
    int32_t partner[kMaxHashedR];
#pragma unroll
    for (int j = 0; j < kMaxHashedR; ++j)
        if (j < R) partner[j] = shuffle_partner(h_sr, w, s, j, N);
    picks_from_partners(partner, w, R, out);
}

// Which block of work (strip, tile, chunk) workgroup `id` takes.  Workgroup ids go round-robin
// over the 8 XCDs; with run == 0 block = id, so XCD x gets every eighth block; else the XCDs take
// turns at runs of `run` consecutive blocks (block ids beyond the work are the caller's to skip).
__device__ __forceinline__ uint32_t xcd_run_block(uint32_t id, uint32_t run) {
    if (run == 0) return id;
    const uint32_t turn = id >> 3;                    // the XCD's turn-th workgroup
    const uint32_t r = turn / run;
    return (r * kXcds + (id & (kXcds - 1))) * run + (turn - r * run);
}

// segment of column e: floor(e / L), the last segment also owning the remainder (Eq. 1)
__device__ __forceinline__ int32_t segment_of(int64_t e, const RoundArgs& a) {
    uint64_t q;
    if (a.p32) q = (uint32_t)e / (uint32_t)a.L;
    else q = (uint64_t)e / (uint64_t)a.L;
    return q >= (uint64_t)a.S ? a.S - 1 : (int32_t)q;
}

// Index of worker `row`'s column e.  Row-major: row*ld + e.  Tiled [T][N][Wt]: tile
// e / Wt holds Wt consecutive columns of all N workers, worker-major inside the tile.
// The front buffer (with the gradients) and the back buffer each have their own layout.
__device__ __forceinline__ size_t layout_offset(int64_t ld, int32_t tile_shift, int32_t N, int32_t row,
                                                int64_t e) {
    if (tile_shift == 0) return (size_t)row * (size_t)ld + (size_t)e;
    const size_t tile = (size_t)e >> tile_shift;
    const size_t in_tile = (size_t)e & (((size_t)1 << tile_shift) - 1);
    return ((tile * (size_t)N + (size_t)row) << tile_shift) + in_tile;
}

__device__ __forceinline__ size_t elem_offset(const RoundArgs& a, int32_t row, int64_t e) {
    return layout_offset(a.ld, a.tile_shift, a.N, row, e);
}

__device__ __forceinline__ size_t elem_offset_dst(const RoundArgs& a, int32_t row, int64_t e) {
    return layout_offset(a.dst_ld, a.dst_tile_shift, a.N, row, e);
}

// pre-aggregation value of worker `row` at column e: the stored parameter, or, when the
// local steps are fused in, the parameter after the tau SGD steps (in slice order)
template <bool FUSED>
__device__ __forceinline__ float served_value(const RoundArgs& a, int32_t row, int64_t e) {
    const size_t k = elem_offset(a, row, e);
    float x = a.src[k];
    if (FUSED)
        for (int32_t t = 0; t < a.tau; ++t)
            x = sgd_step(x, a.lr, a.grad[(size_t)t * (size_t)a.grad_slice + k]);
    return x;
}

// Eq. (3) for one element of any segment: used for tiles that contain a segment
// boundary, ragged row ends and unaligned buffers
template <bool WEIGHTED, bool FUSED, bool HASHED = false>
__device__ __forceinline__ void average_element(const RoundArgs& a, int32_t w, int64_t e) {
    const int32_t s = segment_of(e, a);
    int32_t drawn[kMaxHashedR];
    const int32_t* pl;
    if (HASHED) {
        draw_peers(a.hash_sr, w, s, a.N, a.R, drawn);
        pl = drawn;
    } else {
        pl = a.peers + ((size_t)w * (size_t)a.S + (size_t)s) * (size_t)a.R;
    }
    const float own = served_value<FUSED>(a, w, e);
    float out;
    if (!WEIGHTED) {
        float acc = own;
        for (int32_t j = 0; j < a.R; ++j) acc = __fadd_rn(acc, served_value<FUSED>(a, pl[j], e));
        out = __fmul_rn(acc, a.inv);
    } else {
        float den = a.dsz[w];
        float num = __fmul_rn(den, own);
        for (int32_t j = 0; j < a.R; ++j) {
            const int32_t p = pl[j];
            const float dp = a.dsz[p];
            den = __fadd_rn(den, dp);
            num = __fadd_rn(num, __fmul_rn(dp, served_value<FUSED>(a, p, e)));
        }
        out = __fdiv_rn(num, den);
    }
    a.dst[elem_offset_dst(a, w, e)] = out;
}

// Eq. (3) with dynamic workers (Sec. 4.2) for one element.  status: 0 offline (keeps its
// value), 1 active (own value, then the valid table entries), 2 newcomer (valid table
// entries only; none -> keeps its value).  Table entries < 0 are unused slots.
template <bool WEIGHTED>
__device__ __forceinline__ void average_element_dynamic(const RoundArgs& a, int32_t w, int64_t e) {
    const int32_t s = segment_of(e, a);
    const int32_t* pl = a.peers + ((size_t)w * (size_t)a.S + (size_t)s) * (size_t)a.R;
    const float own = a.src[elem_offset(a, w, e)];
    const int st = a.status[w];
    int cnt = 0;
    float acc = 0.0f, den = 0.0f;
    if (st == 1) {
        if (WEIGHTED) { den = a.dsz[w]; acc = __fmul_rn(den, own); }
        else acc = own;
        cnt = 1;
    }
    if (st != 0) {
        for (int32_t j = 0; j < a.R; ++j) {
            const int32_t p = pl[j];
            if (p < 0) continue;
            const float v = a.src[elem_offset(a, p, e)];
            if (WEIGHTED) {
                const float dp = a.dsz[p];
                const float t = __fmul_rn(dp, v);
                acc = cnt == 0 ? t : __fadd_rn(acc, t);
                den = cnt == 0 ? dp : __fadd_rn(den, dp);
            } else {
                acc = cnt == 0 ? v : __fadd_rn(acc, v);
            }
            ++cnt;
        }
    }
    float out = own;
    if (cnt > 0) out = WEIGHTED ? __fdiv_rn(acc, den) : __fmul_rn(acc, __fdiv_rn(1.0f, (float)cnt));
    a.dst[elem_offset_dst(a, w, e)] = out;
}

}  // namespace combo
#endif
