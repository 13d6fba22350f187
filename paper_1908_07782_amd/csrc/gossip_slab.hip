// Table-driven instantiations of the LDS-slab aggregation kernel (gossip_slab_kernel.h)
// and the host-side choices around it: strip width, workgroup size, LDS budget.
#include <atomic>

#include "gossip_slab_kernel.h"

namespace combo {

size_t slab_lds_bytes(int32_t N, int32_t R, int W, bool hashed) {
    // slab, peer list, dataset sizes, status (or denominators), reciprocals of the
    // denominators; the in-kernel draw adds its swap partners
    return (size_t)N * (size_t)W * 4 + (hashed ? 2 : 1) * (size_t)N * (size_t)R * 4 + 3 * (size_t)N * 4;
}

// 256 threads for slabs of up to 768 128-bit words (12 KiB), 512 beyond; or what the knob says
std::atomic<int> g_slab_threads{0};
void set_slab_threads(int threads) { g_slab_threads.store(threads); }
int get_slab_threads() { return g_slab_threads.load(); }
int slab_threads(int32_t N, int W) {
    const int forced = g_slab_threads.load();
    if (forced != 0) return forced;
    return (int64_t)N * (W / 4) <= 768 ? 256 : 512;
}

// LDS to ask for at launch: at least what the kernel uses.  Asking for more lowers the number
// of workgroups resident per compute unit (160 KiB of LDS each).  Measured on MI355X with
// 256-thread workgroups and 8 KiB slabs, uniform weights, R <= 4: six resident workgroups
// (23..26 KiB each) stream up to 3 % faster than the eight that the wavefront limit allows on
// arenas below about 7 GiB per matrix (c3: 1.00 vs 1.03 ms; fewer requests competing in the
// memory system; c2 and c4 unchanged), five or fewer are slower (c5: 7.72 vs 6.93 ms).  It
// does not hold where a workgroup spends longer between its loads and its stores: with
// dataset-size weights or dynamic workers the two extra workgroups are worth 8-10 % (c2
// weighted: 0.49 vs 0.55 ms), from R = 8 on 2-5 %, and on the largest arena 1 %.  512-thread
// workgroups are four per compute unit anyway.  Slabs between 10 and 12 KiB (worker counts
// between powers of two) do best with five (32 KiB each): 24 workers 6.33 against 6.07 TB/s,
// 48 workers 6.18 against 5.87; about 50-60 KiB of slabs per compute unit in every case.
// With fused local steps a workgroup has the gradient slab in flight as well (and with more than
// one step the next slice on top), and what the memory system takes best is 64-80 KiB of loads
// per compute unit, as for every streaming kernel here: four resident workgroups (36 KiB each)
// for one step, three (44 KiB) for more (c5 with a step: 6.64 against 6.42 TB/s of 12 B per
// element; two steps: 6.41 against 6.15 of 16 B; c2 with two steps 6.50 against 6.20; like the
// rule above only while the aggregation is short: 32 workers with R = 8 lose 5 % that way).
// The knob: 0 = this rule, else the floor in bytes.
std::atomic<int> g_slab_lds_floor{0};
void set_slab_lds_floor(int bytes) { g_slab_lds_floor.store(bytes); }
int get_slab_lds_floor() { return g_slab_lds_floor.load(); }
size_t slab_lds_request(const RoundArgs& a, int W, bool hashed) {
    const size_t used = slab_lds_bytes(a.N, a.R, W, hashed);
    size_t floor_bytes = (size_t)g_slab_lds_floor.load();
    const bool short_aggregation = a.R <= 4 && a.dsz == nullptr && a.status == nullptr;
    const bool small_arena = (uint64_t)a.N * (uint64_t)a.P * sizeof(float) < (7ull << 30);
    const size_t slab_bytes = (size_t)a.N * (size_t)W * sizeof(float);
    if (floor_bytes == 0 && slab_threads(a.N, W) == 256 && short_aggregation) {
        if (a.grad != nullptr) floor_bytes = (a.tau >= 2 ? 44 : 36) * 1024;
        else if (small_arena) floor_bytes = slab_bytes > 10 * 1024 ? 32 * 1024 : 24 * 1024;
    }
    return used > floor_bytes ? used : floor_bytes;
}

namespace {

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

// Slab budget.  Up to 8 replicas the aggregation phase is short and small slabs stream best.
// Beyond, a workgroup spends longer adding (R+1 LDS reads per output word), and what hides
// that is more data in flight per compute unit: 32 KiB slabs with 512 threads (measured, 30
// workers of 25.6 M parameters, R = 16: 1.05 ms against 1.16 ms with 8 KiB slabs and 1.02 ms
// at R = 4; R = 29: 1.38 against 1.59 ms).
size_t slab_budget_bytes(int32_t R, bool tiled) {
    if (R > 8) return 32 * 1024;
    return tiled ? 8 * 1024 : 16 * 1024;
}

// Strip width: the widest power of two in [64, 1024] columns whose slab is within the budget
// (row-major arenas: 16 KiB, two 128-bit words per thread of a 512-thread workgroup; 32 KiB
// for more than 8 replicas); for many workers 64 columns as long as slab, peer list and
// weights fit in 64 KiB of LDS.  `requested` != 0 forces a width if it fits (tiled arenas:
// their tile width, down to 8 columns).
int slab_strip_cols(int32_t N, int32_t R, int requested, bool hashed) {
    const size_t kLimit = 64 * 1024;
    if (requested) {
        const bool pow2 = (requested & (requested - 1)) == 0;
        if (pow2 && requested >= 8 && requested <= 1024 &&
            slab_lds_bytes(N, R, requested, hashed) <= kLimit)
            return requested;
    }
    const size_t budget = slab_budget_bytes(R, false);
    for (int W = 1024; W >= 64; W >>= 1)
        if ((size_t)N * (size_t)W * 4 <= budget && slab_lds_bytes(N, R, W, hashed) <= kLimit) return W;
    return slab_lds_bytes(N, R, 64, hashed) <= kLimit ? 64 : 0;
}

// workgroups of a slab launch: one per strip, or, when the XCDs take turns at runs of
// strips_per_xcd strips, whole rounds of 8 runs (the surplus workgroups return at once);
// 0: beyond the grid limit
uint32_t slab_grid(const RoundArgs& a, int W) {
    const uint64_t strips = ((uint64_t)a.P + (uint64_t)W - 1) / (uint64_t)W;
    if (strips > 0x7FFFFFF0ull || strips != a.nstrips) return 0;
    uint64_t grid = strips;
    if (a.strips_per_xcd != 0) {
        const uint64_t round_strips = (uint64_t)kXcds * a.strips_per_xcd;
        grid = (strips + round_strips - 1) / round_strips * round_strips;
    }
    // a grid dimension holds fewer than 2^32 work-items
    if (grid * (uint64_t)slab_threads(a.N, W) > 0xFFFFFFFFull) return 0;
    return (uint32_t)grid;
}

hipError_t launch_round_slab(const RoundArgs& a, int W, hipStream_t st) {
    const uint32_t grid = slab_grid(a, W);
    if (grid == 0) return hipErrorInvalidValue;
    const size_t lds = slab_lds_request(a, W, false);
    if (a.status != nullptr) return launch_round_slab_dynamic(a, W, grid, lds, st);
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
