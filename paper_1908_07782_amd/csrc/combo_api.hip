// The C ABI of libcombo: argument validation and kernel launches.  See include/combo.h
// for the meaning of every argument; nothing here allocates, copies or synchronises.
#include "../../include/combo.h"

#include <atomic>

#include "combo_internal.h"
#include "round_device.h"

namespace {

std::atomic<int> g_tile_cols{0};              // 0: by the number of workers
std::atomic<int> g_swizzle{1};
std::atomic<int> g_fused_mode{0};
std::atomic<int> g_kernel{0};
std::atomic<int> g_slab_cols{0};
std::atomic<int> g_slab_order{0};             // 0: by size and layout; 1: strip i to workgroup i; 2: contiguous strips per XCD

enum PlanKind { kPlanTile = 0, kPlanSlab = 1 };
struct Plan {
    PlanKind kind;
    int cols;      // strip width for the slab kernels
};

// where a parameter matrix lives: row-major [N][ld] (tile == 0) or tiled [T][N][tile]
struct Layout {
    int64_t ld;
    int tile;
};

// the slab kernels' grid: one workgroup per strip, rounded up to a multiple of 8
constexpr uint64_t kMaxStrips = 0x7FFFFFF0ull;
// tiles per turn of an XCD in kernels that work tile by tile (see enqueue_round): 16, or 32
// for matrices of 7 GiB and more
uint32_t tile_run(int32_t N, int64_t P) {
    return (uint64_t)N * (uint64_t)P * sizeof(float) >= (7ull << 30) ? 32u : 16u;
}

int log2_of(int pow2) {
    int k = 0;
    while ((1 << k) < pow2) ++k;
    return k;
}

bool overlaps(const void* a, uint64_t a_bytes, const void* b, uint64_t b_bytes) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// shared checks of the two aggregation entry points
int check_round_args(const float* dst, const float* src, int64_t ld, const int32_t* peers,
                     int32_t N, int64_t P, int32_t S, int32_t R) {
    if (N < 1 || S < 1 || P < 1 || (int64_t)S > P || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (ld < P || dst == nullptr || src == nullptr) return COMBO_EINVAL;
    if (R > 0 && peers == nullptr) return COMBO_EINVAL;
    if ((uint64_t)ld > (UINT64_MAX / sizeof(float)) / (uint64_t)N) return COMBO_ERANGE;   // N*ld*4 overflows
    const uint64_t bytes = (uint64_t)N * (uint64_t)ld * sizeof(float);
    if (overlaps(dst, bytes, src, bytes)) return COMBO_EALIAS;
    return COMBO_OK;
}

// the small inputs of a round (table, dataset sizes, status) must not lie inside the back buffer
int check_small_inputs(const float* dst, uint64_t dst_bytes, const int32_t* peers, const float* dsz,
                       const uint8_t* status, int32_t N, int32_t S, int32_t R) {
    const uint64_t table_bytes = (uint64_t)N * (uint64_t)S * (uint64_t)R * sizeof(int32_t);
    if (peers != nullptr && table_bytes != 0 && overlaps(dst, dst_bytes, peers, table_bytes)) return COMBO_EALIAS;
    if (dsz != nullptr && overlaps(dst, dst_bytes, dsz, (uint64_t)N * sizeof(float))) return COMBO_EALIAS;
    if (status != nullptr && overlaps(dst, dst_bytes, status, (uint64_t)N)) return COMBO_EALIAS;
    return COMBO_OK;
}

// Columns of one worker per workgroup of the row-tile kernel.  The N workers of a column
// tile run back to back on one XCD and re-read each other's rows from its 4 MiB L2, so
// the tile has to shrink as N grows (measured: N = 1000, 4.50 TB/s at 1024 columns against
// 3.96 at 2048 and 3.24 at 4096; up to N = 300 2048 is at least as good, from N = 500
// on 1024 is better).  A forced value
// or, if the grid would be too large, the next wider tile wins.
int row_tile_cols(int32_t N, int64_t P) {
    const int forced = g_tile_cols.load();
    if (forced != 0) return forced;
    const bool swizzle = g_swizzle.load() != 0;
    const int first = N > 384 ? 1024 : 2048;
    for (int t = first; t <= 4096; t <<= 1)
        if (combo::round_grid_size(N, P, t, swizzle) != 0) return t;
    return 4096;
}

// Enqueue one aggregation round.  grad != nullptr: the local step is fused into the
// round (only possible with the slab kernel); the caller has checked that with
// fused_in_round().
int enqueue_round(float* dst, const float* src, const float* grad, float lr, int64_t ld,
                  const int32_t* peers, const float* dsz, int32_t N, int64_t P, int32_t S,
                  int32_t R, Plan plan, hipStream_t st, const uint8_t* status = nullptr,
                  int32_t tau = 1, int arena_tile = 0, bool hashed = false, uint64_t hash_sr = 0,
                  const Layout* dst_layout = nullptr) {
    const int tile_cols = row_tile_cols(N, P);
    const bool swizzle = g_swizzle.load() != 0;
    combo::RoundArgs a;
    a.dst = dst;
    a.src = src;
    a.peers = peers;
    a.dsz = dsz;
    a.grad = grad;
    a.status = status;
    a.ld = ld;
    a.P = P;
    a.L = P / S;
    a.N = N;
    a.S = S;
    a.R = R;
    a.tiles_per_row = (uint32_t)(((uint64_t)P + (uint64_t)tile_cols - 1) / (uint64_t)tile_cols);
    a.swizzle = swizzle ? 1 : 0;
    a.p32 = P < (int64_t)0x100000000ll ? 1 : 0;
    a.inv = 1.0f / (float)(R + 1);
    a.lr = lr;
    a.tau = tau;
    a.tile_shift = 0;
    a.grad_slice = (int64_t)N * ld;
    if (arena_tile) {         // tiled arena [T][N][Wt]
        a.tile_shift = log2_of(arena_tile);
        const int64_t tiles = (P + arena_tile - 1) / arena_tile;
        a.grad_slice = tiles * (int64_t)N * (int64_t)arena_tile;
    }
    a.dst_ld = ld;            // the back buffer normally has the front buffer's layout
    a.dst_tile_shift = a.tile_shift;
    if (dst_layout != nullptr) {
        a.dst_ld = dst_layout->ld;
        a.dst_tile_shift = dst_layout->tile ? log2_of(dst_layout->tile) : 0;
    }
    a.nstrips = 0;
    a.strips_per_xcd = 0;
    if (plan.kind == kPlanSlab) {
        const uint64_t strips = ((uint64_t)P + (uint64_t)plan.cols - 1) / (uint64_t)plan.cols;
        if (strips > kMaxStrips) return COMBO_ERANGE;
        a.nstrips = (uint32_t)strips;
        // Which strips a workgroup takes.  Workgroup ids go round-robin over the 8 XCDs; with
        // strip = id, XCD x only ever sees the tiles whose address bits just above the tile
        // size equal x.  Letting the XCDs take turns at runs of 16 consecutive tiles (128 KiB
        // for 8 KiB tiles) moves that pattern to higher address bits.  Measured on tiled
        // arenas, both ping-pong directions averaged: runs of 16 gain 1-5 % up to about 7 GiB
        // per matrix (c2 6.42 -> 6.57, c3 6.39 -> 6.65 TB/s) but become erratic beyond (one
        // direction of c5 gains 5 %, the other loses 6 %); runs of 32 gain 1-7 % at every size
        // tried from 6 to 21 GiB (c5 6.31 -> 6.43, 100 x 30 M 5.86 -> 6.27 TB/s); runs of 4 or
        // 8 tiles are 5-10 % slower than strip = id, runs that are not powers of two lose
        // 2-4 %, whole eighths lose 2-10 % on small arenas.  Rounds that change layout gain
        // too when one side is tiled (c2: +3-5 %).  Row-major arenas: what counts is how many
        // consecutive bytes of a row one XCD takes at a time, and 2 KiB is the best (measured over
        // three placements of each arena, both directions): strips of 128 columns in runs of 4
        // (c2 +1.5 %, c3 +3 %, 20 and 30 workers +2.4 %), strips of 64 columns in runs of 8 (64
        // workers +6 %, c4 +1 %), strips of 256 columns and more as they come (c5: runs of 4 lose
        // 2.4 %); runs that are not powers of two and longer runs lose everywhere (the L2 ->
        // fabric request stalls double).
        const int order = g_slab_order.load();
        const bool any_tiled = a.tile_shift != 0 || a.dst_tile_shift != 0;
        if (order == 2) a.strips_per_xcd = (a.nstrips + combo::kXcds - 1) / combo::kXcds;
        else if (order >= 3) a.strips_per_xcd = (uint32_t)order;   // runs of this many strips
        else if (order == 0 && any_tiled) a.strips_per_xcd = tile_run(N, P);
        else if (order == 0 && plan.cols <= 128) a.strips_per_xcd = (uint32_t)(512 / plan.cols);
        if (combo::slab_grid(a, plan.cols) == 0) return COMBO_ERANGE;   // work-items per grid dimension
    }
    a.hash_sr = hash_sr;
    if (hashed)
        return combo::launch_round_slab_hashed(a, plan.cols, st) == hipSuccess ? COMBO_OK : COMBO_EHIP;
    if (plan.kind == kPlanSlab)
        return combo::launch_round_slab(a, plan.cols, st) == hipSuccess ? COMBO_OK : COMBO_EHIP;
    if (status != nullptr)
        return combo::launch_round_dynamic_elementwise(a, st) == hipSuccess ? COMBO_OK : COMBO_EHIP;
    if (combo::round_grid_size(N, P, tile_cols, swizzle) == 0) return COMBO_ERANGE;
    const bool vec = aligned16(dst) && aligned16(src) && (ld % 4 == 0);
    return combo::launch_round(a, tile_cols, vec, st) == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

// Which kernel runs this round.  The slab kernels need 16-byte aligned buffers, a pitch
// that is a multiple of 4 and a slab that fits; everything else goes to the row-tile kernel.
Plan plan_for(const float* dst, const float* src, const float* grad, int64_t ld, int32_t N,
              int64_t P, int32_t R) {
    const Plan tile{kPlanTile, 0};
    const int want = g_kernel.load();
    if (want == 1) return tile;
    if (!(aligned16(dst) && aligned16(src) && aligned16(grad) && ld % 4 == 0)) return tile;
    const int W = combo::slab_strip_cols(N, R, g_slab_cols.load());
    if (W == 0 || ((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W > kMaxStrips) return tile;
    return Plan{kPlanSlab, W};
}

}  // namespace

extern "C" {

int combo_make_peer_table(int32_t* d_peers, int32_t N, int32_t S, int32_t R, uint64_t seed,
                          uint64_t round, void* stream) {
    if (N < 1 || S < 1 || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (R == 0) return COMBO_OK;                       // empty table
    if (d_peers == nullptr) return COMBO_EINVAL;
    if (N > 16384 || (uint64_t)N * (uint64_t)S > 0x7FFFFFFFull) return COMBO_ERANGE;
    const hipError_t e = combo::launch_peer_table(d_peers, N, S, R, seed, round,
                                                  (hipStream_t)stream);
    return e == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_make_peer_table_pooled(int32_t* d_peers, int32_t N, int32_t S, int32_t R, uint64_t seed,
                                 uint64_t round, void* stream) {
    if (N < 1 || S < 1 || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (R == 0) return COMBO_OK;
    if (d_peers == nullptr) return COMBO_EINVAL;
    if (N > 16384) return COMBO_ERANGE;
    const hipError_t e = combo::launch_peer_table_pooled(d_peers, N, S, R, seed, round,
                                                         (hipStream_t)stream);
    return e == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_peer_in_degree(int32_t* d_degree, const int32_t* d_peers, int32_t N, int32_t S, int32_t R,
                         void* stream) {
    if (N < 1 || S < 1 || R < 0 || d_degree == nullptr) return COMBO_EINVAL;
    if (R > 0 && d_peers == nullptr) return COMBO_EINVAL;
    if (N > 16384) return COMBO_ERANGE;
    const uint64_t entries = (uint64_t)N * (uint64_t)S * (uint64_t)R;
    const hipError_t e = combo::launch_peer_in_degree(d_degree, d_peers, N, entries,
                                                      (hipStream_t)stream);
    return e == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_segment_gossip_round(float* d_dst, const float* d_src, int64_t ld,
                               const int32_t* d_peers, const float* d_dataset_sizes, int32_t N,
                               int64_t P, int32_t S, int32_t R, void* stream) {
    int rc = check_round_args(d_dst, d_src, ld, d_peers, N, P, S, R);
    if (rc == COMBO_OK)
        rc = check_small_inputs(d_dst, (uint64_t)N * (uint64_t)ld * 4, d_peers, d_dataset_sizes, nullptr, N, S, R);
    if (rc != COMBO_OK) return rc;
    const Plan plan = plan_for(d_dst, d_src, nullptr, ld, N, P, R);
    return enqueue_round(d_dst, d_src, nullptr, 0.0f, ld, d_peers, d_dataset_sizes, N, P, S, R, plan,
                         (hipStream_t)stream);
}

int combo_make_peer_table_dynamic(int32_t* d_peers, const uint8_t* d_status, int32_t N, int32_t S,
                                  int32_t R, uint64_t seed, uint64_t round, void* stream) {
    if (N < 1 || S < 1 || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (R == 0) return COMBO_OK;
    if (d_peers == nullptr || d_status == nullptr) return COMBO_EINVAL;
    if (N > 16384 || (uint64_t)N * (uint64_t)S > 0x7FFFFFFFull) return COMBO_ERANGE;
    const hipError_t e = combo::launch_peer_table_dynamic(d_peers, d_status, N, S, R, seed, round,
                                                          (hipStream_t)stream);
    return e == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_segment_gossip_round_dynamic(float* d_dst, const float* d_src, int64_t ld,
                                       const int32_t* d_peers, const float* d_dataset_sizes,
                                       const uint8_t* d_status, int32_t N, int64_t P, int32_t S,
                                       int32_t R, void* stream) {
    int rc = check_round_args(d_dst, d_src, ld, d_peers, N, P, S, R);
    if (rc != COMBO_OK) return rc;
    if (d_status == nullptr) return COMBO_EINVAL;
    rc = check_small_inputs(d_dst, (uint64_t)N * (uint64_t)ld * 4, d_peers, d_dataset_sizes, d_status, N, S, R);
    if (rc != COMBO_OK) return rc;
    const Plan plan = plan_for(d_dst, d_src, nullptr, ld, N, P, R);
    if (plan.kind == kPlanTile && ((uint64_t)P + 1023) / 1024 * (uint64_t)N > 0x7FFFFFFFull)
        return COMBO_ERANGE;
    return enqueue_round(d_dst, d_src, nullptr, 0.0f, ld, d_peers, d_dataset_sizes, N, P, S, R, plan,
                         (hipStream_t)stream, d_status);
}

int combo_local_sgd_steps_then_gossip(float* d_dst, float* d_src, const float* d_grads, int32_t tau,
                                      float lr, int64_t ld, const int32_t* d_peers,
                                      const float* d_dataset_sizes, int32_t N, int64_t P, int32_t S,
                                      int32_t R, void* stream) {
    int rc = check_round_args(d_dst, d_src, ld, d_peers, N, P, S, R);
    if (rc != COMBO_OK) return rc;
    if (tau < 0 || (tau > 0 && d_grads == nullptr)) return COMBO_EINVAL;
    const uint64_t bytes = (uint64_t)N * (uint64_t)ld * sizeof(float);
    if (tau > 0 && bytes > UINT64_MAX / (uint64_t)tau) return COMBO_ERANGE;
    if (tau > 0 && (overlaps(d_grads, bytes * (uint64_t)tau, d_src, bytes) ||
                    overlaps(d_grads, bytes * (uint64_t)tau, d_dst, bytes)))
        return COMBO_EALIAS;
    rc = check_small_inputs(d_dst, bytes, d_peers, d_dataset_sizes, nullptr, N, S, R);
    if (rc != COMBO_OK) return rc;
    const hipStream_t st = (hipStream_t)stream;
    const Plan plan = plan_for(d_dst, d_src, d_grads, ld, N, P, R);
    if (tau == 0)   // no local step: the plain round
        return enqueue_round(d_dst, d_src, nullptr, 0.0f, ld, d_peers, d_dataset_sizes, N, P, S, R,
                             plan, st);
    if (plan.kind != kPlanTile && g_fused_mode.load() == 0)   // steps folded into the slab fill
        return enqueue_round(d_dst, d_src, d_grads, lr, ld, d_peers, d_dataset_sizes, N, P, S, R,
                             plan, st, nullptr, tau);
    // separate passes: step every row in place tau times, then the plain round
    if ((plan.kind == kPlanTile &&
         combo::round_grid_size(N, P, row_tile_cols(N, P), g_swizzle.load() != 0) == 0) ||
        combo::round_grid_size(N, P, 4096, false) == 0)
        return COMBO_ERANGE;
    const bool vec = aligned16(d_src) && aligned16(d_grads) && (ld % 4 == 0);
    for (int32_t t = 0; t < tau; ++t)
        if (combo::launch_sgd_step(d_src, d_grads + (size_t)t * (size_t)N * (size_t)ld, lr, ld, N, P,
                                   vec, st) != hipSuccess)
            return COMBO_EHIP;
    return enqueue_round(d_dst, d_src, nullptr, 0.0f, ld, d_peers, d_dataset_sizes, N, P, S, R, plan,
                         st);
}

int combo_local_sgd_then_gossip(float* d_dst, float* d_src, const float* d_grad, float lr,
                                int64_t ld, const int32_t* d_peers, const float* d_dataset_sizes,
                                int32_t N, int64_t P, int32_t S, int32_t R, void* stream) {
    if (d_grad == nullptr) return COMBO_EINVAL;
    return combo_local_sgd_steps_then_gossip(d_dst, d_src, d_grad, 1, lr, ld, d_peers,
                                             d_dataset_sizes, N, P, S, R, stream);
}

// ---- tiled arena layout ---------------------------------------------------------------
namespace {

bool tile_cols_ok(int tile_cols) {
    return tile_cols >= 8 && tile_cols <= 1024 && (tile_cols & (tile_cols - 1)) == 0;
}

// Tile order of the conversion kernels, under the slab kernel's knob: the XCDs take turns at
// runs of 16 tiles (measured against tile i to workgroup i: pack +2-7 %, unpack +3-6 % on c2
// and c3, -2 % on c5).
uint32_t relayout_run(uint64_t tiles, int32_t N, int64_t P) {
    const int order = g_slab_order.load();
    if (order == 1) return 0;
    if (order == 2) return (uint32_t)((tiles + combo::kXcds - 1) / combo::kXcds);
    return order >= 3 ? (uint32_t)order : tile_run(N, P);
}

int64_t tiled_elems(int32_t N, int64_t P, int tile_cols) {
    return (P + tile_cols - 1) / tile_cols * (int64_t)N * (int64_t)tile_cols;
}

// argument checks shared by the tiled aggregation entry points
int check_tiled_args(const float* dst, const float* src, int32_t tile_cols, const int32_t* peers,
                     int32_t N, int64_t P, int32_t S, int32_t R) {
    if (N < 1 || S < 1 || P < 1 || (int64_t)S > P || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (!tile_cols_ok(tile_cols) || dst == nullptr || src == nullptr) return COMBO_EINVAL;
    if (R > 0 && peers == nullptr) return COMBO_EINVAL;
    if (!aligned16(dst) || !aligned16(src)) return COMBO_EINVAL;
    const uint64_t bytes = (uint64_t)tiled_elems(N, P, tile_cols) * sizeof(float);
    if (overlaps(dst, bytes, src, bytes)) return COMBO_EALIAS;
    if (combo::slab_strip_cols(N, R, tile_cols) != tile_cols) return COMBO_ERANGE;   // slab too big
    if (((uint64_t)P + (uint64_t)tile_cols - 1) / (uint64_t)tile_cols > kMaxStrips)
        return COMBO_ERANGE;
    return COMBO_OK;
}

}  // namespace

int64_t combo_tiled_elems(int32_t N, int64_t P, int32_t tile_cols) {
    if (N < 1 || P < 1 || !tile_cols_ok(tile_cols)) return COMBO_EINVAL;
    return tiled_elems(N, P, tile_cols);
}

int32_t combo_tiled_cols(int32_t N, int32_t R) {
    if (N < 1 || R < 0) return COMBO_EINVAL;
    // Up to 8 replicas: the narrowest power of two (from 64 columns) whose tile reaches 8 KiB, so
    // tiles of 8 KiB to just under 16 KiB for N <= 32.  Measured on MI355X: 8 KiB where N is a
    // power of two; for other N the next width down leaves 4-8 KiB tiles, which are 2-18 % slower
    // than the 8-16 KiB ones (20 workers: 5 KiB 5.2 TB/s, 10 KiB 6.1; 30 workers: 7.5 KiB 6.14,
    // 15 KiB 6.26; 12 workers: 6 KiB 5.85, 12 KiB 6.17).  More than 8 replicas: the widest tile
    // within 32 KiB.  For more workers keep the chunk as wide as a slab of at most 32 KiB allows
    // (64 columns up to N = 128, 32 up to 256, 16 up to 512, then 8): a tile is one contiguous
    // block whatever its width, so narrow tiles keep many-worker arenas on the LDS-slab kernel
    const int64_t budget = (int64_t)combo::slab_budget_bytes(R, true);
    if (R <= 8) {
        for (int W = 64; W <= 1024; W <<= 1) {
            const int64_t bytes = (int64_t)N * W * 4;
            if ((bytes >= budget || W == 1024) && bytes <= 32 * 1024 && combo::slab_strip_cols(N, R, W) == W)
                return W;
        }
    } else {
        for (int W = 1024; W >= 64; W >>= 1)
            if ((int64_t)N * W * 4 <= budget && combo::slab_strip_cols(N, R, W) == W) return W;
    }
    for (int W = 64; W >= 8; W >>= 1)
        if ((int64_t)N * W * 4 <= 32 * 1024 && combo::slab_strip_cols(N, R, W) == W) return W;
    return combo::slab_strip_cols(N, R, 8) == 8 ? 8 : COMBO_ERANGE;
}

int combo_pack_tiled(float* d_tiled, const float* d_rows, int64_t ld, int32_t N, int64_t P,
                     int32_t tile_cols, void* stream) {
    if (N < 1 || P < 1 || ld < P || !tile_cols_ok(tile_cols) || d_tiled == nullptr ||
        d_rows == nullptr)
        return COMBO_EINVAL;
    if (overlaps(d_tiled, (uint64_t)tiled_elems(N, P, tile_cols) * 4, d_rows,
                 (uint64_t)N * (uint64_t)ld * 4))
        return COMBO_EALIAS;
    return combo::launch_pack_tiled(d_tiled, d_rows, ld, N, P, tile_cols,
                                    relayout_run(((uint64_t)P + tile_cols - 1) / tile_cols, N, P), (hipStream_t)stream) ==
                   hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_unpack_tiled(float* d_rows, int64_t ld, const float* d_tiled, int32_t N, int64_t P,
                       int32_t tile_cols, void* stream) {
    if (N < 1 || P < 1 || ld < P || !tile_cols_ok(tile_cols) || d_tiled == nullptr ||
        d_rows == nullptr)
        return COMBO_EINVAL;
    if (overlaps(d_tiled, (uint64_t)tiled_elems(N, P, tile_cols) * 4, d_rows,
                 (uint64_t)N * (uint64_t)ld * 4))
        return COMBO_EALIAS;
    return combo::launch_unpack_tiled(d_rows, ld, d_tiled, N, P, tile_cols,
                                    relayout_run(((uint64_t)P + tile_cols - 1) / tile_cols, N, P), (hipStream_t)stream) ==
                   hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_segment_gossip_round_tiled(float* d_dst, const float* d_src, int32_t tile_cols,
                                     const int32_t* d_peers, const float* d_dataset_sizes,
                                     const uint8_t* d_status, int32_t N, int64_t P, int32_t S,
                                     int32_t R, void* stream) {
    int rc = check_tiled_args(d_dst, d_src, tile_cols, d_peers, N, P, S, R);
    if (rc == COMBO_OK)
        rc = check_small_inputs(d_dst, (uint64_t)tiled_elems(N, P, tile_cols) * 4, d_peers, d_dataset_sizes,
                                d_status, N, S, R);
    if (rc != COMBO_OK) return rc;
    return enqueue_round(d_dst, d_src, nullptr, 0.0f, tile_cols, d_peers, d_dataset_sizes, N, P, S, R,
                         Plan{kPlanSlab, tile_cols}, (hipStream_t)stream, d_status, 1, tile_cols);
}

int combo_local_sgd_steps_then_gossip_tiled(float* d_dst, const float* d_src, const float* d_grads,
                                            int32_t tau, float lr, int32_t tile_cols,
                                            const int32_t* d_peers, const float* d_dataset_sizes,
                                            int32_t N, int64_t P, int32_t S, int32_t R, void* stream) {
    int rc = check_tiled_args(d_dst, d_src, tile_cols, d_peers, N, P, S, R);
    if (rc == COMBO_OK)
        rc = check_small_inputs(d_dst, (uint64_t)tiled_elems(N, P, tile_cols) * 4, d_peers, d_dataset_sizes,
                                nullptr, N, S, R);
    if (rc != COMBO_OK) return rc;
    if (tau < 0 || (tau > 0 && (d_grads == nullptr || !aligned16(d_grads)))) return COMBO_EINVAL;
    const uint64_t bytes = (uint64_t)tiled_elems(N, P, tile_cols) * sizeof(float);
    if (tau > 0 && (overlaps(d_grads, bytes * (uint64_t)tau, d_src, bytes) ||
                    overlaps(d_grads, bytes * (uint64_t)tau, d_dst, bytes)))
        return COMBO_EALIAS;
    return enqueue_round(d_dst, d_src, tau > 0 ? d_grads : nullptr, lr, tile_cols, d_peers,
                         d_dataset_sizes, N, P, S, R, Plan{kPlanSlab, tile_cols}, (hipStream_t)stream,
                         nullptr, tau, tile_cols);
}

int combo_round_relayout(float* d_dst, int64_t dst_ld, int32_t dst_tile_cols, const float* d_src,
                         int64_t src_ld, int32_t src_tile_cols, const float* d_grads, int32_t tau,
                         float lr, const int32_t* d_peers, const float* d_dataset_sizes,
                         const uint8_t* d_status, int32_t N, int64_t P, int32_t S, int32_t R,
                         void* stream) {
    if (N < 1 || S < 1 || P < 1 || (int64_t)S > P || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (d_dst == nullptr || d_src == nullptr || (R > 0 && d_peers == nullptr)) return COMBO_EINVAL;
    if (tau < 0 || (tau > 0 && d_grads == nullptr)) return COMBO_EINVAL;
    if (src_tile_cols != 0 && !tile_cols_ok(src_tile_cols)) return COMBO_EINVAL;
    if (dst_tile_cols != 0 && !tile_cols_ok(dst_tile_cols)) return COMBO_EINVAL;
    if (src_tile_cols == 0 && src_ld < P) return COMBO_EINVAL;
    if (dst_tile_cols == 0 && dst_ld < P) return COMBO_EINVAL;
    if (d_status != nullptr && tau > 0) return COMBO_ERANGE;   // no kernel folds steps into a dynamic round
    // one strip of the slab kernel = one tile of the tiled side(s)
    if (src_tile_cols != 0 && dst_tile_cols != 0 && src_tile_cols != dst_tile_cols) return COMBO_ERANGE;
    if ((src_tile_cols == 0 && ((uint64_t)src_ld > (UINT64_MAX / 4) / (uint64_t)N || src_ld % 4 != 0)) ||
        (dst_tile_cols == 0 && ((uint64_t)dst_ld > (UINT64_MAX / 4) / (uint64_t)N || dst_ld % 4 != 0)))
        return COMBO_ERANGE;
    if (!aligned16(d_dst) || !aligned16(d_src) || !aligned16(d_grads)) return COMBO_ERANGE;
    const int tile = src_tile_cols != 0 ? src_tile_cols : dst_tile_cols;
    const int W = combo::slab_strip_cols(N, R, tile ? tile : g_slab_cols.load());
    if (W == 0 || (tile != 0 && W != tile)) return COMBO_ERANGE;          // slab does not fit in LDS
    if (((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W > kMaxStrips) return COMBO_ERANGE;
    const uint64_t src_bytes = 4 * (src_tile_cols ? (uint64_t)tiled_elems(N, P, src_tile_cols)
                                                  : (uint64_t)N * (uint64_t)src_ld);
    const uint64_t dst_bytes = 4 * (dst_tile_cols ? (uint64_t)tiled_elems(N, P, dst_tile_cols)
                                                  : (uint64_t)N * (uint64_t)dst_ld);
    if (overlaps(d_dst, dst_bytes, d_src, src_bytes)) return COMBO_EALIAS;
    if (tau > 0 && src_bytes > UINT64_MAX / (uint64_t)tau) return COMBO_ERANGE;
    if (tau > 0 && (overlaps(d_grads, src_bytes * (uint64_t)tau, d_src, src_bytes) ||
                    overlaps(d_grads, src_bytes * (uint64_t)tau, d_dst, dst_bytes)))
        return COMBO_EALIAS;
    const int rc = check_small_inputs(d_dst, dst_bytes, d_peers, d_dataset_sizes, d_status, N, S, R);
    if (rc != COMBO_OK) return rc;
    const Layout dst_layout{dst_tile_cols ? (int64_t)dst_tile_cols : dst_ld, dst_tile_cols};
    return enqueue_round(d_dst, d_src, tau > 0 ? d_grads : nullptr, lr,
                         src_tile_cols ? (int64_t)src_tile_cols : src_ld, d_peers, d_dataset_sizes, N, P,
                         S, R, Plan{kPlanSlab, W}, (hipStream_t)stream, d_status, tau, src_tile_cols,
                         false, 0, &dst_layout);
}

int combo_round_hashed(float* d_dst, const float* d_src, const float* d_grads, int32_t tau, float lr,
                       int64_t ld, int32_t tile_cols, const float* d_dataset_sizes, int32_t N,
                       int64_t P, int32_t S, int32_t R, uint64_t seed, uint64_t round, void* stream) {
    if (N < 1 || S < 1 || P < 1 || (int64_t)S > P || R < 0 || R > N - 1) return COMBO_EINVAL;
    if (d_dst == nullptr || d_src == nullptr || tau < 0 || (tau > 0 && d_grads == nullptr))
        return COMBO_EINVAL;
    if (R > combo::kMaxHashedR) return COMBO_ERANGE;
    uint64_t elems;
    int W;
    if (tile_cols != 0) {
        if (!tile_cols_ok(tile_cols)) return COMBO_EINVAL;
        elems = (uint64_t)tiled_elems(N, P, tile_cols);
        W = tile_cols;
        if (combo::slab_strip_cols(N, R, W, true) != W) return COMBO_ERANGE;
    } else {
        if (ld < P) return COMBO_EINVAL;
        elems = (uint64_t)N * (uint64_t)ld;
        W = combo::slab_strip_cols(N, R, g_slab_cols.load(), true);
        if (W == 0 || ld % 4 != 0) return COMBO_ERANGE;
    }
    if (!aligned16(d_dst) || !aligned16(d_src) || !aligned16(d_grads)) return COMBO_ERANGE;
    if (((uint64_t)P + (uint64_t)W - 1) / (uint64_t)W > kMaxStrips) return COMBO_ERANGE;
    const uint64_t bytes = elems * sizeof(float);
    if (overlaps(d_dst, bytes, d_src, bytes)) return COMBO_EALIAS;
    if (tau > 0 && (overlaps(d_grads, bytes * (uint64_t)tau, d_src, bytes) ||
                    overlaps(d_grads, bytes * (uint64_t)tau, d_dst, bytes)))
        return COMBO_EALIAS;
    const uint64_t h_sr = combo::hash_take_in(combo::hash_finalise(seed + combo::kHashGamma), round);
    return enqueue_round(d_dst, d_src, tau > 0 ? d_grads : nullptr, lr, tile_cols ? tile_cols : ld,
                         nullptr, d_dataset_sizes, N, P, S, R, Plan{kPlanSlab, W}, (hipStream_t)stream,
                         nullptr, tau, tile_cols, true, h_sr);
}

int64_t combo_aggregation_divergence_workspace(int32_t N, int64_t P) {
    if (N < 1 || P < 1) return COMBO_EINVAL;
    if (combo::divergence_strip_cols(N) == 0) return COMBO_ERANGE;
    // one partial per workgroup and row
    return (int64_t)combo::kDivPartialsPerRow * (int64_t)N * (int64_t)sizeof(double);
}

namespace {

// argument checks shared by the divergence entry points; tile_cols == 0: row-major.
// *strip receives the strip width of the workgroup kernel.
int check_divergence_args(const double* d_dist2, const float* d_x, int64_t ld, int32_t tile_cols,
                          int32_t N, int64_t P, int* strip) {
    if (N < 1 || P < 1 || d_dist2 == nullptr || d_x == nullptr) return COMBO_EINVAL;
    int W = combo::divergence_strip_cols(N);
    if (W == 0) return COMBO_ERANGE;
    if (tile_cols != 0) {
        if (!tile_cols_ok(tile_cols) || !aligned16(d_x)) return COMBO_EINVAL;
        if (W < tile_cols) W = tile_cols;             // a strip spans W / tile_cols whole tiles
        if (!combo::divergence_width_ok(N, W)) return COMBO_ERANGE;
    } else if (ld < P) {
        return COMBO_EINVAL;
    }
    *strip = W;
    return COMBO_OK;
}

// the divergence kernels behind every divergence entry point (arguments already checked)
int enqueue_divergence(double* d_dist2, const float* d_x, int64_t ld, int32_t tile_cols,
                       const float* d_dataset_sizes, int32_t N, int64_t P, int W, void* d_workspace,
                       int64_t workspace_bytes, hipStream_t st) {
    const int64_t need = combo_aggregation_divergence_workspace(N, P);
    if (need < 0) return (int)need;
    if (d_workspace == nullptr || workspace_bytes < need || ((uintptr_t)d_workspace & 7u) != 0)
        return COMBO_EINVAL;
    hipError_t e;
    if (tile_cols == 0)
        e = combo::launch_divergence(d_dist2, (double*)d_workspace, d_x, ld, d_dataset_sizes, N, P, W,
                                     aligned16(d_x) && (ld % 4 == 0), 0, st);
    else if (combo::divergence_tile_fits(N, tile_cols))   // small tiles: one wavefront per tile
        e = combo::launch_divergence_tiles(d_dist2, (double*)d_workspace, d_x, d_dataset_sizes, N, P,
                                           tile_cols, st);
    else
        e = combo::launch_divergence(d_dist2, (double*)d_workspace, d_x, tile_cols, d_dataset_sizes,
                                     N, P, W, true, tile_cols, st);
    return e == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

}  // namespace

int combo_aggregation_divergence(double* d_dist2, const float* d_x, int64_t ld,
                                 const float* d_dataset_sizes, int32_t N, int64_t P,
                                 void* d_workspace, int64_t workspace_bytes, void* stream) {
    int W = 0;
    const int rc = check_divergence_args(d_dist2, d_x, ld, 0, N, P, &W);
    if (rc != COMBO_OK) return rc;
    return enqueue_divergence(d_dist2, d_x, ld, 0, d_dataset_sizes, N, P, W, d_workspace,
                              workspace_bytes, (hipStream_t)stream);
}

int combo_aggregation_divergence_tiled(double* d_dist2, const float* d_x, int32_t tile_cols,
                                       const float* d_dataset_sizes, int32_t N, int64_t P,
                                       void* d_workspace, int64_t workspace_bytes, void* stream) {
    if (tile_cols == 0) return COMBO_EINVAL;
    int W = 0;
    const int rc = check_divergence_args(d_dist2, d_x, 0, tile_cols, N, P, &W);
    if (rc != COMBO_OK) return rc;
    return enqueue_divergence(d_dist2, d_x, 0, tile_cols, d_dataset_sizes, N, P, W, d_workspace,
                              workspace_bytes, (hipStream_t)stream);
}

static_assert(COMBO_DIVERGENCE_NOALLOC_MAX_WORKERS == combo::kDivStaticRows,
              "the header's limit is the number of rows the held array has room for");

int combo_aggregation_divergence_noalloc(double* d_dist2, const float* d_x, int64_t ld,
                                         int32_t tile_cols, const float* d_dataset_sizes, int32_t N,
                                         int64_t P, void* stream) {
    int W = 0;
    const int rc = check_divergence_args(d_dist2, d_x, ld, tile_cols, N, P, &W);
    if (rc != COMBO_OK) return rc;
    if (N > COMBO_DIVERGENCE_NOALLOC_MAX_WORKERS) return COMBO_ERANGE;   // beyond the held array
    double* held = nullptr;
    int64_t held_bytes = 0;
    if (combo::divergence_static_workspace(&held, &held_bytes) != hipSuccess) return COMBO_EHIP;
    return enqueue_divergence(d_dist2, d_x, ld, tile_cols, d_dataset_sizes, N, P, W, held, held_bytes,
                              (hipStream_t)stream);
}

int combo_bandwidth_probe(int kind, float* d_dst, const float* d_src, int32_t N, int64_t ld, int64_t P,
                          int32_t cols, int32_t param, void* stream) {
    if (kind < COMBO_PROBE_COPY || kind > COMBO_PROBE_LDS_READ) return COMBO_EINVAL;
    if (N < 1 || P < 1 || ld < P || d_dst == nullptr) return COMBO_EINVAL;
    if (kind != COMBO_PROBE_WRITE && kind != COMBO_PROBE_LDS_READ && d_src == nullptr) return COMBO_EINVAL;
    if (!aligned16(d_dst) || !aligned16(d_src) || ld % 4 != 0) return COMBO_EINVAL;
    if ((uint64_t)ld > (UINT64_MAX / 4) / (uint64_t)N) return COMBO_ERANGE;
    const uint64_t bytes = (uint64_t)N * (uint64_t)ld * 4;
    if (d_src != nullptr && overlaps(d_dst, bytes, d_src, bytes)) return COMBO_EALIAS;
    const hipError_t e = combo::launch_bandwidth_probe(kind, d_dst, d_src, N, ld, P, cols, param,
                                                       (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return COMBO_EINVAL;
    return e == hipSuccess ? COMBO_OK : COMBO_EHIP;
}

int combo_round_kernel_kind(int32_t N, int32_t R) {
    if (N < 1 || R < 0) return COMBO_EINVAL;
    if (g_kernel.load() == 1) return 0;
    return combo::slab_strip_cols(N, R, g_slab_cols.load()) != 0 ? 1 : 0;
}

int combo_tune(int key, int value) {
    switch (key) {
        case COMBO_TUNE_TILE_COLS:
            if (value != 0 && value != 1024 && value != 2048 && value != 4096) return COMBO_EINVAL;
            g_tile_cols.store(value);
            return COMBO_OK;
        case COMBO_TUNE_XCD_SWIZZLE:
            if (value != 0 && value != 1) return COMBO_EINVAL;
            g_swizzle.store(value);
            return COMBO_OK;
        case COMBO_TUNE_FUSED_MODE:
            if (value != 0 && value != 1) return COMBO_EINVAL;
            g_fused_mode.store(value);
            return COMBO_OK;
        case COMBO_TUNE_KERNEL:
            if (value < 0 || value > 2) return COMBO_EINVAL;
            g_kernel.store(value);
            return COMBO_OK;
        case COMBO_TUNE_SLAB_COLS:
            if (value != 0 && !(value >= 64 && value <= 1024 && (value & (value - 1)) == 0))
                return COMBO_EINVAL;
            g_slab_cols.store(value);
            return COMBO_OK;
        case COMBO_TUNE_SLAB_ORDER:
            if (value < 0 || value > (1 << 24)) return COMBO_EINVAL;
            g_slab_order.store(value);
            return COMBO_OK;
        case COMBO_TUNE_SLAB_THREADS:
            if (value != 0 && value != 256 && value != 512) return COMBO_EINVAL;
            combo::set_slab_threads(value);
            return COMBO_OK;
        case COMBO_TUNE_SLAB_LDS_FLOOR:
            if (value < 0 || value > 64 * 1024) return COMBO_EINVAL;
            combo::set_slab_lds_floor(value);
            return COMBO_OK;
        default:
            return COMBO_EINVAL;
    }
}

int combo_get_tune(int key) {
    switch (key) {
        case COMBO_TUNE_TILE_COLS: return g_tile_cols.load();
        case COMBO_TUNE_XCD_SWIZZLE: return g_swizzle.load();
        case COMBO_TUNE_FUSED_MODE: return g_fused_mode.load();
        case COMBO_TUNE_KERNEL: return g_kernel.load();
        case COMBO_TUNE_SLAB_COLS: return g_slab_cols.load();
        case COMBO_TUNE_SLAB_ORDER: return g_slab_order.load();
        case COMBO_TUNE_SLAB_THREADS: return combo::get_slab_threads();
        case COMBO_TUNE_SLAB_LDS_FLOOR: return combo::get_slab_lds_floor();
        default: return COMBO_EINVAL;
    }
}

const char* combo_strerror(int status) {
    switch (status) {
        case COMBO_OK: return "success";
        case COMBO_EINVAL: return "invalid argument (size out of range or required pointer is NULL)";
        case COMBO_EALIAS: return "buffers overlap: the round needs disjoint front, back and gradient buffers";
        case COMBO_ERANGE: return "argument beyond the supported range (grid or LDS limit)";
        case COMBO_EHIP: return "the HIP runtime reported an error while enqueuing";
        default: return "unknown combo status";
    }
}

}  // extern "C"
