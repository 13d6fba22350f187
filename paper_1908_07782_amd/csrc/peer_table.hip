// Peer selection kernel (Sec. 4.1 step 2 of the segmented-gossip paper: R targets per
// segment, chosen at random among the other workers, without replacement).
//
// One wavefront per (worker, segment).  The N-1 candidates live in LDS as the array of
// a Fisher-Yates shuffle; the lanes initialise it together, then lane 0 performs the R
// dependent swap steps, each driven by one word of the counter-based hash, and writes
// the chosen worker ids straight to the table.  The table is tiny (at most a few
// thousand entries per round), so the kernel is launch-latency bound by construction;
// what matters is that it is a pure function of (seed, round, w, s, j).
#include "combo_internal.h"

namespace combo {
namespace {

constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;   // SplitMix64 increment

__device__ __forceinline__ uint64_t finalise(uint64_t z) {
    // output function of SplitMix64: two xor-shift-multiply rounds and a last xor-shift
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint64_t take_in(uint64_t h, uint64_t counter) {
    return finalise((h ^ counter) + kGamma);
}

__global__ __launch_bounds__(64) void peer_table_kernel(int32_t* __restrict__ peers, int32_t N,
                                                        int32_t S, int32_t R, uint64_t seed,
                                                        uint64_t round) {
    extern __shared__ int32_t cand[];            // N-1 candidate slots
    const int32_t M = N - 1;
    const uint32_t pair = blockIdx.x;            // = w*S + s
    const int32_t w = (int32_t)(pair / (uint32_t)S);
    const int32_t s = (int32_t)(pair - (uint32_t)w * (uint32_t)S);

    for (int32_t i = (int32_t)threadIdx.x; i < M; i += 64) cand[i] = i;
    __syncthreads();

    if (threadIdx.x == 0) {
        uint64_t h = finalise(seed + kGamma);
        h = take_in(h, round);
        h = take_in(h, (uint64_t)w);
        h = take_in(h, (uint64_t)s);
        int32_t* out = peers + (size_t)pair * (size_t)R;
        for (int32_t j = 0; j < R; ++j) {
            const uint64_t word = take_in(h, (uint64_t)j);
            const uint32_t span = (uint32_t)(M - j);
            const int32_t r = j + (int32_t)(((word >> 32) * (uint64_t)span) >> 32);
            const int32_t picked = cand[r];
            cand[r] = cand[j];
            cand[j] = picked;
            out[j] = picked + (picked >= w ? 1 : 0);     // skip over w itself
        }
    }
}

}  // namespace

hipError_t launch_peer_table(int32_t* peers, int32_t N, int32_t S, int32_t R, uint64_t seed,
                             uint64_t round, hipStream_t st) {
    const uint32_t blocks = (uint32_t)N * (uint32_t)S;
    const size_t lds = (size_t)(N > 1 ? N - 1 : 1) * sizeof(int32_t);
    hipLaunchKernelGGL(peer_table_kernel, dim3(blocks), dim3(64), lds, st, peers, N, S, R, seed,
                       round);
    return hipGetLastError();
}

}  // namespace combo
