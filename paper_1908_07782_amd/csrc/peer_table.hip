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
#include "round_device.h"

namespace combo {
namespace {

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
        uint64_t h = hash_finalise(seed + kHashGamma);
        h = hash_take_in(h, round);
        h = hash_take_in(h, (uint64_t)w);
        h = hash_take_in(h, (uint64_t)s);
        int32_t* out = peers + (size_t)pair * (size_t)R;
        for (int32_t j = 0; j < R; ++j) {
            const uint64_t word = hash_take_in(h, (uint64_t)j);
            const uint32_t span = (uint32_t)(M - j);
            const int32_t r = j + (int32_t)(((word >> 32) * (uint64_t)span) >> 32);
            const int32_t picked = cand[r];
            cand[r] = cand[j];
            cand[j] = picked;
            out[j] = picked + (picked >= w ? 1 : 0);     // skip over w itself
        }
    }
}

// Pooled selection (Sec. 4.1 step 2 as written): all S*R requests of a worker draw from
// one queue holding a random permutation of the other workers; an empty queue is
// replaced by the next permutation; a request takes the first queue element that its
// segment has not picked yet, skipped elements keep their place.  Every permutation is
// consumed completely, so ceil(S*R / (N-1)) of them are needed: the wavefront loops over
// them; for each one all lanes fill the queue and evaluate the hash words of the
// Fisher-Yates steps in parallel (LDS, 16-bit entries), then lane 0 applies the swaps and
// serves requests until the queue is empty.  queue[head..M) are the elements still in
// the pool.
constexpr uint64_t kPoolTag = 0x706F6F6C65642121ull;

__global__ __launch_bounds__(64) void peer_table_pooled_kernel(int32_t* __restrict__ peers,
                                                               int32_t N, int32_t S, int32_t R,
                                                               uint64_t seed, uint64_t round) {
    extern __shared__ uint16_t pool_lds[];
    const int32_t M = N - 1;
    uint16_t* queue = pool_lds;                  // [M] worker ids
    uint16_t* partner = pool_lds + M;            // [M] swap partner of every shuffle step
    const int32_t w = (int32_t)blockIdx.x;
    const int lane = (int)threadIdx.x;
    uint64_t hw = hash_finalise((seed ^ kPoolTag) + kHashGamma);
    hw = hash_take_in(hw, round);
    hw = hash_take_in(hw, (uint64_t)w);

    const int64_t requests = (int64_t)S * R;
    const int64_t epochs = (requests + M - 1) / M;
    int64_t served = 0;                           // lane 0: requests done so far
    for (int64_t epoch = 0; epoch < epochs; ++epoch) {
        const uint64_t he = hash_take_in(hw, (uint64_t)epoch);
        for (int32_t i = lane; i < M; i += 64) {
            queue[i] = (uint16_t)(i + (i >= w ? 1 : 0));
            const uint64_t word = hash_take_in(he, (uint64_t)i);
            partner[i] = (uint16_t)(i + (int32_t)(((word >> 32) * (uint64_t)(uint32_t)(M - i)) >> 32));
        }
        __syncthreads();
        if (lane == 0) {
            // Fisher-Yates fixes position i at step i, and this permutation hands out at most
            // `left` elements after skipping at most R-1: later steps cannot change what is used
            const int64_t left = requests - served;
            const int32_t steps = left + R < (int64_t)(M - 1) ? (int32_t)(left + R) : M - 1;
            for (int32_t i = 0; i < steps; ++i) {
                const int32_t r = partner[i];
                const uint16_t t = queue[i];
                queue[i] = queue[r];
                queue[r] = t;
            }
            // Only the picks this segment received from EARLIER permutations can reappear in
            // the new queue (picks taken from this queue have left it): copy those once into
            // the now unused partner array and compare against them while the segment lasts.
            int32_t carried = (int32_t)(served % R);
            {
                const int32_t* seg = peers + ((size_t)w * (size_t)S) * (size_t)R + (size_t)(served - carried);
                for (int32_t k = 0; k < carried; ++k) partner[k] = (uint16_t)seg[k];
            }
            int32_t head = 0;
            while (head < M && served < requests) {
                const int32_t j = (int32_t)(served % R);
                if (j == 0) carried = 0;          // a new segment starts with an empty pick set
                int32_t* picks = peers + ((size_t)w * (size_t)S) * (size_t)R + (size_t)(served - j);
                // first pool element this segment has not picked; at most `carried` are skipped
                int32_t pos = head;
                for (; pos < M; ++pos) {
                    const uint16_t c = queue[pos];
                    bool taken = false;
                    for (int32_t k = 0; k < carried; ++k) taken = taken || (partner[k] == c);
                    if (!taken) break;
                }
                if (pos == M) pos = M - 1;        // unreachable while R <= N-1; keeps indices in range
                const uint16_t c = queue[pos];
                for (int32_t q = pos; q > head; --q) queue[q] = queue[q - 1];   // skipped keep their order
                ++head;
                picks[j] = (int32_t)c;
                ++served;
            }
        }
        __syncthreads();
    }
}

// The same selection for N <= 65, where one permutation fits the wavefront: lane l holds
// queue element l, so the queue, the swap partners and the current segment's picks live in
// registers (c2's 4096 entries: 45 us with the LDS kernel above).
//   - Shuffle: every lane tracks where ITS element goes while the swaps are replayed (one
//     cross-lane read of the partner per step), then one forward permute places the elements.
//   - Serving: only the segment that straddles the refill can meet a pick it already has, and
//     it always completes within the new permutation (it lacks at most R-1 <= M-1 picks and
//     only its own earlier picks are skipped).  Those few requests go one by one (ballot for
//     the first lane holding a candidate the segment does not have yet; skipped elements move
//     up one lane).  After that no request of this permutation can collide, so the rest of the
//     queue is handed out in order with ONE coalesced store.
__global__ __launch_bounds__(64) void peer_table_pooled_wave_kernel(int32_t* __restrict__ peers,
                                                                    int32_t N, int32_t S, int32_t R,
                                                                    uint64_t seed, uint64_t round) {
    const int32_t M = N - 1;                      // 1..64 candidates
    const int32_t w = (int32_t)blockIdx.x;
    const int lane = (int)threadIdx.x;
    uint64_t hw = hash_finalise((seed ^ kPoolTag) + kHashGamma);
    hw = hash_take_in(hw, round);
    hw = hash_take_in(hw, (uint64_t)w);

    const int64_t requests = (int64_t)S * R;
    int32_t* out = peers + (size_t)w * (size_t)S * (size_t)R;
    int64_t served = 0;
    int32_t j = 0;                                // position of the next request in its segment
    int32_t cpick = -1;                           // lane k: k-th pick of the segment in progress
    for (int64_t epoch = 0; served < requests; ++epoch) {
        const uint64_t he = hash_take_in(hw, (uint64_t)epoch);
        int32_t partner = lane;
        if (lane < M) {
            const uint64_t word = hash_take_in(he, (uint64_t)lane);
            partner = lane + (int32_t)(((word >> 32) * (uint64_t)(uint32_t)(M - lane)) >> 32);
        }
        int32_t where = lane;                     // position of the element that starts in this lane
        // Fisher-Yates: step i swaps positions i and r >= i, so position i is final after step
        // i; this permutation hands out at most `left` elements after skipping at most R-1,
        // and later steps cannot change what is used
        const int64_t left_now = requests - served;
        const int32_t steps = left_now + R < (int64_t)(M - 1) ? (int32_t)(left_now + R) : M - 1;
        for (int32_t i = 0; i < steps; ++i) {
            const int32_t r = __builtin_amdgcn_readlane(partner, i);
            where = where == i ? r : (where == r ? i : where);
        }
        // lane l sends its element (identity order, skipping w) to lane where[l]
        int32_t q = __builtin_amdgcn_ds_permute(where << 2, lane + (lane >= w ? 1 : 0));

        int32_t head = 0;                         // lanes head..M-1 are still in the pool
        // the straddling segment: its first j picks (cpick lanes 0..j-1) came from earlier permutations
        const int32_t carried = j;
        while (j != 0 && head < M && served < requests) {
            bool is_free = lane >= head && lane < M;
            for (int32_t k = 0; k < carried; ++k)
                is_free = is_free && q != __builtin_amdgcn_readlane(cpick, k);
            const uint64_t mask = __ballot(is_free);
            // never empty while R <= N-1; the fallback keeps the lane index in range
            const int32_t pos = mask != 0 ? (int32_t)__ffsll((unsigned long long)mask) - 1 : M - 1;
            const int32_t c = __builtin_amdgcn_readlane(q, pos);
            if (pos != head) {                    // skipped elements keep their order
                const int32_t below = __shfl_up(q, 1, 64);
                if (lane > head && lane <= pos) q = below;
            }
            ++head;
            if (lane == j) cpick = c;
            if (lane == 0) out[served] = c;
            ++served;
            if (++j == R) j = 0;
        }
        if (j == 0) {                             // always, while R <= N-1
            // the rest of the queue goes out in order
            const int64_t left = requests - served;
            const int32_t count = (int32_t)(left < (int64_t)(M - head) ? left : (int64_t)(M - head));
            if (lane >= head && lane < head + count) out[served + (lane - head)] = q;
            served += count;
            j = count % R;
            // picks of the segment now in progress: the last j elements handed out
            cpick = __shfl(q, head + count - j + lane, 64);
        }
    }
}

// Selection with dynamic workers (Sec. 4.2): candidates are the ACTIVE others (offline
// workers are not asked, newcomers are not yet known to anyone); an offline requester
// asks nobody.  One wavefront per (w, s): the lanes compact the candidate list into LDS
// with ballots (increasing worker order), lane 0 performs min(R, #candidates) swap steps
// of the same hashed Fisher-Yates; unused slots are -1.
__global__ __launch_bounds__(64) void peer_table_dynamic_kernel(int32_t* __restrict__ peers,
                                                                const uint8_t* __restrict__ status,
                                                                int32_t N, int32_t S, int32_t R,
                                                                uint64_t seed, uint64_t round) {
    extern __shared__ int32_t cand[];            // up to N-1 candidates
    const uint32_t pair = blockIdx.x;
    const int32_t w = (int32_t)(pair / (uint32_t)S);
    const int32_t s = (int32_t)(pair - (uint32_t)w * (uint32_t)S);
    const int lane = (int)threadIdx.x;
    int32_t* out = peers + (size_t)pair * (size_t)R;

    int32_t count = 0;
    if (status[w] != 0) {
        for (int32_t base = 0; base < N; base += 64) {
            const int32_t v = base + lane;
            const bool ok = v < N && v != w && status[v] == 1;
            const uint64_t mask = __ballot(ok);
            if (ok) cand[count + __popcll(mask & ((1ull << lane) - 1ull))] = v;
            count += (int32_t)__popcll(mask);
        }
    }
    __syncthreads();

    if (lane == 0) {
        uint64_t h = hash_finalise(seed + kHashGamma);
        h = hash_take_in(h, round);
        h = hash_take_in(h, (uint64_t)w);
        h = hash_take_in(h, (uint64_t)s);
        const int32_t take = R < count ? R : count;
        for (int32_t j = 0; j < take; ++j) {
            const uint64_t word = hash_take_in(h, (uint64_t)j);
            const int32_t r = j + (int32_t)(((word >> 32) * (uint64_t)(uint32_t)(count - j)) >> 32);
            const int32_t picked = cand[r];
            cand[r] = cand[j];
            cand[j] = picked;
            out[j] = picked;
        }
        for (int32_t j = take; j < R; ++j) out[j] = -1;
    }
}

// Serve load: deg[v] = number of requests (w, s, j) whose target is v.  One workgroup,
// LDS histogram, integer atomics (the result does not depend on their order).
__global__ __launch_bounds__(1024) void peer_in_degree_kernel(int32_t* __restrict__ deg,
                                                              const int32_t* __restrict__ peers,
                                                              int32_t N, uint64_t entries) {
    extern __shared__ int32_t hist[];
    for (int32_t i = threadIdx.x; i < N; i += 1024) hist[i] = 0;
    __syncthreads();
    for (uint64_t i = threadIdx.x; i < entries; i += 1024) {
        const int32_t v = peers[i];
        if (v >= 0 && v < N) atomicAdd(&hist[v], 1);
    }
    __syncthreads();
    for (int32_t i = threadIdx.x; i < N; i += 1024) deg[i] = hist[i];
}

}  // namespace

hipError_t launch_peer_table_pooled(int32_t* peers, int32_t N, int32_t S, int32_t R, uint64_t seed,
                                    uint64_t round, hipStream_t st) {
    if (N - 1 <= 64 && R <= 64) {                 // one permutation per wavefront, all in registers
        hipLaunchKernelGGL(peer_table_pooled_wave_kernel, dim3((uint32_t)N), dim3(64), 0, st, peers, N,
                           S, R, seed, round);
        return hipGetLastError();
    }
    const size_t lds = (size_t)(N > 1 ? N - 1 : 1) * 2 * sizeof(uint16_t);
    hipLaunchKernelGGL(peer_table_pooled_kernel, dim3((uint32_t)N), dim3(64), lds, st, peers, N, S,
                       R, seed, round);
    return hipGetLastError();
}

hipError_t launch_peer_table_dynamic(int32_t* peers, const uint8_t* status, int32_t N, int32_t S,
                                     int32_t R, uint64_t seed, uint64_t round, hipStream_t st) {
    const uint32_t blocks = (uint32_t)N * (uint32_t)S;
    const size_t lds = (size_t)(N > 1 ? N - 1 : 1) * sizeof(int32_t);
    hipLaunchKernelGGL(peer_table_dynamic_kernel, dim3(blocks), dim3(64), lds, st, peers, status, N,
                       S, R, seed, round);
    return hipGetLastError();
}

hipError_t launch_peer_in_degree(int32_t* deg, const int32_t* peers, int32_t N, uint64_t entries,
                                 hipStream_t st) {
    hipLaunchKernelGGL(peer_in_degree_kernel, dim3(1), dim3(1024), (size_t)N * sizeof(int32_t), st,
                       deg, peers, N, entries);
    return hipGetLastError();
}

hipError_t launch_peer_table(int32_t* peers, int32_t N, int32_t S, int32_t R, uint64_t seed,
                             uint64_t round, hipStream_t st) {
    const uint32_t blocks = (uint32_t)N * (uint32_t)S;
    const size_t lds = (size_t)(N > 1 ? N - 1 : 1) * sizeof(int32_t);
    hipLaunchKernelGGL(peer_table_kernel, dim3(blocks), dim3(64), lds, st, peers, N, S, R, seed,
                       round);
    return hipGetLastError();
}

}  // namespace combo
