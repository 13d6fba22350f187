// Reference ("oracle") implementation of the segmented-gossip aggregation round.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-threaded
// CPU program whose only purpose is to state, as directly as possible, what the
// GPU library must compute.  It shares no source, header, table or helper with the
// HIP path and must never be linked into, imported by, or called from it.  Only the
// tests, the smoke check and the CPU-baseline leg of the benchmark may use it.
//
// What it follows (Hu, Jiang, Wang: "Decentralized Federated Learning: A Segmented
// Gossip Approach", IJCAI-19 workshop / arXiv 1908.07782):
//   * Sec. 3 "Segmented Pulling", Eq. (1): the flat parameter vector is cut into S
//     non-overlapping segments.
//   * Sec. 4.1 step (2): for every segment a worker picks R peers among the other
//     workers, at random, without replacement.
//   * Sec. 3 "Segmented Aggregation", Eq. (3): segment l of worker i becomes the
//     dataset-size-weighted mean over P_l = {i} U {the R providers of segment l}.
//   * Eq. (4): the aggregated segments are concatenated into the new model.
//   * Sec. 4.1 steps (1),(3),(4) and Sec. 5.1: the local update strictly precedes
//     serving, serving precedes aggregation, and the process is synchronous - every
//     pulled segment is the provider's post-update, pre-aggregation state.
//
// Where the paper is silent the reading taken here is spelled out next to the code.
//
// Parity status of each function ("pinned" = checked by the CPU test-suite against
// something other than itself):
//   combo_ref_segment_bounds      pinned  (closed forms, exhaustive cover checks)
//   combo_ref_mix64               pinned  (published SplitMix64 output vectors)
//   combo_ref_hash / _reduce      pinned  (hand-expanded chain of pinned mix64 calls;
//                                          exhaustive range/monotonicity checks)
//   combo_ref_make_peer_table     pinned for structure and distribution (textbook
//                                 Fisher-Yates re-run in Python on the same hash
//                                 words, permutation / distinctness / chi-square).
//                                 The VALUES of the table depend on this repository's
//                                 own choice of hash chaining: parity unpinned
//                                 externally for those.
//   combo_ref_gossip_round[_f64]  pinned  (hand-worked literal examples, dense
//                                 row-stochastic matmul, FedAvg limit, identity, ...)
//   combo_ref_local_sgd_then_gossip  pinned (lr = 0, constant-gradient closed form,
//                                 matmul of the stepped matrix)
//   combo_ref_local_sgd_steps_then_gossip  pinned (tau = 1 is the single step; tau
//                                 numpy binary32 multiply/subtract passes then the round)
//   combo_ref_make_peer_table_pooled pinned for structure (all S*R targets distinct
//                                 when they fit, serve counts differ by at most one,
//                                 independent queue re-implementation on the same hash
//                                 words); values: parity unpinned externally, as above
//   combo_ref_peer_in_degree      pinned (numpy bincount)
//   combo_ref_aggregation_divergence  pinned (numpy float64 mean / squared norms,
//                                 closed forms: identical workers, +x/-x pair)
//   combo_ref_make_peer_table_dynamic / combo_ref_gossip_round_dynamic
//                                 pinned (reduce to the static functions when every
//                                 worker is active; hand-worked examples with offline
//                                 workers and newcomers; NaN-poisoned rows that must not
//                                 be read; dense matmul)

#include <cstddef>
#include <cstdint>
#include <cmath>
#include <vector>

namespace {

// ---- Eq. (1): segment partition -------------------------------------------------
// The paper asks for segments "of the same number of parameters".  When S does not
// divide P that is impossible; the reading taken: every segment has floor(P/S)
// parameters except the last, which also takes the remainder.
inline int64_t seg_len(int64_t P, int32_t S) { return P / S; }
inline int64_t seg_lo(int64_t P, int32_t S, int32_t s) { return (int64_t)s * seg_len(P, S); }
inline int64_t seg_hi(int64_t P, int32_t S, int32_t s) {
    return (s == S - 1) ? P : (int64_t)(s + 1) * seg_len(P, S);
}

// ---- the counter-based hash -----------------------------------------------------
// The paper only says "randomly selected".  A stateless, seeded function of
// (round, worker, segment, draw) is used so that any entry of any round's table can
// be recomputed anywhere.  Building block: the output function of SplitMix64
// (Steele, Lea, Flood, OOPSLA 2014), whose generator is  state += GAMMA; return
// mix64(state).
const uint64_t GAMMA = 0x9E3779B97F4A7C15ull;

inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Start from the first SplitMix64 output for `seed`, then absorb the four counters
// one at a time: xor the counter in, advance by GAMMA, mix.
inline uint64_t absorb(uint64_t h, uint64_t c) { return mix64((h ^ c) + GAMMA); }

inline uint64_t peer_hash(uint64_t seed, uint64_t round, uint64_t w, uint64_t s, uint64_t j) {
    uint64_t h = mix64(seed + GAMMA);
    h = absorb(h, round);
    h = absorb(h, w);
    h = absorb(h, s);
    h = absorb(h, j);
    return h;
}

// Map a hash word to [0, m): multiply the top 32 bits by m and keep the top 32 bits
// of the 64-bit product.  No modulo, no rejection; bias below m / 2^32.
inline uint32_t reduce(uint64_t h, uint32_t m) {
    return (uint32_t)(((h >> 32) * (uint64_t)m) >> 32);
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------------
// Eq. (1).  lo[s], hi[s] for s in [0,S): segment s is columns [lo, hi).
// Returns 0, or -1 when S < 1 or S > P.
int combo_ref_segment_bounds(int64_t P, int32_t S, int64_t* lo, int64_t* hi) {
    if (S < 1 || (int64_t)S > P) return -1;
    for (int32_t s = 0; s < S; ++s) {
        lo[s] = seg_lo(P, S, s);
        hi[s] = seg_hi(P, S, s);
    }
    return 0;
}

uint64_t combo_ref_mix64(uint64_t z) { return mix64(z); }

uint64_t combo_ref_hash(uint64_t seed, uint64_t round, uint64_t w, uint64_t s, uint64_t j) {
    return peer_hash(seed, round, w, s, j);
}

uint32_t combo_ref_reduce(uint64_t h, uint32_t m) { return reduce(h, m); }

// ---------------------------------------------------------------------------------
// Sec. 4.1 step (2): the peer table of one round.
// peers[(w*S + s)*R + j], j in [0,R): R distinct workers, none equal to w.
//
// Reading: the draw is "without replacement" within one (worker, segment) - that is
// what makes P_l of Eq. (3) a set - and independent between segments.  It is done as
// the first R steps of a Fisher-Yates shuffle of the N-1 other workers, numbered
// 0..N-2 in increasing worker order with w itself skipped, step j drawing its swap
// partner from hash(seed, round, w, s, j).  The order of the R entries matters: it is
// the order in which Eq. (3)'s sum is accumulated.
// Returns 0, or -1 for N < 1, S < 1, R < 0 or R > N-1.
int combo_ref_make_peer_table(int32_t* peers, int32_t N, int32_t S, int32_t R,
                              uint64_t seed, uint64_t round) {
    if (N < 1 || S < 1 || R < 0 || R > N - 1) return -1;
    const int32_t M = N - 1;
    std::vector<int32_t> a((size_t)(M > 0 ? M : 1));
    for (int32_t w = 0; w < N; ++w) {
        for (int32_t s = 0; s < S; ++s) {
            for (int32_t i = 0; i < M; ++i) a[(size_t)i] = i;
            for (int32_t j = 0; j < R; ++j) {
                const uint64_t h = peer_hash(seed, round, (uint64_t)w, (uint64_t)s, (uint64_t)j);
                const int32_t r = j + (int32_t)reduce(h, (uint32_t)(M - j));
                const int32_t t = a[(size_t)j];
                a[(size_t)j] = a[(size_t)r];
                a[(size_t)r] = t;
                const int32_t c = a[(size_t)j];
                peers[((size_t)w * (size_t)S + (size_t)s) * (size_t)R + (size_t)j] = c + (c >= w ? 1 : 0);
            }
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------------
// Sec. 4.1 step (2) read literally: the targets of ALL S*R requests of a worker are drawn
// from one pool of the other workers without replacement "until there is no option
// left", so that requests spread evenly over the workers and, when S*R <= N-1, all
// segments come from different workers.
//
// Reading of what the text leaves open:
//   * requests are issued segment by segment, replica by replica (s-major, j-minor);
//   * the pool is a queue holding a uniformly random permutation of the N-1 others
//     (a full Fisher-Yates shuffle; swap partner of step i of the t-th permutation from
//     hash(seed ^ POOL_TAG, round, w, t, i)); when the queue is empty the next
//     permutation becomes the queue ("no option left" -> start over);
//   * P_l of Eq. (3) is a set, so a request takes the first queue element that this
//     segment has not already picked (this can only matter right after a refill inside
//     a segment); skipped elements keep their place at the front of the queue.
const uint64_t POOL_TAG = 0x706F6F6C65642121ull;

int combo_ref_make_peer_table_pooled(int32_t* peers, int32_t N, int32_t S, int32_t R,
                                     uint64_t seed, uint64_t round) {
    if (N < 1 || S < 1 || R < 0 || R > N - 1) return -1;
    const int32_t M = N - 1;
    for (int32_t w = 0; w < N; ++w) {
        std::vector<int32_t> queue;
        uint64_t epoch = 0;
        for (int32_t s = 0; s < S; ++s) {
            int32_t* picks = peers + ((size_t)w * (size_t)S + (size_t)s) * (size_t)R;
            for (int32_t j = 0; j < R; ++j) {
                if (queue.empty()) {
                    for (int32_t v = 0; v < N; ++v)
                        if (v != w) queue.push_back(v);
                    for (int32_t i = 0; i + 1 < M; ++i) {
                        const uint64_t h = peer_hash(seed ^ POOL_TAG, round, (uint64_t)w, epoch, (uint64_t)i);
                        const int32_t r = i + (int32_t)reduce(h, (uint32_t)(M - i));
                        const int32_t t = queue[(size_t)i];
                        queue[(size_t)i] = queue[(size_t)r];
                        queue[(size_t)r] = t;
                    }
                    ++epoch;
                }
                size_t pos = 0;
                for (; pos < queue.size(); ++pos) {
                    bool taken = false;
                    for (int32_t k = 0; k < j; ++k) taken = taken || picks[k] == queue[pos];
                    if (!taken) break;
                }
                if (pos == queue.size()) return -2;   // cannot happen while R <= N-1
                picks[j] = queue[pos];
                queue.erase(queue.begin() + (std::ptrdiff_t)pos);
            }
        }
    }
    return 0;
}

// Serve load of a table: deg[v] = number of (w, s, j) requests whose target is v.
int combo_ref_peer_in_degree(int32_t* deg, const int32_t* peers, int32_t N, int32_t S, int32_t R) {
    if (N < 1 || S < 1 || R < 0) return -1;
    for (int32_t v = 0; v < N; ++v) deg[v] = 0;
    const size_t n = (size_t)N * (size_t)S * (size_t)R;
    for (size_t i = 0; i < n; ++i) {
        if (peers[i] < 0 || peers[i] >= N) return -1;
        deg[peers[i]] += 1;
    }
    return 0;
}

// ---------------------------------------------------------------------------------
// Eq. (3) + Eq. (4): one aggregation round in single precision.
//
// X, Y hold a window of `ncols` columns that starts at global column `col0`
// (0 <= col0, col0 + ncols <= P); row w starts at X + w*ld.  With col0 = 0 and
// ncols = P this is the whole round.  (An output column depends only on the same
// column of the inputs, so a window of the full result equals the result on the
// window; the window form exists so that samples of very large rounds can be checked.)
//
// d = dataset sizes |D_j| (length N), or NULL for equal sizes.
//   equal sizes:  acc = X[w][e]; acc += X[p_0][e]; ...; acc += X[p_{R-1}][e];
//                 Y[w][e] = acc * inv  with inv = 1.0f / (float)(R+1)
//   general:      num = d[w]*X[w][e]; num += d[p_j]*X[p_j][e] (product rounded, then
//                 the sum rounded), den = d[w] + d[p_0] + ... in the same order,
//                 Y[w][e] = num / den.
// All arithmetic is IEEE binary32, one rounding per operation, no fused multiply-add.
// Every read is from X and every write to Y, so all workers see the pre-round state.
// Columns outside the window and the padding [ncols, ld) are not touched.
int combo_ref_gossip_round(float* Y, const float* X, int64_t ld, const int32_t* peers,
                           const float* d, int32_t N, int64_t P, int32_t S, int32_t R,
                           int64_t col0, int64_t ncols) {
    if (N < 1 || S < 1 || (int64_t)S > P || R < 0 || R > N - 1) return -1;
    if (col0 < 0 || ncols < 0 || col0 + ncols > P || ld < ncols) return -1;
    const float inv = 1.0f / (float)(R + 1);
    for (int32_t w = 0; w < N; ++w) {
        for (int32_t s = 0; s < S; ++s) {
            const int32_t* pl = peers + ((size_t)w * (size_t)S + (size_t)s) * (size_t)R;
            int64_t lo = seg_lo(P, S, s), hi = seg_hi(P, S, s);
            if (lo < col0) lo = col0;
            if (hi > col0 + ncols) hi = col0 + ncols;
            float den = 0.0f;
            if (d) {
                den = d[w];
                for (int32_t j = 0; j < R; ++j) den = den + d[pl[j]];
            }
            for (int64_t e = lo; e < hi; ++e) {
                const size_t c = (size_t)(e - col0);
                if (!d) {
                    float acc = X[(size_t)w * (size_t)ld + c];
                    for (int32_t j = 0; j < R; ++j) acc = acc + X[(size_t)pl[j] * (size_t)ld + c];
                    Y[(size_t)w * (size_t)ld + c] = acc * inv;
                } else {
                    float num = d[w] * X[(size_t)w * (size_t)ld + c];
                    for (int32_t j = 0; j < R; ++j) {
                        const float term = d[pl[j]] * X[(size_t)pl[j] * (size_t)ld + c];
                        num = num + term;
                    }
                    Y[(size_t)w * (size_t)ld + c] = num / den;
                }
            }
        }
    }
    return 0;
}

// The same round with every sum, product and quotient in binary64 and a binary64
// result: Eq. (3) evaluated (almost) exactly, used to report how far the
// single-precision arithmetic is from the mathematical value.
int combo_ref_gossip_round_f64(double* Y, const float* X, int64_t ld, const int32_t* peers,
                               const float* d, int32_t N, int64_t P, int32_t S, int32_t R,
                               int64_t col0, int64_t ncols) {
    if (N < 1 || S < 1 || (int64_t)S > P || R < 0 || R > N - 1) return -1;
    if (col0 < 0 || ncols < 0 || col0 + ncols > P || ld < ncols) return -1;
    for (int32_t w = 0; w < N; ++w) {
        for (int32_t s = 0; s < S; ++s) {
            const int32_t* pl = peers + ((size_t)w * (size_t)S + (size_t)s) * (size_t)R;
            int64_t lo = seg_lo(P, S, s), hi = seg_hi(P, S, s);
            if (lo < col0) lo = col0;
            if (hi > col0 + ncols) hi = col0 + ncols;
            double den = d ? (double)d[w] : 1.0;
            for (int32_t j = 0; j < R; ++j) den += d ? (double)d[pl[j]] : 1.0;
            for (int64_t e = lo; e < hi; ++e) {
                const size_t c = (size_t)(e - col0);
                double num = (d ? (double)d[w] : 1.0) * (double)X[(size_t)w * (size_t)ld + c];
                for (int32_t j = 0; j < R; ++j)
                    num += (d ? (double)d[pl[j]] : 1.0) * (double)X[(size_t)pl[j] * (size_t)ld + c];
                Y[(size_t)w * (size_t)ld + c] = num / den;
            }
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------------
// Sec. 4.2 "Dynamic Workers".  status[w]: 0 = offline, 1 = active, 2 = newcomer (joins in
// this round).
//
// Selection: an offline worker sends no request (its entries are -1).  Any other worker
// draws, per segment, among the ACTIVE others: offline workers have been marked offline
// and the request re-sent elsewhere, and a newcomer is not yet on anybody's worker list
// in the round it joins.  With A candidates (listed in increasing worker order) the
// picks are the first min(R, A) steps of the same hashed Fisher-Yates as in the static
// table, the span of step j being A - j; unused entries are -1.  With every worker
// active this is exactly the static table.
int combo_ref_make_peer_table_dynamic(int32_t* peers, const uint8_t* status, int32_t N, int32_t S,
                                      int32_t R, uint64_t seed, uint64_t round) {
    if (N < 1 || S < 1 || R < 0 || R > N - 1) return -1;
    std::vector<int32_t> cand;
    for (int32_t w = 0; w < N; ++w) {
        for (int32_t s = 0; s < S; ++s) {
            int32_t* out = peers + ((size_t)w * (size_t)S + (size_t)s) * (size_t)R;
            for (int32_t j = 0; j < R; ++j) out[j] = -1;
            if (status[w] == 0) continue;
            cand.clear();
            for (int32_t v = 0; v < N; ++v)
                if (v != w && status[v] == 1) cand.push_back(v);
            const int32_t A = (int32_t)cand.size();
            const int32_t take = R < A ? R : A;
            for (int32_t j = 0; j < take; ++j) {
                const uint64_t h = peer_hash(seed, round, (uint64_t)w, (uint64_t)s, (uint64_t)j);
                const int32_t r = j + (int32_t)reduce(h, (uint32_t)(A - j));
                const int32_t t = cand[(size_t)j];
                cand[(size_t)j] = cand[(size_t)r];
                cand[(size_t)r] = t;
                out[j] = cand[(size_t)j];
            }
        }
    }
    return 0;
}

// Aggregation with dynamic workers (Sec. 4.2 + Eq. 3):
//   offline worker:  keeps its parameters, Y[w] = X[w];
//   active worker:   terms = own value, then the valid (>= 0) table entries in order;
//   newcomer:        terms = the valid table entries only - it aggregates "without its
//                    local model"; with no valid entry it keeps what it has.
//   equal sizes:     acc = first term; acc += each further term; Y = acc * (1.0f/(float)count)
//   dataset sizes:   num = d*x of the first term, += d*x of the others (product rounded,
//                    then the sum); den = sum of the terms' d in the same order; Y = num/den
int combo_ref_gossip_round_dynamic(float* Y, const float* X, int64_t ld, const int32_t* peers,
                                   const float* d, const uint8_t* status, int32_t N, int64_t P,
                                   int32_t S, int32_t R, int64_t col0, int64_t ncols) {
    if (N < 1 || S < 1 || (int64_t)S > P || R < 0 || R > N - 1) return -1;
    if (col0 < 0 || ncols < 0 || col0 + ncols > P || ld < ncols) return -1;
    std::vector<int32_t> terms;
    for (int32_t w = 0; w < N; ++w) {
        for (int32_t s = 0; s < S; ++s) {
            const int32_t* pl = peers + ((size_t)w * (size_t)S + (size_t)s) * (size_t)R;
            int64_t lo = seg_lo(P, S, s), hi = seg_hi(P, S, s);
            if (lo < col0) lo = col0;
            if (hi > col0 + ncols) hi = col0 + ncols;
            terms.clear();
            if (status[w] == 1) terms.push_back(w);
            if (status[w] != 0)
                for (int32_t j = 0; j < R; ++j)
                    if (pl[j] >= 0) terms.push_back(pl[j]);
            const size_t n = terms.size();
            float inv = 0.0f, den = 0.0f;
            if (n > 0) {
                inv = 1.0f / (float)n;
                if (d) {
                    den = d[terms[0]];
                    for (size_t k = 1; k < n; ++k) den = den + d[terms[k]];
                }
            }
            for (int64_t e = lo; e < hi; ++e) {
                const size_t c = (size_t)(e - col0);
                float out;
                if (n == 0) {
                    out = X[(size_t)w * (size_t)ld + c];
                } else if (!d) {
                    float acc = X[(size_t)terms[0] * (size_t)ld + c];
                    for (size_t k = 1; k < n; ++k) acc = acc + X[(size_t)terms[k] * (size_t)ld + c];
                    out = acc * inv;
                } else {
                    float num = d[terms[0]] * X[(size_t)terms[0] * (size_t)ld + c];
                    for (size_t k = 1; k < n; ++k) {
                        const float term = d[terms[k]] * X[(size_t)terms[k] * (size_t)ld + c];
                        num = num + term;
                    }
                    out = num / den;
                }
                Y[(size_t)w * (size_t)ld + c] = out;
            }
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------------
// Sec. 4.3, Definition 2 (aggregation divergence): the distance between a worker's model
// W_{t,i} and W_t, the aggregate of ALL workers (the FedAvg output: the dataset-size
// weighted mean, plain mean for equal sizes).  dist2[i] = sum_e (X[i][e] - mean[e])^2;
// rho of the definition is bounded below by max_i sqrt(dist2[i]).
// Accumulated in extended precision so that the result is the exact value to far below
// the comparison tolerance; the mean is formed in worker order.
int combo_ref_aggregation_divergence(double* dist2, const float* X, int64_t ld, const float* d,
                                     int32_t N, int64_t P) {
    if (N < 1 || P < 1 || ld < P) return -1;
    std::vector<long double> acc((size_t)N, 0.0L);
    long double den = 0.0L;
    for (int32_t w = 0; w < N; ++w) den += d ? (long double)d[w] : 1.0L;
    for (int64_t e = 0; e < P; ++e) {
        long double num = 0.0L;
        for (int32_t w = 0; w < N; ++w)
            num += (d ? (long double)d[w] : 1.0L) * (long double)X[(size_t)w * (size_t)ld + (size_t)e];
        const long double mean = num / den;
        for (int32_t w = 0; w < N; ++w) {
            const long double diff = (long double)X[(size_t)w * (size_t)ld + (size_t)e] - mean;
            acc[(size_t)w] += diff * diff;
        }
    }
    for (int32_t w = 0; w < N; ++w) dist2[w] = (double)acc[(size_t)w];
    return 0;
}

// ---------------------------------------------------------------------------------
// Sec. 4.1 step (1) with one SGD step of a given gradient, followed by steps (3),(4):
// first X[w][e] <- X[w][e] - lr*G[w][e] for EVERY worker and column of the window
// (product rounded, then the difference rounded), and only then the round above on
// the stepped X.  X is overwritten by the stepped values.
int combo_ref_local_sgd_then_gossip(float* Y, float* X, const float* G, float lr, int64_t ld,
                                    const int32_t* peers, const float* d, int32_t N, int64_t P,
                                    int32_t S, int32_t R, int64_t col0, int64_t ncols) {
    if (N < 1 || S < 1 || (int64_t)S > P || R < 0 || R > N - 1) return -1;
    if (col0 < 0 || ncols < 0 || col0 + ncols > P || ld < ncols) return -1;
    for (int32_t w = 0; w < N; ++w) {
        for (int64_t c = 0; c < ncols; ++c) {
            const size_t k = (size_t)w * (size_t)ld + (size_t)c;
            const float step = lr * G[k];
            X[k] = X[k] - step;
        }
    }
    return combo_ref_gossip_round(Y, X, ld, peers, d, N, P, S, R, col0, ncols);
}

// Sec. 4.1 step (1) with a communication interval tau > 1: tau SGD steps with given
// gradients G[k] (k = 0..tau-1, each [N][ld], slice k starting at G + k*N*ld) are applied
// one after the other, x <- x - lr*G[k] (product rounded, then the difference), on every
// worker and column of the window; then the round on the stepped X.  X is overwritten
// by the stepped values.
int combo_ref_local_sgd_steps_then_gossip(float* Y, float* X, const float* G, int32_t tau, float lr,
                                          int64_t ld, const int32_t* peers, const float* d,
                                          int32_t N, int64_t P, int32_t S, int32_t R, int64_t col0,
                                          int64_t ncols) {
    if (tau < 0) return -1;
    if (N < 1 || S < 1 || (int64_t)S > P || R < 0 || R > N - 1) return -1;
    if (col0 < 0 || ncols < 0 || col0 + ncols > P || ld < ncols) return -1;
    for (int32_t k = 0; k < tau; ++k) {
        const float* Gk = G + (size_t)k * (size_t)N * (size_t)ld;
        for (int32_t w = 0; w < N; ++w) {
            for (int64_t c = 0; c < ncols; ++c) {
                const size_t i = (size_t)w * (size_t)ld + (size_t)c;
                const float step = lr * Gk[i];
                X[i] = X[i] - step;
            }
        }
    }
    return combo_ref_gossip_round(Y, X, ld, peers, d, N, P, S, R, col0, ncols);
}

}  // extern "C"
