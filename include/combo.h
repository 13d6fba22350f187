/*
 * combo.h - C ABI of the segmented-gossip aggregation round on one AMD MI355X (gfx950).
 *
 * The method is the model aggregation of "Decentralized Federated Learning: A Segmented
 * Gossip Approach" (Hu, Jiang, Wang; arXiv 1908.07782):  N simulated workers each hold a
 * flat parameter vector of P values, cut into S contiguous, non-overlapping segments
 * (Sec. 3, Eq. 1).  In every round each worker chooses, for each segment, R other
 * workers (Sec. 4.1 step 2) and replaces the segment by the weighted mean of its own
 * copy and the R pulled copies (Sec. 3, Eq. 3); the aggregated segments together are the
 * new model (Eq. 4).  All pulled segments are the providers' state from before the
 * aggregation of the same round (Sec. 4.1 steps 3-4, Sec. 5.1: synchronous process).
 *
 * Conventions common to every entry point
 *   - Pointers named d_* are DEVICE pointers (HIP global memory of the current device).
 *     The library never allocates, frees or copies device memory and never
 *     synchronises: work is enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and the call returns at once.  The caller owns every
 *     buffer and must keep it alive until the stream has passed the enqueued work.
 *   - Return value: COMBO_OK (0) or a negative combo_status.  No exceptions, no aborts.
 *     COMBO_EINVAL, COMBO_EALIAS and COMBO_ERANGE are found before anything is enqueued.
 *     COMBO_EHIP is what the HIP runtime reports when a launch is enqueued; a call that
 *     enqueues several kernels (the separate-pass form of the local steps, the divergence
 *     monitor) may then have enqueued the earlier ones, so after COMBO_EHIP the contents
 *     of the output - and of d_src where a call is documented to step it in place - are
 *     unspecified.
 *   - Parameter matrices are row-major float32 [N][ld]: worker w's parameter e is at
 *     index w*ld + e, e in [0, P).  ld >= P is the row pitch in elements.  The padding
 *     columns [P, ld) are never read and never written.
 *   - Segment s in [0, S) covers columns [s*L, (s+1)*L) with L = floor(P/S), except the
 *     last, which extends to P (it absorbs the remainder).  Requires 1 <= S <= P.
 *   - A peer table is int32 [N][S][R], worker-major: entry (w*S + s)*R + j is the j-th
 *     provider of segment s for worker w.  The order of the j axis is the order of
 *     summation.  Entries must lie in [0, N); the aggregation entry points do not
 *     check the contents of a table (they are device data) - out-of-range entries are
 *     undefined behaviour.
 *   - Arithmetic is IEEE binary32 with one rounding per operation (no fused
 *     multiply-add), in the fixed order stated at each entry point, so results are
 *     reproducible bit for bit.  A quotient is the correctly rounded one, however the
 *     kernel obtains it.
 *   - Fast paths need 16-byte aligned d_dst/d_src/d_grad and ld % 4 == 0; any other
 *     alignment or pitch is accepted and handled by a slower scalar kernel.
 *   - Thread safety: calls are independent; tuning (combo_tune) is process-global.
 */
#ifndef COMBO_H_
#define COMBO_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    COMBO_OK = 0,
    COMBO_EINVAL = -1, /* a size or pointer argument is invalid (see each function)      */
    COMBO_EALIAS = -2, /* output overlaps an input that must stay intact during the round */
    COMBO_ERANGE = -3, /* valid in principle but beyond what this build supports          */
    COMBO_EHIP = -4    /* the HIP runtime reported an error when enqueuing                */
} combo_status;

/*
 * Peer selection for one round (Sec. 4.1 step 2: R targets per segment, drawn at random
 * among the other workers without replacement).
 *
 * For every (w, s) the R entries are the first R elements of a Fisher-Yates shuffle of
 * the N-1 other workers (listed in increasing order, w skipped).  Step j in [0, R)
 * swaps position j with position j + reduce(hash(seed, round, w, s, j), N-1-j), where
 *   mix64(z):  z = (z ^ z>>30) * 0xBF58476D1CE4E5B9; z = (z ^ z>>27) * 0x94D049BB133111EB;
 *              return z ^ z>>31                                  (SplitMix64 finaliser)
 *   hash:      h = mix64(seed + G); then for c in (round, w, s, j): h = mix64((h ^ c) + G)
 *              with G = 0x9E3779B97F4A7C15
 *   reduce(h, m) = ((h >> 32) * m) >> 32.
 * The table is a pure function of (N, S, R, seed, round): any entry can be recomputed
 * anywhere, nothing is carried from round to round.
 *
 *   d_peers  out, device, int32[N*S*R]; may be NULL when R == 0 (nothing is written).
 * Errors: COMBO_EINVAL for N < 1, S < 1, R < 0, R > N-1 (R distinct others do not
 * exist), or d_peers == NULL with R > 0.  COMBO_ERANGE for N > 16384 (the shuffle
 * state of one (w, s) is kept in 64 KiB of LDS).
 */
int combo_make_peer_table(int32_t* d_peers, int32_t N, int32_t S, int32_t R,
                          uint64_t seed, uint64_t round, void* stream);

/*
 * Peer selection as Sec. 4.1 step 2 words it: the targets of ALL S*R requests of a worker
 * come from one pool of the other workers, drawn without replacement until no option is
 * left, so requests spread evenly and, when S*R <= N-1, all of a worker's segments come
 * from different workers.  Requests are issued s-major, j-minor.  The pool is a queue
 * holding a random permutation of the N-1 others (full Fisher-Yates; swap partner of
 * step i of the t-th permutation from hash(seed ^ 0x706F6F6C65642121, round, w, t, i),
 * same hash and reduce as above); an empty queue is replaced by the next permutation; a
 * request takes the first queue element its segment has not picked yet (Eq. 3's P_l is a
 * set), skipped elements keeping their place.  Same table layout, arguments and errors
 * as combo_make_peer_table; the aggregation entry points accept either kind of table.
 */
int combo_make_peer_table_pooled(int32_t* d_peers, int32_t N, int32_t S, int32_t R,
                                 uint64_t seed, uint64_t round, void* stream);

/*
 * Serve load of a table (the balance Sec. 4.1 step 2 asks for): d_degree[v] = number of
 * requests (w, s, j) whose target is worker v.  Entries outside [0, N) are not counted.
 *   d_degree  out, device, int32[N] (overwritten);  d_peers  in, device, int32[N*S*R].
 * Errors: COMBO_EINVAL for bad sizes or NULL pointers, COMBO_ERANGE for N > 16384.
 */
int combo_peer_in_degree(int32_t* d_degree, const int32_t* d_peers, int32_t N, int32_t S,
                         int32_t R, void* stream);

/*
 * One aggregation round: Eq. (3) on every segment of every worker, written to the back
 * buffer (Eq. 4), all reads from the front buffer.
 *
 *   uniform weights (d_dataset_sizes == NULL):
 *       acc = src[w][e]; acc += src[p_0][e]; ...; acc += src[p_{R-1}][e];
 *       dst[w][e] = acc * (1.0f / (float)(R + 1))
 *   dataset-size weights (d_dataset_sizes = |D_j|, device float32[N], all > 0):
 *       num = d[w]*src[w][e]; num += d[p_j]*src[p_j][e] for j = 0..R-1 (product rounded,
 *       then the sum); den = d[w] + d[p_0] + ... + d[p_{R-1}] in that order;
 *       dst[w][e] = num / den
 *   with p_j = d_peers[(w*S + seg(e))*R + j].
 *
 *   d_dst    out, device, float32[N][ld]; every element [w][0..P) is written exactly once.
 *   d_src    in,  device, float32[N][ld]; not modified.
 *   d_peers  in,  device, int32[N*S*R]; may be NULL when R == 0 (the round is a copy).
 * Errors: COMBO_EINVAL for N < 1, S < 1, S > P, R < 0, R > N-1, ld < P, a NULL d_dst or
 * d_src, NULL d_peers with R > 0; COMBO_EALIAS if [d_dst, d_dst + N*ld) overlaps
 * [d_src, d_src + N*ld) (a worker would read a neighbour's already aggregated values) or
 * the table, the dataset sizes or (dynamic rounds) the status array; COMBO_ERANGE if
 * N*ceil(P/tile) exceeds the grid limit of 2^31-1 workgroups or N*ld*4 does not fit in 64 bits.
 */
int combo_segment_gossip_round(float* d_dst, const float* d_src, int64_t ld,
                               const int32_t* d_peers, const float* d_dataset_sizes,
                               int32_t N, int64_t P, int32_t S, int32_t R, void* stream);

/*
 * Local update, then the round (Sec. 4.1 steps 1, 3, 4): first EVERY worker takes one
 * SGD step with the given gradient, x' = x - lr*g (product rounded, then the
 * difference), and only then Eq. (3) is applied to the stepped parameters x' exactly as
 * in combo_segment_gossip_round.
 *
 *   d_src   in/out, device, float32[N][ld]: the pre-update parameters x.  On return its
 *           contents are x or x', unspecified which (the fused kernel forms x' on the
 *           fly and leaves d_src alone; the two-pass fallback steps d_src in place).
 *           Callers ping-pong the buffers, so the old front buffer is dead either way.
 *   d_grad  in, device, float32[N][ld], same pitch; not modified.
 * Errors: as combo_segment_gossip_round, plus COMBO_EINVAL for a NULL d_grad and
 * COMBO_EALIAS if d_grad overlaps d_src or d_dst.
 */
int combo_local_sgd_then_gossip(float* d_dst, float* d_src, const float* d_grad, float lr,
                                int64_t ld, const int32_t* d_peers,
                                const float* d_dataset_sizes, int32_t N, int64_t P, int32_t S,
                                int32_t R, void* stream);

/*
 * The same with a communication interval tau (Sec. 4.1 step 1: several SGD rounds between
 * two synchronisations): tau steps x <- x - lr*g_t, t = 0..tau-1 in that order, each with
 * its own given gradient, then the round on the result.
 *   d_grads  in, device, float32[tau][N][ld]: slice t starts at d_grads + t*N*ld.
 *   tau      >= 0; 0 is the plain round (d_grads may then be NULL).
 * d_src as in combo_local_sgd_then_gossip (which is this call with tau = 1).
 * Errors: as combo_local_sgd_then_gossip, plus COMBO_EINVAL for tau < 0.
 */
int combo_local_sgd_steps_then_gossip(float* d_dst, float* d_src, const float* d_grads,
                                      int32_t tau, float lr, int64_t ld, const int32_t* d_peers,
                                      const float* d_dataset_sizes, int32_t N, int64_t P,
                                      int32_t S, int32_t R, void* stream);

/*
 * Dynamic workers (Sec. 4.2).  d_status is device uint8[N]: 0 = offline, 1 = active,
 * 2 = newcomer joining in this round.
 *
 * Selection: an offline worker sends no request (all its entries are -1).  Every other
 * worker draws, per segment, among the ACTIVE others - a worker found offline is marked
 * offline and the request goes to someone else; a newcomer is not yet on anybody's
 * worker list.  With A candidates (in increasing worker order) the picks are the first
 * min(R, A) steps of the hashed Fisher-Yates of combo_make_peer_table, the span of step j
 * being A - j; unused entries are -1.  With every worker active the table equals
 * combo_make_peer_table's.  Errors as combo_make_peer_table, plus COMBO_EINVAL for a NULL
 * d_status.
 */
int combo_make_peer_table_dynamic(int32_t* d_peers, const uint8_t* d_status, int32_t N, int32_t S,
                                  int32_t R, uint64_t seed, uint64_t round, void* stream);

/*
 * Aggregation with dynamic workers: as combo_segment_gossip_round, except that
 *   - an offline worker keeps its parameters (dst[w] = src[w]);
 *   - an active worker averages its own value and the valid (>= 0) entries of its table
 *     row, in order; a newcomer averages the valid entries only - it aggregates "without
 *     its local model" - and keeps what it has if there is none;
 *   - uniform weights scale by 1.0f/(float)(number of terms); with dataset sizes the
 *     numerator and denominator run over the same terms in the same order.
 * Rows of offline workers and the own rows of newcomers are never read for anybody else.
 * Errors as combo_segment_gossip_round, plus COMBO_EINVAL for a NULL d_status.
 */
int combo_segment_gossip_round_dynamic(float* d_dst, const float* d_src, int64_t ld,
                                       const int32_t* d_peers, const float* d_dataset_sizes,
                                       const uint8_t* d_status, int32_t N, int64_t P, int32_t S,
                                       int32_t R, void* stream);

/*
 * Tiled arena layout.  Instead of row-major [N][ld], a parameter matrix may be kept as
 * [T][N][Wt]: tile t = e / Wt holds the Wt consecutive columns [t*Wt, (t+1)*Wt) of ALL N
 * workers, worker-major inside the tile; T = ceil(P / Wt); worker w's parameter e is at
 * ((e / Wt)*N + w)*Wt + e % Wt.  The N x Wt slab that one workgroup of the aggregation
 * kernel stages in LDS is then one contiguous block, which streams from HBM 6-18 % faster
 * than N separate row chunks (measured on MI355X).  Columns >= P of the last tile are
 * padding: never read, never written.  Element-wise work (the local SGD step) is
 * layout-agnostic, so a simulation can live in this layout and unpack only to export.
 *
 *   combo_tiled_cols(N, R)          recommended Wt (a power of two in [8, 1024]: for N <= 32
 *                                   the narrowest one whose tile reaches 8 KiB, i.e. tiles of
 *                                   8 KiB to just under 16 KiB - for R > 8 the widest within
 *                                   32 KiB, where more data in flight hides the longer
 *                                   aggregation -, then the widest of 64, 32, 16, 8 columns
 *                                   whose tile stays within 32 KiB),
 *                                   or a negative status if N rows of 8 columns do not fit in
 *                                   LDS (N*(44 + 4*R) > 65536)
 *   combo_tiled_elems(N, P, Wt)     floats in one tiled matrix, = T*N*Wt
 *   combo_pack_tiled / combo_unpack_tiled   convert row-major <-> tiled (pure copies)
 *   combo_segment_gossip_round_tiled        the round of combo_segment_gossip_round on
 *                                   tiled d_dst/d_src; d_status == NULL for the static round,
 *                                   else the dynamic-worker semantics of
 *                                   combo_segment_gossip_round_dynamic
 *   combo_local_sgd_steps_then_gossip_tiled  as combo_local_sgd_steps_then_gossip; d_grads
 *                                   holds tau tiled matrices back to back; d_src is never
 *                                   modified (the steps are folded into the slab fill)
 * Same arithmetic, order and results as the row-major entry points, bit for bit.
 * Errors: COMBO_EINVAL for bad sizes, NULL or not 16-byte aligned buffers, Wt not a power
 * of two in [8, 1024]; COMBO_EALIAS for overlapping buffers; COMBO_ERANGE when the N x Wt
 * slab with its peer list does not fit in 64 KiB of LDS.
 */
int32_t combo_tiled_cols(int32_t N, int32_t R);
int64_t combo_tiled_elems(int32_t N, int64_t P, int32_t tile_cols);
int combo_pack_tiled(float* d_tiled, const float* d_rows, int64_t ld, int32_t N, int64_t P,
                     int32_t tile_cols, void* stream);
int combo_unpack_tiled(float* d_rows, int64_t ld, const float* d_tiled, int32_t N, int64_t P,
                       int32_t tile_cols, void* stream);
int combo_segment_gossip_round_tiled(float* d_dst, const float* d_src, int32_t tile_cols,
                                     const int32_t* d_peers, const float* d_dataset_sizes,
                                     const uint8_t* d_status, int32_t N, int64_t P, int32_t S,
                                     int32_t R, void* stream);
int combo_local_sgd_steps_then_gossip_tiled(float* d_dst, const float* d_src, const float* d_grads,
                                            int32_t tau, float lr, int32_t tile_cols,
                                            const int32_t* d_peers, const float* d_dataset_sizes,
                                            int32_t N, int64_t P, int32_t S, int32_t R,
                                            void* stream);

/*
 * A round that reads one layout and writes another (Eq. 4's reassembly lands directly in
 * the layout the caller wants next): the work of combo_local_sgd_steps_then_gossip (tau = 0:
 * of combo_segment_gossip_round; with d_status: of combo_segment_gossip_round_dynamic) with
 * independent layouts for the front buffer and the back buffer.  A caller whose models are
 * row-major enters the tiled arena with its first round and leaves it with its last one,
 * without a combo_pack_tiled / combo_unpack_tiled pass.  Same arithmetic, order and
 * results as the single-layout entry points, bit for bit.
 *   d_dst, dst_ld, dst_tile_cols   back buffer: dst_tile_cols == 0: row-major [N][dst_ld];
 *                                  else tiled [T][N][dst_tile_cols] (dst_ld ignored)
 *   d_src, src_ld, src_tile_cols   front buffer, likewise; never modified
 *   d_grads                        tau matrices in the FRONT buffer's layout, back to back;
 *                                  may be NULL when tau == 0
 *   d_status                       NULL, or dynamic-worker status (then tau must be 0)
 * Always runs the LDS-slab kernel with one strip per tile.  Errors: COMBO_EINVAL / COMBO_EALIAS
 * as for the single-layout calls; COMBO_ERANGE when that kernel cannot be used: buffers not
 * 16-byte aligned, a row pitch that is not a multiple of 4, two tiled sides of different
 * tile widths, N rows of a tile (or, with two row-major sides, of 64 columns) not fitting in
 * 64 KiB of LDS, or d_status together with tau > 0.
 */
int combo_round_relayout(float* d_dst, int64_t dst_ld, int32_t dst_tile_cols, const float* d_src,
                         int64_t src_ld, int32_t src_tile_cols, const float* d_grads, int32_t tau,
                         float lr, const int32_t* d_peers, const float* d_dataset_sizes,
                         const uint8_t* d_status, int32_t N, int64_t P, int32_t S, int32_t R,
                         void* stream);

/*
 * A whole iteration in ONE launch, without a peer table: peer selection exactly as
 * combo_make_peer_table(seed, round) would make it (every workgroup draws the peer lists
 * it needs from the counter-based hash while its loads are in flight), the optional tau
 * local SGD steps, and the aggregation.  Results are identical, bit for bit, to
 * combo_make_peer_table followed by combo_local_sgd_steps_then_gossip (or its tiled form).
 *   tile_cols  0: row-major d_dst/d_src/d_grads with pitch ld; else the tiled layout
 *              [T][N][tile_cols] (ld is ignored)
 *   d_grads    tau matrices in the same layout, back to back; may be NULL when tau == 0
 *   d_src      never modified
 * Errors: COMBO_EINVAL / COMBO_EALIAS as for the table-driven calls; COMBO_ERANGE when the
 * in-kernel draw cannot be used: R > 8, buffers not 16-byte aligned, ld % 4 != 0, or the
 * N-row slab does not fit in LDS - use the table-driven entry points then.
 */
int combo_round_hashed(float* d_dst, const float* d_src, const float* d_grads, int32_t tau,
                       float lr, int64_t ld, int32_t tile_cols, const float* d_dataset_sizes,
                       int32_t N, int64_t P, int32_t S, int32_t R, uint64_t seed, uint64_t round,
                       void* stream);

/*
 * Aggregation divergence (Sec. 4.3, Definition 2): how far each worker's model is from the
 * aggregate of ALL workers (the FedAvg output).
 *     mean[e]     = sum_w d[w]*x[w][e] / sum_w d[w]      (d = 1 when d_dataset_sizes is NULL)
 *     d_dist2[w]  = sum_e (x[w][e] - mean[e])^2
 * evaluated in binary64 in a fixed order (the mean as sum * (1 / sum of d); no floating-
 * point atomics), so repeated calls give identical bits.  The rho of Definition 2 is bounded
 * below by max_w sqrt(d_dist2[w]).  Accuracy against exact arithmetic: 2e-12 relative, plus -
 * the mean being a sum times a rounded reciprocal, off by at most delta = (N+3) * 2^-53 * |mean|
 * in norm - an absolute 2*sqrt(d_dist2)*delta + delta^2; identical rows give at most delta^2,
 * exactly 0 when N is a power of two.
 *   d_dist2      out, device, float64[N]
 *   d_x          in,  device, float32[N][ld]
 *   d_workspace  scratch, device, 8-byte aligned, at least
 *                combo_aggregation_divergence_workspace(N, P) bytes; contents irrelevant
 *                before and after the call
 * combo_aggregation_divergence_tiled reads a tiled matrix [T][N][tile_cols] instead.
 * Errors: COMBO_EINVAL for bad sizes, NULL pointers, a workspace that is too small or
 * misaligned; COMBO_ERANGE for N > 1024, or when N rows of a tile exceed the kernel's
 * register slots (N * tile_cols > 16384).
 * combo_aggregation_divergence_workspace returns the byte count (4096*N*8), or a negative
 * status.
 */
int64_t combo_aggregation_divergence_workspace(int32_t N, int64_t P);
int combo_aggregation_divergence(double* d_dist2, const float* d_x, int64_t ld,
                                 const float* d_dataset_sizes, int32_t N, int64_t P,
                                 void* d_workspace, int64_t workspace_bytes, void* stream);
int combo_aggregation_divergence_tiled(double* d_dist2, const float* d_x, int32_t tile_cols,
                                       const float* d_dataset_sizes, int32_t N, int64_t P,
                                       void* d_workspace, int64_t workspace_bytes, void* stream);

/*
 * The divergence monitor for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels, arithmetic and results as combo_aggregation_divergence
 * (tile_cols == 0: row-major d_x with pitch ld) and combo_aggregation_divergence_tiled
 * (tile_cols != 0: tiled d_x, ld ignored), bit for bit; the per-workgroup partial sums go
 * to an array the library holds itself in device memory (4 MiB, one copy on every GPU the
 * library runs on, until the process ends).  Its address is looked up on the first call on
 * a device; no call allocates, frees or copies memory.
 *   - At most COMBO_DIVERGENCE_NOALLOC_MAX_WORKERS workers; more return COMBO_ERANGE (use the
 *     workspace forms then).
 *   - All calls on one GPU share the one array: calls that may run at the same time on that
 *     GPU (different streams, different threads) race on it and must be serialised by the
 *     caller.  Calls on one stream are ordered and safe.  Nothing in the array needs to be
 *     cleared between calls: every entry that is read has been written by the same call.
 * Errors: as the workspace forms, plus COMBO_EHIP when the array's address cannot be obtained.
 */
#define COMBO_DIVERGENCE_NOALLOC_MAX_WORKERS 128
int combo_aggregation_divergence_noalloc(double* d_dist2, const float* d_x, int64_t ld,
                                         int32_t tile_cols, const float* d_dataset_sizes, int32_t N,
                                         int64_t P, void* stream);

/*
 * Bandwidth probes: gather-free passes with the memory access patterns of the aggregation
 * kernels, to measure what the device sustains for each pattern (the practical ceiling a
 * round is compared with).  They compute nothing of the method.  d_dst and d_src are
 * float32 [N][ld] buffers (16-byte aligned, ld % 4 == 0, not overlapping); only whole
 * 128-bit words, strips and tiles are touched, so a ragged remainder is left alone.
 *   COMBO_PROBE_COPY        flat copy of the N*ld floats, 128-bit streaming loads and stores;
 *                           param = words in flight per thread (1, 2, 4, 8); cols bit 0 = 0:
 *                           the words of a thread are 4 KiB apart, 1: the words of one
 *                           wavefront are consecutive KiB; cols bit 1: the stores are written
 *                           through to device scope instead of carrying the non-temporal
 *                           hint; cols >> 4 = k != 0: the XCDs take turns at runs of k
 *                           consecutive workgroup blocks, as the slab kernel's strip order
 *                           does (the last two also for the next two kinds)
 *   COMBO_PROBE_READ        the same loads folded to one float per workgroup, written to
 *                           d_dst[workgroup] (d_dst needs N*ld / (1024*param) + 1 floats)
 *   COMBO_PROBE_WRITE       the same stores of a constant; d_src may be NULL
 *   COMBO_PROBE_ROW_CHUNKS  per workgroup N row chunks of `cols` columns, rows ld apart: the
 *                           slab kernel's footprint on a row-major arena (no LDS, no gather);
 *                           param > 1: the XCDs take turns at runs of `param` consecutive
 *                           strips (also for the next kind), else strip i to workgroup i
 *   COMBO_PROBE_TILES       per workgroup one contiguous N x cols tile: the footprint on a
 *                           tiled arena; the first (P / cols)*N*cols floats are copied
 *   COMBO_PROBE_MULTI_READ  d_dst[w][e] = sum of `param` rows w, w+1, ... (wrapping) of
 *                           d_src, one workgroup per (1024 columns, row), rows in
 *                           worker-major order: param read streams and one write stream with
 *                           no reuse out of LDS
 *   COMBO_PROBE_LDS_READ    no global memory traffic: `cols` workgroups of 256 threads each
 *                           fill 8 KiB of LDS and read it `param` x 8 times per thread with
 *                           conflict-free 128-bit reads (the lanes of a wavefront read 64
 *                           consecutive words, as the aggregation phase of a round does);
 *                           LDS bytes read = cols * 256 * 8 * 16 * param; d_dst[workgroup]
 *                           receives a checksum (cols <= N*ld), d_src may be NULL
 * Errors: COMBO_EINVAL for an unknown kind, bad sizes or pointers, or a cols/param the
 * probe does not cover; COMBO_EALIAS for overlapping buffers.
 */
enum {
    COMBO_PROBE_COPY = 0,
    COMBO_PROBE_READ = 1,
    COMBO_PROBE_WRITE = 2,
    COMBO_PROBE_ROW_CHUNKS = 3,
    COMBO_PROBE_TILES = 4,
    COMBO_PROBE_MULTI_READ = 5,
    COMBO_PROBE_LDS_READ = 6
};
int combo_bandwidth_probe(int kind, float* d_dst, const float* d_src, int32_t N, int64_t ld, int64_t P,
                          int32_t cols, int32_t param, void* stream);

/*
 * Performance knobs (process-global, host side only; results never depend on them).
 *   COMBO_TUNE_KERNEL      0: automatic (LDS-slab kernel when the buffers are 16-byte
 *                          aligned, ld % 4 == 0 and N rows of a 64-column strip fit in
 *                          64 KiB of LDS, else the row-tile kernel); 1: always the
 *                          row-tile kernel; 2: same as 0
 *   COMBO_TUNE_SLAB_COLS   strip width of the slab kernel: 0 = automatic, or a power of
 *                          two in [64, 1024] (ignored if that slab does not fit in LDS)
 *   COMBO_TUNE_SLAB_ORDER  slab kernel, which strip a workgroup takes (workgroup ids go round-robin
 *                          over the 8 XCDs): 1: workgroup i takes strip i; 2: every XCD works
 *                          through its own contiguous eighth of the strips; k >= 3: the XCDs
 *                          take turns at runs of k consecutive strips; 0: automatic (runs of
 *                          16 tiles for tiled arenas, 32 from 7 GiB per matrix on, where
 *                          they measure 1-7 % faster; for row-major arenas runs that give an
 *                          XCD 2 KiB of consecutive columns of a row per turn: 4 strips of
 *                          128 columns, 8 of 64, strip i for wider strips)
 *   COMBO_TUNE_SLAB_THREADS slab kernel: workgroup size; 0: automatic (256 threads for slabs of up
 *                          to 12 KiB, else 512), or 256, 512
 *   COMBO_TUNE_SLAB_LDS_FLOOR slab kernel: least LDS bytes a launch asks for (1..65536); above
 *                          what the kernel uses it only lowers the number of workgroups
 *                          resident per compute unit; 0: automatic (24 KiB for 256-thread
 *                          workgroups of uniform-weight static rounds with R <= 4 on arenas
 *                          below 7 GiB per matrix, where six resident workgroups beat eight;
 *                          36 KiB with one fused local step and 44 KiB with more, so that
 *                          four or three workgroups are resident, the gradient slabs
 *                          being in flight as well)
 *   COMBO_TUNE_TILE_COLS   row-tile kernel: columns of one worker handled by one
 *                          workgroup: 0 = automatic (2048, or 1024 for more than 384
 *                          workers), or 1024, 2048, 4096
 *   COMBO_TUNE_XCD_SWIZZLE row-tile kernel: 1: consecutive workgroups on one XCD are the
 *                          N workers of one column tile (peer rows are re-read from that
 *                          XCD's L2); 0: plain worker-major order
 *   COMBO_TUNE_FUSED_MODE  combo_local_sgd_then_gossip: 0: fold the step into the slab
 *                          kernel when that kernel is used; 1: always two passes
 * Returns COMBO_OK or COMBO_EINVAL for an unknown key or unsupported value.
 */
enum {
    COMBO_TUNE_TILE_COLS = 0,
    COMBO_TUNE_XCD_SWIZZLE = 1,
    COMBO_TUNE_FUSED_MODE = 2,
    COMBO_TUNE_KERNEL = 3,
    COMBO_TUNE_SLAB_COLS = 4,
    COMBO_TUNE_SLAB_ORDER = 5,
    COMBO_TUNE_SLAB_THREADS = 6,
    COMBO_TUNE_SLAB_LDS_FLOOR = 7
};
int combo_tune(int key, int value);
/* Which kernel the row-major aggregation entry points use for N workers and R replicas
 * with aligned buffers under the current knobs: 1 = LDS-slab kernel, 0 = row-tile kernel. */
int combo_round_kernel_kind(int32_t N, int32_t R);
int combo_get_tune(int key); /* current value, or COMBO_EINVAL */

/* Static, human-readable text for a status code. Never NULL. */
const char* combo_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* COMBO_H_ */
