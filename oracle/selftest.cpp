// Memory-safety self-test of the CPU oracle (test infrastructure): calls every exported
// function on small, awkward shapes with exactly sized heap buffers.  Built together with
// combo_ref.cpp under -fsanitize=address,undefined by the CPU test-suite; any out-of-bounds
// access or undefined behaviour aborts the run.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
int combo_ref_segment_bounds(int64_t, int32_t, int64_t*, int64_t*);
int combo_ref_make_peer_table(int32_t*, int32_t, int32_t, int32_t, uint64_t, uint64_t);
int combo_ref_make_peer_table_pooled(int32_t*, int32_t, int32_t, int32_t, uint64_t, uint64_t);
int combo_ref_make_peer_table_dynamic(int32_t*, const uint8_t*, int32_t, int32_t, int32_t, uint64_t, uint64_t);
int combo_ref_peer_in_degree(int32_t*, const int32_t*, int32_t, int32_t, int32_t);
int combo_ref_gossip_round(float*, const float*, int64_t, const int32_t*, const float*, int32_t, int64_t,
                           int32_t, int32_t, int64_t, int64_t);
int combo_ref_gossip_round_f64(double*, const float*, int64_t, const int32_t*, const float*, int32_t,
                               int64_t, int32_t, int32_t, int64_t, int64_t);
int combo_ref_gossip_round_dynamic(float*, const float*, int64_t, const int32_t*, const float*,
                                   const uint8_t*, int32_t, int64_t, int32_t, int32_t, int64_t, int64_t);
int combo_ref_local_sgd_then_gossip(float*, float*, const float*, float, int64_t, const int32_t*,
                                    const float*, int32_t, int64_t, int32_t, int32_t, int64_t, int64_t);
int combo_ref_local_sgd_steps_then_gossip(float*, float*, const float*, int32_t, float, int64_t,
                                          const int32_t*, const float*, int32_t, int64_t, int32_t,
                                          int32_t, int64_t, int64_t);
int combo_ref_aggregation_divergence(double*, const float*, int64_t, const float*, int32_t, int64_t);
}

#define REQUIRE(x) do { if (!(x)) { std::printf("FAILED %s line %d\n", #x, __LINE__); return 1; } } while (0)

static int run_case(int32_t N, int64_t P, int32_t S, int32_t R, int64_t pad) {
    const int64_t ld = P + pad;
    std::vector<int64_t> lo((size_t)S), hi((size_t)S);
    REQUIRE(combo_ref_segment_bounds(P, S, lo.data(), hi.data()) == 0);
    std::vector<int32_t> t((size_t)N * S * R + 0), tp(t.size()), td(t.size()), deg((size_t)N);
    std::vector<uint8_t> status((size_t)N, 1);
    if (N > 2) { status[1] = 0; status[(size_t)N - 1] = 2; }
    REQUIRE(combo_ref_make_peer_table(t.data(), N, S, R, 3, 4) == 0);
    REQUIRE(combo_ref_make_peer_table_pooled(tp.data(), N, S, R, 3, 4) == 0);
    REQUIRE(combo_ref_make_peer_table_dynamic(td.data(), status.data(), N, S, R, 3, 4) == 0);
    REQUIRE(combo_ref_peer_in_degree(deg.data(), tp.data(), N, S, R) == 0);
    std::vector<float> X((size_t)(N * ld)), Y(X.size()), G((size_t)(3 * N * ld)), d((size_t)N);
    std::vector<double> Y64(X.size()), dist((size_t)N);
    for (size_t i = 0; i < X.size(); ++i) X[i] = (float)((i * 2654435761u) % 1000) * 1e-3f - 0.5f;
    for (size_t i = 0; i < G.size(); ++i) G[i] = (float)((i * 40503u) % 100) * 1e-4f;
    for (int32_t w = 0; w < N; ++w) d[(size_t)w] = 100.0f + (float)w;
    for (const float* dd : {(const float*)nullptr, (const float*)d.data()}) {
        REQUIRE(combo_ref_gossip_round(Y.data(), X.data(), ld, t.data(), dd, N, P, S, R, 0, P) == 0);
        REQUIRE(combo_ref_gossip_round(Y.data(), X.data(), ld, tp.data(), dd, N, P, S, R, 0, P) == 0);
        REQUIRE(combo_ref_gossip_round_f64(Y64.data(), X.data(), ld, t.data(), dd, N, P, S, R, 0, P) == 0);
        REQUIRE(combo_ref_gossip_round_dynamic(Y.data(), X.data(), ld, td.data(), dd, status.data(), N, P,
                                               S, R, 0, P) == 0);
        REQUIRE(combo_ref_aggregation_divergence(dist.data(), X.data(), ld, dd, N, P) == 0);
        std::vector<float> Xc = X;
        REQUIRE(combo_ref_local_sgd_then_gossip(Y.data(), Xc.data(), G.data(), 0.01f, ld, t.data(), dd, N,
                                                P, S, R, 0, P) == 0);
        Xc = X;
        REQUIRE(combo_ref_local_sgd_steps_then_gossip(Y.data(), Xc.data(), G.data(), 3, 0.01f, ld, t.data(),
                                                      dd, N, P, S, R, 0, P) == 0);
    }
    // a column window in the middle, tightly allocated
    if (P > 10) {
        const int64_t c0 = P / 3, nc = P / 2;
        std::vector<float> Xw((size_t)(N * nc)), Yw((size_t)(N * nc));
        for (int32_t w = 0; w < N; ++w)
            for (int64_t c = 0; c < nc; ++c) Xw[(size_t)(w * nc + c)] = X[(size_t)(w * ld + c0 + c)];
        REQUIRE(combo_ref_gossip_round(Yw.data(), Xw.data(), nc, t.data(), nullptr, N, P, S, R, c0, nc) == 0);
    }
    return 0;
}

int main() {
    const struct { int32_t N; int64_t P; int32_t S, R; int64_t pad; } cases[] = {
        {1, 1, 1, 0, 0}, {2, 2, 2, 1, 0}, {3, 6, 2, 2, 1}, {4, 65, 8, 2, 3}, {5, 97, 97, 4, 0},
        {7, 1003, 7, 3, 5}, {9, 50, 3, 8, 0}, {16, 333, 1, 15, 2}, {6, 10, 10, 0, 0},
    };
    for (const auto& c : cases)
        if (run_case(c.N, c.P, c.S, c.R, c.pad)) return 1;
    // rejected arguments must be rejected, not crash
    int32_t dummy[8];
    if (combo_ref_make_peer_table(dummy, 2, 2, 2, 0, 0) == 0) return 1;
    if (combo_ref_make_peer_table_pooled(dummy, 0, 2, 0, 0, 0) == 0) return 1;
    std::printf("oracle selftest ok\n");
    return 0;
}
