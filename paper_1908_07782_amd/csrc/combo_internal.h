// Internal declarations shared by the translation units of libcombo (HIP path only).
#ifndef COMBO_INTERNAL_H_
#define COMBO_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace combo {

constexpr int kThreads = 256;          // 4 wavefronts of 64 lanes per workgroup
constexpr int kXcds = 8;               // accelerator complex dies of one MI355X

// Arguments of one aggregation round, passed by value to the kernels.
struct RoundArgs {
    float* dst;
    const float* src;
    const int32_t* peers;
    const float* dsz;        // dataset sizes |D_j| or nullptr (uniform weights)
    const float* grad;       // gradients for the fused local step, or nullptr
    const uint8_t* status;   // dynamic workers: 0 offline, 1 active, 2 newcomer; or nullptr
    int64_t ld;              // row pitch in elements
    int64_t P;               // parameters per worker
    int64_t L;               // floor(P / S): length of every segment but the last
    int32_t N, S, R;
    uint32_t tiles_per_row;  // ceil(P / tile columns)
    int32_t swizzle;         // 1: XCD-aware workgroup order
    int32_t p32;             // 1: P < 2^32, segment lookup may divide in 32 bits
    float inv;               // 1.0f / (float)(R + 1)
    float lr;                // learning rate of the fused local step
    int32_t tau;             // number of fused local steps (gradient slices)
    int64_t grad_slice;      // elements between consecutive gradient slices
    int32_t tile_shift;      // front buffer and gradients: 0: row-major [N][ld]; else log2(Wt) of the tiled layout [T][N][Wt]
    int64_t dst_ld;          // back buffer: its own pitch and layout (normally the front buffer's)
    int32_t dst_tile_shift;
    uint32_t nstrips;        // slab kernels: ceil(P / strip width)
    uint32_t strips_per_xcd; // slab kernels: 0: workgroup i takes strip i; else the XCDs (i mod 8) take turns
                             // at runs of this many consecutive strips
    uint64_t hash_sr;        // table-free rounds: peer-hash state after seed and round
};

// launchers; each returns hipGetLastError() of its launch
hipError_t launch_round(const RoundArgs& a, int tile_cols, bool vec, hipStream_t st);
hipError_t launch_round_dynamic_elementwise(const RoundArgs& a, hipStream_t st);
hipError_t launch_peer_table_dynamic(int32_t* peers, const uint8_t* status, int32_t N, int32_t S,
                                     int32_t R, uint64_t seed, uint64_t round, hipStream_t st);
hipError_t launch_sgd_step(float* x, const float* g, float lr, int64_t ld, int32_t N, int64_t P,
                           bool vec, hipStream_t st);
hipError_t launch_peer_table(int32_t* peers, int32_t N, int32_t S, int32_t R, uint64_t seed,
                             uint64_t round, hipStream_t st);

hipError_t launch_peer_table_pooled(int32_t* peers, int32_t N, int32_t S, int32_t R,
                                    uint64_t seed, uint64_t round, hipStream_t st);
hipError_t launch_peer_in_degree(int32_t* deg, const int32_t* peers, int32_t N, uint64_t entries,
                                 hipStream_t st);

// Aggregation divergence (divergence.hip)
constexpr int kDivPartialsPerRow = 4096;   // workspace: at most this many workgroup partials per worker row
constexpr int kDivStaticRows = 128;        // worker rows the library-held workspace has room for
int divergence_strip_cols(int32_t N);
bool divergence_width_ok(int32_t N, int strip_cols);
hipError_t launch_divergence(double* dist2, double* workspace, const float* x, int64_t ld,
                             const float* dsz, int32_t N, int64_t P, int strip_cols, bool vec,
                             int arena_tile, hipStream_t st);
// tiled arena whose tiles fit the register slots of one wavefront (divergence_tile_fits):
// one wavefront per tile, no workgroup-level exchange
bool divergence_tile_fits(int32_t N, int tile_cols);
hipError_t launch_divergence_tiles(double* dist2, double* workspace, const float* x,
                                   const float* dsz, int32_t N, int64_t P, int tile_cols,
                                   hipStream_t st);

// the workspace the library holds itself (a static device array, one per GPU) and its size
hipError_t divergence_static_workspace(double** workspace, int64_t* bytes);

// layout conversion kernels (layout.hip)
// run: 0: workgroup i converts tile i; else the XCDs take turns at runs of `run` tiles
hipError_t launch_pack_tiled(float* tiled, const float* rows, int64_t ld, int32_t N, int64_t P,
                             int tile_cols, uint32_t run, hipStream_t st);
hipError_t launch_unpack_tiled(float* rows, int64_t ld, const float* tiled, int32_t N, int64_t P,
                               int tile_cols, uint32_t run, hipStream_t st);

// gather-free passes with the kernels' memory access patterns (probe.hip)
hipError_t launch_bandwidth_probe(int kind, float* dst, const float* src, int32_t N, int64_t ld, int64_t P,
                                  int cols, int param, hipStream_t st);

// Slab kernel: one workgroup stages all N rows of a strip of `strip_cols` columns in
// LDS.  slab_strip_cols() picks the strip width for N workers (0: does not fit in LDS).
int slab_strip_cols(int32_t N, int32_t R, int requested, bool hashed = false);
size_t slab_budget_bytes(int32_t R, bool tiled);   // slab size the strip and tile widths aim for
hipError_t launch_round_slab(const RoundArgs& a, int strip_cols, hipStream_t st);
// the same kernel drawing its peers in-kernel from a.hash_sr (R <= 8, no table)
hipError_t launch_round_slab_hashed(const RoundArgs& a, int strip_cols, hipStream_t st);
// dynamic-worker variants (a.status != nullptr); grid and LDS size as computed by launch_round_slab
hipError_t launch_round_slab_dynamic(const RoundArgs& a, int strip_cols, uint32_t grid, size_t lds,
                                     hipStream_t st);
size_t slab_lds_bytes(int32_t N, int32_t R, int strip_cols, bool hashed);
uint32_t slab_grid(const RoundArgs& a, int strip_cols);
size_t slab_lds_request(const RoundArgs& a, int strip_cols, bool hashed);
void set_slab_lds_floor(int bytes);   // least LDS a slab launch asks for (limits resident workgroups)
int get_slab_lds_floor();
int slab_threads(int32_t N, int strip_cols);
void set_slab_threads(int threads);   // 0: automatic, else 256 or 512
int get_slab_threads();

// number of workgroups launch_round would use, or 0 if that exceeds the grid limit
uint64_t round_grid_size(int32_t N, int64_t P, int tile_cols, bool swizzle);

}  // namespace combo
#endif
