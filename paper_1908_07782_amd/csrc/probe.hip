// Bandwidth probes: gather-free passes with the memory access patterns of the aggregation
// kernels, for measuring what this device's HBM sustains for each pattern (the practical
// ceiling that the round is compared with).  They compute nothing of the method.
//
//   linear copy        every thread streams 128-bit words of one flat array to another
//   read only          the same loads, folded into one value per workgroup
//   write only         the same stores, of a constant
//   row-chunk copy     one workgroup copies N row chunks of `cols` columns of a row-major
//                      [N][ld] matrix: the slab kernel's footprint on a row-major arena,
//                      without LDS staging and without the gather
//   tile copy          one workgroup copies one contiguous N x cols tile: the footprint on
//                      a tiled arena [T][N][cols]
//   multi-read pass    dst[w][e] = src[w][e] + src[w+1][e] + ... (k rows, wrapping): k
//                      read streams and one write stream with no LDS reuse, the footprint
//                      of a gather kernel that fetches every provider row from memory
#include "combo_internal.h"
#include "round_device.h"

namespace combo {
namespace {

constexpr int kProbeThreads = 256;

// 128-bit word u (of FLIGHT) of a thread.  Strided: the words of a thread are a workgroup's
// width (4 KiB) apart, so each of the FLIGHT instructions of a workgroup covers 4 KiB.
// Adjacent: the FLIGHT instructions of one wavefront cover FLIGHT consecutive KiB.
// `run` != 0: the workgroups of one XCD (ids congruent modulo 8) take turns at runs of `run`
// consecutive blocks instead of every eighth block (see the strip order of the slab kernel).
__device__ __forceinline__ uint32_t probe_block(uint32_t run) { return xcd_run_block(blockIdx.x, run); }

template <int FLIGHT, bool ADJACENT>
__device__ __forceinline__ uint64_t probe_word(int u, uint32_t run) {
    const uint64_t base = (uint64_t)probe_block(run) * (kProbeThreads * FLIGHT);
    if (ADJACENT) {
        const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        return base + (uint64_t)((wave * FLIGHT + u) * 64 + lane);
    }
    return base + (uint64_t)u * kProbeThreads + threadIdx.x;
}

// A 128-bit store with the hint the aggregation kernels use (non-temporal), or, `through` set,
// one that is written through to device scope (the sc1 bit) instead of waiting in the L2 for
// its eviction.  Plain copies run about 3.5 % faster with the latter; the aggregation kernels do
// not (their stores come in bursts of a whole slab, which the write-back L2 absorbs).
__device__ __forceinline__ void probe_store(v4f* p, v4f v, uint32_t through) {
    if (through) asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
    else __builtin_nontemporal_store(v, p);
}

template <int FLIGHT, bool ADJACENT>
__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(float* __restrict__ dst,
                                                                   const float* __restrict__ src,
                                                                   uint64_t n4, uint32_t run, uint32_t through) {
    v4f v[FLIGHT];
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) {
        const uint64_t i = probe_word<FLIGHT, ADJACENT>(u, run);
        if (i < n4) v[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src) + i);
    }
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) {
        const uint64_t i = probe_word<FLIGHT, ADJACENT>(u, run);
        if (i < n4) probe_store(reinterpret_cast<v4f*>(dst) + i, v[u], through);
    }
}

template <int FLIGHT, bool ADJACENT>
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(float* __restrict__ dst,
                                                                   const float* __restrict__ src,
                                                                   uint64_t n4, uint32_t run) {
    __shared__ float part[kProbeThreads];
    v4f v[FLIGHT];
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) {
        const uint64_t i = probe_word<FLIGHT, ADJACENT>(u, run);
        v[u] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        if (i < n4) v[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src) + i);
    }
    float s = 0.0f;
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int half = kProbeThreads / 2; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) part[threadIdx.x] += part[threadIdx.x + half];
        __syncthreads();
    }
    const uint32_t block = probe_block(run);
    if (threadIdx.x == 0 && (uint64_t)block * (kProbeThreads * FLIGHT) < n4) dst[block] = part[0];
}

template <int FLIGHT, bool ADJACENT>
__global__ __launch_bounds__(kProbeThreads) void probe_write_kernel(float* __restrict__ dst, uint64_t n4, uint32_t run,
                                                                    uint32_t through) {
    const v4f c = v4f{1.0f, 2.0f, 3.0f, 4.0f};
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) {
        const uint64_t i = probe_word<FLIGHT, ADJACENT>(u, run);
        if (i < n4) probe_store(reinterpret_cast<v4f*>(dst) + i, c, through);
    }
}

// one workgroup per strip of `cols` columns (a multiple of 4; only whole strips are copied);
// TILED: the strip's N chunks are adjacent, else ld apart
template <bool TILED>
__global__ __launch_bounds__(kProbeThreads) void probe_strip_copy_kernel(float* __restrict__ dst,
                                                                         const float* __restrict__ src,
                                                                         int64_t ld, int32_t N, int cols,
                                                                         uint32_t nstrips, uint32_t run) {
    const uint32_t strip = xcd_run_block(blockIdx.x, run);
    if (strip >= nstrips) return;                  // surplus workgroup of the last round of runs
    const int W4 = cols >> 2;
    const int total4 = N * W4;
    const size_t stride = TILED ? (size_t)cols : (size_t)ld;
    const size_t base = TILED ? (size_t)strip * (size_t)N * (size_t)cols : (size_t)strip * (size_t)cols;
    for (int b = 0; b < total4; b += kProbeThreads * 4) {
        v4f v[4];
        size_t off[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = b + u * kProbeThreads + (int)threadIdx.x;
            if (idx < total4) {
                const int row = idx / W4;
                off[u] = (size_t)row * stride + base + (size_t)(idx - row * W4) * 4;
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src + off[u]));
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = b + u * kProbeThreads + (int)threadIdx.x;
            if (idx < total4) store4_stream(dst + off[u], v[u]);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // all loads of the pass consumed (see gossip_slab_kernel.h)
    }
}

// k read streams, one write stream, one workgroup per (1024-column tile, row); whole tiles only
__global__ __launch_bounds__(kProbeThreads) void probe_multi_read_kernel(float* __restrict__ dst,
                                                                         const float* __restrict__ src,
                                                                         int64_t ld, int32_t N, int k,
                                                                         uint32_t tiles) {
    const uint32_t tile = blockIdx.x % tiles;
    const int32_t w = (int32_t)(blockIdx.x / tiles);
    const size_t col = (size_t)tile * 1024 + (size_t)threadIdx.x * 4;
    v4f acc = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src + (size_t)w * (size_t)ld + col));
    for (int j = 1; j < k; ++j) {
        const int32_t p = (w + j) % N;
        acc = add4(acc, load4(src + (size_t)p * (size_t)ld + col));
    }
    store4_stream(dst + (size_t)w * (size_t)ld + col, acc);
}

// LDS read rate: every workgroup fills an 8 KiB block of LDS with its word indices and reads
// it `iters` x 8 times per thread with conflict-free 128-bit reads (the lanes of a wavefront read
// 64 consecutive words, as the aggregation phase of the slab kernel does), adding what it reads;
// the workgroup's sum goes to dst[workgroup].  No global memory traffic to speak of.
constexpr int kLdsProbeWords = 512;
__global__ __launch_bounds__(kProbeThreads) void probe_lds_read_kernel(float* __restrict__ dst, int iters) {
    __shared__ v4f block[kLdsProbeWords];
    __shared__ float part[kProbeThreads];
    for (int i = threadIdx.x; i < kLdsProbeWords; i += kProbeThreads)
        block[i] = v4f{(float)i, 0.0f, 0.0f, 1.0f};
    __syncthreads();
    v4f acc = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    int idx = (int)threadIdx.x;
    for (int it = 0; it < iters; ++it) {
        // the index is made opaque to the compiler in every iteration, so that no read is carried
        // over from the iteration before (the eight words of a thread recur)
        asm volatile("" : "+v"(idx));
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const v4f v = block[(idx + u * 64) & (kLdsProbeWords - 1)];
            acc.x += v.x;
            acc.y += v.y;
            acc.z += v.z;
            acc.w += v.w;
        }
        idx = (idx + 64) & (kLdsProbeWords - 1);
    }
    part[threadIdx.x] = acc.x + acc.w;
    __syncthreads();
    for (int half = kProbeThreads / 2; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) part[threadIdx.x] += part[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) dst[blockIdx.x] = part[0];
}

}  // namespace

// kind: 0 linear copy, 1 read only, 2 write only (n = N*ld floats, `param` = 128-bit words in
// flight per thread: 1, 2, 4 or 8; cols bit 0: the words of a wavefront are adjacent; cols bit 1:
// stores written through to device scope; cols >> 4: blocks per XCD turn);
// 3 row-chunk copy, 4 tile copy (`cols` columns per strip; `param` > 1: the XCDs take turns at
// runs of `param` consecutive strips);
// 5 multi-read pass (`param` = rows read per output); 6 LDS read rate (`cols` workgroups, each
// reading 8 KiB of LDS `param` x 8 times per thread; dst[workgroup] receives a checksum).  Only
// whole 128-bit words, strips and tiles are touched.  Returns hipErrorInvalidValue for shapes the probes do not cover.
hipError_t launch_bandwidth_probe(int kind, float* dst, const float* src, int32_t N, int64_t ld, int64_t P,
                                  int cols, int param, hipStream_t st) {
    const uint64_t n4 = (uint64_t)N * (uint64_t)ld / 4;
    if (kind >= 0 && kind <= 2) {
        if (param != 1 && param != 2 && param != 4 && param != 8) return hipErrorInvalidValue;
        const uint64_t per_wg = (uint64_t)kProbeThreads * (uint64_t)param;
        uint64_t grid64 = (n4 + per_wg - 1) / per_wg;
        const bool adjacent = (cols & 1) != 0;
        const uint32_t through = (cols & 2) != 0 ? 1u : 0u;
        const uint32_t run = (uint32_t)(cols >> 4);              // blocks per XCD turn, 0: block = id
        if (run != 0) grid64 = (grid64 + 8ull * run - 1) / (8ull * run) * (8ull * run);   // surplus blocks are out of range
        // a grid dimension holds fewer than 2^32 work-items
        if (cols < 0 || grid64 == 0 || grid64 * kProbeThreads > 0xFFFFFFFFull) return hipErrorInvalidValue;
        const dim3 grid((uint32_t)grid64), block(kProbeThreads);
#define COMBO_PROBE_FLIGHT(KERNEL, ...)                                                                   \
        switch (param * 2 + (adjacent ? 1 : 0)) {                                                         \
            case 2: case 3: hipLaunchKernelGGL((KERNEL<1, false>), grid, block, 0, st, __VA_ARGS__); break; \
            case 4: hipLaunchKernelGGL((KERNEL<2, false>), grid, block, 0, st, __VA_ARGS__); break;       \
            case 5: hipLaunchKernelGGL((KERNEL<2, true>), grid, block, 0, st, __VA_ARGS__); break;        \
            case 8: hipLaunchKernelGGL((KERNEL<4, false>), grid, block, 0, st, __VA_ARGS__); break;       \
            case 9: hipLaunchKernelGGL((KERNEL<4, true>), grid, block, 0, st, __VA_ARGS__); break;        \
            case 16: hipLaunchKernelGGL((KERNEL<8, false>), grid, block, 0, st, __VA_ARGS__); break;      \
            default: hipLaunchKernelGGL((KERNEL<8, true>), grid, block, 0, st, __VA_ARGS__); break;       \
        }
        if (kind == 0) { COMBO_PROBE_FLIGHT(probe_copy_kernel, dst, src, n4, run, through) }
        else if (kind == 1) { COMBO_PROBE_FLIGHT(probe_read_kernel, dst, src, n4, run) }
        else { COMBO_PROBE_FLIGHT(probe_write_kernel, dst, n4, run, through) }
#undef COMBO_PROBE_FLIGHT
        return hipGetLastError();
    }
    if (kind == 3 || kind == 4) {
        if (cols < 4 || cols % 4 != 0 || P < cols) return hipErrorInvalidValue;
        const uint64_t strips = (uint64_t)P / (uint64_t)cols;        // whole strips only
        if (param < 0 || param > 65536) return hipErrorInvalidValue;
        const uint32_t run = param > 1 ? (uint32_t)param : 0u;
        uint64_t grid64 = strips;
        if (run != 0) grid64 = (strips + 8ull * run - 1) / (8ull * run) * (8ull * run);
        // a grid dimension holds fewer than 2^32 work-items
        if (strips > 0x7FFFFFF0ull || grid64 * kProbeThreads > 0xFFFFFFFFull) return hipErrorInvalidValue;
        if (kind == 3)
            hipLaunchKernelGGL(probe_strip_copy_kernel<false>, dim3((uint32_t)grid64), dim3(kProbeThreads), 0,
                               st, dst, src, ld, N, cols, (uint32_t)strips, run);
        else
            hipLaunchKernelGGL(probe_strip_copy_kernel<true>, dim3((uint32_t)grid64), dim3(kProbeThreads), 0,
                               st, dst, src, ld, N, cols, (uint32_t)strips, run);
        return hipGetLastError();
    }
    if (kind == 5) {
        const uint64_t tiles = (uint64_t)P / 1024;
        if (param < 1 || param > N || tiles == 0 || tiles * (uint64_t)N > 0x7FFFFFFFull)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL(probe_multi_read_kernel, dim3((uint32_t)(tiles * (uint64_t)N)), dim3(kProbeThreads), 0,
                           st, dst, src, ld, N, param, (uint32_t)tiles);
        return hipGetLastError();
    }
    if (kind == 6) {
        if (cols < 1 || (uint64_t)cols > n4 * 4 || param < 1 || param > (1 << 20)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(probe_lds_read_kernel, dim3((uint32_t)cols), dim3(kProbeThreads), 0, st, dst, param);
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

}  // namespace combo
