// Internal declarations shared by the translation units of libbgl.
// Host-side error plumbing, handle layouts and the small device helpers
// (hashing, block scan) that more than one kernel file uses.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <exception>
#include <new>

#include "bgl.h"

namespace bgl {

// ----------------------------------------------------------------- errors
void set_error(const char *fmt, ...);

#define BGL_FAIL(code, ...)            \
    do {                               \
        ::bgl::set_error(__VA_ARGS__); \
        return (code);                 \
    } while (0)

#define BGL_HIP(call)                                                               \
    do {                                                                            \
        hipError_t e__ = (call);                                                    \
        if (e__ != hipSuccess) {                                                    \
            ::bgl::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), \
                             __FILE__, __LINE__);                                   \
            return e__ == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP;              \
        }                                                                           \
    } while (0)

// The C ABI promises that nothing throws: every entry point is a function-try-block whose
// handler returns this (called inside the handler: it looks at the exception in flight).
inline int caught()
{
    try {
        throw;
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return BGL_ENOMEM;
    } catch (const std::exception &e) {
        set_error("unexpected exception: %s", e.what());
        return BGL_EHIP;
    } catch (...) {
        set_error("unexpected exception");
        return BGL_EHIP;
    }
}
#define BGL_NOTHROW_END catch (...) { return ::bgl::caught(); }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace bgl

// ----------------------------------------------------------------- handles
struct bgl_graph {
    const void *row_ptr;  // device-visible
    const int32_t *col;   // device-visible
    int64_t num_nodes;
    int64_t num_edges;
    int bits;
    int placement;
    void *owned_row_ptr;  // hipMalloc'd copies (BGL_DEVICE), else null
    void *owned_col;
    int device;
};

// ----------------------------------------------------------------- device helpers
#if defined(__HIPCC__)
namespace bgl {

constexpr int kWave = 64;

// MurmurHash3 32-bit finaliser: spreads node ids over table positions.
__device__ __forceinline__ uint32_t hash32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}

__device__ __forceinline__ int wave_incl_scan(int v)
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive prefix sum of one int per thread over a block of THREADS threads
// (a multiple of 64, at most 1024).  `total` receives the block sum.  `sh` is
// LDS scratch of THREADS/64 ints.  Ends with a barrier, so `sh` may be reused.
template <int THREADS>
__device__ __forceinline__ int block_excl_scan(int v, int *sh, int &total)
{
    constexpr int NW = THREADS / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    int inc = wave_incl_scan(v);
    if (lane == kWave - 1) sh[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        int s = sh[i];
        if (i < w) base += s;
        tot += s;
    }
    total = tot;
    __syncthreads();
    return base + inc - v;
}

// Exclusive prefix sums of `tiles` per-tile counts, computed by ONE workgroup of
// THREADS threads (prefix may alias counts).  The list kernels use it for calls of
// many tiles, where every workgroup summing its predecessors' counts itself
// would make the work quadratic in the tile count.
template <int THREADS>
__device__ __forceinline__ void scan_tile_counts(const int32_t *counts, int64_t tiles, int32_t *prefix, int *sh)
{
    int carry = 0;
    for (int64_t base = 0; base < tiles; base += THREADS) {
        const int64_t t = base + threadIdx.x;
        const int v = t < tiles ? counts[t] : 0;
        int tot;
        const int ex = block_excl_scan<THREADS>(v, sh, tot);
        if (t < tiles) prefix[t] = carry + ex;
        carry += tot;
    }
}

constexpr int kScanThreads = 1024;
// From this many tiles on the list kernels read prefixes made by scan_tile_counts.
constexpr int64_t kSelfSumTiles = 4096;

}  // namespace bgl
#endif
