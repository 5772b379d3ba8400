// Shared host/device helpers of the HIP library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "adacomp.h"

namespace adacomp {

constexpr int WAVE = 64;
constexpr uint32_t KEY_MASK = 0x7fffffffu;

// Magnitude key: IEEE-754 bit pattern with the sign cleared.  Unsigned order of
// the key is the order of |x| ("largest ... in absolute value", Alg. 1,
// SELECT_GRAD); denormals keep their exact order, +-0 map to 0.
__device__ __forceinline__ uint32_t mag_key(uint32_t bits) { return bits & KEY_MASK; }

// Number of set bits of `m` below the calling lane (wave64).
__device__ __forceinline__ uint32_t lanes_below(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t popc64(uint64_t m) { return (uint32_t)__popcll(m); }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// The card hands the workgroups of a launch to its 8 XCDs (each with an L2 of its own) in turn.
// For kernels whose consecutive workgroups read consecutive memory this gives every XCD one
// contiguous eighth of the launch instead of every eighth piece: position in the launch of
// the calling workgroup (a bijection of 0 .. gridDim.x - 1 whatever the real hand-out is).
constexpr uint32_t XCDS = 8;
__device__ __forceinline__ uint32_t xcd_contiguous_block() {
    const uint32_t q = gridDim.x / XCDS, r = gridDim.x % XCDS, x = blockIdx.x % XCDS, i = blockIdx.x / XCDS;
    return x * q + (x < r ? x : r) + i;
}

// Exclusive prefix sum of x over a workgroup of NWAVES full waves; `total` receives the
// sum.  s_wave: NWAVES words of LDS, free for reuse when the call returns.
template <uint32_t NWAVES>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t *s_wave, uint32_t &total) {
    const uint32_t lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    uint32_t incl = x;
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        const uint32_t y = __shfl_up(incl, d);
        if (lane >= (uint32_t)d) incl += y;
    }
    if (lane == WAVE - 1) s_wave[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
    total = 0;
#pragma unroll
    for (uint32_t w = 0; w < NWAVES; ++w) {
        const uint32_t s = s_wave[w];
        if (w < wave) base += s;
        total += s;
    }
    __syncthreads();
    return base + incl - x;
}

// Asynchronous host->device upload of small tables through kernel arguments.
// The payload travels inside the launch packet, so the host buffer may be freed
// as soon as the call returns, no pinned memory is needed and the copy can be
// captured into a graph like any other kernel.
constexpr uint32_t PUT_WORDS = 448;  // 3584 bytes of payload per launch
struct PutPayload {
    uint64_t w[PUT_WORDS];
};
hipError_t put_async(void *dst_dev, const void *src_host, size_t bytes, hipStream_t s);

// dst[i] = value for i < n (32-bit words)
hipError_t fill_u32_async(uint32_t *dst_dev, uint32_t value, size_t n, hipStream_t s);

// Start/stop events for one kernel dispatch when timing of kernel `id` is switched on.
class ProfScope {
public:
    explicit ProfScope(int id);
    bool active() const { return beg_ != nullptr; }
    hipEvent_t beg() const { return beg_; }
    hipEvent_t end() const { return end_; }

private:
    hipEvent_t beg_, end_;
};

// Launch `kernel` on stream `s`; with timing on, the dispatch carries its own events.
#define ADACOMP_LAUNCH(id, kernel, grid, block, s, ...)                                       \
    do {                                                                                      \
        ::adacomp::ProfScope prof_scope_(id);                                                 \
        if (prof_scope_.active())                                                             \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, s, prof_scope_.beg(), prof_scope_.end(), 0, \
                                  __VA_ARGS__);                                               \
        else                                                                                  \
            hipLaunchKernelGGL(kernel, grid, block, 0, s, __VA_ARGS__);                       \
    } while (0)

}  // namespace adacomp
