// Measurement support: a kernel that does nothing but issue 32-bit integer VALU instructions, so
// that the benchmark can divide by the rate this GPU actually sustains (clock under load, issue
// limits) as well as by the nominal 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.
#include "harp_internal.h"

namespace harp {

namespace {

constexpr int kChains = 8;   // independent dependency chains per lane: hides the VALU latency

__global__ __launch_bounds__(256) void k5_valu_int32(uint32_t *sink, int iters, uint32_t key) {
    uint32_t a[kChains];
#pragma unroll
    for (int k = 0; k < kChains; ++k) a[k] = threadIdx.x * 2654435761u + k;
    const uint32_t x = (blockIdx.x << 1) | 1u;
    uint32_t y = threadIdx.x ^ key;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kChains; ++k) {
            a[k] += x;                         // one add
            a[k] = a[k] > y ? a[k] : y;        // one max
        }
        y ^= key >> 7;                         // keeps the loop body from being hoisted or folded
    }
    uint32_t all = 0;
#pragma unroll
    for (int k = 0; k < kChains; ++k) all ^= a[k];
    if (all == key) sink[0] = all;             // one chance in 2^32 per lane: keeps the chains alive
}

}  // namespace

void launch_valu_int32(int blocks, int iters, uint32_t *sink, hipStream_t st) {
    hipLaunchKernelGGL(k5_valu_int32, dim3(blocks), dim3(256), 0, st, sink, iters, 0x9E3779B9u * uint32_t(iters));
}

}  // namespace harp
