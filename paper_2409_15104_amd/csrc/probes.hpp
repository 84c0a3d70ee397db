// Measurement aids for the rooflines, no part of the method.
//  * mfma_probe_kernel: bare matrix-pipe rate of the chip as it stands (clocks, power cap, operand
//    data): a loop of independent v_mfma_f32_32x32x16_bf16 and nothing else.  The attention kernel's
//    rate is reported against this as well as against the nominal peak.
//  * hbm_read_probe_kernel: a streaming read of a large buffer with many 16-byte loads in flight per
//    thread: the read bandwidth the memory system delivers, against which the HBM-bound kernels
//    (decode, layout exchange) are reported as well as against the nominal 8 TB/s.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace pec {

constexpr int kProbeWaves = 8;        // two wavefronts per SIMD, as in the attention kernel
constexpr int kProbeFrags = 8;        // distinct A and B fragments cycled through
constexpr int kProbeMfmaPerIter = 32; // MFMAs per loop iteration and wavefront

// operands: at least kProbeFrags * 2 * 64 * 16 bytes of bf16 (A fragments, then B fragments; lane l
// takes 16 bytes at (frag * 64 + l) * 16).  sink: one float per thread, written once so that the
// accumulators count as used.
__global__ __launch_bounds__(kProbeWaves * 64) void mfma_probe_kernel(const u32x4* __restrict__ operands, int iters,
                                                                      float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[kProbeFrags], b[kProbeFrags];
#pragma unroll
    for (int f = 0; f < kProbeFrags; ++f) {
        a[f] = __builtin_bit_cast(bf16x8, operands[f * 64 + lane]);
        b[f] = __builtin_bit_cast(bf16x8, operands[(kProbeFrags + f) * 64 + lane]);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kProbeMfmaPerIter; ++m)
            acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m % kProbeFrags], b[(m / 4) % kProbeFrags], acc[m & 3], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Reads n chunks of 16 bytes, eight independent loads in flight per thread; writes one word per thread
// to `sink` only if the xor of everything read has an improbable value, so that the loads cannot be
// dropped.
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const u32x4* __restrict__ src, size_t n,
                                                             uint32_t* __restrict__ sink) {
    constexpr int kBatch = 8;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += kBatch * stride) {
        u32x4 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (i + u * stride < n) v[u] = __builtin_nontemporal_load(src + i + u * stride);
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) acc ^= v[u];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = 1u;
}

}  // namespace pec
