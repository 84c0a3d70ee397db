// Bare matrix-pipe rate of the chip as it stands (clocks, power cap, operand data): a loop of
// independent v_mfma_f32_32x32x16_bf16 and nothing else.  Measurement aid for the roofline: the
// attention kernel's rate is reported against this as well as against the nominal peak.
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

}  // namespace pec
