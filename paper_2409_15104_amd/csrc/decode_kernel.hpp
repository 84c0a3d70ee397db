// Split-KV decode attention for one new token (gfx950): every WAVEFRONT streams one KV head of a
// range of keys on its own, no workgroup barrier anywhere.
//
// The step is HBM-bound (K and V are read once, 512 bytes per key and KV head, against 1 Kflop),
// so the design goal is bytes in flight: each wavefront owns private LDS rings of 32-key tiles filled
// by direct global->LDS loads, two stages for K and three for V (all of the 160 KiB of LDS: V is
// consumed last in a tile, so the extra stage goes to it), i.e. up to 40 KiB outstanding per
// wavefront and 160 KiB per compute unit (4 wavefronts) to cover the memory latency at the HBM rate.  The g query heads that share a KV head are the 32 "query columns" of the same
// transposed-score MFMA scheme as the prefill kernels (columns >= g carry zeros): the matrix
// pipe is mostly idle and does not matter here.
//
// Each wavefront writes a normalised partial O and its LSE for its key range; the ranges are
// merged by combine_splits_kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace pec {

struct DecodeParams {
    const __bf16* q;          // [n_q_heads][128], the one query token
    const unsigned char* k;   // [sk][n_kv_heads][128] bf16
    const unsigned char* v;
    float* o_part;            // [n_ranges][n_q_heads][128]
    float* lse_part;          // [n_ranges][n_q_heads], natural log
    int32_t sk;
    int32_t n_q_heads, n_kv_heads, group;
    int32_t n_ranges;         // key ranges (each wavefront takes one range of one KV head)
    int32_t range_len;        // keys per range, a multiple of 32
    float scale_log2;
};

constexpr int kDecTile = 32;                          // keys per tile
constexpr int kDecTileBytes = kDecTile * kRowBytes;   // 8 KiB for K, 8 KiB for V
constexpr int kDecWaves = 4;
constexpr int kDecKStages = 2, kDecVStages = 3;      // ring depths: K(j) is requested two tiles ahead, V(j) three

__global__ __launch_bounds__(kDecWaves * 64) void decode_kernel(const DecodeParams p) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds_k[kDecWaves][kDecKStages][kDecTileBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_v[kDecWaves][kDecVStages][kDecTileBytes];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, hl = lane >> 5;

    // workgroup -> (key range, group of four KV heads), wavefront -> KV head: the wavefronts of a
    // workgroup (and the neighbouring workgroups of a range) read the same tokens, so HBM sees whole
    // token rows instead of one 256-byte head slice per reader.  One contiguous logical range per XCD.
    const int head_groups = (p.n_kv_heads + kDecWaves - 1) / kDecWaves;
    const int total = p.n_ranges * head_groups;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (logical >= total) return;
    const int range = logical / head_groups;
    const int kvh = (logical % head_groups) * kDecWaves + wave;
    if (kvh >= p.n_kv_heads) return;

    const int64_t key_begin = (int64_t)range * p.range_len;
    const int len = (int)max((int64_t)0, min((int64_t)p.range_len, (int64_t)p.sk - key_begin));
    const int n_tiles = (len + kDecTile - 1) / kDecTile;
    const int g = p.group;

    // ---- Q fragments: column l32 = head l32 of the group
    bf16x8 qf[8];
    {
        const __bf16* qrow = p.q + ((int64_t)kvh * g + l32) * kHeadDim + 8 * hl;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (l32 < g) raw = *reinterpret_cast<const u32x4*>(qrow + 16 * t);
            qf[t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // ---- tile loads (asm: M0 = LDS address, SGPR base + 32-bit lane offset).  One instruction moves
    // four key rows; rows past the end of the range re-read its last row (finite data, masked below).
    const uint32_t kv_stride_b = (uint32_t)p.n_kv_heads * kHeadDim * 2;
    const unsigned char* kbase = p.k + (key_begin * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);
    const unsigned char* vbase = p.v + (key_begin * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);
    const int ld_row = lane >> 4, ld_pos = lane & 15;
    auto dma16 = [](const unsigned char* sbase, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(voff), "s"(sbase), "s"(lds_addr)
                     : "memory", "m0");
    };
    auto issue_half = [&](const unsigned char* base, bool is_v, int tile, unsigned char* stage) {
        if (tile >= n_tiles) return;
        const int key0 = tile * kDecTile;
        const int last = len - 1 - key0;   // last valid row of this tile (>= 0)
        const unsigned char* tb = base + (int64_t)key0 * kv_stride_b;
        const uint32_t l0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)stage;
#pragma unroll
        for (int i = 0; i < kDecTile / 4; ++i) {
            const int key = 4 * i + ld_row;
            const uint32_t row_off = (uint32_t)min(key, last) * kv_stride_b;
            const uint32_t col = is_v ? (uint32_t)((((ld_pos >> 2) ^ (key & 3)) << 2) | (ld_pos & 3)) * 16u
                                      : (uint32_t)(ld_pos ^ (key & 15)) * 16u;
            dma16(tb, row_off + col, l0 + i * 1024);
        }
    };
    auto issue_k = [&](int tile) { issue_half(kbase, false, tile, lds_k[wave][tile % kDecKStages]); };
    auto issue_v = [&](int tile) { issue_half(vbase, true, tile, lds_v[wave][tile % kDecVStages]); };
    constexpr int kLoadsPerHalf = kDecTile / 4;   // 8 load instructions per K or V tile and wavefront

    // ---- LDS operand offsets
    uint32_t k_off[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) k_off[t] = k_lds_off(l32, 2 * t + hl);
    uint32_t v_off[4];
    {
        const int gi = l32 & 15, gg = l32 >> 4;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) v_off[dt] = v_lds_off(4 * hl + (gi >> 2), dt * 64 + gg * 32 + (gi & 3) * 8);
    }

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2 = p.scale_log2;

    // Issue order: K(0) V(0) K(1) V(1) V(2), then per tile j: K(j+2) V(j+3).  Loads retire in order, so
    // when tile j starts the requests younger than K(j) and V(j) are V(j+1) | K(j+1) V(j+2): 24 of them
    // in the steady state, fewer at the end of the range (tiles past the end are not requested).
    issue_k(0);
    issue_v(0);
    issue_k(1);
    issue_v(1);
    issue_v(2);
    static_assert(kLoadsPerHalf == 8 && kDecKStages == 2 && kDecVStages == 3, "the vmcnt immediates below assume this");
    for (int j = 0; j < n_tiles; ++j) {
        const int left = n_tiles - 1 - j;   // tiles after this one
        if (left >= 2) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");        // V(j+1) K(j+1) V(j+2)
        else if (left == 1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");   // V(j+1) K(j+1)
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const unsigned char* kst = lds_k[wave][j % kDecKStages];
        const unsigned char* vst = lds_v[wave][j % kDecVStages];

        // S^T = K Q^T for 32 keys
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kst + k_off[t]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s, 0, 0, 0);
        }
        // keys past the end of the range (only in its last tile)
        const int lim = len - 1 - j * kDecTile - 4 * hl;   // compare against 8*(r/4) + r%4
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
        {
            const uint32_t u = __builtin_bit_cast(uint32_t, mx);
            const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
            mx = fmaxf(__builtin_bit_cast(float, (uint32_t)sw[0]), __builtin_bit_cast(float, (uint32_t)sw[1]));
        }
        // every tile has at least one valid key, so the reference is finite from the first tile on
        const float mx2 = mx * sl2;
        const float m_new = (mx2 > m_run + 8.f) ? mx2 : m_run;   // lazy reference, as in the prefill kernel
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float rs = 0.f;
        bf16x8 pp[2];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            u32x4 packed;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f32x2 x = {__builtin_amdgcn_exp2f(fmaf(s[8 * t2 + 2 * e], sl2, -m_new)),
                                 __builtin_amdgcn_exp2f(fmaf(s[8 * t2 + 2 * e + 1], sl2, -m_new))};
                rs += x[0] + x[1];
                packed[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
            }
            pp[t2] = __builtin_bit_cast(bf16x8, packed);
        }
        l_run = l_run * alpha + rs;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
        // O^T += V^T P^T
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const unsigned char* src = vst + v_off[dt] + ks * 16 * kRowBytes;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(src));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (__attribute__((address_space(3))) bf16x4*)(src + 8 * kRowBytes));
                const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pp[ks], o[dt], 0, 0, 0);
            }
        // the LDS reads of this tile's stages are consumed (the MFMAs above needed them): refill them
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        issue_k(j + 2);
        issue_v(j + 3);
    }

    // ---- partial result of this range
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (l32 < g) {
        const int head = kvh * g + l32;
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
        if (hl == 0) p.lse_part[(int64_t)range * p.n_q_heads + head] = lse;
        float* orow = p.o_part + ((int64_t)range * p.n_q_heads + head) * kHeadDim + 4 * hl;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f32x4 x;
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = o[dt][4 * b + i] * inv;
                *reinterpret_cast<f32x4*>(orow + 32 * dt + 8 * b) = x;
            }
    }
}

}  // namespace pec
