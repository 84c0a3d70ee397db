// Plain blockwise attention forward kernel for gfx950 (CDNA4), kept as the cross-check of the
// pipelined kernel in fwd_kernel_il.hpp (selected per call with PEC_FLAG_SIMPLE_KERNEL): the same
// mathematics -- S^T = K Q^T and O^T = V^T P^T on v_mfma_f32_32x32x16_bf16, online softmax in
// registers (Eq. 2-3 of the paper evaluated tile by tile with the exact running row maximum and
// denominator) -- in the most direct organisation: 8 wavefronts x 32 query rows per workgroup, K/V
// tiles of 64 keys staged global -> registers -> LDS (double buffered), one workgroup per (query
// tile, head), no persistence, no lazy softmax reference, no fused split-KV mode.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace pec {

constexpr int kSimpleWaves = 8;
constexpr int kSimpleBM = kSimpleWaves * 32;   // query rows per workgroup

__global__ __launch_bounds__(kSimpleWaves * 64) void fwd_simple_kernel(const FwdParams p) {
    constexpr int NT = 1, NWAVES = kSimpleWaves;
    constexpr int NTHREADS = NWAVES * 64;
    constexpr int BM = NWAVES * NT * 32;
    constexpr int LOADS = (kBN * 16) / NTHREADS;  // 16-byte chunks per thread per tile

    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * kTileBytes];  // K0 V0 K1 V1

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int hl = lane >> 5;

    // ---- block -> (kv head, work item, head in group); XCD-aware: consecutive block ids
    // go round-robin to the 8 XCDs, so give each XCD one contiguous range of the
    // (kv head major) logical order and its L2 sees as few KV heads as possible.
    const int64_t total = (int64_t)p.n_items * p.n_q_heads;
    const int64_t per_xcd = (total + 7) >> 3;
    const int64_t logical = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int per_kvh = p.n_items * p.group;
    const int kvh = (int)(logical / per_kvh);
    const int rem = (int)(logical % per_kvh);
    const int item = rem / p.group;
    const int head = kvh * p.group + rem % p.group;

    int sq, sk, delta, qt;
    int64_t q_tok0, kv_tok0;
    if (p.cu_seqlens) {
        if (item >= *p.n_work) return;
        const WorkItem w = p.work[item];
        const int b0 = min(max(p.cu_seqlens[w.seq], 0), p.total_tokens);
        const int b1 = min(max(p.cu_seqlens[w.seq + 1], b0), p.total_tokens);
        sq = sk = b1 - b0;
        delta = 0;
        qt = w.qtile;
        q_tok0 = kv_tok0 = b0;
    } else {
        sq = p.sq;
        sk = p.sk;
        delta = p.delta;
        qt = p.causal ? (p.n_items - 1 - item) : item;  // longest rows first
        q_tok0 = kv_tok0 = 0;
    }
    const int causal = p.causal;
    const int row0 = qt * BM;                    // first local row of the block
    const int rw0 = row0 + wave * (NT * 32);     // first local row of the wave
    const int blk_last = min(sq, row0 + BM) - 1;

    // keys [0, kv_end) can be visible to some row of the block
    int kv_end = sk;
    if (causal) kv_end = max(0, min(sk, blk_last + delta + 1));
    const int n_tiles = (kv_end + kBN - 1) / kBN;

    const int64_t q_stride = (int64_t)p.n_q_heads * kHeadDim;
    const int64_t kv_stride = (int64_t)p.n_kv_heads * kHeadDim;
    const __bf16* kbase = p.k + kv_tok0 * kv_stride + (int64_t)kvh * kHeadDim;
    const __bf16* vbase = p.v + kv_tok0 * kv_stride + (int64_t)kvh * kHeadDim;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds 8 head-dim values per 16-wide step
    bf16x8 qf[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = rw0 + nt * 32 + l32;
        const __bf16* qrow = p.q + (q_tok0 + row) * q_stride + (int64_t)head * kHeadDim + 8 * hl;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row < sq) raw = *reinterpret_cast<const u32x4*>(qrow + 16 * t);
            qf[nt][t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // ---- running state
    f32x16 o[4][NT];
    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = -INFINITY;
        l_run[nt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][nt][r] = 0.f;
    }
    if (p.acc_in) {
        // continue from a normalised partial: weight 1 at maximum lse_in
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int row = rw0 + nt * 32 + l32;
            if (row < sq) {
                const float lin = p.lse_in[(int64_t)head * p.lse_stride + q_tok0 + row];
                if (lin != -INFINITY) {
                    m_run[nt] = lin * kLog2e;
                    l_run[nt] = hl == 0 ? 1.f : 0.f;   // the halves' partial sums are added at the end
                    const float* arow = p.acc_in + (q_tok0 + row) * q_stride + (int64_t)head * kHeadDim + 4 * hl;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const f32x4 x = *reinterpret_cast<const f32x4*>(arow + 32 * dt + 8 * b);
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[dt][nt][4 * b + i] = x[i];
                        }
                }
            }
        }
    }

    // ---- K/V tile staging: global -> registers -> LDS
    u32x4 kreg[LOADS], vreg[LOADS];
    auto load_tile = [&](int tile) {
        const int key0 = tile * kBN;
#pragma unroll
        for (int it = 0; it < LOADS; ++it) {
            const int cid = it * NTHREADS + tid;
            const int key = cid >> 4, c = cid & 15;
            const int64_t off = (int64_t)(key0 + key) * kv_stride + c * 8;
            u32x4 kz = {0u, 0u, 0u, 0u}, vz = {0u, 0u, 0u, 0u};
            if (key0 + key < sk) {
                kz = *reinterpret_cast<const u32x4*>(kbase + off);
                vz = *reinterpret_cast<const u32x4*>(vbase + off);
            }
            kreg[it] = kz;
            vreg[it] = vz;
        }
    };
    auto store_tile = [&](int buf) {
        unsigned char* kb = smem + buf * 2 * kTileBytes;
        unsigned char* vb = kb + kTileBytes;
#pragma unroll
        for (int it = 0; it < LOADS; ++it) {
            const int cid = it * NTHREADS + tid;
            const int key = cid >> 4, c = cid & 15;
            *reinterpret_cast<u32x4*>(kb + k_lds_off(key, c)) = kreg[it];
            *reinterpret_cast<u32x4*>(vb + v_lds_off(key, c * 16)) = vreg[it];
        }
    };

    if (n_tiles > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();

    const float sl2 = p.scale_log2;
    const int wave_last = rw0 + NT * 32 - 1;

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const int key0 = tile * kBN;
        const bool more = tile + 1 < n_tiles;
        if (more) load_tile(tile + 1);

        // a wave whose rows all lie before this tile has nothing to add
        const bool wave_active = !causal || key0 <= wave_last + delta;
        if (wave_active) {
            const unsigned char* kb = smem + buf * 2 * kTileBytes;
            const unsigned char* vb = kb + kTileBytes;

            // ---- S^T tile: [2 key sub-tiles][NT query sub-tiles]
            f32x16 s[2][NT];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[mt][nt][r] = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kb + k_lds_off(mt * 32 + l32, 2 * t + hl));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        s[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nt][t], s[mt][nt], 0, 0, 0);
                }

            // ---- mask (only tiles that straddle the causal boundary or the end of the keys)
            const bool need_mask = (key0 + kBN > sk) || (causal && key0 + kBN - 1 > rw0 + delta);
            if (need_mask) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int row = rw0 + nt * 32 + l32;
                    int last_vis = sk - 1;                      // last visible key of this row
                    if (causal) last_vis = min(last_vis, row + delta);
                    const int lim = last_vis - key0 - 4 * hl;   // compare against 32*mt + 8*(r/4) + r%4
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (mt * 32 + 8 * (r >> 2) + (r & 3) > lim) s[mt][nt][r] = -INFINITY;
                }
            }

            // ---- online softmax, per query column (lane) and sub-tile
            bf16x8 pf[NT][2][2];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float mx = s[0][nt][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][nt][r]);
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][nt][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[nt], mx * sl2);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;   // a row that has seen no key yet
                const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_use);
                float rs = 0.f;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = __builtin_amdgcn_exp2f(fmaf(s[mt][nt][r], sl2, -m_use));
                        s[mt][nt][r] = e;
                        rs += e;
                    }
                l_run[nt] = l_run[nt] * alpha + rs;
                m_run[nt] = m_new;
                if (__any(alpha != 1.f)) {
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[dt][nt][r] *= alpha;
                }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2) {
                        f32x8 x;
#pragma unroll
                        for (int e = 0; e < 8; ++e) x[e] = s[mt][nt][8 * t2 + e];
                        pf[nt][mt][t2] = __builtin_convertvector(x, bf16x8);
                    }
            }

            // ---- O^T += V^T P^T : 4 key steps of 16, 4 head-dim sub-tiles of 32
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int mt = ks >> 1, t2 = ks & 1;
                const int kb0 = mt * 32 + t2 * 16 + 4 * hl;      // keys kb0..kb0+3 and kb0+8..kb0+11
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    bf16x8 vf;
                    // 16 lanes cooperate: lane i of a group supplies key kb0 + i/4, columns 4*(i%4)..+3
                    // of the group's 16 columns and receives 4 consecutive keys of column i.
                    const int gi = l32 & 15, gg = l32 >> 4;
                    const int col_byte = dt * 64 + gg * 32 + (gi & 3) * 8;
                    const int ka = kb0 + (gi >> 2);
                    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) bf16x4*)(vb + v_lds_off(ka, col_byte)));
                    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) bf16x4*)(vb + v_lds_off(ka + 8, col_byte)));
                    vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nt][mt][t2], o[dt][nt], 0, 0, 0);
                }
            }
        }

        if (more) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, LSE = m + ln l, store
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = rw0 + nt * 32 + l32;
        const float l_tot = l_run[nt] + __shfl_xor(l_run[nt], 32);
        if (row >= sq) continue;
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const float lse = l_tot > 0.f ? (m_run[nt] + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
        if (hl == 0) p.lse[(int64_t)head * p.lse_stride + q_tok0 + row] = lse;
        const int64_t obase = (q_tok0 + row) * q_stride + (int64_t)head * kHeadDim + 4 * hl;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f32x4 x;
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = o[dt][nt][4 * b + i] * inv;
                const int64_t idx = obase + 32 * dt + 8 * b;
                if (p.acc_out) *reinterpret_cast<f32x4*>(p.acc_out + idx) = x;
                if (p.out) {
                    if (p.out_f32)
                        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + idx) = x;
                    else
                        *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + idx) =
                            __builtin_convertvector(x, bf16x4);
                }
            }
    }
}

}  // namespace pec
