// Blockwise attention forward kernel, second generation: same mathematics and MFMA
// operand layouts as fwd_kernel.hpp, restructured around the measured issue limits of
// gfx950 (one VALU instruction costs ~4 issue cycles per SIMD, a transcendental ~12, an
// MFMA 32x32x16 keeps the matrix pipe busy for 32), so the tile loop carries as few
// VALU instructions as possible:
//   * K/V tiles go global -> LDS directly (global_load_lds_dwordx4): no staging
//     registers, no ds_write; the XOR swizzles are applied on the global side by
//     choosing which 16-byte chunk each lane fetches (a permutation inside one 256 B
//     row, so the global access stays fully coalesced);
//   * every LDS operand address is a VGPR plus an immediate; the VGPRs are flipped
//     between the two LDS stages once per tile;
//   * masking lives in a separate copy of the tile body that only the tiles straddling
//     the causal diagonal or the end of the keys take.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fwd_kernel.hpp"

namespace pec {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kStageBytes = 2 * kTileBytes;   // K tile then V tile

template <int NT, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) void fwd_dma_kernel(const FwdParams p) {
    constexpr int BM = NWAVES * NT * 32;
    constexpr int BLOCKS_PER_WAVE = 32 / NWAVES;   // 1 KiB LDS blocks each wave fills per tile (K: 16, V: 16)
    static_assert(32 % NWAVES == 0, "tile blocks must divide evenly over the waves");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * kStageBytes];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int hl = lane >> 5;

    // ---- block -> (kv head, work item, head in group), one contiguous logical range per XCD
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
    const int row0 = qt * BM;
    const int rw0 = row0 + wave * (NT * 32);
    const int blk_last = min(sq, row0 + BM) - 1;
    int kv_end = sk;
    if (causal) kv_end = max(0, min(sk, blk_last + delta + 1));
    const int n_tiles = (kv_end + kBN - 1) / kBN;

    const int64_t q_stride = (int64_t)p.n_q_heads * kHeadDim;
    const uint32_t kv_stride_b = (uint32_t)p.n_kv_heads * kHeadDim * 2;   // bytes per token
    const unsigned char* kbase =
        reinterpret_cast<const unsigned char*>(p.k) + (kv_tok0 * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);
    const unsigned char* vbase =
        reinterpret_cast<const unsigned char*>(p.v) + (kv_tok0 * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);

    // ---- Q fragments
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
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int row = rw0 + nt * 32 + l32;
            if (row < sq) {
                const float lin = p.lse_in[(int64_t)head * p.lse_stride + q_tok0 + row];
                if (lin != -INFINITY) {
                    m_run[nt] = lin * kLog2e;
                    l_run[nt] = hl == 0 ? 1.f : 0.f;
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

    // ---- tile staging: each wave instruction fills one 1 KiB LDS block = 4 key rows; lane s
    // lands at byte 16*s of the block and fetches the chunk the swizzle wants there.
    const int ld_row = lane >> 4;            // row inside the block
    const int ld_pos = lane & 15;            // physical 16 B position inside the row
    uint32_t ld_off[BLOCKS_PER_WAVE];        // byte offset inside a tile's global rows (full tiles)
    int ld_key[BLOCKS_PER_WAVE], ld_chunk[BLOCKS_PER_WAVE];
#pragma unroll
    for (int it = 0; it < BLOCKS_PER_WAVE; ++it) {
        const int bi = it * NWAVES + wave;           // 0..15 K blocks, 16..31 V blocks
        const int key = 4 * (bi & 15) + ld_row;
        const bool is_v = (it * NWAVES) >= 16;       // compile-time per `it`
        const int chunk = is_v ? ((((ld_pos >> 2) ^ (key & 3)) << 2) | (ld_pos & 3)) : (ld_pos ^ (key & 15));
        ld_key[it] = key;
        ld_chunk[it] = chunk;
        ld_off[it] = (uint32_t)key * kv_stride_b + (uint32_t)chunk * 16u;
    }
    auto issue_tile = [&](int tile, int stage) {
        const int key0 = tile * kBN;
        const bool full = key0 + kBN <= sk;
        const unsigned char* kt = kbase + (int64_t)key0 * kv_stride_b;
        const unsigned char* vt = vbase + (int64_t)key0 * kv_stride_b;
#pragma unroll
        for (int it = 0; it < BLOCKS_PER_WAVE; ++it) {
            const bool is_v = (it * NWAVES) >= 16;
            uint32_t off = ld_off[it];
            if (!full)  // rows past the end re-read the last valid row: finite data, weight zero
                off = (uint32_t)min(ld_key[it], sk - 1 - key0) * kv_stride_b + (uint32_t)ld_chunk[it] * 16u;
            const unsigned char* src = (is_v ? vt : kt) + off;
            unsigned char* dst = smem + stage * kStageBytes + (it * NWAVES + wave) * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };

    // ---- loop-invariant LDS operand addresses
    uint32_t k_addr[8];   // K fragment (sub-tile 0) for head-dim step t
#pragma unroll
    for (int t = 0; t < 8; ++t) k_addr[t] = k_lds_off(l32, 2 * t + hl);
    uint32_t v_addr[4];   // V^T fragment source for head-dim sub-tile dt, key offset 0
    {
        const int gi = l32 & 15, gg = l32 >> 4;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
            v_addr[dt] = v_lds_off(4 * hl + (gi >> 2), dt * 64 + gg * 32 + (gi & 3) * 8);
    }

    const float sl2 = p.scale_log2;
    const int wave_last = rw0 + NT * 32 - 1;

    // One KV tile.  STAGE is the LDS stage as a compile-time constant (so every LDS
    // address is register + immediate); MASK selects the copy that applies the causal /
    // end-of-keys mask.
    auto compute_tile = [&](auto mask_tag, int key0) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const unsigned char* kb = smem;               // the stage offset lives in k_addr / v_addr
        const unsigned char* vb = kb + kTileBytes;

        f32x16 s[2][NT];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[mt][nt][r] = 0.f;
        {
            // all 16 K fragments are requested up front so that LDS latency overlaps the MFMAs
            bf16x8 kf[8][2];
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    kf[t][mt] = *reinterpret_cast<const bf16x8*>(kb + k_addr[t] + mt * 32 * kRowBytes);
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        s[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t][mt], qf[nt][t], s[mt][nt], 0, 0, 0);
            // schedule: 6 reads ahead, then one read per MFMA group, then drain
            __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
            for (int i = 0; i < 10; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 6 * NT, 0);
        }

        if constexpr (MASK) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int row = rw0 + nt * 32 + l32;
                int last_vis = sk - 1;
                if (causal) last_vis = min(last_vis, row + delta);
                const int lim = last_vis - key0 - 4 * hl;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (mt * 32 + 8 * (r >> 2) + (r & 3) > lim) s[mt][nt][r] = -INFINITY;
            }
        }

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
            float m_use = m_new;
            if constexpr (MASK) m_use = (m_new == -INFINITY) ? 0.f : m_new;   // only masked tiles can leave a row empty
            const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_use);
            float rs = 0.f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {
                    u32x4 packed;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const f32x2 x = {__builtin_amdgcn_exp2f(fmaf(s[mt][nt][8 * t2 + 2 * e], sl2, -m_use)),
                                         __builtin_amdgcn_exp2f(fmaf(s[mt][nt][8 * t2 + 2 * e + 1], sl2, -m_use))};
                        // the denominator keeps the unrounded weights: a bf16-rounded sum would cost
                        // up to 2^-8 relative error on short rows, more than the LSE tolerance allows
                        rs += x[0] + x[1];
                        packed[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
                    }
                    pf[nt][mt][t2] = __builtin_bit_cast(bf16x8, packed);
                }
            l_run[nt] = l_run[nt] * alpha + rs;
            m_run[nt] = m_new;
            if (__any(alpha != 1.f)) {
                // in-place multiply (tied operand) so the rarely taken branch costs no register copies;
                // the wait states cover an MFMA still writing O (inline asm gets no hazard handling)
                asm volatile("s_nop 15\n\ts_nop 15");
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        asm volatile("v_mul_f32 %0, %0, %1" : "+v"(o[dt][nt][r]) : "v"(alpha));
            }
        }

#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int mt = ks >> 1, t2 = ks & 1;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const unsigned char* src = vb + v_addr[dt] + (mt * 32 + t2 * 16) * kRowBytes;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (__attribute__((address_space(3))) bf16x4*)(src));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (__attribute__((address_space(3))) bf16x4*)(src + 8 * kRowBytes));
                const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nt][mt][t2], o[dt][nt], 0, 0, 0);
            }
        }
    };

    // Tiles come in three runs for a wave: first those it can take without any mask,
    // then those straddling its causal boundary or the end of the keys, then (causal
    // only) tiles that lie wholly after its rows, where it just keeps the block's
    // load/barrier cadence.  Separate loops keep each accumulator in place.
    int n_full = sk / kBN;
    int n_act = n_tiles;
    if (causal) {
        n_full = min(n_full, max(0, rw0 + delta + 1) / kBN);
        n_act = min(n_tiles, max(0, wave_last + delta + kBN) / kBN);
    }
    n_full = min(n_full, n_tiles);
    n_act = max(n_act, n_full);

    auto flip_stage = [&]() {
#pragma unroll
        for (int t = 0; t < 8; ++t) k_addr[t] ^= (uint32_t)kStageBytes;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) v_addr[dt] ^= (uint32_t)kStageBytes;
    };
    auto end_of_tile = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of the next tile has landed
        __syncthreads();
    };

    if (n_tiles > 0) issue_tile(0, 0);
    end_of_tile();
    int tile = 0;
    for (; tile < n_full; ++tile) {
        if (tile + 1 < n_tiles) issue_tile(tile + 1, (tile + 1) & 1);
        compute_tile(std::false_type{}, tile * kBN);
        flip_stage();
        end_of_tile();
    }
    for (; tile < n_act; ++tile) {
        if (tile + 1 < n_tiles) issue_tile(tile + 1, (tile + 1) & 1);
        compute_tile(std::true_type{}, tile * kBN);
        flip_stage();
        end_of_tile();
    }
    for (; tile < n_tiles; ++tile) {
        if (tile + 1 < n_tiles) issue_tile(tile + 1, (tile + 1) & 1);
        end_of_tile();
    }

    // ---- epilogue
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
