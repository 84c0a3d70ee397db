// Blockwise attention forward kernel, "ping-pong" organisation for gfx950.
//
// Same mathematics, MFMA operand layouts, LDS swizzles and direct global->LDS tile
// loads as fwd_kernel_dma.hpp (8 wavefronts x 32 query rows, 64-key tiles).  What
// changes is WHEN each wavefront does what.  A SIMD holds two wavefronts of the
// workgroup; the matrix pipe and the vector ALU can work at the same time, but only
// if the two wavefronts are in different phases.  So every wavefront's tile loop is
// software-pipelined into an MFMA block  M(j) = [O += P(j-1) V(j-1) ; S(j) = K(j) Q^T]
// and a VALU block  V(j) = online softmax of S(j) -> P(j),  each closed by a workgroup
// barrier, and one half of the wavefronts runs one barrier behind the other half:
//
//     half-step      0      1      2      3      4
//     group A      M(0)   V(0)   M(1)   V(1)   M(2)  ...
//     group B       --    M(0)   V(0)   M(1)   V(1)  ...
//
// so that in every half-step one wavefront of each SIMD feeds the matrix pipe while
// the other does softmax.  K and V tiles have three LDS stages each (96 KiB in all); the
// loads for K(j+2) and V(j+1) are issued by every wavefront at the start of its own
// M(j) -- after the last reader of the stage being overwritten (M(j-1) of group B, one
// barrier earlier) -- and are only waited for at the end of its M(j+1), two half-steps
// and about two microseconds later, which is still one barrier before the first reader
// (M(j+2) of group A).  Every M block issues exactly four loads per wavefront (tile
// indices past the end are clamped, the stage they land in is free), so the wait is the
// constant `vmcnt(4)`: everything but the loads issued in this block.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fwd_kernel.hpp"
#include "fwd_kernel_dma.hpp"
#include "mblock_asm.inc"

namespace pec {

constexpr int kPpLdsBytes = 6 * kTileBytes;   // three K stages + three V stages

// x *= a with the destination tied to the source register, so that a rarely taken branch
// around it does not make the compiler copy the accumulator.
__device__ __forceinline__ void scale_in_place(f32x16& x, float a) {
#pragma unroll
    for (int r = 0; r < 16; ++r) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x[r]) : "v"(a));
}

// PAIR_STRIDE4: wavefronts w and w+4 share a SIMD (round-robin placement) -> group = w / 4;
// otherwise w and w+1 are taken to share one -> group = w % 2.
template <bool PAIR_STRIDE4>
__global__ __launch_bounds__(512) void fwd_pp_kernel(const FwdParams p) {
    constexpr int NWAVES = 8;
    constexpr int BM = NWAVES * 32;

    // K stages 0..2, then V stages 0..2 (kPpLdsBytes of dynamic LDS)
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int hl = lane >> 5;
    const int group = PAIR_STRIDE4 ? (wave >> 2) : (wave & 1);

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
    const int rw0 = row0 + wave * 32;
    const int wave_last = rw0 + 31;
    const int blk_last = min(sq, row0 + BM) - 1;
    int kv_end = sk;
    if (causal) kv_end = max(0, min(sk, blk_last + delta + 1));
    const int n_tiles = (kv_end + kBN - 1) / kBN;

    // runs of tiles for this wavefront: [0, n_full) need no mask, [n_full, n_act) do,
    // [n_act, n_tiles) lie wholly after its rows (causal only)
    int n_full = sk / kBN;
    int n_act = n_tiles;
    if (causal) {
        n_full = min(n_full, max(0, rw0 + delta + 1) / kBN);
        n_act = min(n_tiles, max(0, wave_last + delta + kBN) / kBN);
    }
    n_full = min(n_full, n_tiles);
    n_act = max(n_act, n_full);

    const int64_t q_stride = (int64_t)p.n_q_heads * kHeadDim;
    const uint32_t kv_stride_b = (uint32_t)p.n_kv_heads * kHeadDim * 2;   // bytes per token
    const unsigned char* kbase =
        reinterpret_cast<const unsigned char*>(p.k) + (kv_tok0 * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);
    const unsigned char* vbase =
        reinterpret_cast<const unsigned char*>(p.v) + (kv_tok0 * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);

    // ---- Q fragments
    bf16x8 qf[8];
    {
        const int row = rw0 + l32;
        const __bf16* qrow = p.q + (q_tok0 + row) * q_stride + (int64_t)head * kHeadDim + 8 * hl;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row < sq) raw = *reinterpret_cast<const u32x4*>(qrow + 16 * t);
            qf[t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // ---- running state
    f32x16 o[4];
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    if (p.acc_in) {
        const int row = rw0 + l32;
        if (row < sq) {
            const float lin = p.lse_in[(int64_t)head * p.lse_stride + q_tok0 + row];
            if (lin != -INFINITY) {
                m_run = lin * kLog2e;
                l_run = hl == 0 ? 1.f : 0.f;
                const float* arow = p.acc_in + (q_tok0 + row) * q_stride + (int64_t)head * kHeadDim + 4 * hl;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const f32x4 x = *reinterpret_cast<const f32x4*>(arow + 32 * dt + 8 * b);
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[dt][4 * b + i] = x[i];
                    }
            }
        }
    }

    // ---- tile staging.  Per tile and per matrix each wavefront fills two 1 KiB LDS blocks of
    // 4 key rows; lane s lands at byte 16*s of its block and fetches the chunk the swizzle wants there.
    const int ld_row = lane >> 4, ld_pos = lane & 15;
    int ld_key[2];
    uint32_t ldk_col[2], ldv_col[2], ldk_off[2], ldv_off[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int key = 4 * (it * NWAVES + wave) + ld_row;
        ld_key[it] = key;
        ldk_col[it] = (uint32_t)(ld_pos ^ (key & 15)) * 16u;
        ldv_col[it] = (uint32_t)((((ld_pos >> 2) ^ (key & 3)) << 2) | (ld_pos & 3)) * 16u;
        ldk_off[it] = (uint32_t)key * kv_stride_b + ldk_col[it];   // offsets inside a full tile
        ldv_off[it] = (uint32_t)key * kv_stride_b + ldv_col[it];
    }
    auto issue_tile = [&](const unsigned char* base, const uint32_t (&col)[2], const uint32_t (&full_off)[2], int tile,
                          int lds_base) {
        if (n_tiles <= 0) return;
        const int stage = tile % 3;
        tile = min(tile, n_tiles - 1);    // past the end: reload the last tile into a free stage (keeps load counts uniform)
        const int key0 = tile * kBN;
        const int last = sk - 1 - key0;   // rows past the end re-read the last valid row: finite, weight zero
        const unsigned char* tb = base + (int64_t)key0 * kv_stride_b;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            uint32_t off = full_off[it];
            if (last < kBN - 1) off = (uint32_t)min(ld_key[it], last) * kv_stride_b + col[it];
            unsigned char* dst = smem + lds_base + stage * kTileBytes + (it * NWAVES + wave) * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(tb + off),
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };
    auto issue_k = [&](int tile) { issue_tile(kbase, ldk_col, ldk_off, tile, 0); };
    auto issue_v = [&](int tile) { issue_tile(vbase, ldv_col, ldv_off, tile, 3 * kTileBytes); };

    // ---- LDS operand addresses as raw LDS byte addresses (the hand-scheduled sequences use them
    // directly).  They include the stage and move to the other stage after every use.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    uint32_t k_addr[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) k_addr[t] = lds0 + k_lds_off(l32, 2 * t + hl);
    uint32_t v_addr[4];
    {
        const int gi = l32 & 15, gg = l32 >> 4;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
            v_addr[dt] = lds0 + 3 * kTileBytes + v_lds_off(4 * hl + (gi >> 2), dt * 64 + gg * 32 + (gi & 3) * 8);
    }
    int k_stage = 0, v_stage = 0;   // stage the addresses point at

    const float sl2 = p.scale_log2;
    f32x16 s[2];     // S^T tile of the next softmax
    bf16x8 pf[2][2]; // P^T operands of the next PV product

    // MFMA block: O += P V (tile j-1) and/or S = K Q^T (tile j).  The two instruction
    // sequences are scheduled by hand (mblock_asm.inc): the compiler would otherwise wait for
    // each LDS fragment right where it is requested, and it has no way to know that the LDS
    // stage being read is not the one the in-flight tile loads are writing.
    auto m_block = [&](auto pv_tag, auto qk_tag) {
        constexpr bool DO_PV = decltype(pv_tag)::value;
        constexpr bool DO_QK = decltype(qk_tag)::value;
        if constexpr (DO_PV) {
            asm volatile(PEC_PV_ASM
                         : [o0] "+v"(o[0]), [o1] "+v"(o[1]), [o2] "+v"(o[2]), [o3] "+v"(o[3])
                         : [p0] "v"(pf[0][0]), [p1] "v"(pf[0][1]), [p2] "v"(pf[1][0]), [p3] "v"(pf[1][1]),
                           [va0] "v"(v_addr[0]), [va1] "v"(v_addr[1]), [va2] "v"(v_addr[2]), [va3] "v"(v_addr[3])
                         : PEC_MBLOCK_CLOBBERS);
            const int step = v_stage == 2 ? -2 * kTileBytes : kTileBytes;
            v_stage = v_stage == 2 ? 0 : v_stage + 1;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) v_addr[dt] += (uint32_t)step;
        }
        if constexpr (DO_QK) {
            asm volatile(PEC_QK_ASM
                         : [s0] "=&v"(s[0]), [s1] "=&v"(s[1])
                         : [q0] "v"(qf[0]), [q1] "v"(qf[1]), [q2] "v"(qf[2]), [q3] "v"(qf[3]), [q4] "v"(qf[4]),
                           [q5] "v"(qf[5]), [q6] "v"(qf[6]), [q7] "v"(qf[7]), [ka0] "v"(k_addr[0]),
                           [ka1] "v"(k_addr[1]), [ka2] "v"(k_addr[2]), [ka3] "v"(k_addr[3]), [ka4] "v"(k_addr[4]),
                           [ka5] "v"(k_addr[5]), [ka6] "v"(k_addr[6]), [ka7] "v"(k_addr[7])
                         : PEC_MBLOCK_CLOBBERS);
            const int step = k_stage == 2 ? -2 * kTileBytes : kTileBytes;
            k_stage = k_stage == 2 ? 0 : k_stage + 1;
#pragma unroll
            for (int t = 0; t < 8; ++t) k_addr[t] += (uint32_t)step;
        }
    };

    // VALU block: online softmax of s (tile at key0) -> pf, running max / sum, rescale of O
    auto v_block = [&](auto mask_tag, int key0) {
        constexpr bool MASK = decltype(mask_tag)::value;
        if constexpr (MASK) {
            const int row = rw0 + l32;
            int last_vis = sk - 1;
            if (causal) last_vis = min(last_vis, row + delta);
            const int lim = last_vis - key0 - 4 * hl;   // compare against 32*mt + 8*(r/4) + r%4
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (mt * 32 + 8 * (r >> 2) + (r & 3) > lim) s[mt][r] = -INFINITY;
        }
        float mx = s[0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
        {   // other lane half holds the other 32 keys of the same query
            const uint32_t u = __builtin_bit_cast(uint32_t, mx);
            const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
            mx = fmaxf(__builtin_bit_cast(float, (uint32_t)sw[0]), __builtin_bit_cast(float, (uint32_t)sw[1]));
        }
        const float m_new = fmaxf(m_run, mx * sl2);
        float m_use = m_new;
        if constexpr (MASK) m_use = (m_new == -INFINITY) ? 0.f : m_new;   // only masked tiles can leave a row empty
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        float rs = 0.f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                u32x4 packed;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const f32x2 x = {__builtin_amdgcn_exp2f(fmaf(s[mt][8 * t2 + 2 * e], sl2, -m_use)),
                                     __builtin_amdgcn_exp2f(fmaf(s[mt][8 * t2 + 2 * e + 1], sl2, -m_use))};
                    rs += x[0] + x[1];   // denominator from the unrounded weights (LSE tolerance)
                    packed[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
                }
                pf[mt][t2] = __builtin_bit_cast(bf16x8, packed);
            }
        l_run = l_run * alpha + rs;
        m_run = m_new;
        // the weights must exist before the barrier that ends this block (keeps the exp work out of the MFMA block)
        asm volatile("" : "+v"(l_run), "+v"(m_run) : "v"(pf[0][0]), "v"(pf[0][1]), "v"(pf[1][0]), "v"(pf[1][1]));
        if (__any(alpha != 1.f)) {
            // in-place multiply (tied operand): the rarely taken branch costs no register copies;
            // wait states in case an MFMA is still writing O (inline asm gets no hazard handling)
            asm volatile("s_nop 15\n\ts_nop 15");
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) scale_in_place(o[dt], alpha);
        }
    };

    // Barrier closing an M block: the loads issued one M block earlier have landed (the four
    // issued in this block may still be in flight).  Barrier closing a V block: nothing to wait for.
    auto sync_m = [&]() {
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };
    auto sync_v = [&]() { __builtin_amdgcn_s_barrier(); };

    // ---- schedule (every wavefront passes 2*n_tiles + 3 barriers)
    issue_k(0);
    issue_k(1);
    issue_v(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (group == 1) sync_v();        // group B runs one half-step behind
    issue_k(2);
    issue_v(1);
    if (n_act > 0) m_block(std::false_type{}, std::true_type{});   // M(0) = S(0)
    sync_m();
    int j = 0;
    const int e1 = max(0, min(n_full, n_act - 1));
    for (; j < e1; ++j) {
        v_block(std::false_type{}, j * kBN);
        sync_v();
        issue_k(j + 3);
        issue_v(j + 2);
        m_block(std::true_type{}, std::true_type{});
        sync_m();
    }
    for (; j < n_act - 1; ++j) {
        v_block(std::true_type{}, j * kBN);
        sync_v();
        issue_k(j + 3);
        issue_v(j + 2);
        m_block(std::true_type{}, std::true_type{});
        sync_m();
    }
    if (n_act > 0) {   // last active tile: nothing left to multiply by K
        v_block(std::true_type{}, j * kBN);
        sync_v();
        issue_k(j + 3);
        issue_v(j + 2);
        m_block(std::true_type{}, std::false_type{});
        sync_m();
        ++j;
    }
    for (; j < n_tiles; ++j) {   // keep the workgroup's load / barrier cadence
        sync_v();
        issue_k(j + 3);
        issue_v(j + 2);
        sync_m();
    }
    if (group == 0) sync_v();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no tile load may outlive the workgroup's LDS

    // ---- epilogue
    {
        const int row = rw0 + l32;
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        if (row < sq) {
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
            if (hl == 0) p.lse[(int64_t)head * p.lse_stride + q_tok0 + row] = lse;
            const int64_t obase = (q_tok0 + row) * q_stride + (int64_t)head * kHeadDim + 4 * hl;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    f32x4 x;
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[i] = o[dt][4 * b + i] * inv;
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
}

}  // namespace pec
