// Blockwise attention forward kernel with MFMA and softmax interleaved inside every
// wavefront's instruction stream (gfx950).
//
// Measurements on MI355X behind this organisation: a wavefront that issues MFMAs back
// to back keeps the vector ALU of its SIMD from serving the other resident wavefront,
// so running softmax in one wavefront while another does MFMAs gains nothing; but VALU
// instructions that FOLLOW an MFMA in the same wavefront do execute under it.  So the
// tile loop is software-pipelined in each wavefront: iteration j carries
//     S(j+1) = K(j+1) Q^T               16 MFMAs
//     O     += P(j-1) V(j-1)            16 MFMAs   (P(j-1) from the previous iteration)
//     P(j)   = exp2(S(j) - m(j)) etc.   ~112 VALU  (S(j), m(j) from the previous iteration)
//     m(j+1), alpha(j+1) from S(j+1)    ~30 VALU   (masked tiles only, after the first 16 MFMAs)
// which are independent of each other and get issued round-robin (3 to 4 VALU per MFMA).
// Measured: an MFMA of this shape keeps the SIMD's vector issue port for about 23 of its 32
// cycles, so only 4 to 5 plain VALU instructions per MFMA are free; every one beyond that costs
// about 2 cycles, a transcendental about 5.  Hence the softmax reference m is kept lazily
// (see row_max) and unmasked tiles do without a row maximum (see body).
// MFMA operand layouts and LDS swizzles as described in common.hpp; K/V tiles go global -> LDS
// directly (global_load_lds_dwordx4: no staging registers, no ds_write; the XOR swizzles are applied
// on the global side by choosing which 16-byte chunk each lane fetches, a permutation inside one
// 256 B row, so the global access stays fully coalesced); 8 wavefronts x 32 query rows; one
// workgroup barrier per tile.
//
// LDS: two stages each for K and V (four 16 KiB pieces of one block; every access names its stage because
// the loop is unrolled by two).  Iteration j, parity
// r = j % 2: loads K(j+2) -> K[r] and V(j) -> V[r]; reads K(j+1) from K[1-r] and V(j-1)
// from V[1-r].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "common.hpp"

namespace pec {

typedef __attribute__((address_space(3))) unsigned char lds_byte;

// In-place rescale of the four O accumulators.  The compiler's hazard recogniser does not look inside
// inline asm, and the hardware does not interlock a VALU read of a register an MFMA is still writing,
// so the wait states sit in ONE asm statement that takes all four accumulators as read-write operands:
// every MFMA that produces them is ordered before it by the data dependence, and nothing can move
// between the wait and the multiplications that follow it in the same statement sequence.
__device__ __forceinline__ void scale_acc_in_place(f32x16 (&o)[4], float a) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]));
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(o[dt][r]) : "v"(a));
}

// Three instances, so that each carries only its own bookkeeping through the (register-starved) work-item code:
// kFwdDense -- one call = one problem, work items dealt in fixed rounds (ring step, fused merge, key splits, the
// plain sweep); kFwdSweep -- the resumable sweep (progress table, stop word, state of stopped items);
// kFwdList -- device-built work lists (packed and colocated batch), work items drawn at run time.
enum { kFwdDense = 0, kFwdSweep = 1, kFwdList = 2 };

template <int MODE>
__global__ __launch_bounds__(512) void fwd_il_kernel(const FwdParams p) {
    constexpr bool kSweep = MODE == kFwdSweep;
    constexpr bool kList = MODE == kFwdList;
    constexpr int NWAVES = 8;
    constexpr int BM = NWAVES * 32;

    // One LDS block laid out by hand, the four tile stages inside the first 64 KiB: every operand read
    // of the tile loop is then "lane offset + 16-bit immediate".  (Separate arrays are placed by the
    // compiler in an order of its own; a stage that lands above 64 KiB needs its address in a register,
    // and the tile loop has none to spare.)
    __shared__ __attribute__((aligned(1024))) unsigned char lds_all[4 * kTileBytes + 256 + 64];
    unsigned char* const lds_k0 = lds_all;
    unsigned char* const lds_k1 = lds_all + kTileBytes;
    unsigned char* const lds_v0 = lds_all + 2 * kTileBytes;
    unsigned char* const lds_v1 = lds_all + 3 * kTileBytes;

    // ---- persistent workgroups: the grid holds n_slots workgroups per XCD (hardware deals block
    // ids round-robin over the 8 XCDs); each XCD owns one contiguous logical range of the
    // (KV-head-major, longest-rows-first) work order.  Dense calls: its workgroups walk it in snake order
    // (slot, then reversed slot, ...), which evens out the causal length differences.  Work-list calls
    // (p.sched): items differ in length by orders of magnitude and the XCDs do not run at the same speed, so
    // every workgroup draws its next item from its XCD's counter, and from the next XCD's once that share is
    // used up; the heaviest items come first in the list, so the launch ends on the lightest ones.
    constexpr bool dynamic = kList;
    const int n_items_eff = dynamic ? min(*p.n_work, p.n_items) : p.n_items;
    const int64_t total = (int64_t)n_items_eff * p.n_q_heads;
    const int64_t per_xcd = (total + 7) >> 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_slots = (int)(gridDim.x >> 3);
    const int slot = (int)(blockIdx.x >> 3);
    // 64 copies of the stop word of a resumable sweep, brought in by wavefront 0 with a tile-style load
    const uint32_t lds_stop = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_all + 4 * kTileBytes;
    auto request_stop_word = [&]() {   // lands with the tile loads; visible to everyone after the next barrier
        if (wave == 0) {
            uint32_t zero;
            asm volatile("v_mov_b32 %0, 0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 sc0 sc1"
                         : "=&v"(zero)
                         : "s"(p.stop), "s"(lds_stop)
                         : "memory", "m0");
        }
    };
    auto read_stop_word = [&]() -> int {
        const int v = *(const __attribute__((address_space(3))) volatile int*)(lds_all + 4 * kTileBytes);
        return __builtin_amdgcn_readfirstlane(v);
    };
    bool first_item = true;   // of this workgroup in this launch: it is never abandoned before its first segment
    // Drawing (work-list calls): lane 0 of wavefront 0 takes the next index and leaves it in one of two LDS
    // words used in turn; everyone reads it after the next barrier.  The draw for item i + 1 is made while item
    // i waits for its first tiles, so its latency is hidden; only the first draw, and the one after an index
    // that turns out to hold no work, is waited for.  Words 2 and 3 (lane 0's own): the XCD share being drawn
    // from and how many shares were found used up.
    typedef __attribute__((address_space(3))) volatile int lds_int;
    lds_int* const lds_sched = (lds_int*)(lds_all + 4 * kTileBytes + 256);
    int sched_par = 0;         // which of the two words holds the index to take next
    bool have_next = false;
    auto draw_next = [&](int into) {
        if (wave == 0) {
            int ln;
            asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
            if (ln == 0) {
                int x = lds_sched[2], t = lds_sched[3], got = -1;
                while (t < 8) {
                    const int v = atomicAdd(&p.sched[x], 1);
                    if (v < per_xcd && (int64_t)x * per_xcd + v < total) {
                        got = (int)(x * per_xcd + v);
                        break;
                    }
                    x = (x + 1) & 7;
                    ++t;
                }
                lds_sched[into] = got;
                lds_sched[2] = x;
                lds_sched[3] = t;
            }
        }
    };
    if (dynamic && threadIdx.x == 0) {
        lds_sched[2] = (int)(blockIdx.x & 7);
        lds_sched[3] = 0;
    }
    for (int64_t round0 = 0; dynamic || round0 < per_xcd; round0 += n_slots) {
    // Lane-derived values are recomputed for every work item (the empty asm hides that they are
    // loop invariant): hoisted out of this loop they would stay live through the tile loop, which
    // has no register to spare -- a spill reload there waits on the tile loads just issued.
    int lane;   // volatile asm: not hoisted, and no vector register carries it from item to item
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
    const int l32 = lane & 31;
    const int hl = lane >> 5;
    int64_t logical;
    if (dynamic) {
        if (!have_next) {
            draw_next(sched_par);
            __builtin_amdgcn_s_barrier();
        }
        have_next = false;
        const int got = __builtin_amdgcn_readfirstlane(lds_sched[sched_par]);
        sched_par ^= 1;
        if (got < 0) break;
        logical = got;
    } else {
        const int64_t idx_in_xcd = round0 + (((round0 / n_slots) & 1) ? (n_slots - 1 - slot) : slot);
        if (idx_in_xcd >= per_xcd) continue;
        logical = (int64_t)(blockIdx.x & 7) * per_xcd + idx_in_xcd;
        if (logical >= total) continue;
    }
    const int per_kvh = n_items_eff * p.group;
    const int kvh = (int)(logical / per_kvh);
    const int rem = (int)(logical % per_kvh);
    const int item = rem / p.group;
    const int head = kvh * p.group + rem % p.group;

    // Per-item geometry and addressing: rows sq x keys sk with diagonal offset delta; element offsets of
    // row 0 in q (q_off0), in out / acc (o_off0) and in lse (lse_off0), the row stride of q / out / acc.
    int sq, sk, delta, qt;
    int64_t kv_tok0, q_off0, o_off0, lse_off0;
    int64_t q_stride = p.q_row_stride ? p.q_row_stride : (int64_t)p.n_q_heads * kHeadDim;
    void* out_ptr = p.out;
    float* lse_ptr = p.lse;
    int out_f32 = p.out_f32;
    const float* acc_in = p.acc_in;
    float* acc_out = p.acc_out;
    int seg_done = 0;          // resumable sweep: key segments this item has behind it
    if constexpr (kList) {
        if (item >= *p.n_work) continue;
        const WorkItem w = p.work[item];
        const int b0 = min(max(p.cu_seqlens[w.seq], 0), p.total_tokens);
        const int b1 = min(max(p.cu_seqlens[w.seq + 1], b0), p.total_tokens);
        int k0 = b0, k1 = b1;
        if (p.cu_seqlens_k) {
            k0 = min(max(p.cu_seqlens_k[w.seq], 0), p.total_k);
            k1 = min(max(p.cu_seqlens_k[w.seq + 1], k0), p.total_k);
        }
        if (w.qtile >= 0) {   // a query tile of a prompt: its rows are the last b1 - b0 positions of k1 - k0
            sq = b1 - b0;
            sk = k1 - k0;
            delta = sk - sq;
            qt = w.qtile;
            kv_tok0 = k0;
            q_off0 = b0 * q_stride + (int64_t)head * kHeadDim;
            o_off0 = q_off0;
            lse_off0 = (int64_t)head * p.lse_stride + b0;
        } else {              // a key range of a one-token sequence: the heads of a KV group are the rows
            if (rem % p.group != 0) continue;   // one unit per KV head
            const int r = -1 - w.qtile;
            const int64_t slot_no = (int64_t)p.seq_slot0[w.seq] + r;
            sq = p.group;
            kv_tok0 = (int64_t)k0 + (int64_t)r * p.coloc_range_len;
            sk = (int)max((int64_t)0, min((int64_t)p.coloc_range_len, (int64_t)k1 - kv_tok0));
            delta = sk;       // every key of the range is visible
            qt = 0;
            q_off0 = b0 * q_stride + (int64_t)kvh * p.group * kHeadDim;
            q_stride = kHeadDim;
            o_off0 = (slot_no * p.n_q_heads + (int64_t)kvh * p.group) * kHeadDim;
            lse_off0 = slot_no * p.n_q_heads + (int64_t)kvh * p.group;
            out_ptr = p.part_out;
            lse_ptr = p.part_lse;
            out_f32 = 1;
        }
    } else {
        sq = p.sq;
        sk = p.sk;
        delta = p.delta;
        qt = p.causal ? (p.n_items - 1 - item) : item;  // longest rows first
        kv_tok0 = 0;
        q_off0 = (int64_t)head * (p.q_head_stride ? p.q_head_stride : kHeadDim);
        o_off0 = q_off0;
        lse_off0 = (int64_t)head * p.lse_stride;
        if constexpr (kSweep) {     // continue behind the segments already folded in
            seg_done = p.progress[logical];
            // (a table that was never initialised must not send the loads out of bounds: anything that is
            // not a count of segments inside the key range is taken as "through" or as "not started")
            if (seg_done == kSweepDone || (seg_done > 0 && (int64_t)seg_done * p.seg_tiles * kBN >= (int64_t)sk)) continue;
            seg_done = max(seg_done, 0);
            if (seg_done == 0) acc_in = nullptr;
            kv_tok0 = (int64_t)seg_done * p.seg_tiles * kBN;
            sk -= (int)kv_tok0;
            delta -= (int)kv_tok0;
        }
        if (!kSweep && p.kv_split_len > 0) {   // the work item is a key range; all of it is visible (decode)
            qt = 0;
            kv_tok0 = (int64_t)item * p.kv_split_len;
            sk = (int)max((int64_t)0, min((int64_t)p.kv_split_len, (int64_t)p.sk - kv_tok0));
            o_off0 += item * p.split_out_stride;
            lse_off0 += item * p.split_lse_stride;
        }
    }
    const int causal = p.causal;
    const int row0 = qt * BM;
    const int rw0 = row0 + wave * 32;
    const int wave_last = rw0 + 31;
    const int blk_last = min(sq, row0 + BM) - 1;
    int kv_end = sk;
    if (causal) kv_end = max(0, min(sk, blk_last + delta + 1));
    int n_tiles = (kv_end + kBN - 1) / kBN;

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
    if (rw0 >= sq) n_full = n_act = 0;   // a wavefront without a valid row only helps loading tiles

    const uint32_t kv_stride_b = (uint32_t)p.n_kv_heads * kHeadDim * 2;   // bytes per token
    const unsigned char* kbase =
        reinterpret_cast<const unsigned char*>(p.k) + (kv_tok0 * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);
    const unsigned char* vbase =
        reinterpret_cast<const unsigned char*>(p.v) + (kv_tok0 * p.n_kv_heads + kvh) * (int64_t)(kHeadDim * 2);

    // ---- Q fragments
    bf16x8 qf[8];
    {
        const int row = rw0 + l32;
        const __bf16* qrow = p.q + q_off0 + row * q_stride + 8 * hl;
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
    if (acc_in) {
        const int row = rw0 + l32;
        if (row < sq) {
            const float lin = p.lse_in[lse_off0 + row];
            constexpr bool raw = kSweep;   // state of a stopped sweep item, stored as the registers held it
            if (raw || lin != -INFINITY) {
                m_run = raw ? lin : lin * kLog2e;
                l_run = raw ? p.l_part[(lse_off0 + row) * 2 + hl] : (hl == 0 ? 1.f : 0.f);
                const float* arow = acc_in + o_off0 + row * q_stride + 4 * hl;
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

    // ---- tile loads: per tile and matrix each wavefront fills two 1 KiB LDS blocks of 4 key rows;
    // lane s lands at byte 16*s of its block and fetches the chunk the swizzle wants there.  The
    // load is written as asm (M0 = LDS block address, SGPR base + 32-bit lane offset): three
    // instructions per load, and the compiler does not serialise later LDS reads behind it --
    // the stage being filled is never the one being read, which it cannot see.
    const int ld_row = lane >> 4, ld_pos = lane & 15;
    // byte offsets inside a full tile of this lane's first block; its second block lies 32 keys
    // further (same swizzle, since 32 is a multiple of both swizzle periods)
    uint32_t ldk_off0, ldv_off0;
    {
        const int key = 4 * wave + ld_row;
        ldk_off0 = (uint32_t)key * kv_stride_b + (uint32_t)(ld_pos ^ (key & 15)) * 16u;
        ldv_off0 = (uint32_t)key * kv_stride_b + (uint32_t)((((ld_pos >> 2) ^ (key & 3)) << 2) | (ld_pos & 3)) * 16u;
    }
    const uint32_t block_stride_b = 4u * NWAVES * kv_stride_b;
    auto dma16 = [](const unsigned char* sbase, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(voff), "s"(sbase), "s"(lds_addr)
                     : "memory", "m0");
    };
    auto issue_tile = [&](const unsigned char* base, bool is_v, uint32_t full_off0, int tile, unsigned char* stage) {
        if (tile >= n_tiles) return;
        const int key0 = tile * kBN;
        const unsigned char* tb = base + (int64_t)key0 * kv_stride_b;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)stage + wave * 1024;
        if (key0 + kBN <= sk) {
#pragma unroll
            for (int it = 0; it < 2; ++it) dma16(tb + it * block_stride_b, full_off0, lds0 + it * NWAVES * 1024);
        } else {   // rows past the end re-read the last valid row: finite data, weight zero
            // (at most once per work item: everything is rebuilt from the lane id here, so that the
            // tile loop carries no register for this path)
            int ln;
            asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
            const int r_row = ln >> 4, r_pos = ln & 15;
            const int last = sk - 1 - key0;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int key = 4 * (it * NWAVES + wave) + r_row;
                const uint32_t col = is_v ? (uint32_t)((((r_pos >> 2) ^ (key & 3)) << 2) | (r_pos & 3)) * 16u
                                          : (uint32_t)(r_pos ^ (key & 15)) * 16u;
                dma16(tb, (uint32_t)min(key, last) * kv_stride_b + col, lds0 + it * NWAVES * 1024);
            }
        }
    };
    auto issue_k = [&](int tile, unsigned char* stage) { issue_tile(kbase, false, ldk_off0, tile, stage); };
    auto issue_v = [&](int tile, unsigned char* stage) { issue_tile(vbase, true, ldv_off0, tile, stage); };

    // ---- LDS operand offsets inside a stage
    uint32_t k_off[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) k_off[t] = k_lds_off(l32, 2 * t + hl);
    uint32_t v_off[4];
    {
        const int gi = l32 & 15, gg = l32 >> 4;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) v_off[dt] = v_lds_off(4 * hl + (gi >> 2), dt * 64 + gg * 32 + (gi & 3) * 8);
    }

    const float sl2 = p.scale_log2;
    f32x16 s_a[2], s_b[2];        // score tiles of even / odd iterations
    bf16x8 p_a[2][2], p_b[2][2];  // probability operands produced by even / odd iterations
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            p_a[i][k2] = __builtin_bit_cast(bf16x8, z);
            p_b[i][k2] = __builtin_bit_cast(bf16x8, z);
        }

    auto qk_mfma = [&](f32x16 (&s)[2], const unsigned char* kst) {
        bf16x8 kf[8][2];
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                kf[t][mt] = *reinterpret_cast<const bf16x8*>(kst + k_off[t] + mt * 32 * kRowBytes);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t][mt], qf[t], s[mt], 0, 0, 0);
    };
    auto pv_mfma = [&](const bf16x8 (&pp)[2][2], const unsigned char* vst) {
        bf16x8 vf[4][4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const unsigned char* src = vst + v_off[dt] + ks * 16 * kRowBytes;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(src));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (__attribute__((address_space(3))) bf16x4*)(src + 8 * kRowBytes));
                vf[ks][dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks][dt], pp[ks >> 1][ks & 1], o[dt], 0, 0, 0);
    };
    // Softmax, split in two so that every iteration has VALU work that is ready from its first
    // cycle.  row_max(): mask / row maximum of a fresh score tile -> new running maximum and the
    // factor alpha by which everything accumulated so far shrinks.  weights(): exp2 of a score
    // tile against the reference fixed one iteration earlier -> P operands and the denominator.
    constexpr float kRefSlack = 8.f;   // log2 units
    constexpr float kSumLimit = 65536.f;   // per-lane sum of 32 weights that triggers a reference update
    float m_use = 0.f;    // reference the pending tile's weights are taken against (0 for a row without keys)
    float alpha = 1.f;    // exp2(previous reference - m_use)
    auto row_max = [&](auto mask_tag, f32x16 (&s)[2], int key0) {
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
        {   // the other lane half holds the other 32 keys of the same query
            const uint32_t u = __builtin_bit_cast(uint32_t, mx);
            const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
            mx = fmaxf(__builtin_bit_cast(float, (uint32_t)sw[0]), __builtin_bit_cast(float, (uint32_t)sw[1]));
        }
        // Lazy reference: any reference value gives the same softmax as long as numerator and
        // denominator share it, so m_run only moves when the tile maximum exceeds it by more than
        // kRefSlack (weights stay below 2^kRefSlack).  With the exact running maximum some row of a
        // wavefront sets a new record in most tiles and O would be rescaled nearly every iteration.
        const float mx2 = mx * sl2;
        const float m_new = (mx2 > m_run + kRefSlack) ? mx2 : m_run;
        m_use = m_new;
        if constexpr (MASK) m_use = (m_new == -INFINITY) ? 0.f : m_new;   // only masked tiles can leave a row empty
        alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
    };
    auto weights_rs = [&](const f32x16 (&s)[2], bf16x8 (&pp)[2][2]) -> float {
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
                pp[mt][t2] = __builtin_bit_cast(bf16x8, packed);
            }
        return rs;
    };
    auto weights = [&](const f32x16 (&s)[2], bf16x8 (&pp)[2][2]) {
        const float rs = weights_rs(s, pp);
        l_run = l_run * alpha + rs;
    };

    auto end_of_iteration = [&]() {
        // vmcnt(0): this wavefront's tile loads have landed.  Issued through the builtin so that the
        // compiler's own counter bookkeeping knows nothing is outstanding here: it cannot see the
        // asm tile loads, and a leftover wait of its own inside the loop would stall on them.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt 0, expcnt / lgkmcnt unconstrained
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };

    // One pipelined iteration j, parity PAR = j % 2:
    //   MFMA : S(j+1) = K(j+1) Q^T (if DO_QK), then O += P(j-1) V(j-1)
    //   VALU : P(j) = weights of S(j); then (if DO_QK) mask / row maximum of S(j+1)
    //   last : O *= alpha(j), once the MFMAs above are done and before P(j) V(j) is added
    auto body = [&](auto par_tag, auto mask_next_tag, auto qk_tag, int j) {
        constexpr int PAR = decltype(par_tag)::value;
        constexpr bool DO_QK = decltype(qk_tag)::value;
        unsigned char* k_wr = PAR ? lds_k1 : lds_k0;
        unsigned char* v_wr = PAR ? lds_v1 : lds_v0;
        const unsigned char* k_rd = PAR ? lds_k0 : lds_k1;
        const unsigned char* v_rd = PAR ? lds_v0 : lds_v1;
        issue_k(j + 2, k_wr);
        issue_v(j, v_wr);
        // An iteration whose next tile needs no mask skips the row maximum altogether: the weights of
        // tile j are taken against the reference as it stands, and only a row sum above kSumLimit
        // (some score far ahead of the reference) sends the wavefront through row_max() and a second
        // pass over the tile, after the MFMAs.  Every row in such an iteration has a finite reference:
        // tile 0 is fully visible to it and went through row_max() in the prologue.
        constexpr bool FAST = DO_QK && !decltype(mask_next_tag)::value;
        float alpha_j = alpha;
        float rs_fast = 0.f;
        if constexpr (FAST) {
            if constexpr (PAR == 0) {
                qk_mfma(s_b, k_rd);
                pv_mfma(p_b, v_rd);
                rs_fast = weights_rs(s_a, p_a);
                asm volatile("" : "+v"(rs_fast), "+v"(m_run), "+v"(m_use), "+v"(alpha)
                             : "v"(p_a[0][0]), "v"(p_a[0][1]), "v"(p_a[1][0]), "v"(p_a[1][1]));
            } else {
                qk_mfma(s_a, k_rd);
                pv_mfma(p_a, v_rd);
                rs_fast = weights_rs(s_b, p_b);
                asm volatile("" : "+v"(rs_fast), "+v"(m_run), "+v"(m_use), "+v"(alpha)
                             : "v"(p_b[0][0]), "v"(p_b[0][1]), "v"(p_b[1][0]), "v"(p_b[1][1]));
            }
        } else if constexpr (PAR == 0) {
            if constexpr (DO_QK) qk_mfma(s_b, k_rd);
            pv_mfma(p_b, v_rd);
            weights(s_a, p_a);
            if constexpr (DO_QK) row_max(mask_next_tag, s_b, (j + 1) * kBN);
            asm volatile("" : "+v"(l_run), "+v"(m_run), "+v"(m_use), "+v"(alpha)
                         : "v"(p_a[0][0]), "v"(p_a[0][1]), "v"(p_a[1][0]), "v"(p_a[1][1]));
        } else {
            if constexpr (DO_QK) qk_mfma(s_a, k_rd);
            pv_mfma(p_a, v_rd);
            weights(s_b, p_b);
            if constexpr (DO_QK) row_max(mask_next_tag, s_a, (j + 1) * kBN);
            asm volatile("" : "+v"(l_run), "+v"(m_run), "+v"(m_use), "+v"(alpha)
                         : "v"(p_b[0][0]), "v"(p_b[0][1]), "v"(p_b[1][0]), "v"(p_b[1][1]));
        }
        // issue order: operand fragments a few MFMAs ahead; after every MFMA a slice of the softmax
        if constexpr (DO_QK) {
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int i = 0; i < 12; ++i) {   // QK MFMAs, remaining K fragments
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {   // last QK MFMAs and first PV MFMAs, V fragments
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
            }
        } else {
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int i = 0; i < 14; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
            }
        }
        if constexpr (FAST) {
            // no factor is pending on entry (the prologue applies its own), so the one test decides
            // everything; alpha_j is only set on the rare path
            if (__any(!(rs_fast <= kSumLimit))) {   // also catches an overflowed (infinite) sum
                if constexpr (PAR == 0) {
                    row_max(std::false_type{}, s_a, j * kBN);
                    rs_fast = weights_rs(s_a, p_a);
                } else {
                    row_max(std::false_type{}, s_b, j * kBN);
                    rs_fast = weights_rs(s_b, p_b);
                }
                l_run *= alpha;
                scale_acc_in_place(o, alpha);
                alpha = 1.f;        // nothing pending for tile j + 1: its reference is the current one
                m_use = m_run;
            }
            l_run += rs_fast;
        } else {
            if (__any(alpha_j != 1.f)) scale_acc_in_place(o, alpha_j);
        }
        end_of_iteration();
    };
    using T = std::true_type;
    using F = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    // ---- prologue: K(0), K(1); V(0) also into the stage iteration 0 reads with P = 0 (finite data)
    issue_k(0, lds_k0);
    issue_k(1, lds_k1);
    issue_v(0, lds_v1);
    const bool may_stop = kSweep && p.stop != nullptr;
    if (may_stop && !first_item) request_stop_word();
    if (dynamic) {   // the next item's index, while this one waits for its first tiles
        draw_next(sched_par);
        have_next = true;
    }
    end_of_iteration();
    if (may_stop && !first_item && read_stop_word() != 0) return;   // nothing of this item has been touched
    first_item = false;
    if (n_act > 0) {
        qk_mfma(s_a, lds_k0);
        row_max(T{}, s_a, 0);
        // the factor tile 0 puts on what was carried in is applied here, so that the unmasked
        // iterations start with nothing pending
        l_run *= alpha;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
        alpha = 1.f;
    }
    asm volatile("" : "+v"(s_a[0]), "+v"(s_a[1]), "+v"(m_run), "+v"(m_use), "+v"(alpha));
    __builtin_amdgcn_s_barrier();     // K stage 0 may be overwritten from here on

    // ---- schedule: every wavefront passes one barrier per tile.  Iteration j needs the mask
    // for tile j + 1, so the unmasked run ends one tile early; it is taken in whole pairs.
    int j = 0;
    int e1 = max(0, min(n_full - 1, n_act - 1)) & ~1;
    // Resumable sweep: the stop word is looked at ahead of every segment boundary b that all eight
    // wavefronts reach inside their unmasked run (and only in items whose 256 rows are all valid, so that
    // every wavefront is in that run): requested at tile b - 8, read at tile b - 4 -- at least two barriers
    // later -- by everyone from the same LDS word.  When it is set, the item ends at b: the loop limits
    // shrink and the code below drains the pipeline as it does at the end of the keys.
    int stop_b = 0x7fffffff, stop_evt = 0x7fffffff, stop_limit = 0;
    bool stop_requested = false, stopped = false;
    if (may_stop && p.seg_tiles >= 16 && row0 + BM <= sq) {
        int nf0 = sk / kBN, na0 = n_tiles;
        if (causal) {
            nf0 = min(nf0, max(0, row0 + delta + 1) / kBN);
            na0 = min(n_tiles, max(0, row0 + 31 + delta + kBN) / kBN);
        }
        stop_limit = min(max(0, min(nf0 - 1, na0 - 1)) & ~1, n_tiles - 1);
        stop_b = p.seg_tiles;
        if (stop_b <= stop_limit) stop_evt = (stop_b & ~1) - 8;
    }
    for (;;) {
        const int e_span = min(e1, stop_evt);
        for (; j < e_span; j += 2) {
            body(P0{}, F{}, T{}, j);
            body(P1{}, F{}, T{}, j + 1);
        }
        if (j >= e1) break;
        if (!stop_requested) {
            request_stop_word();
            stop_requested = true;
            stop_evt += 4;
        } else if (read_stop_word() != 0) {
            stopped = true;
            n_tiles = n_act = n_full = stop_b;
            e1 = max(0, stop_b - 1) & ~1;
            stop_evt = 0x7fffffff;
        } else {
            stop_requested = false;
            stop_b += p.seg_tiles;
            stop_evt = stop_b <= stop_limit ? (stop_b & ~1) - 8 : 0x7fffffff;
        }
    }
    if (e1 > 0) {
        // S(e1) left the unmasked run without a row maximum, and the iterations below take their
        // tile's weights without the overflow check: settle its reference here, once
        row_max(F{}, s_a, e1 * kBN);
        asm volatile("" : "+v"(m_run), "+v"(m_use), "+v"(alpha));
    }
    for (; j + 1 < n_act - 1; j += 2) {
        body(P0{}, T{}, T{}, j);
        body(P1{}, T{}, T{}, j + 1);
    }
    if (j < n_act - 1) {
        body(P0{}, T{}, T{}, j);
        ++j;
    }
    if (n_act > 0) {   // last active tile (no further scores), then the product still owed
        if (j & 1) {
            body(P1{}, T{}, F{}, j);
            pv_mfma(p_b, lds_v1);
        } else {
            body(P0{}, T{}, F{}, j);
            pv_mfma(p_a, lds_v0);
        }
        ++j;
    }
    for (; j < n_tiles; ++j) {   // keep the workgroup's load / barrier cadence
        issue_k(j + 2, (j & 1) ? lds_k1 : lds_k0);
        issue_v(j, (j & 1) ? lds_v1 : lds_v0);
        end_of_iteration();
    }

    // ---- epilogue
    if constexpr (kSweep) {   // an item stopped short keeps its fp32 state; one that is through writes the result
        if (stopped) out_ptr = nullptr; else acc_out = nullptr;
    }
    {
        const int row = rw0 + l32;
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        if (row < sq) {
            const bool raw = kSweep && stopped;   // a stopped sweep item keeps its state as it stands
            const float inv = raw ? 1.f : (l_tot > 0.f ? 1.f / l_tot : 0.f);
            const float lse = raw ? m_run : (l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY);
            if (raw) p.l_part[(lse_off0 + row) * 2 + hl] = l_run;
            if (hl == 0) lse_ptr[lse_off0 + row] = lse;
            const int64_t obase = o_off0 + row * q_stride + 4 * hl;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    f32x4 x;
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[i] = o[dt][4 * b + i] * inv;
                    const int64_t idx = obase + 32 * dt + 8 * b;
                    if (acc_out) *reinterpret_cast<f32x4*>(acc_out + idx) = x;
                    if (out_ptr) {
                        if (out_f32)
                            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out_ptr) + idx) = x;
                        else
                            *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(out_ptr) + idx) =
                                __builtin_convertvector(x, bf16x4);
                    }
                }
        }
    }
    if (kSweep && threadIdx.x == 0) {
        p.progress[logical] = stopped ? seg_done + stop_b / p.seg_tiles : kSweepDone;
        if (!stopped) atomicSub(p.pending, 1);
    }
    if (kSweep && stopped) return;  // a stop request: this workgroup takes no further item
    __builtin_amdgcn_s_barrier();   // every wavefront is done with the LDS stages before the next item's loads
    }   // work items of this workgroup
}

}  // namespace pec
