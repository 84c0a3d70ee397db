// HBM-bound helpers around the attention kernel: the log-sum-exp merge of two
// partial results, the fp32 -> bf16 finalisation, and the device-side work list for
// packed variable-length batches.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace pec {

// o_acc <- o_acc * exp(la - L) + o_part * exp(lb - L),  L = ln(exp(la) + exp(lb)).
// One thread per 4 consecutive head-dim values; the 32 threads of one (row, head)
// sit in one wavefront, so all of them read lse_acc before thread 0 overwrites it.
template <bool F32>
__global__ __launch_bounds__(256) void merge_kernel(void* __restrict__ o_acc_v, float* __restrict__ lse_acc,
                                                    const void* __restrict__ o_part_v,
                                                    const float* __restrict__ lse_part, int64_t sq, int n_q_heads) {
    const int64_t n_groups = sq * n_q_heads * 32;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n_groups;
         g += (int64_t)gridDim.x * blockDim.x) {
        const int64_t rh = g >> 5;
        const int64_t row = rh / n_q_heads;
        const int h = (int)(rh % n_q_heads);
        const int64_t li = (int64_t)h * sq + row;
        const float la = lse_acc[li], lb = lse_part[li];
        const float mx = fmaxf(la, lb);
        float wa = 0.f, wb = 0.f, L = -INFINITY;
        if (mx != -INFINITY) {
            const float ea = expf(la - mx), eb = expf(lb - mx);
            const float den = ea + eb;
            wa = ea / den;
            wb = eb / den;
            L = mx + logf(den);
        }
        f32x4 a, b;
        if constexpr (F32) {
            a = reinterpret_cast<const f32x4*>(o_acc_v)[g];
            b = reinterpret_cast<const f32x4*>(o_part_v)[g];
        } else {
            a = __builtin_convertvector(reinterpret_cast<const bf16x4*>(o_acc_v)[g], f32x4);
            b = __builtin_convertvector(reinterpret_cast<const bf16x4*>(o_part_v)[g], f32x4);
        }
        f32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = a[i] * wa + b[i] * wb;
        if constexpr (F32)
            reinterpret_cast<f32x4*>(o_acc_v)[g] = r;
        else
            reinterpret_cast<bf16x4*>(o_acc_v)[g] = __builtin_convertvector(r, bf16x4);
        if ((g & 31) == 0) lse_acc[li] = L;
    }
}

__global__ __launch_bounds__(256) void finalize_kernel(const float* __restrict__ src, __bf16* __restrict__ dst,
                                                       int64_t n_groups) {
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n_groups;
         g += (int64_t)gridDim.x * blockDim.x)
        reinterpret_cast<bf16x4*>(dst)[g] = __builtin_convertvector(reinterpret_cast<const f32x4*>(src)[g], bf16x4);
}

// Combines the partial results of a split-KV decode: for one head, L = ln sum_s exp(lse_s) and
// O = sum_s O_s exp(lse_s - L) over the n_splits disjoint key ranges (the two-set merge applied to
// all ranges at once).  One workgroup of kCombineGroups x 128 threads per call: thread (grp, d) sums
// the ranges s = grp, grp + kCombineGroups, ... for dimension d, LDS adds the groups up.  Partials
// are fp32 [n_splits][n_heads][128] and [n_splits][n_heads]; out_row points at the 128 outputs.
constexpr int kCombineGroups = 8;
template <bool OUT_F32>
__device__ __forceinline__ void combine_one_head(const float* __restrict__ o_part, const float* __restrict__ lse_part,
                                                 int n_splits, int n_heads, int h, void* __restrict__ out_row,
                                                 float* __restrict__ lse_dst) {
    __shared__ float red[kCombineGroups][kHeadDim];
    __shared__ float red_s[kCombineGroups * 2];
    const int d = threadIdx.x & 127, grp = threadIdx.x >> 7;
    const int tid = threadIdx.x, nthr = kCombineGroups * 128;
    // maximum LSE of the head: every wavefront reduces its share, LDS the 16 wavefronts
    float mx = -INFINITY;
    for (int s = tid; s < n_splits; s += nthr) mx = fmaxf(mx, lse_part[(int64_t)s * n_heads + h]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    __syncthreads();                 // a previous call's readers of red_s / red are done
    if ((tid & 63) == 0) red_s[tid >> 6] = mx;
    __syncthreads();
    mx = red_s[0];
#pragma unroll
    for (int w = 1; w < kCombineGroups * 2; ++w) mx = fmaxf(mx, red_s[w]);
    float den = 0.f, acc = 0.f;
    if (mx != -INFINITY) {
        for (int s = grp; s < n_splits; s += kCombineGroups) {
            const float w = expf(lse_part[(int64_t)s * n_heads + h] - mx);
            den += w;   // every thread of a group carries the group's share of the denominator
            acc += w * o_part[((int64_t)s * n_heads + h) * kHeadDim + d];
        }
    }
    red[grp][d] = acc;
    __syncthreads();                 // also orders the reads of red_s above before its reuse below
    if (d == 0) red_s[grp] = den;
    __syncthreads();
    if (grp == 0) {
        float a = 0.f, dn = 0.f;
#pragma unroll
        for (int g2 = 0; g2 < kCombineGroups; ++g2) {
            a += red[g2][d];
            dn += red_s[g2];
        }
        if (mx != -INFINITY) a /= dn;
        if constexpr (OUT_F32)
            reinterpret_cast<float*>(out_row)[d] = a;
        else
            reinterpret_cast<__bf16*>(out_row)[d] = (__bf16)a;
        if (d == 0) *lse_dst = mx != -INFINITY ? mx + logf(dn) : -INFINITY;
    }
}

template <bool OUT_F32>
__global__ __launch_bounds__(kCombineGroups * 128) void combine_splits_kernel(const float* __restrict__ o_part,
                                                                              const float* __restrict__ lse_part,
                                                                              int n_splits, int n_heads,
                                                                              void* __restrict__ out,
                                                                              float* __restrict__ lse) {
    const int h = blockIdx.x;
    void* out_row = OUT_F32 ? static_cast<void*>(reinterpret_cast<float*>(out) + (int64_t)h * kHeadDim)
                            : static_cast<void*>(reinterpret_cast<__bf16*>(out) + (int64_t)h * kHeadDim);
    combine_one_head<OUT_F32>(o_part, lse_part, n_splits, n_heads, h, out_row, lse + h);
}

// The same combination for the one-token sequences of a colocated batch: split_seqs lists
// (sequence, first slot, number of key ranges); the result goes to the sequence's row of the packed
// out [total_q, n_heads, 128] / lse [n_heads, total_q].  grid = (n_heads, up to batch).
struct SplitSeq {
    int32_t seq, slot0, n_ranges, pad;
};
template <bool OUT_F32>
__global__ __launch_bounds__(kCombineGroups * 128) void combine_colocated_kernel(
    const float* __restrict__ o_part, const float* __restrict__ lse_part, const SplitSeq* __restrict__ split_seqs,
    const int32_t* __restrict__ n_split_seqs, const int32_t* __restrict__ cu_q, int total_q, int n_heads,
    void* __restrict__ out, float* __restrict__ lse) {
    const int h = blockIdx.x;
    const int n = *n_split_seqs;
    for (int i = blockIdx.y; i < n; i += gridDim.y) {
        const SplitSeq ss = split_seqs[i];
        const int64_t row = min(max(cu_q[ss.seq], 0), total_q - 1);
        void* out_row = OUT_F32 ? static_cast<void*>(reinterpret_cast<float*>(out) + (row * n_heads + h) * kHeadDim)
                                : static_cast<void*>(reinterpret_cast<__bf16*>(out) + (row * n_heads + h) * kHeadDim);
        combine_one_head<OUT_F32>(o_part + (int64_t)ss.slot0 * n_heads * kHeadDim, lse_part + (int64_t)ss.slot0 * n_heads,
                                  ss.n_ranges, n_heads, h, out_row, lse + (int64_t)h * total_q + row);
    }
}

// Ulysses-style layout exchange, the on-GPU halves.  A GPU holding a sequence segment of all heads,
// x [s, H, 128], packs it into G messages of s x H/G heads, y [G, s, H/G, 128] (message g = the heads
// GPU g will own); the inverse turns G received messages back into [s, H, 128].  16 bytes per thread,
// both sides contiguous in runs of H/G * 256 bytes.  TO_MESSAGES selects the direction.
template <bool TO_MESSAGES>
__global__ __launch_bounds__(256) void ulysses_layout_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                             int64_t s, int n_heads, int n_gpus) {
    constexpr int kBatch = 4;                        // loads in flight per thread before the first store
    const int hg = n_heads / n_gpus;                 // heads per message
    const int64_t chunks_per_tok = (int64_t)n_heads * 16;   // 16-byte chunks per token (all heads)
    const int64_t total = s * chunks_per_tok;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    auto other_side = [&](int64_t i) {               // i indexes the [s, H, 16] side; returns the [G, s, H/G, 16] index
        const int64_t t = i / chunks_per_tok;
        const int r = (int)(i % chunks_per_tok);
        const int h = r >> 4, c = r & 15;
        const int g = h / hg, hh = h % hg;
        return (((int64_t)g * s + t) * hg + hh) * 16 + c;
    };
    for (int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < total; i0 += kBatch * stride) {
        u32x4 v[kBatch];
        int64_t j[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int64_t i = i0 + u * stride;
            if (i < total) {
                j[u] = other_side(i);
                v[u] = __builtin_nontemporal_load(src + (TO_MESSAGES ? i : j[u]));
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int64_t i = i0 + u * stride;
            if (i < total) __builtin_nontemporal_store(v[u], dst + (TO_MESSAGES ? j[u] : i));
        }
    }
}

// Exclusive suffix sum in place over a[0..n), by one workgroup of 1024 threads: a[t] <- sum of the old
// a[t'] for t' > t.  Returns the sum of all old elements.  `red` is int32[1024] in LDS.
__device__ inline int block_suffix_sum_1024(int32_t* a, int n, int32_t* red) {
    const int tid = threadIdx.x;
    const int chunk = (n + 1023) / 1024;
    const int lo = min(n, tid * chunk), hi = min(n, lo + chunk);
    int mine = 0;
    for (int t = lo; t < hi; ++t) mine += a[t];
    red[tid] = mine;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {   // inclusive suffix scan of the per-thread sums
        const int add = tid + off < 1024 ? red[tid + off] : 0;
        __syncthreads();
        red[tid] += add;
        __syncthreads();
    }
    const int total = red[0];
    int run = red[tid] - mine;                   // everything owned by later threads
    __syncthreads();
    for (int t = hi - 1; t >= lo; --t) {
        const int x = a[t];
        a[t] = run;
        run += x;
    }
    __syncthreads();
    return total;
}

// Work list for a packed batch: one item per (sequence, query tile), ordered by descending
// query-tile index so that the longest causal rows start first.  Single workgroup of 1024 threads;
// `bucket` (int32[cap + 1]) and `cursor` (int32[cap]) are scratch, cap >= total_tokens / bm + 1.
// Sequence bounds are clamped into [0, total_tokens] exactly as the attention kernel clamps them, so
// no sequence can have more than total_tokens / bm + 1 tiles and none is ever cut short.
__global__ __launch_bounds__(1024) void build_worklist_kernel(const int32_t* __restrict__ cu, int batch,
                                                              int total_tokens, int bm, int capacity,
                                                              WorkItem* __restrict__ work,
                                                              int32_t* __restrict__ n_work,
                                                              int32_t* __restrict__ bucket,
                                                              int32_t* __restrict__ cursor) {
    __shared__ int32_t red[1024];
    const int tid = threadIdx.x;
    auto tiles_of = [&](int b) {
        const int b0 = min(max(cu[b], 0), total_tokens);
        const int b1 = min(max(cu[b + 1], b0), total_tokens);
        return (b1 - b0 + bm - 1) / bm;
    };
    // largest tile count of any sequence: only that many buckets are touched
    int mx = 0;
    for (int b = tid; b < batch; b += 1024) mx = max(mx, tiles_of(b));
    red[tid] = mx;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if (tid < off) red[tid] = max(red[tid], red[tid + off]);
        __syncthreads();
    }
    const int n_t = red[0];
    __syncthreads();
    for (int t = tid; t <= n_t; t += 1024) bucket[t] = 0;
    for (int t = tid; t < n_t; t += 1024) cursor[t] = 0;
    __syncthreads();
    for (int b = tid; b < batch; b += 1024) atomicAdd(&bucket[tiles_of(b)], 1);   // histogram of tile counts
    __syncthreads();
    block_suffix_sum_1024(bucket, n_t + 1, red);                   // bucket[t] = sequences with more than t tiles
    const int total = block_suffix_sum_1024(bucket, n_t, red);     // bucket[t] = list position of the first item of tile t
    if (tid == 0) *n_work = min(total, capacity);
    if (tid >= 8 && tid < 16) n_work[tid] = 0;   // the attention kernel's draw counters, one per XCD
    // placement: one wavefront per sequence, one lane per tile
    const int wave = tid >> 6, lane = tid & 63;
    for (int b = wave; b < batch; b += 16) {
        const int nq = tiles_of(b);
        for (int t = lane; t < nq; t += 64) {
            const int pos = bucket[t] + atomicAdd(&cursor[t], 1);
            if (pos < capacity) {   // cannot overflow: capacity bounds the item count of any clamped cu_seqlens
                work[pos].seq = b;
                work[pos].qtile = t;
            }
        }
    }
}

// Work list of a colocated batch (separate query and key offsets per sequence).  A sequence with one
// query token and more than range_len keys (the decode step of a long request) is cut into key ranges
// of range_len keys, every other sequence into query tiles of bm rows; items are ordered by
// descending number of 256-key blocks they have to read, so the long ones start first.
// Single workgroup of 1024 threads.  counters: [0] number of items, [1] slots handed out, [2] number
// of split sequences.  bucket is int32[n_buckets + 1], cursor int32[n_buckets], n_buckets >= total_k / 256 + 2.
__global__ __launch_bounds__(1024) void build_colocated_worklist_kernel(
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k, int batch, int total_q, int total_k, int bm,
    int range_len, int capacity, int slot_capacity, int n_buckets, WorkItem* __restrict__ work,
    int32_t* __restrict__ counters, int32_t* __restrict__ bucket, int32_t* __restrict__ cursor,
    int32_t* __restrict__ seq_slot0, SplitSeq* __restrict__ split_seqs) {
    __shared__ int32_t red[1024];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int t = tid; t <= n_buckets; t += 1024) bucket[t] = 0;
    for (int t = tid; t < n_buckets; t += 1024) cursor[t] = 0;
    if (tid < 3) counters[tid] = 0;
    __syncthreads();
    struct Seq {
        int len_q, len_k, n_items;
        bool split;
    };
    auto seq_of = [&](int b) {
        const int q0 = min(max(cu_q[b], 0), total_q), q1 = min(max(cu_q[b + 1], q0), total_q);
        const int k0 = min(max(cu_k[b], 0), total_k), k1 = min(max(cu_k[b + 1], k0), total_k);
        Seq s;
        s.len_q = q1 - q0;
        s.len_k = k1 - k0;
        s.split = s.len_q == 1 && s.len_k > range_len;
        s.n_items = s.split ? (s.len_k + range_len - 1) / range_len : (s.len_q + bm - 1) / bm;
        return s;
    };
    auto weight_of = [&](const Seq& s, int i) {   // 256-key blocks item i of the sequence reads
        int keys;
        if (s.split) keys = min(range_len, s.len_k - i * range_len);
        else keys = min(s.len_k, max(0, s.len_k - s.len_q + min(s.len_q, bm * (i + 1))));
        return min(n_buckets - 1, (keys + 255) / 256);
    };
    // slots of the split sequences first: a sequence that finds no room (only possible with offsets that
    // are not monotone, whose clamped lengths can add up to more than total_k) is left out altogether
    for (int b = tid; b < batch; b += 1024) {
        const Seq s = seq_of(b);
        int slot0 = -1;
        if (s.split) {
            slot0 = atomicAdd(&counters[1], s.n_items);
            if (slot0 + s.n_items <= slot_capacity) {
                const int idx = atomicAdd(&counters[2], 1);
                split_seqs[idx] = SplitSeq{b, slot0, s.n_items, 0};
            } else {
                slot0 = -2;
            }
        }
        seq_slot0[b] = slot0;
    }
    __syncthreads();
    // histogram of item weights
    for (int b = wave; b < batch; b += 16) {
        const Seq s = seq_of(b);
        if (seq_slot0[b] == -2) continue;
        for (int i = lane; i < s.n_items; i += 64) atomicAdd(&bucket[weight_of(s, i)], 1);
    }
    __syncthreads();
    // bucket[w] <- number of items heavier than w = list position of the first item of weight w
    const int total = block_suffix_sum_1024(bucket, n_buckets, red);
    if (tid == 0) counters[0] = min(total, capacity);
    if (tid >= 8 && tid < 16) counters[tid] = 0;   // the attention kernel's draw counters, one per XCD
    for (int b = wave; b < batch; b += 16) {
        const Seq s = seq_of(b);
        if (seq_slot0[b] == -2) continue;
        for (int i = lane; i < s.n_items; i += 64) {
            const int w = weight_of(s, i);
            const int pos = bucket[w] + atomicAdd(&cursor[w], 1);
            if (pos < capacity) {
                work[pos].seq = b;
                work[pos].qtile = s.split ? -1 - i : i;
            }
        }
    }
}

// Start of a resumable sweep: no item has a segment behind it, all of them are pending.
__global__ void sweep_init_kernel(int32_t* progress, int64_t n_items, int32_t* pending) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_items; i += (int64_t)gridDim.x * blockDim.x)
        progress[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) *pending = (int32_t)n_items;
}

}  // namespace pec
