// Types, constants, launch parameters and LDS layouts shared by the attention kernels (gfx950).
//
// MFMA 32x32x16 operand layout (lane l, l32 = l % 32, hl = l / 32):
//   A[M=32][K=16]: lane holds row l32, k-slots 8*hl .. 8*hl+7
//   B[K=16][N=32]: lane holds column l32, k-slots 8*hl .. 8*hl+7
//   C[M=32][N=32]: lane holds column l32, rows 8*(r/4) + 4*hl + r%4 for register r
// Scores are computed TRANSPOSED, S^T = K Q^T (keys along M, queries along N), so each lane owns one
// query column: row max / row sum are in-lane reductions plus one exchange between the two lane
// halves, and the running rescale of O is a per-lane scalar.  The contraction O^T += V^T P^T only
// needs A and B to agree on which key sits in which k-slot, so P (taken straight from the score
// registers) fixes the key order of the V^T operand: slots 0..3 <- keys 16*t2 + 4*hl + 0..3,
// slots 4..7 <- +8.
//
// LDS layout: a tile is 64 rows (keys) of 256 B (128 bf16).  K rows are XOR-swizzled at 16 B
// granularity (chunk c -> c ^ (key & 15)) for conflict-free b128 operand reads; V rows at 64 B
// granularity (segment s -> s ^ (key & 3)) for the transposing ds_read_b64_tr_b16 reads that
// deliver 4 consecutive keys of one head-dim column.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pec {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kHeadDim = 128;
constexpr int kBN = 64;               // keys per LDS tile
constexpr int kRowBytes = 256;        // one key row of 128 bf16
constexpr int kTileBytes = kBN * kRowBytes;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct WorkItem {   // one (sequence, query tile) of a packed batch; in a colocated batch a negative
    int32_t seq;    // qtile stands for key range number -1 - qtile of a one-token (decode) sequence
    int32_t qtile;
};

constexpr int32_t kSweepDone = 0x7fffffff;

struct FwdParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    void* out;              // [tokens, Hq, 128] bf16 or fp32 (may be null when only acc_out is wanted)
    float* lse;             // [Hq, lse_stride]
    const float* acc_in;    // running O (fp32, normalised) to continue from, or null
    const float* lse_in;    // running LSE matching acc_in
    float* acc_out;         // fp32 copy of the result (running state), or null
    int64_t lse_stride;     // tokens per head row in lse arrays
    int32_t sq, sk;         // dense mode: rows / keys of this call
    int32_t delta;          // q_off - kv_off, clamped to [-sq-1, sk]
    int32_t causal;
    int32_t n_q_heads, n_kv_heads, group;
    int32_t n_items;        // query tiles (dense) or work-list capacity (varlen)
    int32_t out_f32;
    float scale_log2;       // scale * log2(e)
    // varlen mode (cu_seqlens != null): work list built on the device
    const int32_t* cu_seqlens;
    const WorkItem* work;
    const int32_t* n_work;  // number of valid work items
    int32_t* sched;         // eight zeroed counters (fwd_il_kernel only): work items are drawn from them, one
                            // counter per XCD's share of the work order, instead of being dealt in fixed rounds
    int32_t total_tokens;   // rows of the packed arrays (bounds every index taken from cu_seqlens)
    // split-KV mode (kv_split_len > 0; fwd_il_kernel only): work item = key range
    // [item * kv_split_len, ...), partial results go to out / lse + item * split_*_stride
    int32_t kv_split_len;
    int64_t split_out_stride, split_lse_stride;   // elements
    // element strides of q / out / acc between rows and between heads (0 = the packed
    // [tokens, n_q_heads, 128] layout; fwd_il_kernel only)
    int64_t q_row_stride, q_head_stride;
    // colocated batch (cu_seqlens_k != null; fwd_il_kernel only): sequence b has queries
    // cu_seqlens[b] .. and keys cu_seqlens_k[b] ..; its query i sits at position len_k - len_q + i.
    // One-token sequences with long caches are cut into key ranges of coloc_range_len keys whose
    // partial results go to part_out / part_lse at slot seq_slot0[seq] + range.
    const int32_t* cu_seqlens_k;
    const int32_t* seq_slot0;
    float* part_out;            // [slots][n_q_heads][128] fp32
    float* part_lse;            // [slots][n_q_heads]
    int32_t total_k;            // rows of the packed k / v arrays
    int32_t coloc_range_len;    // keys per range, a multiple of 64
    // resumable sweep (dense mode, progress != null; fwd_il_kernel only): work item i has finished its first
    // progress[i] key segments of seg_tiles tiles each (kSweepDone: all of them) and continues from there, its
    // running state in acc_in / lse_in / l_part.  A nonzero *stop makes a workgroup end the item in hand at the next
    // segment boundary (state to acc_out / lse / l_part, progress updated) and take no further item; an item that
    // gets through its last key writes out / lse and takes one off *pending.  The state of a stopped item is kept
    // as the registers hold it -- un-normalised O, the softmax reference (log2 units) in the LSE slot, and the two
    // lane halves' partial denominators in l_part [n_q_heads][lse_stride][2] -- so a stop adds no rounding step.
    float* l_part;
    int32_t* progress;
    int32_t* pending;
    const int32_t* stop;
    int32_t seg_tiles;
};

__device__ __forceinline__ uint32_t k_lds_off(int key, int chunk16) {
    return (uint32_t)(key * kRowBytes + ((chunk16 ^ (key & 15)) << 4));
}
__device__ __forceinline__ uint32_t v_lds_off(int key, int byte_in_row) {
    const int seg = byte_in_row >> 6;
    return (uint32_t)(key * kRowBytes + (((seg ^ (key & 3)) << 6) | (byte_in_row & 63)));
}

}  // namespace pec
