/*
 * pec_attn -- blockwise causal prefill attention for one GPU's share of a
 * sequence-parallel (ring) prefill, for AMD MI355X (gfx950).
 *
 * C ABI: plain pointers and sizes only.  Unless said otherwise every pointer is a
 * DEVICE pointer owned by the caller, 16-byte aligned, and every call is
 * asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default
 * stream).  The library keeps no state between calls (every option travels in
 * pec_shape_t.flags, so concurrent callers cannot disturb each other), allocates
 * no device memory, and never synchronises the device.
 *
 * Layouts (row-major, contiguous, counts in elements):
 *   q, out  : [tokens, n_q_heads, 128]   bf16 (out: bf16 or fp32, see out_dtype)
 *   k, v    : [tokens, n_kv_heads, 128]  bf16
 *   lse     : [n_q_heads, tokens]        fp32, natural log of sum_j exp(q.k_j * scale)
 * Query head h reads KV head h / (n_q_heads / n_kv_heads)  (grouped-query
 * attention as assumed by the paper's cost model, section "Fast Sequence
 * Parallelism for Long-Request Prefill").
 *
 * Positions: local query row i sits at global position q_off + i, local key j at
 * kv_off + j.  With causal != 0 key j is visible to row i iff
 * kv_off + j <= q_off + i  (Eq. 3: the softmax denominator runs up to the row's
 * own token, which is included).  A row with no visible key gets out = 0 and
 * lse = -inf; that pair is the identity of pec_attn_merge.
 *
 * Every function returns PEC_OK (0) or a negative pec_status; nothing throws or
 * aborts across this boundary.  Zero-sized problems (sq == 0) are PEC_OK no-ops.
 */
#ifndef PEC_ATTN_H
#define PEC_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PEC_OK = 0,
    PEC_ERR_INVALID_ARGUMENT = -1, /* null pointer, negative size, n_q_heads % n_kv_heads != 0, scale <= 0 ... */
    PEC_ERR_UNSUPPORTED = -2,      /* head_dim != 128, unknown dtype / option, size beyond 2^30 rows */
    PEC_ERR_MISALIGNED = -3,       /* a pointer is not 16-byte aligned */
    PEC_ERR_WORKSPACE = -4,        /* workspace missing or smaller than pec_*_workspace_bytes() */
    PEC_ERR_HIP = -5,              /* the HIP runtime reported an error at launch */
    PEC_ERR_SCRATCH_LIMIT = -6     /* pec_decode_splitkv_static: the problem needs more than the static scratch buffer */
} pec_status;

enum { PEC_BF16 = 0, PEC_F32 = 1 };

typedef struct {
    int32_t n_q_heads;  /* N_h */
    int32_t n_kv_heads; /* N_h^KV, divides n_q_heads */
    int32_t head_dim;   /* d_h, must be 128 */
    int32_t out_dtype;  /* dtype of `out` / `o_acc` / `o_part`: PEC_BF16 (final) or PEC_F32 (partials kept
                           exact across merges) */
    float scale;        /* multiplies q.k; 0 selects 1/sqrt(head_dim) (Eq. 2) */
    uint32_t flags;     /* PEC_FLAG_* or-ed together; 0 = defaults */
} pec_shape_t;

/* Per-call options (pec_shape_t.flags). */
enum {
    PEC_FLAG_SIMPLE_KERNEL = 1u,     /* run the plain, unpipelined attention kernel (exact running maximum, no
                                        persistence) instead of the default one: a cross-check, several times slower */
    PEC_FLAG_SP_SEPARATE_MERGE = 2u, /* pec_sp_prefill: one launch per ring step, pec_attn_chunk -> fp32 partial ->
                                        pec_attn_merge, instead of the default single sweep */
    PEC_FLAG_SP_STEP_LAUNCHES = 4u   /* pec_sp_prefill: one launch per ring step with the merge fused into the kernel
                                        (what issuing pec_sp_prefill_step back to back does), instead of the
                                        default single sweep */
};

/*
 * One ring step: attention of a local query segment against ONE key/value
 * segment (Eq. 2 with the softmax of Eq. 3 restricted to that segment's keys),
 * returned as the partial pair (out, lse).
 *   q [sq, Hq, 128], k/v [sk, Hkv, 128], out [sq, Hq, 128] (out_dtype), lse [Hq, sq].
 * sk == 0 or a segment wholly in the future gives out = 0, lse = -inf.
 */
int pec_attn_chunk(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                   int64_t sq, int64_t sk, int64_t q_off, int64_t kv_off, int causal,
                   void* out, float* lse, void* stream);

/*
 * Same ring step, folded straight into running accumulators: on entry
 * (o_acc, lse_acc) is the exact result over the keys seen so far, on return it is
 * the exact result over those keys plus this segment's (the log-sum-exp merge of
 * pec_attn_merge applied inside the kernel, so the partial never reaches HBM).
 * o_acc is always fp32 [sq, Hq, 128]; lse_acc [Hq, sq].  If out_final is not NULL
 * the merged result is ALSO written there in shape->out_dtype (used for the last
 * ring step); o_acc/lse_acc are updated in either case.
 */
int pec_attn_chunk_merge(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                         int64_t sq, int64_t sk, int64_t q_off, int64_t kv_off, int causal,
                         float* o_acc, float* lse_acc, void* out_final, void* stream);

/*
 * Exact merge of two partial results over disjoint key sets (the online-softmax
 * step of ring attention, section "Sequence Parallelism for Long Requests"):
 *   L = ln(exp(lse_acc) + exp(lse_part)),
 *   o_acc = o_acc * exp(lse_acc - L) + o_part * exp(lse_part - L),  lse_acc = L.
 * In place on (o_acc, lse_acc).  o_acc and o_part are [sq, Hq, 128] in
 * shape->out_dtype, the lse arrays [Hq, sq] fp32.  (0, -inf) is the identity.
 */
int pec_attn_merge(const pec_shape_t* shape, void* o_acc, float* lse_acc,
                   const void* o_part, const float* lse_part, int64_t sq, void* stream);

/* fp32 [sq, Hq, 128] -> bf16, round to nearest even.  For callers that merged fp32 partials. */
int pec_finalize(const pec_shape_t* shape, const float* o_f32, void* o_bf16, int64_t sq, void* stream);

/*
 * One ring member's whole prefill on one GPU: the query segment q [s_q, Hq, 128]
 * at global offset q_off attends over k/v [s_kv, Hkv, 128] (global positions
 * 0..s_kv-1) cut into contiguous segments of `chunk` tokens (the last may be
 * short); under the causal mask segments wholly in the future are skipped.
 * By default ONE launch sweeps all visible segments in position order, the running
 * (O, LSE) of every query tile staying in registers from segment to segment; this
 * call cannot be stopped half way (pec_sp_prefill_resumable and pec_sp_prefill_step
 * can).  PEC_FLAG_SP_STEP_LAUNCHES and PEC_FLAG_SP_SEPARATE_MERGE instead launch
 * once per ring step, in ring order starting from the member's own segment,
 * (r - t) mod P for step t with r = q_off / chunk, the running fp32 pair going
 * through the workspace between steps (merged inside the next step's kernel, or by
 * pec_attn_merge).  All three give the same result up to fp32 rounding order.
 *   out [s_q, Hq, 128] in shape->out_dtype, lse [Hq, s_q].
 * workspace: device scratch of at least pec_sp_workspace_bytes() bytes, 16-byte
 * aligned; contents undefined on return (not used by the default sweep).
 */
int pec_sp_prefill(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                   int64_t s_q, int64_t q_off, int64_t s_kv, int64_t chunk, int causal,
                   void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream);
size_t pec_sp_workspace_bytes(const pec_shape_t* shape, int64_t s_q);

/*
 * The sweep of pec_sp_prefill as a launch that a scheduler can stop between two key
 * segments and continue later (section "Preemption of Long-Request Prefill": the
 * long prefill yields at operation granularity and only the intermediate data of
 * the interrupted operation is kept).  Every workgroup looks at *stop shortly
 * before each segment boundary of the query tile it is working on; once it reads a
 * nonzero value it finishes the segment in hand, puts the tile's running state
 * and the number of segments done into the workspace, and takes no further tile.
 * A later call with resume = 1 and the same arguments and workspace continues every
 * tile from where it stopped; *pending is then the number of query tiles x heads
 * that have not yet seen their last key (0: out and lse are complete).  A launch
 * always takes each workgroup's first unfinished tile through at least one more
 * segment, so repeated calls end even if *stop stays set.  A stopped tile's state
 * is stored as the kernel held it (un-normalised O, softmax reference, partial
 * denominators), so a stop adds no rounding step: the result equals the
 * uninterrupted sweep's bit for bit, except that a row with a score, within two
 * tiles of a cut, more than 2^8 above its running softmax reference may differ by
 * one fp32 rescale.
 *   stop    : int32 the GPU can read while the kernel runs: pinned host memory written by the
 *             host, or device memory written by a copy or a kernel on another stream (it is
 *             read past the caches); NULL = never stop.  Segments
 *             shorter than 1024 keys, and query tiles with fewer than 256 rows, are
 *             only left between tiles, not between segments.
 *   pending : DEVICE int32, written by the call (resume = 0 sets it to the tile count).
 *   resume  : 0 starts from the first segment and ignores the workspace contents.
 *   chunk   : a multiple of 64 (PEC_ERR_UNSUPPORTED otherwise).
 *   workspace: pec_sp_resumable_workspace_bytes() bytes, 16-byte aligned; holds the
 *             state between calls (the caller may copy it away and back, together
 *             with lse, which holds part of the state of unfinished tiles meanwhile).
 * PEC_FLAG_SIMPLE_KERNEL is refused (PEC_ERR_UNSUPPORTED).  Two calls that use one
 * workspace at the same time race; one sweep needs one workspace.
 */
int pec_sp_prefill_resumable(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                             int64_t s_q, int64_t q_off, int64_t s_kv, int64_t chunk, int causal,
                             void* out, float* lse, void* workspace, size_t workspace_bytes,
                             const int32_t* stop, int32_t* pending, int resume, void* stream);
size_t pec_sp_resumable_workspace_bytes(const pec_shape_t* shape, int64_t s_q);

/*
 * The same prefill one ring step at a time, for a scheduler that pauses a long prefill between
 * two kernel operations and resumes it later (section "Preemption of Long-Request Prefill": only
 * the intermediate data passed between the two operations has to be kept).  Here that data is the
 * running pair (o_acc fp32 [s_q, Hq, 128], lse_acc fp32 [Hq, s_q]) plus the index of the next step.
 *   pec_sp_prefill_num_steps: number of KV segments this member visits (>= 0), or a negative status.
 *   pec_sp_prefill_step: executes visited segment number `step` (0-based, ring order).  Step 0
 *   initialises (o_acc, lse_acc) and ignores their previous contents; steps must be issued in
 *   order, each exactly once; anything may run on the GPU, and the state may be copied away and
 *   back, between two steps.  If out_final is not NULL on the last step the result is written
 *   there in shape->out_dtype (and o_acc is then left unchanged); lse_acc always ends as the LSE.
 * Issuing all steps back to back is what pec_sp_prefill does with PEC_FLAG_SP_STEP_LAUNCHES.
 */
int64_t pec_sp_prefill_num_steps(const pec_shape_t* shape, int64_t s_q, int64_t q_off, int64_t s_kv,
                                 int64_t chunk, int causal);
int pec_sp_prefill_step(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                        int64_t s_q, int64_t q_off, int64_t s_kv, int64_t chunk, int causal, int64_t step,
                        float* o_acc, float* lse_acc, void* out_final, void* stream);

/*
 * Packed batch of independent prompts (batched short prefills colocated with a
 * long request, section "Coordinated Prefill-Decode Colocation and
 * Disaggregation"): sequence b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1 of
 * q/k/v/out, attends only to itself, positions restart at 0.
 *   cu_seqlens: DEVICE int32 [batch + 1], non-decreasing, cu_seqlens[0] == 0,
 *               cu_seqlens[batch] == total_tokens (not checked; otherwise undefined).
 *               Entries are clamped into [0, total_tokens] and made non-decreasing on the
 *               device, so malformed values can misplace results but never index out of bounds.
 *   max_seqlen: the caller's bound on the sequence lengths (host value); a HINT only -- the work
 *               list is sized from total_tokens, so a sequence longer than max_seqlen is still
 *               processed in full, never cut short.
 *   lse [Hq, total_tokens].  Zero-length sequences are legal.
 * workspace: at least pec_varlen_workspace_bytes() bytes (the device-built work list).
 */
int pec_attn_varlen(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                    const int32_t* cu_seqlens, int32_t batch, int64_t total_tokens, int32_t max_seqlen,
                    int causal, void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream);
size_t pec_varlen_workspace_bytes(int32_t batch, int64_t total_tokens);

/*
 * Colocated batch in ONE attention launch (section "Coordinated Prefill-Decode Colocation and
 * Disaggregation": the GPUs that hold a long request's KV cache run its decode step batched together
 * with the prefills of short requests).  Sequence b has len_q = cu_seqlens_q[b+1] - cu_seqlens_q[b]
 * query tokens (rows of q / out) and len_k = cu_seqlens_k[b+1] - cu_seqlens_k[b] keys (rows of k / v);
 * its queries are the LAST len_q positions of the sequence, query i at position len_k - len_q + i, so
 * with causal != 0 key j is visible to query i iff j <= len_k - len_q + i (Eq. 3).  A prompt has
 * len_q == len_k; the decode step of a request has len_q == 1 and len_k = its cache length including
 * the new token; anything in between is a chunk of new tokens behind a cached prefix.
 *   q, out [total_q, Hq, 128]; k, v [total_k, Hkv, 128]; lse [Hq, total_q].
 *   cu_seqlens_q, cu_seqlens_k: DEVICE int32 [batch + 1], non-decreasing from 0 (values are clamped on
 *   the device; malformed ones can misplace or drop results but never index out of bounds).
 * One-token sequences with more than 4096 keys are cut into key ranges of 4096 keys that run as work
 * items of the same launch (the query heads of a KV group share one pass over the keys); a second,
 * small launch merges their partial (O, LSE) pairs by log-sum-exp.  Rows without a visible key get
 * out = 0, lse = -inf.  workspace: pec_colocated_workspace_bytes() bytes.
 * PEC_FLAG_SIMPLE_KERNEL is not supported here (PEC_ERR_UNSUPPORTED).
 */
int pec_attn_colocated(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                       const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int32_t batch,
                       int64_t total_q, int64_t total_k, int causal, void* out, float* lse,
                       void* workspace, size_t workspace_bytes, void* stream);
size_t pec_colocated_workspace_bytes(const pec_shape_t* shape, int32_t batch, int64_t total_q, int64_t total_k);

/*
 * Decode attention of a long request kept on its prefill GPUs while short prefills share them
 * (section "Coordinated Prefill-Decode Colocation and Disaggregation"): ONE new token, q [1, Hq, 128],
 * against this GPU's shard of the KV cache, k/v [sk, Hkv, 128]; every key is visible.  The shard is
 * cut into n_splits key ranges (0 = pick a default: one workgroup per compute unit), each KV head of
 * a range is streamed by one wavefront on its own, the partial (O, LSE) pairs are combined exactly
 * by log-sum-exp.  out [1, Hq, 128] in shape->out_dtype and
 * lse [Hq] form a partial pair over this shard: results of several shards / GPUs (the paper's
 * example merges the outputs of two GPUs) combine with pec_attn_merge (use out_dtype PEC_F32).
 * sk == 0 gives out = 0, lse = -inf.  workspace: pec_decode_workspace_bytes() bytes.
 * HBM-bound: K and V are read once, 2 * sk * Hkv * 128 * 2 bytes.
 */
int pec_decode_splitkv(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sk,
                       int32_t n_splits, void* out, float* lse, void* workspace, size_t workspace_bytes,
                       void* stream);
int32_t pec_decode_default_splits(const pec_shape_t* shape, int64_t sk);
size_t pec_decode_workspace_bytes(const pec_shape_t* shape, int32_t n_splits);

/*
 * pec_decode_splitkv for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results (bit-identical) as pec_decode_splitkv, but the partial (O, LSE) pairs of the
 * key ranges live in a buffer of PEC_DECODE_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (one copy per GPU, held until the process ends).  The call allocates and frees
 * nothing, on the device or through any library.
 *   Limit: pec_decode_workspace_bytes(shape, n_splits) = n_splits * n_q_heads * 129 * 4 bytes must
 *   not exceed PEC_DECODE_STATIC_SCRATCH_BYTES (e.g. 128 key ranges x 64 query heads = 4.2 MB);
 *   beyond it the call returns PEC_ERR_SCRATCH_LIMIT and launches nothing.
 *   The first call on a device looks up the buffer's device address (hipGetSymbolAddress); make that
 *   first call outside any stream capture.
 *   Every call on a GPU uses that GPU's one buffer: two calls that overlap in time on the same GPU
 *   (different streams, different threads) race on it and give undefined results.  Calls on one
 *   stream, or otherwise ordered, are safe; nothing in the buffer needs clearing between calls
 *   (every partial a call reads it has written itself).
 */
#define PEC_DECODE_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
int pec_decode_splitkv_static(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sk,
                              int32_t n_splits, void* out, float* lse, void* stream);

/*
 * On-GPU halves of the head <-> sequence exchange of Ulysses-style sequence parallelism (section
 * "Sequence Parallelism of Megatron and Ulysses": an all-to-all turns "my sequence segment, all
 * heads" into "the whole sequence, my heads" before attention, and back afterwards).  bf16,
 * head_dim 128.
 *   to_messages != 0: src [s, n_heads, 128] -> dst [n_gpus, s, n_heads/n_gpus, 128]; message g holds
 *     the heads GPU g owns and is what the all-to-all sends to it.  (The messages a GPU receives,
 *     ordered by source rank, already are its [n_gpus*s, n_heads/n_gpus, 128] input: no kernel.)
 *   to_messages == 0: the inverse, src [n_gpus, s, n_heads/n_gpus, 128] (messages received after
 *     attention, ordered by source rank) -> dst [s, n_heads, 128].
 * src and dst must not overlap.  HBM-bound copy: every byte is read once and written once.
 * The all-to-all itself is not part of this library.
 */
int pec_ulysses_layout(const void* src, void* dst, int64_t s, int32_t n_heads, int32_t head_dim, int32_t n_gpus,
                       int to_messages, void* stream);

/*
 * Intra-node strategy selection of fast Sequence Parallelism (section "Fast Sequence Parallelism for
 * Long-Request Prefill"): for the attention stage and for the MLP stage either Megatron SP or Ulysses
 * SP; the paper gives the communication volume per node and the computation volume per GPU of each
 * choice in closed form, estimates the time of the four combinations and takes the smallest.  Host
 * arithmetic only; no GPU work.  Volumes are in elements / flop exactly as the paper's formulas give
 * them; the time estimate of a combination is, for both stages,
 *     comm_elements * bytes_per_element / node_bandwidth + compute_flop / gpu_flops
 * (the paper does not say how the two are combined; they are added).  Index 0 = Megatron, 1 = Ulysses.
 */
typedef struct {
    int64_t d_model;          /* d */
    int32_t n_heads;          /* N_h */
    int32_t n_kv_heads;       /* N_h^KV */
    int32_t head_dim;         /* d_h */
    int64_t seg_len;          /* s: sequence segment length per GPU */
    int32_t tp;               /* T: tensor-parallel size */
    int32_t gpus_per_node;    /* G */
    double bytes_per_element; /* 2 for bf16 */
    double node_bandwidth;    /* bytes/s available to the node's collectives */
    double gpu_flops;         /* flop/s one GPU sustains on these GEMMs / attention */
} pec_sp_model_t;

typedef struct {
    double attn_comm[2], attn_compute[2]; /* attention stage: [Megatron, Ulysses] */
    double mlp_comm[2], mlp_compute[2];   /* MLP stage */
    double seconds[2][2];                 /* [attention choice][MLP choice] */
    int32_t best_attn, best_mlp;          /* argmin of seconds (ties: Megatron first) */
} pec_sp_choice_t;

int pec_sp_select_strategy(const pec_sp_model_t* model, pec_sp_choice_t* choice);

/*
 * Measurement aid, not part of the method: launches a loop of independent bf16 MFMAs
 * (v_mfma_f32_32x32x16_bf16, the instruction of the attention kernels; one workgroup of 8
 * wavefronts per compute unit, `iters` x 32 MFMAs per wavefront) on operands the caller supplies,
 * so that the matrix-pipe rate the chip sustains at its clocks and power limit can be measured with
 * the caller's own timer, for constant and for random operand data.
 *   operands: DEVICE, at least 16 KiB (8 A and 8 B fragments of 64 lanes x 16 bytes of bf16).
 *   sink: DEVICE, at least compute units x 512 floats; receives one value per thread.
 * Returns the number of floating-point operations the launch performs (> 0), or a negative status.
 */
int64_t pec_mfma_probe(const void* operands, size_t operand_bytes, int32_t iters, float* sink, size_t sink_floats,
                       void* stream);

/*
 * Measurement aid, not part of the method: one streaming read of `bytes` bytes (a multiple of 16) at
 * `src` (DEVICE), eight 16-byte loads in flight per thread, 32 workgroups per compute unit; `sink`
 * (DEVICE, 4 bytes) is only there so that the loads count as used.  Timed by the caller, it gives the
 * read bandwidth the memory system delivers, the ceiling of the HBM-bound kernels of this library.
 */
int pec_hbm_read_probe(const void* src, size_t bytes, void* sink, void* stream);

const char* pec_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PEC_ATTN_H */
