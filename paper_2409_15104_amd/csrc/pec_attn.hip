// C-ABI host side of pec_attn: argument validation, launch geometry, ring-order
// chunk schedule.  All arithmetic of the method runs in the kernels.
#include "../../include/pec_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <mutex>

#include "aux_kernels.hpp"
#include "common.hpp"
#include "decode_kernel.hpp"
#include "fwd_kernel.hpp"
#include "fwd_kernel_il.hpp"
#include "probes.hpp"

namespace {

using namespace pec;

// Compute units of the current device (cached per device id).
int compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}
// The pipelined kernel is persistent: one workgroup per compute unit (its registers allow no
// second one), each walking its share of the `grid` logical work items.
void launch_il(const FwdParams& p, unsigned grid, hipStream_t st) {
    const unsigned per_xcd = grid / 8;
    const unsigned slots = std::max(1u, std::min(per_xcd, (unsigned)compute_units() / 8));
    if (p.progress)
        hipLaunchKernelGGL(fwd_il_kernel<kFwdSweep>, dim3(8 * slots), dim3(512), 0, st, p);
    else if (p.cu_seqlens)
        hipLaunchKernelGGL(fwd_il_kernel<kFwdList>, dim3(8 * slots), dim3(512), 0, st, p);
    else
        hipLaunchKernelGGL(fwd_il_kernel<kFwdDense>, dim3(8 * slots), dim3(512), 0, st, p);
}

// Both kernels take 256 query rows per workgroup, so work lists and launch geometry do not depend
// on which one a call selects.
constexpr int kBM = 256;
static_assert(kSimpleBM == kBM, "the two kernels must agree on the query tile");

constexpr int64_t kMaxRows = (int64_t)1 << 30;

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_shape(const pec_shape_t* s, float* scale_out) {
    if (!s) return PEC_ERR_INVALID_ARGUMENT;
    if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->n_q_heads % s->n_kv_heads != 0) return PEC_ERR_INVALID_ARGUMENT;
    if (s->head_dim != kHeadDim) return PEC_ERR_UNSUPPORTED;
    if (s->out_dtype != PEC_BF16 && s->out_dtype != PEC_F32) return PEC_ERR_UNSUPPORTED;
    if (s->flags & ~(uint32_t)(PEC_FLAG_SIMPLE_KERNEL | PEC_FLAG_SP_SEPARATE_MERGE | PEC_FLAG_SP_STEP_LAUNCHES))
        return PEC_ERR_UNSUPPORTED;
    if ((s->flags & PEC_FLAG_SP_SEPARATE_MERGE) && (s->flags & PEC_FLAG_SP_STEP_LAUNCHES)) return PEC_ERR_INVALID_ARGUMENT;
    float scale = s->scale;
    if (scale == 0.f) scale = 1.0f / std::sqrt((float)s->head_dim);
    if (!(scale > 0.f) || !std::isfinite(scale)) return PEC_ERR_INVALID_ARGUMENT;
    if (scale_out) *scale_out = scale;
    return PEC_OK;
}

int launch_fwd(const FwdParams& p, bool simple, hipStream_t stream) {
    const int64_t total = (int64_t)p.n_items * p.n_q_heads;
    if (total <= 0) return PEC_OK;
    const int64_t per_xcd = (total + 7) / 8;
    const int64_t grid = per_xcd * 8;
    if (grid > 0x7fffffffLL) return PEC_ERR_UNSUPPORTED;
    if (simple)
        hipLaunchKernelGGL(fwd_simple_kernel, dim3((unsigned)grid), dim3(kSimpleWaves * 64), 0, stream, p);
    else
        launch_il(p, (unsigned)grid, stream);
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

// Common body of pec_attn_chunk / pec_attn_chunk_merge.
struct Sweep {   // resumable sweep: per-item progress table, count of unfinished items, stop word, tiles per segment
    float* l_part;
    int32_t* progress;
    int32_t* pending;
    const int32_t* stop;
    int32_t seg_tiles;
};

int chunk_impl(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sq, int64_t sk,
               int64_t q_off, int64_t kv_off, int causal, void* out, int out_f32, float* lse, const float* acc_in,
               const float* lse_in, float* acc_out, int64_t lse_stride, void* stream, const Sweep* sweep = nullptr) {
    float scale;
    if (int rc = check_shape(shape, &scale)) return rc;
    if (sq < 0 || sk < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (sq > kMaxRows || sk > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (sq == 0) return PEC_OK;
    if (!q || !lse || (!out && !acc_out) || (sk > 0 && (!k || !v))) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(acc_in) ||
        misaligned(acc_out) || (reinterpret_cast<uintptr_t>(lse) & 3u))
        return PEC_ERR_MISALIGNED;

    FwdParams p{};
    p.q = static_cast<const __bf16*>(q);
    p.k = static_cast<const __bf16*>(k);
    p.v = static_cast<const __bf16*>(v);
    p.out = out;
    p.lse = lse;
    p.acc_in = acc_in;
    p.lse_in = lse_in;
    p.acc_out = acc_out;
    p.lse_stride = lse_stride;
    p.sq = (int32_t)sq;
    p.sk = (int32_t)sk;
    // key j visible to row i  <=>  j <= i + (q_off - kv_off); beyond [-sq-1, sk] the value no longer matters
    const int64_t d = q_off - kv_off;
    p.delta = (int32_t)std::max<int64_t>(-sq - 1, std::min<int64_t>(d, sk));
    p.causal = causal ? 1 : 0;
    p.n_q_heads = shape->n_q_heads;
    p.n_kv_heads = shape->n_kv_heads;
    p.group = shape->n_q_heads / shape->n_kv_heads;
    p.n_items = (int32_t)((sq + kBM - 1) / kBM);
    p.out_f32 = out_f32;
    p.scale_log2 = scale * kLog2e;
    if (sweep) {
        p.l_part = sweep->l_part;
        p.progress = sweep->progress;
        p.pending = sweep->pending;
        p.stop = sweep->stop;
        p.seg_tiles = sweep->seg_tiles;
    }
    return launch_fwd(p, (shape->flags & PEC_FLAG_SIMPLE_KERNEL) != 0, static_cast<hipStream_t>(stream));
}

// Ring schedule of one member: step t brings segment (r - t) mod P with r = q_off / chunk (own
// segment first); under the causal mask segments wholly in the future of every local query are
// skipped.  Returns the number of visited segments; if `want` is in range, *lo / *len get the
// want-th visited segment.
int64_t ring_visit(int64_t s_q, int64_t q_off, int64_t s_kv, int64_t chunk, int causal, int64_t want, int64_t* lo,
                   int64_t* len) {
    if (s_kv <= 0) return 0;
    const int64_t n_chunks = (s_kv + chunk - 1) / chunk;
    const int64_t r = std::min(q_off / chunk, n_chunks - 1);
    int64_t visited = 0;
    for (int64_t t = 0; t < n_chunks; ++t) {
        const int64_t c = ((r - t) % n_chunks + n_chunks) % n_chunks;
        if (causal && c * chunk > q_off + s_q - 1) continue;
        if (visited == want) {
            *lo = c * chunk;
            *len = std::min(chunk, s_kv - c * chunk);
        }
        ++visited;
    }
    return visited;
}

int grid_for(int64_t n_groups) { return (int)std::min<int64_t>((n_groups + 255) / 256, 256 * 32); }

}  // namespace

extern "C" {

int pec_attn_chunk(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sq, int64_t sk,
                   int64_t q_off, int64_t kv_off, int causal, void* out, float* lse, void* stream) {
    if (sq > 0 && !out) return PEC_ERR_INVALID_ARGUMENT;
    return chunk_impl(shape, q, k, v, sq, sk, q_off, kv_off, causal, out, shape ? shape->out_dtype == PEC_F32 : 0, lse,
                      nullptr, nullptr, nullptr, sq, stream);
}

int pec_attn_chunk_merge(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sq, int64_t sk,
                         int64_t q_off, int64_t kv_off, int causal, float* o_acc, float* lse_acc, void* out_final,
                         void* stream) {
    if (sq > 0 && (!o_acc || !lse_acc)) return PEC_ERR_INVALID_ARGUMENT;
    return chunk_impl(shape, q, k, v, sq, sk, q_off, kv_off, causal, out_final,
                      shape ? shape->out_dtype == PEC_F32 : 0, lse_acc, o_acc, lse_acc, o_acc, sq, stream);
}

int pec_attn_merge(const pec_shape_t* shape, void* o_acc, float* lse_acc, const void* o_part, const float* lse_part,
                   int64_t sq, void* stream) {
    if (int rc = check_shape(shape, nullptr)) return rc;
    if (sq < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (sq > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (sq == 0) return PEC_OK;
    if (!o_acc || !lse_acc || !o_part || !lse_part) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(o_acc) || misaligned(o_part)) return PEC_ERR_MISALIGNED;
    const int64_t n_groups = sq * shape->n_q_heads * 32;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (shape->out_dtype == PEC_F32)
        hipLaunchKernelGGL((merge_kernel<true>), dim3(grid_for(n_groups)), dim3(256), 0, st, o_acc, lse_acc, o_part,
                           lse_part, sq, shape->n_q_heads);
    else
        hipLaunchKernelGGL((merge_kernel<false>), dim3(grid_for(n_groups)), dim3(256), 0, st, o_acc, lse_acc, o_part,
                           lse_part, sq, shape->n_q_heads);
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

int pec_finalize(const pec_shape_t* shape, const float* o_f32, void* o_bf16, int64_t sq, void* stream) {
    if (int rc = check_shape(shape, nullptr)) return rc;
    if (sq < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (sq > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (sq == 0) return PEC_OK;
    if (!o_f32 || !o_bf16) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(o_f32) || misaligned(o_bf16)) return PEC_ERR_MISALIGNED;
    const int64_t n_groups = sq * shape->n_q_heads * 32;
    hipLaunchKernelGGL(finalize_kernel, dim3(grid_for(n_groups)), dim3(256), 0, static_cast<hipStream_t>(stream), o_f32,
                       static_cast<__bf16*>(o_bf16), n_groups);
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

size_t pec_sp_workspace_bytes(const pec_shape_t* shape, int64_t s_q) {
    if (!shape || s_q <= 0 || shape->n_q_heads <= 0) return 0;
    // running fp32 O, one fp32 partial O, one partial LSE (the last two only with PEC_FLAG_SP_SEPARATE_MERGE)
    const size_t o = (size_t)s_q * shape->n_q_heads * kHeadDim * sizeof(float);
    const size_t l = (((size_t)s_q * shape->n_q_heads * sizeof(float)) + 255) & ~(size_t)255;
    return 2 * o + l;
}

int pec_sp_prefill(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t s_q, int64_t q_off,
                   int64_t s_kv, int64_t chunk, int causal, void* out, float* lse, void* workspace,
                   size_t workspace_bytes, void* stream) {
    float scale;
    if (int rc = check_shape(shape, &scale)) return rc;
    if (s_q < 0 || s_kv < 0 || chunk <= 0 || q_off < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (s_q > kMaxRows || s_kv > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (s_q == 0) return PEC_OK;
    if (!q || !out || !lse || (s_kv > 0 && (!k || !v))) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(out) || misaligned(workspace)) return PEC_ERR_MISALIGNED;
    const int out_f32 = shape->out_dtype == PEC_F32;
    const int64_t kv_row = (int64_t)shape->n_kv_heads * kHeadDim;  // elements per token
    const __bf16* kp = static_cast<const __bf16*>(k);
    const __bf16* vp = static_cast<const __bf16*>(v);

    if (!(shape->flags & (PEC_FLAG_SP_STEP_LAUNCHES | PEC_FLAG_SP_SEPARATE_MERGE)) || s_kv == 0)
        return chunk_impl(shape, q, k, v, s_q, s_kv, q_off, 0, causal, out, out_f32, lse, nullptr, nullptr, nullptr, s_q,
                          stream);

    int64_t lo = 0, len = 0;
    const int64_t n_steps = ring_visit(s_q, q_off, s_kv, chunk, causal, 0, &lo, &len);
    if (n_steps == 0)  // nothing visible at all: out = 0, lse = -inf
        return chunk_impl(shape, q, k, v, s_q, 0, q_off, 0, causal, out, out_f32, lse, nullptr, nullptr, nullptr, s_q,
                          stream);
    if (n_steps == 1)
        return chunk_impl(shape, q, kp + lo * kv_row, vp + lo * kv_row, s_q, len, q_off, lo, causal, out, out_f32, lse,
                          nullptr, nullptr, nullptr, s_q, stream);

    if (!workspace || workspace_bytes < pec_sp_workspace_bytes(shape, s_q)) return PEC_ERR_WORKSPACE;
    const size_t o_bytes = (size_t)s_q * shape->n_q_heads * kHeadDim * sizeof(float);
    float* o_acc = static_cast<float*>(workspace);

    if (!(shape->flags & PEC_FLAG_SP_SEPARATE_MERGE)) {
        for (int64_t t = 0; t < n_steps; ++t) {
            const int rc = pec_sp_prefill_step(shape, q, k, v, s_q, q_off, s_kv, chunk, causal, t, o_acc, lse,
                                               t == n_steps - 1 ? out : nullptr, stream);
            if (rc != PEC_OK) return rc;
        }
        return PEC_OK;
    }

    // PEC_FLAG_SP_SEPARATE_MERGE: fp32 partial of every step through HBM, stand-alone merge kernel
    float* o_part = reinterpret_cast<float*>(static_cast<char*>(workspace) + o_bytes);
    float* lse_part = reinterpret_cast<float*>(static_cast<char*>(workspace) + 2 * o_bytes);
    pec_shape_t part_shape = *shape;
    part_shape.out_dtype = PEC_F32;
    for (int64_t t = 0; t < n_steps; ++t) {
        ring_visit(s_q, q_off, s_kv, chunk, causal, t, &lo, &len);
        int rc;
        if (t == 0) {
            rc = chunk_impl(&part_shape, q, kp + lo * kv_row, vp + lo * kv_row, s_q, len, q_off, lo, causal, o_acc, 1,
                            lse, nullptr, nullptr, nullptr, s_q, stream);
        } else {
            rc = chunk_impl(&part_shape, q, kp + lo * kv_row, vp + lo * kv_row, s_q, len, q_off, lo, causal, o_part, 1,
                            lse_part, nullptr, nullptr, nullptr, s_q, stream);
            if (rc == PEC_OK) rc = pec_attn_merge(&part_shape, o_acc, lse, o_part, lse_part, s_q, stream);
        }
        if (rc != PEC_OK) return rc;
    }
    if (out_f32) {
        if (hipMemcpyAsync(out, o_acc, o_bytes, hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)) != hipSuccess)
            return PEC_ERR_HIP;
        return PEC_OK;
    }
    return pec_finalize(shape, o_acc, out, s_q, stream);
}

size_t pec_sp_resumable_workspace_bytes(const pec_shape_t* shape, int64_t s_q) {
    if (!shape || s_q <= 0 || shape->n_q_heads <= 0) return 0;
    // un-normalised fp32 O, two partial denominators per (head, row), progress table
    const size_t o = (size_t)s_q * shape->n_q_heads * kHeadDim * sizeof(float);
    const size_t l = (((size_t)s_q * shape->n_q_heads * 2 * sizeof(float)) + 255) & ~(size_t)255;
    const size_t items = (size_t)((s_q + kBM - 1) / kBM) * shape->n_q_heads;
    return o + l + ((items * sizeof(int32_t) + 255) & ~(size_t)255);
}

int pec_sp_prefill_resumable(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t s_q,
                             int64_t q_off, int64_t s_kv, int64_t chunk, int causal, void* out, float* lse,
                             void* workspace, size_t workspace_bytes, const int32_t* stop, int32_t* pending, int resume,
                             void* stream) {
    if (int rc = check_shape(shape, nullptr)) return rc;
    if (shape->flags & PEC_FLAG_SIMPLE_KERNEL) return PEC_ERR_UNSUPPORTED;   // the plain kernel keeps no progress
    if (s_q < 0 || s_kv < 0 || chunk <= 0 || q_off < 0 || !pending) return PEC_ERR_INVALID_ARGUMENT;
    if (s_q > kMaxRows || s_kv > kMaxRows || chunk % kBN != 0 || chunk / kBN > 0x3fffffff) return PEC_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(stop) & 3u) || (reinterpret_cast<uintptr_t>(pending) & 3u)) return PEC_ERR_MISALIGNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t items = ((s_q + kBM - 1) / kBM) * shape->n_q_heads;
    if (s_q > 0) {
        if (!q || !out || !lse || (s_kv > 0 && (!k || !v))) return PEC_ERR_INVALID_ARGUMENT;
        if (misaligned(out) || misaligned(workspace)) return PEC_ERR_MISALIGNED;
        if (!workspace || workspace_bytes < pec_sp_resumable_workspace_bytes(shape, s_q)) return PEC_ERR_WORKSPACE;
    }
    float* o_acc = static_cast<float*>(workspace);
    const size_t o_bytes = (size_t)s_q * shape->n_q_heads * kHeadDim * sizeof(float);
    const size_t l_bytes = (((size_t)s_q * shape->n_q_heads * 2 * sizeof(float)) + 255) & ~(size_t)255;
    float* l_part = s_q > 0 ? reinterpret_cast<float*>(static_cast<char*>(workspace) + o_bytes) : nullptr;
    int32_t* progress = s_q > 0 ? reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + o_bytes + l_bytes) : nullptr;
    if (!resume || s_q == 0) {
        hipLaunchKernelGGL(sweep_init_kernel, dim3((unsigned)std::max<int64_t>(1, std::min<int64_t>((items + 255) / 256, 1024))),
                           dim3(256), 0, st, progress, items, pending);
        if (hipGetLastError() != hipSuccess) return PEC_ERR_HIP;
    }
    if (s_q == 0) return PEC_OK;
    const Sweep sweep{l_part, progress, pending, stop, (int32_t)(chunk / kBN)};
    return chunk_impl(shape, q, k, v, s_q, s_kv, q_off, 0, causal, out, shape->out_dtype == PEC_F32, lse, o_acc, lse, o_acc,
                      s_q, stream, &sweep);
}

int64_t pec_sp_prefill_num_steps(const pec_shape_t* shape, int64_t s_q, int64_t q_off, int64_t s_kv, int64_t chunk,
                                 int causal) {
    if (int rc = check_shape(shape, nullptr)) return rc;
    if (s_q < 0 || s_kv < 0 || chunk <= 0 || q_off < 0) return PEC_ERR_INVALID_ARGUMENT;
    int64_t lo, len;
    return ring_visit(s_q, q_off, s_kv, chunk, causal, -1, &lo, &len);
}

int pec_sp_prefill_step(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t s_q,
                        int64_t q_off, int64_t s_kv, int64_t chunk, int causal, int64_t step, float* o_acc,
                        float* lse_acc, void* out_final, void* stream) {
    if (int rc = check_shape(shape, nullptr)) return rc;
    if (s_q < 0 || s_kv < 0 || chunk <= 0 || q_off < 0 || step < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (s_q > kMaxRows || s_kv > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (s_q == 0) return PEC_OK;
    if (!o_acc || !lse_acc) return PEC_ERR_INVALID_ARGUMENT;
    int64_t lo = 0, len = 0;
    const int64_t n_steps = ring_visit(s_q, q_off, s_kv, chunk, causal, step, &lo, &len);
    const int out_f32 = shape->out_dtype == PEC_F32;
    const int64_t kv_row = (int64_t)shape->n_kv_heads * kHeadDim;
    const __bf16* kp = static_cast<const __bf16*>(k) + lo * kv_row;
    const __bf16* vp = static_cast<const __bf16*>(v) + lo * kv_row;
    if (n_steps == 0 && step == 0) {  // nothing visible: the state (and the result) is the empty pair
        int rc = chunk_impl(shape, q, k, v, s_q, 0, q_off, 0, causal, o_acc, 1, lse_acc, nullptr, nullptr, nullptr, s_q,
                            stream);
        if (rc == PEC_OK && out_final)
            rc = chunk_impl(shape, q, k, v, s_q, 0, q_off, 0, causal, out_final, out_f32, lse_acc, nullptr, nullptr,
                            nullptr, s_q, stream);
        return rc;
    }
    if (step >= n_steps) return PEC_ERR_INVALID_ARGUMENT;
    const bool last = step == n_steps - 1;
    if (step == 0) {  // starts the running state; a one-step prefill may also emit the final output
        int rc = chunk_impl(shape, q, kp, vp, s_q, len, q_off, lo, causal, o_acc, 1, lse_acc, nullptr, nullptr, nullptr,
                            s_q, stream);
        if (rc == PEC_OK && last && out_final) {
            if (out_f32) {
                const size_t o_bytes = (size_t)s_q * shape->n_q_heads * kHeadDim * sizeof(float);
                if (hipMemcpyAsync(out_final, o_acc, o_bytes, hipMemcpyDeviceToDevice,
                                   static_cast<hipStream_t>(stream)) != hipSuccess)
                    rc = PEC_ERR_HIP;
            } else {
                rc = pec_finalize(shape, o_acc, out_final, s_q, stream);
            }
        }
        return rc;
    }
    // later steps fold the segment into the running state; on the last one the merged result can go
    // straight to out_final, and the fp32 state, no longer needed, is then left as it was
    float* acc_out = (last && out_final) ? nullptr : o_acc;
    return chunk_impl(shape, q, kp, vp, s_q, len, q_off, lo, causal, out_final, out_f32, lse_acc, o_acc, lse_acc, acc_out,
                      s_q, stream);
}

int32_t pec_decode_default_splits(const pec_shape_t* shape, int64_t sk) {
    if (!shape || shape->n_kv_heads <= 0 || sk <= 0) return 1;
    const int g = shape->n_q_heads / shape->n_kv_heads;
    const int64_t per_cu = std::max<int64_t>(1, compute_units() / shape->n_kv_heads);
    if (g <= 32) {   // one workgroup (four KV heads of one range) per compute unit, at least 8 tiles of 32 keys each
        const int64_t head_groups = (shape->n_kv_heads + kDecWaves - 1) / kDecWaves;
        return (int32_t)std::max<int64_t>(1, std::min<int64_t>(compute_units() / head_groups, sk / 256));
    }
    // wide groups run on the prefill kernel: one workgroup per compute unit, at least 16 tiles of 64 keys each
    return (int32_t)std::max<int64_t>(1, std::min<int64_t>(per_cu, sk / 1024));
}

size_t pec_decode_workspace_bytes(const pec_shape_t* shape, int32_t n_splits) {
    if (!shape || shape->n_q_heads <= 0 || n_splits <= 0) return 0;
    return (size_t)n_splits * shape->n_q_heads * (kHeadDim + 1) * sizeof(float);
}

}  // extern "C"

namespace {

// Scratch of pec_decode_splitkv_static: the fp32 partial (O, LSE) of every (key range, query head).
// One copy per GPU, held until the process ends; its device address is looked up once per device.
constexpr size_t kStaticScratchBytes = PEC_DECODE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch(void** out) {
    static void* ptr[64] = {nullptr};
    static std::mutex lock;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PEC_ERR_HIP;
    std::lock_guard<std::mutex> guard(lock);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PEC_ERR_HIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return PEC_OK;
}

// Common body of the two decode entry points; `workspace` holds pec_decode_workspace_bytes(shape, n_splits) bytes.
int decode_impl(const pec_shape_t* shape, float scale, const void* q, const void* k, const void* v, int64_t sk,
                int32_t n_splits, void* out, float* lse, void* workspace, void* stream) {
    const int g = shape->n_q_heads / shape->n_kv_heads;
    float* o_part = static_cast<float*>(workspace);
    float* lse_part = o_part + (size_t)n_splits * shape->n_q_heads * kHeadDim;
    hipStream_t st = static_cast<hipStream_t>(stream);

    if (g <= 32) {   // one key range per wavefront (decode_kernel.hpp)
        DecodeParams d{};
        d.q = static_cast<const __bf16*>(q);
        d.k = static_cast<const unsigned char*>(k);
        d.v = static_cast<const unsigned char*>(v);
        d.o_part = o_part;
        d.lse_part = lse_part;
        d.sk = (int32_t)sk;
        d.n_q_heads = shape->n_q_heads;
        d.n_kv_heads = shape->n_kv_heads;
        d.group = g;
        d.n_ranges = n_splits;
        const int64_t per = ((sk + n_splits - 1) / n_splits + kDecTile - 1) / kDecTile * kDecTile;
        d.range_len = (int32_t)std::max<int64_t>(per, kDecTile);
        d.scale_log2 = scale * kLog2e;
        const int64_t blocks = (int64_t)n_splits * ((shape->n_kv_heads + kDecWaves - 1) / kDecWaves);
        const int64_t grid = ((blocks + 7) / 8) * 8;
        if (grid > 0x7fffffffLL) return PEC_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(decode_kernel, dim3((unsigned)grid), dim3(kDecWaves * 64), 0, st, d);
        if (hipGetLastError() != hipSuccess) return PEC_ERR_HIP;
    } else {
    // The g query heads of one KV head become the g rows of one query tile: row stride 128, "head"
    // (= KV head) stride g*128; the work items are the key ranges.
    FwdParams p{};
    p.q = static_cast<const __bf16*>(q);
    p.k = static_cast<const __bf16*>(k);
    p.v = static_cast<const __bf16*>(v);
    p.out = o_part;
    p.lse = lse_part;
    p.lse_stride = g;
    p.sq = g;
    p.sk = (int32_t)sk;
    p.delta = (int32_t)sk;
    p.causal = 0;
    p.n_q_heads = shape->n_kv_heads;
    p.n_kv_heads = shape->n_kv_heads;
    p.group = 1;
    p.n_items = n_splits;
    p.out_f32 = 1;
    p.scale_log2 = scale * kLog2e;
    const int64_t split_len = ((sk + n_splits - 1) / n_splits + kBN - 1) / kBN * kBN;   // whole tiles
    p.kv_split_len = (int32_t)std::max<int64_t>(split_len, kBN);
    p.split_out_stride = (int64_t)shape->n_q_heads * kHeadDim;
    p.split_lse_stride = shape->n_q_heads;
    p.q_row_stride = kHeadDim;
    p.q_head_stride = (int64_t)g * kHeadDim;
    const int64_t total = (int64_t)n_splits * shape->n_kv_heads;
    launch_il(p, (unsigned)(((total + 7) / 8) * 8), st);
    if (hipGetLastError() != hipSuccess) return PEC_ERR_HIP;
    }
    if (shape->out_dtype == PEC_F32)
        hipLaunchKernelGGL((combine_splits_kernel<true>), dim3(shape->n_q_heads), dim3(kCombineGroups * 128), 0, st, o_part, lse_part,
                           (int)n_splits, (int)shape->n_q_heads, out, lse);
    else
        hipLaunchKernelGGL((combine_splits_kernel<false>), dim3(shape->n_q_heads), dim3(kCombineGroups * 128), 0, st, o_part, lse_part,
                           (int)n_splits, (int)shape->n_q_heads, out, lse);
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

}  // namespace

extern "C" {

int pec_decode_splitkv(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sk,
                       int32_t n_splits, void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    float scale;
    if (int rc = check_shape(shape, &scale)) return rc;
    if (sk < 0 || n_splits < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (sk > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (!q || !out || !lse || (sk > 0 && (!k || !v))) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(workspace))
        return PEC_ERR_MISALIGNED;
    if (n_splits == 0) n_splits = pec_decode_default_splits(shape, sk);
    if (shape->n_q_heads / shape->n_kv_heads > 256) return PEC_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < pec_decode_workspace_bytes(shape, n_splits)) return PEC_ERR_WORKSPACE;
    return decode_impl(shape, scale, q, k, v, sk, n_splits, out, lse, workspace, stream);
}

int pec_decode_splitkv_static(const pec_shape_t* shape, const void* q, const void* k, const void* v, int64_t sk,
                              int32_t n_splits, void* out, float* lse, void* stream) {
    float scale;
    if (int rc = check_shape(shape, &scale)) return rc;
    if (sk < 0 || n_splits < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (sk > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (!q || !out || !lse || (sk > 0 && (!k || !v))) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out)) return PEC_ERR_MISALIGNED;
    if (n_splits == 0) n_splits = pec_decode_default_splits(shape, sk);
    if (shape->n_q_heads / shape->n_kv_heads > 256) return PEC_ERR_UNSUPPORTED;
    if (pec_decode_workspace_bytes(shape, n_splits) > kStaticScratchBytes) return PEC_ERR_SCRATCH_LIMIT;
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return decode_impl(shape, scale, q, k, v, sk, n_splits, out, lse, ws, stream);
}

int pec_ulysses_layout(const void* src, void* dst, int64_t s, int32_t n_heads, int32_t head_dim, int32_t n_gpus,
                       int to_messages, void* stream) {
    if (s < 0 || n_heads <= 0 || n_gpus <= 0 || n_heads % n_gpus != 0) return PEC_ERR_INVALID_ARGUMENT;
    if (head_dim != kHeadDim) return PEC_ERR_UNSUPPORTED;
    if (s > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (s == 0) return PEC_OK;
    if (!src || !dst || src == dst) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(src) || misaligned(dst)) return PEC_ERR_MISALIGNED;
    const int64_t total = s * n_heads * 16;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (to_messages)
        hipLaunchKernelGGL((ulysses_layout_kernel<true>), dim3(grid_for(total)), dim3(256), 0, st,
                           static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), s, (int)n_heads, (int)n_gpus);
    else
        hipLaunchKernelGGL((ulysses_layout_kernel<false>), dim3(grid_for(total)), dim3(256), 0, st,
                           static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), s, (int)n_heads, (int)n_gpus);
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

int pec_sp_select_strategy(const pec_sp_model_t* m, pec_sp_choice_t* c) {
    if (!m || !c) return PEC_ERR_INVALID_ARGUMENT;
    if (m->d_model <= 0 || m->n_heads <= 0 || m->n_kv_heads <= 0 || m->head_dim <= 0 || m->seg_len <= 0 ||
        m->tp <= 0 || m->gpus_per_node <= 0 || !(m->bytes_per_element > 0) || !(m->node_bandwidth > 0) ||
        !(m->gpu_flops > 0))
        return PEC_ERR_INVALID_ARGUMENT;
    const double d = (double)m->d_model, s = (double)m->seg_len, T = m->tp, G = m->gpus_per_node;
    const double qkv = ((double)m->n_heads + m->n_kv_heads) * m->head_dim;   // (N_h + N_h^KV) d_h
    // attention stage
    c->attn_comm[0] = 2 * s * d * (T - 1) * G;                                           // all-gather + reduce-scatter
    c->attn_compute[0] = 2 * s * d * qkv / T + 4 * (s * T) * (s * T) * d / T + 2 * s * d * d;
    c->attn_comm[1] = 2 * s * qkv * (G - 1) + (d * qkv + d * d) * G * (T - 1) / T;       // two all-to-alls + parameters
    c->attn_compute[1] = 2 * s * d * qkv + 4 * (s * G) * (s * G) * d / G + 2 * s * d * d;
    // MLP stage
    c->mlp_comm[0] = 2 * s * d * (T - 1) * G;
    c->mlp_compute[0] = 16 * s * d * d;
    c->mlp_comm[1] = 8 * d * d * (T - 1) * G / T;
    c->mlp_compute[1] = 16 * s * d * d;
    double best = 0;
    c->best_attn = c->best_mlp = 0;
    for (int a = 0; a < 2; ++a)
        for (int l = 0; l < 2; ++l) {
            const double t = (c->attn_comm[a] + c->mlp_comm[l]) * m->bytes_per_element / m->node_bandwidth +
                             (c->attn_compute[a] + c->mlp_compute[l]) / m->gpu_flops;
            c->seconds[a][l] = t;
            if ((a == 0 && l == 0) || t < best) {
                best = t;
                c->best_attn = a;
                c->best_mlp = l;
            }
        }
    return PEC_OK;
}

size_t pec_varlen_workspace_bytes(int32_t batch, int64_t total_tokens) {
    if (batch < 0 || total_tokens < 0) return 0;
    // every sequence contributes at most len / 256 + 1 items
    const size_t cap = (size_t)(total_tokens / kBM) + (size_t)batch + 1;
    // work list + counter (padded) + two int32 arrays indexed by query-tile number
    return cap * sizeof(WorkItem) + 256 + (2 * cap + 1) * sizeof(int32_t);
}

int pec_attn_varlen(const pec_shape_t* shape, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                    int32_t batch, int64_t total_tokens, int32_t max_seqlen, int causal, void* out, float* lse,
                    void* workspace, size_t workspace_bytes, void* stream) {
    float scale;
    if (int rc = check_shape(shape, &scale)) return rc;
    if (batch < 0 || total_tokens < 0 || max_seqlen < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (total_tokens > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (batch == 0 || total_tokens == 0) return PEC_OK;
    if (!q || !k || !v || !out || !lse || !cu_seqlens) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(workspace) ||
        (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u))
        return PEC_ERR_MISALIGNED;
    if (!workspace || workspace_bytes < pec_varlen_workspace_bytes(batch, total_tokens)) return PEC_ERR_WORKSPACE;
    (void)max_seqlen;   // a hint only: the work list is sized from total_tokens, so an understated value costs nothing

    const size_t cap = (size_t)(total_tokens / kBM) + (size_t)batch + 1;
    const int capacity = (int)std::min<size_t>(cap, 0x7fffffff);
    char* ws = static_cast<char*>(workspace);
    WorkItem* work = reinterpret_cast<WorkItem*>(ws);
    int32_t* n_work = reinterpret_cast<int32_t*>(ws + cap * sizeof(WorkItem));
    int32_t* bucket = reinterpret_cast<int32_t*>(ws + cap * sizeof(WorkItem) + 256);
    int32_t* cursor = bucket + cap + 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(build_worklist_kernel, dim3(1), dim3(1024), 0, st, cu_seqlens, (int)batch, (int)total_tokens, kBM,
                       capacity, work, n_work, bucket, cursor);
    if (hipGetLastError() != hipSuccess) return PEC_ERR_HIP;

    FwdParams p{};
    p.q = static_cast<const __bf16*>(q);
    p.k = static_cast<const __bf16*>(k);
    p.v = static_cast<const __bf16*>(v);
    p.out = out;
    p.lse = lse;
    p.lse_stride = total_tokens;
    p.causal = causal ? 1 : 0;
    p.n_q_heads = shape->n_q_heads;
    p.n_kv_heads = shape->n_kv_heads;
    p.group = shape->n_q_heads / shape->n_kv_heads;
    p.n_items = capacity;
    p.out_f32 = shape->out_dtype == PEC_F32;
    p.scale_log2 = scale * kLog2e;
    p.cu_seqlens = cu_seqlens;
    p.work = work;
    p.n_work = n_work;
    p.sched = n_work + 8;   // same 256-byte block, zeroed by the builder
    p.total_tokens = (int32_t)total_tokens;
    return launch_fwd(p, (shape->flags & PEC_FLAG_SIMPLE_KERNEL) != 0, st);
}

namespace {
constexpr int kColocRange = 4096;   // keys per range of a split one-token sequence (64 tiles)
struct ColocLayout {
    size_t cap_items, n_buckets, slot_cap;
    size_t off_counters, off_bucket, off_cursor, off_slot0, off_split, off_part_lse, off_part_out, bytes;
};
ColocLayout coloc_layout(int n_q_heads, int32_t batch, int64_t total_q, int64_t total_k) {
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    ColocLayout L;
    L.slot_cap = (size_t)(total_k / kColocRange) + (size_t)batch;
    L.cap_items = (size_t)(total_q / kBM) + (size_t)batch + L.slot_cap + 1;
    L.n_buckets = (size_t)(total_k / 256) + 2;
    size_t o = up(L.cap_items * sizeof(WorkItem));
    L.off_counters = o;  o += 256;
    L.off_bucket = o;    o = up(o + (L.n_buckets + 1) * sizeof(int32_t));
    L.off_cursor = o;    o = up(o + L.n_buckets * sizeof(int32_t));
    L.off_slot0 = o;     o = up(o + (size_t)batch * sizeof(int32_t));
    L.off_split = o;     o = up(o + (size_t)batch * sizeof(SplitSeq));
    L.off_part_lse = o;  o = up(o + L.slot_cap * n_q_heads * sizeof(float));
    L.off_part_out = o;  o = up(o + L.slot_cap * n_q_heads * kHeadDim * sizeof(float));
    L.bytes = o;
    return L;
}
}  // namespace

size_t pec_colocated_workspace_bytes(const pec_shape_t* shape, int32_t batch, int64_t total_q, int64_t total_k) {
    if (!shape || shape->n_q_heads <= 0 || batch < 0 || total_q < 0 || total_k < 0) return 0;
    return coloc_layout(shape->n_q_heads, batch, total_q, total_k).bytes;
}

int pec_attn_colocated(const pec_shape_t* shape, const void* q, const void* k, const void* v,
                       const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int32_t batch, int64_t total_q,
                       int64_t total_k, int causal, void* out, float* lse, void* workspace, size_t workspace_bytes,
                       void* stream) {
    float scale;
    if (int rc = check_shape(shape, &scale)) return rc;
    if (shape->flags & PEC_FLAG_SIMPLE_KERNEL) return PEC_ERR_UNSUPPORTED;   // the plain kernel knows no key ranges
    if (shape->n_q_heads / shape->n_kv_heads > 256) return PEC_ERR_UNSUPPORTED;   // a KV group's heads are the rows of one query tile
    if (batch < 0 || total_q < 0 || total_k < 0) return PEC_ERR_INVALID_ARGUMENT;
    if (total_q > kMaxRows || total_k > kMaxRows) return PEC_ERR_UNSUPPORTED;
    if (batch == 0 || total_q == 0) return PEC_OK;
    if (!q || !out || !lse || !cu_seqlens_q || !cu_seqlens_k || (total_k > 0 && (!k || !v))) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(workspace) ||
        (reinterpret_cast<uintptr_t>(cu_seqlens_q) & 3u) || (reinterpret_cast<uintptr_t>(cu_seqlens_k) & 3u))
        return PEC_ERR_MISALIGNED;
    const ColocLayout L = coloc_layout(shape->n_q_heads, batch, total_q, total_k);
    if (!workspace || workspace_bytes < L.bytes) return PEC_ERR_WORKSPACE;
    if (L.cap_items > 0x7fffffff || L.n_buckets > 0x7fffffff) return PEC_ERR_UNSUPPORTED;

    char* ws = static_cast<char*>(workspace);
    WorkItem* work = reinterpret_cast<WorkItem*>(ws);
    int32_t* counters = reinterpret_cast<int32_t*>(ws + L.off_counters);
    int32_t* seq_slot0 = reinterpret_cast<int32_t*>(ws + L.off_slot0);
    SplitSeq* split_seqs = reinterpret_cast<SplitSeq*>(ws + L.off_split);
    float* part_lse = reinterpret_cast<float*>(ws + L.off_part_lse);
    float* part_out = reinterpret_cast<float*>(ws + L.off_part_out);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(build_colocated_worklist_kernel, dim3(1), dim3(1024), 0, st, cu_seqlens_q, cu_seqlens_k, (int)batch,
                       (int)total_q, (int)total_k, kBM, kColocRange, (int)L.cap_items, (int)L.slot_cap, (int)L.n_buckets,
                       work, counters, reinterpret_cast<int32_t*>(ws + L.off_bucket),
                       reinterpret_cast<int32_t*>(ws + L.off_cursor), seq_slot0, split_seqs);
    if (hipGetLastError() != hipSuccess) return PEC_ERR_HIP;

    FwdParams p{};
    p.q = static_cast<const __bf16*>(q);
    p.k = static_cast<const __bf16*>(k);
    p.v = static_cast<const __bf16*>(v);
    p.out = out;
    p.lse = lse;
    p.lse_stride = total_q;
    p.causal = causal ? 1 : 0;
    p.n_q_heads = shape->n_q_heads;
    p.n_kv_heads = shape->n_kv_heads;
    p.group = shape->n_q_heads / shape->n_kv_heads;
    p.n_items = (int32_t)L.cap_items;
    p.out_f32 = shape->out_dtype == PEC_F32;
    p.scale_log2 = scale * kLog2e;
    p.cu_seqlens = cu_seqlens_q;
    p.work = work;
    p.n_work = counters;
    p.sched = counters + 8;   // same 256-byte block, zeroed by the builder
    p.total_tokens = (int32_t)total_q;
    p.cu_seqlens_k = cu_seqlens_k;
    p.seq_slot0 = seq_slot0;
    p.part_out = part_out;
    p.part_lse = part_lse;
    p.total_k = (int32_t)total_k;
    p.coloc_range_len = kColocRange;
    if (int rc = launch_fwd(p, false, st)) return rc;

    const dim3 grid((unsigned)shape->n_q_heads, (unsigned)std::min<int32_t>(batch, 1024));
    if (shape->out_dtype == PEC_F32)
        hipLaunchKernelGGL((combine_colocated_kernel<true>), grid, dim3(kCombineGroups * 128), 0, st, part_out, part_lse,
                           split_seqs, counters + 2, cu_seqlens_q, (int)total_q, (int)shape->n_q_heads, out, lse);
    else
        hipLaunchKernelGGL((combine_colocated_kernel<false>), grid, dim3(kCombineGroups * 128), 0, st, part_out, part_lse,
                           split_seqs, counters + 2, cu_seqlens_q, (int)total_q, (int)shape->n_q_heads, out, lse);
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

int64_t pec_mfma_probe(const void* operands, size_t operand_bytes, int32_t iters, float* sink, size_t sink_floats,
                       void* stream) {
    const size_t need = (size_t)kProbeFrags * 2 * 64 * 16;
    if (!operands || !sink || iters <= 0) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(operands) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return PEC_ERR_MISALIGNED;
    const int grid = compute_units();
    if (operand_bytes < need || sink_floats < (size_t)grid * kProbeWaves * 64) return PEC_ERR_WORKSPACE;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(grid), dim3(kProbeWaves * 64), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(operands), (int)iters, sink);
    if (hipGetLastError() != hipSuccess) return PEC_ERR_HIP;
    // flop of the launch: every MFMA is 32 x 32 x 16 multiply-adds
    return (int64_t)grid * kProbeWaves * iters * kProbeMfmaPerIter * (2LL * 32 * 32 * 16);
}

int pec_hbm_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes < 16) return PEC_ERR_INVALID_ARGUMENT;
    if (misaligned(src) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return PEC_ERR_MISALIGNED;
    hipLaunchKernelGGL(hbm_read_probe_kernel, dim3(compute_units() * 32), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? PEC_OK : PEC_ERR_HIP;
}

const char* pec_status_string(int status) {
    switch (status) {
        case PEC_OK:
            return "ok";
        case PEC_ERR_INVALID_ARGUMENT:
            return "invalid argument";
        case PEC_ERR_UNSUPPORTED:
            return "unsupported configuration";
        case PEC_ERR_MISALIGNED:
            return "pointer not 16-byte aligned";
        case PEC_ERR_WORKSPACE:
            return "workspace missing or too small";
        case PEC_ERR_HIP:
            return "HIP runtime error";
        case PEC_ERR_SCRATCH_LIMIT:
            return "problem needs more than the library's static scratch buffer";
        default:
            return "unknown status";
    }
}

}  // extern "C"
