"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle.

Tolerances (from the task definition): max-abs 2e-2 on bf16 outputs,
|dLSE| <= 1e-3 * max(1, |LSE|) on fp32 LSE, -inf exactly where no key is visible;
mask / offset / cu_seqlens indexing is checked bit-exactly through closed forms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import reference as oracle
from paper_2409_15104_amd import binding as pec
from paper_2409_15104_amd import synth

pytestmark = pytest.mark.gpu

O_ATOL = 2e-2
LSE_RTOL = 1e-3
DEV = "cuda:0"
# per-call kernel selection: the default pipelined kernel and the plain cross-check kernel
KERNELS = [0, pec.PEC_FLAG_SIMPLE_KERNEL]
# pec_sp_prefill: the default single sweep, and the two modes that launch once per ring step
SP_MODES = [0, pec.PEC_FLAG_SP_SEPARATE_MERGE, pec.PEC_FLAG_SP_STEP_LAUNCHES]


@pytest.fixture(autouse=True)
def _sync_after():
    yield
    torch.cuda.synchronize()


def assert_close(out, lse, o_ref, l_ref, what=""):
    o = out.float().cpu().numpy().astype(np.float64)
    l = lse.float().cpu().numpy().astype(np.float64)
    assert not np.isnan(o).any() and not np.isnan(l).any(), what
    err = np.abs(o - o_ref).max() if o.size else 0.0
    assert err <= O_ATOL, "%s: max-abs O error %.4g" % (what, err)
    fin = np.isfinite(l_ref)
    assert np.array_equal(np.isfinite(l), fin), what + ": -inf pattern of LSE differs"
    assert np.all(l[~fin] == -np.inf)
    if fin.any():
        rel = (np.abs(l[fin] - l_ref[fin]) / np.maximum(1.0, np.abs(l_ref[fin]))).max()
        assert rel <= LSE_RTOL, "%s: LSE error %.4g" % (what, rel)
    # rows without a visible key are exactly zero
    assert np.all(o[np.transpose(~fin)] == 0.0), what


def gpu(*ts):
    return [t.to(DEV) for t in ts]


CHUNK_CASES = [
    # sq, sk, hq, hkv, q_off, kv_off, causal
    (300, 333, 4, 2, 33, 0, True),      # ragged both ways, several tiles, all rows see something
    (257, 130, 2, 1, 0, 0, True),       # one row into the second query tile
    (64, 64, 2, 2, 0, 0, True),         # exactly one tile
    (520, 200, 4, 1, 0, 100, True),     # first 100 rows see nothing of this segment
    (96, 128, 2, 2, 0, 1000, True),     # segment wholly in the future
    (200, 450, 8, 2, 5000, 0, True),    # segment wholly in the past: no masking
    (130, 77, 4, 4, 0, 0, False),       # non-causal
    (1, 1, 2, 1, 0, 0, True),
    (1, 700, 8, 8, 699, 0, True),       # a decode-like single row
    (40, 0, 2, 2, 0, 0, True),          # no keys at all
]


@pytest.mark.parametrize("variant", KERNELS)
@pytest.mark.parametrize("case", CHUNK_CASES)
def test_chunk_matches_oracle(case, variant):
    sq, sk, hq, hkv, q_off, kv_off, causal = case
    q, k, v = synth.qkv(7 + sq + sk, sq, sk, hq, hkv)
    o_ref, l_ref = oracle.attention(q, k, v, q_off=q_off, kv_off=kv_off, causal=causal)
    for out_dtype in (torch.bfloat16, torch.float32):
        out, lse = pec.pec_attn_chunk(*gpu(q, k, v), q_off, kv_off, causal, out_dtype=out_dtype, flags=variant)
        assert_close(out, lse, o_ref, l_ref, "chunk %s v%d %s" % (case, variant, out_dtype))


@pytest.mark.parametrize("variant", KERNELS)
@pytest.mark.parametrize("q_off", [0, 4096])
def test_late_jumps_of_the_row_maximum(q_off, variant):
    # keys that lift single rows' scores 16 ... 130 log2 units above the bulk, placed in tiles after the
    # first one, in masked (diagonal) and unmasked tiles: the kernels' softmax reference has to follow
    s = 1024
    outliers = [(70, 950, 1), (300, 400, 2), (301, 1000, 4), (640, 700, 8), (900, 901, 8), (999, 1023, 2),
                (130, 5, 4), (515, 33, 1)]   # the last two are invisible under the causal mask when q_off = 0
    q, k, v = synth.qkv_with_outlier_keys(4242, s, s, 8, 2, outliers)
    o_ref, l_ref = oracle.attention(q, k, v, q_off=q_off, kv_off=0, causal=True)
    out, lse = pec.pec_attn_chunk(*gpu(q, k, v), q_off, 0, True, out_dtype=torch.float32, flags=variant)
    assert_close(out, lse, o_ref, l_ref, "outlier keys q_off %d v%d" % (q_off, variant))
    # and continued from a first half computed separately (fused merge across the jump)
    h = s // 2
    o1, l1 = pec.pec_attn_chunk(*gpu(q, k[:h].contiguous(), v[:h].contiguous()), q_off, 0, True, out_dtype=torch.float32,
                                flags=variant)
    o2, l2 = pec.pec_attn_chunk_merge(*gpu(q, k[h:].contiguous(), v[h:].contiguous()), q_off, h, o1, l1, True,
                                      flags=variant)
    assert_close(o2, l2, o_ref, l_ref, "outlier keys, two segments, q_off %d v%d" % (q_off, variant))


def test_late_jumps_in_a_packed_batch_and_without_a_mask():
    # the same outlier keys inside one sequence of a packed batch, and in a non-causal call whose last
    # tile is ragged
    lengths = [200, 1024, 77]
    cu = synth.cu_seqlens_of(lengths)
    t = int(cu[-1])
    lo = int(cu[1])
    outliers = [(lo + 70, lo + 950, 2), (lo + 640, lo + 700, 8), (lo + 900, lo + 901, 4), (10, 150, 8)]
    q, k, v = synth.qkv_with_outlier_keys(4343, t, t, 8, 2, outliers)
    o_ref, l_ref = oracle.varlen(q, k, v, cu)
    out, lse = pec.pec_attn_varlen(*gpu(q, k, v), torch.from_numpy(cu).to(DEV), max(lengths), True,
                                   out_dtype=torch.float32)
    assert_close(out, lse, o_ref, l_ref, "outlier keys, packed batch")
    q, k, v = synth.qkv_with_outlier_keys(4344, 300, 1000, 4, 4, [(500, 17, 8), (998, 250, 2), (999, 299, 8)])
    o_ref, l_ref = oracle.attention(q, k, v, causal=False)
    out, lse = pec.pec_attn_chunk(*gpu(q, k, v), 0, 0, False, out_dtype=torch.float32)
    assert_close(out, lse, o_ref, l_ref, "outlier keys, non-causal")


def test_chunk_empty_query_is_a_noop():
    q, k, v = synth.qkv(3, 0, 16, 2, 2)
    out, lse = pec.pec_attn_chunk(*gpu(q, k, v), 0, 0)
    assert out.shape == (0, 2, 128) and lse.shape == (2, 0)


@pytest.mark.parametrize("variant", KERNELS)
@pytest.mark.parametrize("q_off,kv_off,sq,sk", [(0, 0, 600, 600), (1000, 937, 333, 700), (5, 200, 300, 90),
                                               (0, 64, 256, 256), (255, 0, 258, 515)])
def test_mask_is_bit_exact_via_zero_query(q_off, kv_off, sq, sk, variant):
    """Q = 0 gives LSE_i = ln n_i with n_i the visible-key count; a one-hot V column gives
    exactly 1/n_i or exactly 0: any off-by-one in mask or offsets shows."""
    hq, hkv = 4, 2
    _, k, _ = synth.qkv(11, sq, sk, hq, hkv)
    q = torch.zeros(sq, hq, 128, dtype=torch.bfloat16)
    jstar = sk // 2
    v = torch.zeros(sk, hkv, 128, dtype=torch.bfloat16)
    v[jstar] = 1.0
    out, lse = pec.pec_attn_chunk(*gpu(q, k, v), q_off, kv_off, True, out_dtype=torch.float32, flags=variant)
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    n = np.clip(q_off + np.arange(sq) - kv_off + 1, 0, sk)
    vis = n > 0
    assert np.all(lse[:, ~vis] == -np.inf)
    assert np.array_equal(np.rint(np.exp(lse[:, vis].astype(np.float64))).astype(np.int64),
                          np.tile(n[vis], (hq, 1)))
    sees = n > jstar
    assert np.all(out[~sees] == 0.0)
    np.testing.assert_allclose(out[sees], np.broadcast_to((1.0 / n[sees])[:, None, None], out[sees].shape),
                               rtol=2e-3, atol=0)


def test_row_zero_returns_first_value_exactly():
    q, k, v = synth.qkv(13, 70, 70, 4, 2)
    out, lse = pec.pec_attn_chunk(*gpu(q, k, v), 0, 0, True)
    assert torch.equal(out[0].cpu(), v[0].repeat_interleave(2, dim=0))
    ref = (q[0].double() * k[0].repeat_interleave(2, dim=0).double()).sum(-1) / math.sqrt(128.0)
    np.testing.assert_allclose(lse[:, 0].cpu().numpy(), ref.numpy(), rtol=1e-3, atol=1e-3)


def test_constant_value_is_reproduced():
    q, k, _ = synth.qkv(14, 300, 300, 4, 4)
    v = torch.full((300, 4, 128), -2.5, dtype=torch.bfloat16)
    out, _ = pec.pec_attn_chunk(*gpu(q, k, v), 0, 0, True, out_dtype=torch.float32)
    np.testing.assert_allclose(out.cpu().numpy(), -2.5, rtol=0, atol=2e-2)


def test_gqa_is_bit_identical_to_mha_with_repeated_kv():
    q, k, v = synth.qkv(15, 300, 400, 8, 2)
    o_g, l_g = pec.pec_attn_chunk(*gpu(q, k, v), 150, 0, True)
    kr, vr = k.repeat_interleave(4, dim=1).contiguous(), v.repeat_interleave(4, dim=1).contiguous()
    o_m, l_m = pec.pec_attn_chunk(*gpu(q, kr, vr), 150, 0, True)
    assert torch.equal(o_g, o_m) and torch.equal(l_g, l_m)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_merge_matches_oracle_and_identity_is_exact(dtype):
    sq, hq = 333, 4
    g = torch.Generator().manual_seed(16)
    o_a = torch.randn(sq, hq, 128, generator=g).to(dtype)
    o_b = torch.randn(sq, hq, 128, generator=g).to(dtype)
    l_a = torch.randn(hq, sq, generator=g) * 3
    l_b = torch.randn(hq, sq, generator=g) * 3
    l_a[0, :7] = -math.inf          # rows known only to B
    l_b[1, 5:9] = -math.inf         # rows known only to A
    l_a[2, 100], l_b[2, 100] = -math.inf, -math.inf
    o_a[:7, 0] = 0
    o_b[5:9, 1] = 0
    o_a[100, 2] = 0
    o_b[100, 2] = 0
    o_ref, l_ref = oracle.merge(o_a.double().numpy(), l_a.double().numpy(), o_b.double().numpy(),
                                l_b.double().numpy())
    o, lse = pec.pec_attn_merge(o_a.to(DEV).clone(), l_a.to(DEV).clone(), o_b.to(DEV), l_b.to(DEV))
    assert_close(o, lse, o_ref, l_ref, "merge %s" % dtype)
    # (0, -inf) is the identity, bit for bit, on either side
    zero = torch.zeros_like(o_a).to(DEV)
    ninf = torch.full_like(l_a, -math.inf).to(DEV)
    o, lse = pec.pec_attn_merge(o_b.to(DEV).clone(), l_b.to(DEV).clone(), zero, ninf)
    keep = torch.isfinite(l_b)
    assert torch.equal(lse.cpu(), l_b)
    assert torch.equal(o.cpu()[keep.T], o_b[keep.T])
    o, lse = pec.pec_attn_merge(zero.clone(), ninf.clone(), o_b.to(DEV), l_b.to(DEV))
    assert torch.equal(lse.cpu(), l_b) and torch.equal(o.cpu()[keep.T], o_b[keep.T])


@pytest.mark.parametrize("variant", KERNELS)
def test_chunk_merge_folds_segments_exactly(variant):
    sq, s, hq, hkv, q_off = 300, 900, 4, 2, 600
    q, k, v = synth.qkv(17, sq, s, hq, hkv)
    o_ref, l_ref = oracle.attention(q, k, v, q_off=q_off, kv_off=0, causal=True)
    qd, kd, vd = gpu(q, k, v)
    o_acc = torch.zeros(sq, hq, 128, dtype=torch.float32, device=DEV)
    l_acc = torch.full((hq, sq), -math.inf, dtype=torch.float32, device=DEV)
    final = torch.empty(sq, hq, 128, dtype=torch.bfloat16, device=DEV)
    edges = [0, 250, 251, 640, 900]                 # uneven segments, one of a single key
    order = [2, 0, 3, 1]                            # any order gives the same result
    for n, c in enumerate(order):
        lo, hi = edges[c], edges[c + 1]
        pec.pec_attn_chunk_merge(qd, kd[lo:hi], vd[lo:hi], q_off, lo, o_acc, l_acc, True,
                                 out_final=final if n == len(order) - 1 else None, flags=variant)
    assert_close(o_acc, l_acc, o_ref, l_ref, "chunk_merge acc")
    assert_close(final, l_acc, o_ref, l_ref, "chunk_merge final")
    # separate-kernel route: fp32 partials + pec_attn_merge + pec_finalize
    o2 = torch.zeros_like(o_acc)
    l2 = torch.full_like(l_acc, -math.inf)
    for c in order:
        lo, hi = edges[c], edges[c + 1]
        o_p, l_p = pec.pec_attn_chunk(qd, kd[lo:hi], vd[lo:hi], q_off, lo, True, out_dtype=torch.float32,
                                      flags=variant)
        pec.pec_attn_merge(o2, l2, o_p, l_p)
    assert_close(pec.pec_finalize(o2), l2, o_ref, l_ref, "chunk + merge + finalize")


@pytest.mark.parametrize("mode", SP_MODES)
@pytest.mark.parametrize("variant", KERNELS)
def test_sp_prefill_small_config_in_full(mode, variant):
    """8 heads = 8 KV heads, seq 2048 as 4 segments of 512: every ring member, every row."""
    w = synth.WORKLOADS["c1_mha_2k"]
    q, k, v = synth.qkv(w.seed, w.seq, w.seq, w.n_q_heads, w.n_kv_heads)
    o_ref, l_ref = oracle.attention(q, k, v, causal=True)
    qd, kd, vd = gpu(q, k, v)
    for r in range(w.seq // w.chunk):
        lo, hi = r * w.chunk, (r + 1) * w.chunk
        out, lse = pec.pec_sp_prefill(qd[lo:hi], kd, vd, lo, w.chunk, True, flags=mode | variant)
        assert_close(out, lse, o_ref[lo:hi], l_ref[:, lo:hi], "sp_prefill c1 member %d mode %d" % (r, mode))


@pytest.mark.parametrize("mode", SP_MODES)
def test_sp_prefill_ragged_and_noncausal(mode):
    s, hq, hkv, chunk = 1000, 4, 2, 300                         # last segment has 100 tokens
    q, k, v = synth.qkv(18, s, s, hq, hkv)
    qd, kd, vd = gpu(q, k, v)
    o_ref, l_ref = oracle.attention(q, k, v, causal=True)
    for r in range(4):
        lo, hi = r * chunk, min(s, (r + 1) * chunk)
        out, lse = pec.pec_sp_prefill(qd[lo:hi], kd, vd, lo, chunk, True, out_dtype=torch.float32, flags=mode)
        assert_close(out, lse, o_ref[lo:hi], l_ref[:, lo:hi], "ragged member %d" % r)
    o_nc, l_nc = oracle.attention(q[300:600], k, v, causal=False)
    out, lse = pec.pec_sp_prefill(qd[300:600], kd, vd, 300, chunk, False, flags=mode)
    assert_close(out, lse, o_nc, l_nc, "non-causal ring")


def _resumable_run(qd, kd, vd, q_off, chunk, causal, stop, out_dtype=torch.bfloat16, max_calls=10000, between=None):
    """Calls pec_sp_prefill_resumable until nothing is pending; returns (out, lse, number of calls, pending after each)."""
    s_q, hq = qd.shape[0], qd.shape[1]
    out = torch.full((s_q, hq, 128), float("nan"), dtype=out_dtype, device=DEV)
    lse = torch.full((hq, s_q), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(max(16, pec.pec_sp_resumable_workspace_bytes(qd, kd)), dtype=torch.uint8, device=DEV)
    pending = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    history = []
    for call in range(max_calls):
        pec.pec_sp_prefill_resumable(qd, kd, vd, q_off, chunk, out, lse, ws, pending, stop=stop, resume=call > 0,
                                     causal=causal)
        history.append(int(pending.item()))
        if history[-1] == 0:
            return out, lse, call + 1, history
        if between is not None:
            between(call, ws)
    raise AssertionError("sweep did not finish: pending %s" % history[-5:])


RESUMABLE_CASES = [
    # s_q, s_kv, hq, hkv, q_off, chunk, causal
    (512, 4096, 4, 2, 3584, 1024, True),     # last member of 4 x 1024 ... with two query tiles; poll points inside
    (512, 4096, 4, 2, 1024, 1024, True),     # an early member: two segments visible
    (768, 5000, 2, 1, 4232, 1024, True),     # ragged key total (last segment 904 keys), three query tiles
    (300, 4096, 2, 2, 3796, 2048, True),     # second query tile has 44 rows: only left between tiles
    (256, 3072, 8, 2, 0, 1024, False),       # non-causal: all three segments for every row
    (256, 2048, 2, 2, 1792, 128, True),      # segments too short to be left half way
    (200, 0, 2, 1, 0, 1024, True),           # no keys at all
    (2048, 6144, 2, 2, 4096, 1024, True),    # the query segment spans two key segments: tiles end in different ones
    (256, 3000, 4, 2, 0, 1024, False),       # non-causal with a short last segment (952 keys)
    (512, 4096, 16, 2, 3584, 2048, True),    # groups of 8 query heads per KV head
]


@pytest.mark.parametrize("case", RESUMABLE_CASES)
def test_resumable_sweep_uninterrupted_and_stopped_at_every_boundary(case):
    """The stoppable sweep against the oracle: with the stop word clear one call finishes everything; with it set from
    the start every call takes each workgroup's first unfinished tile through exactly one more segment, so the sweep
    is cut at every boundary it can be cut at, and the result must not depend on that."""
    s_q, s_kv, hq, hkv, q_off, chunk, causal = case
    q, k, v = synth.qkv(41 + s_q + s_kv, s_q, max(s_kv, 1), hq, hkv)
    k, v = k[:s_kv], v[:s_kv]
    o_ref, l_ref = oracle.attention(q, k, v, q_off=q_off, kv_off=0, causal=causal)
    qd, kd, vd = gpu(q, k, v)
    clear = torch.zeros(1, dtype=torch.int32, device=DEV)
    for stop in (None, clear):
        out, lse, calls, hist = _resumable_run(qd, kd, vd, q_off, chunk, causal, stop)
        assert calls == 1, hist
        assert_close(out, lse, o_ref, l_ref, "resumable %s uninterrupted" % (case,))
    out_f, lse_f, _, _ = _resumable_run(qd, kd, vd, q_off, chunk, causal, clear, out_dtype=torch.float32)
    assert_close(out_f, lse_f, o_ref, l_ref, "resumable %s fp32 out" % (case,))
    out_u, lse_u = out, lse
    raised = torch.ones(1, dtype=torch.int32, device=DEV)
    out, lse, calls, hist = _resumable_run(qd, kd, vd, q_off, chunk, causal, raised)
    assert_close(out, lse, o_ref, l_ref, "resumable %s stopped after every segment" % (case,))
    # a stopped tile keeps its state exactly as the registers held it, so on such data (no score near a cut far
    # above the running softmax reference) the cuts do not change a single bit
    assert torch.equal(out, out_u) and torch.equal(lse, lse_u), "cuts changed the result of %s" % (case,)
    assert all(a >= b for a, b in zip(hist, hist[1:])), hist          # pending never grows
    n_tiles_q = (s_q + 255) // 256
    assert hist[0] <= n_tiles_q * hq
    # how many calls it must have taken: the grid holds min(items, CUs) workgroups, each leaves after one segment
    # of one tile when that tile can be cut (256 valid rows, segments of at least 1024 keys, a boundary inside
    # the part of the keys no row has masked) -- at least one extra call whenever some tile has two such segments
    vis_end = min(s_kv, q_off + 256) if causal else s_kv                 # keys the first tile's first row block sees
    if s_q >= 256 and chunk >= 1024 and vis_end // chunk >= 2:
        assert calls >= 2, (calls, hist)


def test_resumable_sweep_with_jumps_of_the_row_maximum_around_the_cuts():
    """Keys that lift single rows' scores 16 ... 130 log2 units above the bulk, placed in the last two tiles before a
    segment boundary (the tiles a stopped item drains through), on the boundary itself and right behind it (the first
    tile of the continued item): the softmax reference has to follow on both sides of every cut.  Here cut and
    uninterrupted sweeps may differ in the rounding of single rows, so both are held to the oracle, not to each other."""
    s_q, s_kv, hq, hkv, q_off, chunk = 256, 4096, 8, 2, 3840, 1024
    outliers = [(896, 3, 2), (960, 40, 8), (1023, 77, 4), (1024, 100, 8), (1025, 101, 1), (1088, 130, 2),
                (2047, 180, 8), (2048, 181, 8), (3008, 200, 4), (3071, 220, 1), (3072, 221, 8), (3073, 255, 2),
                (3100, 0, 8), (4000, 250, 8)]
    q, k, v = synth.qkv_with_outlier_keys(4545, s_q, s_kv, hq, hkv, outliers)
    o_ref, l_ref = oracle.attention(q, k, v, q_off=q_off, kv_off=0, causal=True)
    qd, kd, vd = gpu(q, k, v)
    for stop_value, what in ((0, "uninterrupted"), (1, "cut at every boundary")):
        stop = torch.full((1,), stop_value, dtype=torch.int32, device=DEV)
        out, lse, calls, hist = _resumable_run(qd, kd, vd, q_off, chunk, True, stop, out_dtype=torch.float32)
        assert calls == (1 if stop_value == 0 else 4), hist
        assert_close(out, lse, o_ref, l_ref, "outlier keys around the cuts, " + what)


def test_resumable_sweep_state_survives_being_copied_away_and_other_work():
    """Between two calls the workspace and the running LSE are copied away, overwritten, and copied back while another
    prefill runs: only that data (plus q / k / v) carries the interrupted sweep."""
    s_q, s_kv, hq, hkv, q_off, chunk = 512, 6144, 4, 2, 5632, 1024
    q, k, v = synth.qkv(77, s_q, s_kv, hq, hkv)
    o_ref, l_ref = oracle.attention(q, k, v, q_off=q_off, kv_off=0, causal=True)
    qd, kd, vd = gpu(q, k, v)
    raised = torch.ones(1, dtype=torch.int32, device=DEV)
    out = torch.empty((s_q, hq, 128), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((hq, s_q), dtype=torch.float32, device=DEV)
    ws = torch.empty(pec.pec_sp_resumable_workspace_bytes(qd, kd), dtype=torch.uint8, device=DEV)
    pending = torch.zeros(1, dtype=torch.int32, device=DEV)
    calls = 0
    while True:
        pec.pec_sp_prefill_resumable(qd, kd, vd, q_off, chunk, out, lse, ws, pending, stop=raised, resume=calls > 0)
        calls += 1
        if int(pending.item()) == 0:
            break
        saved_ws, saved_lse, saved_out = ws.clone(), lse.clone(), out.clone()
        ws.fill_(0xA5), lse.fill_(float("nan")), out.fill_(float("nan"))
        pec.pec_sp_prefill(qd[:256], kd[:512], vd[:512], 256, 256, True)      # a short request gets the GPU meanwhile
        ws.copy_(saved_ws), lse.copy_(saved_lse), out.copy_(saved_out)
        assert calls < 200
    assert calls > 2
    assert_close(out, lse, o_ref, l_ref, "resumable with state moved between calls")


@pytest.mark.parametrize("where", ["pinned host word", "device word, copy on a side stream", "device word, kernel on a side stream"])
def test_resumable_sweep_stop_raised_while_the_kernel_runs(where):
    """The stop word is raised while the sweep runs -- by the host in pinned memory, or in device memory by a copy or
    a fill kernel on another stream; after every call it is cleared, then raised again a little later.  However
    far each call got, the end result is the same."""
    w = synth.WORKLOADS["c3_gqa_128k"]                                     # the last member's sweep runs ~14 ms
    s_q, q_off = w.chunk, w.seq - w.chunk
    qd, kd, vd = synth.qkv(w.seed + 7, s_q, w.seq, w.n_q_heads, w.n_kv_heads, device=DEV)
    ref_out, ref_lse = pec.pec_sp_prefill(qd, kd, vd, q_off, w.chunk, True)
    pinned = where.startswith("pinned")
    stop = torch.zeros(1, dtype=torch.int32).pin_memory() if pinned else torch.zeros(1, dtype=torch.int32, device=DEV)
    one = torch.ones(1, dtype=torch.int32).pin_memory()
    side = torch.cuda.Stream()
    out = torch.empty_like(ref_out)
    lse = torch.empty_like(ref_lse)
    ws = torch.empty(pec.pec_sp_resumable_workspace_bytes(qd, kd), dtype=torch.uint8, device=DEV)
    pending = torch.zeros(1, dtype=torch.int32, device=DEV)
    calls, hist, fresh, sweeps = 0, [], True, 1
    while True:
        raise_it = calls < 3
        if pinned:
            stop[0] = 0
        else:
            stop.zero_()
            torch.cuda.synchronize()
            if raise_it:    # queued up front: the side stream starts with the sweep, idles ~1 ms, then raises the word
                start = torch.cuda.Event()
                start.record()
                side.wait_event(start)
                with torch.cuda.stream(side):
                    torch.cuda._sleep(2000000)
                    if "copy" in where:
                        stop.copy_(one, non_blocking=True)
                    else:
                        stop.fill_(1)
        pec.pec_sp_prefill_resumable(qd, kd, vd, q_off, w.chunk, out, lse, ws, pending, stop=stop, resume=not fresh)
        calls, fresh = calls + 1, False
        if pinned and raise_it:
            stop[0] = 1                                                    # lands somewhere inside the running kernel
        torch.cuda.synchronize()
        hist.append(int(pending.item()))
        if hist[-1] == 0:
            if max(hist) > 0 or sweeps == 3:
                break
            # the host was held up for the whole 14 ms of the kernel: nothing was interrupted, so start over
            calls, hist, fresh, sweeps = 0, [], True, sweeps + 1
        assert calls < 50, hist
    # same arithmetic per tile wherever it was cut, and the state goes through memory as the registers held it
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    assert max(hist) > 0, "no call was interrupted in three sweeps: %s" % hist
    # and against the oracle, on sampled rows of one KV group
    _sampled_check(qd, kd, vd, out, lse, q_off, _edge_rows(s_q, [256, 32 * 9], 5, 6), heads=3, what="resumable c3 " + where)


@pytest.mark.parametrize("variant", KERNELS)
def test_varlen_matches_oracle_and_dense_calls(variant):
    lengths = [5, 0, 1, 300, 257, 0, 64, 700, 256]
    cu = synth.cu_seqlens_of(lengths)
    t, hq, hkv = int(cu[-1]), 4, 2
    q, k, v = synth.qkv(19, t, t, hq, hkv)
    o_ref, l_ref = oracle.varlen(q, k, v, cu)
    qd, kd, vd = gpu(q, k, v)
    cud = torch.from_numpy(cu).to(DEV)
    out, lse = pec.pec_attn_varlen(qd, kd, vd, cud, max(lengths), True, flags=variant)
    assert_close(out, lse, o_ref, l_ref, "varlen")
    for b, n in enumerate(lengths):                 # bit-identical to one dense call per sequence
        lo, hi = int(cu[b]), int(cu[b + 1])
        if n == 0:
            continue
        o_b, l_b = pec.pec_attn_chunk(qd[lo:hi].contiguous(), kd[lo:hi].contiguous(), vd[lo:hi].contiguous(), 0, 0,
                                      flags=variant)
        assert torch.equal(out[lo:hi], o_b) and torch.equal(lse[:, lo:hi], l_b), "sequence %d" % b
    # Q = 0: LSE = ln(position + 1) exposes any leak across sequence boundaries
    _, lse0 = pec.pec_attn_varlen(torch.zeros_like(qd), kd, vd, cud, max(lengths), True, flags=variant)
    pos = np.concatenate([np.arange(n) for n in lengths])
    got = np.rint(np.exp(lse0.cpu().numpy().astype(np.float64))).astype(np.int64)
    assert np.array_equal(got, np.tile(pos + 1, (hq, 1)))


def test_varlen_max_seqlen_is_only_a_hint_through_the_c_abi():
    """A sequence longer than the max_seqlen the caller states is still processed in full: no row of
    out / lse stays unwritten (they start as NaN) and the result matches the oracle."""
    import ctypes

    lengths = [300, 1100, 0, 17, 520]
    cu = synth.cu_seqlens_of(lengths)
    t, hq, hkv = int(cu[-1]), 4, 2
    q, k, v = synth.qkv(29, t, t, hq, hkv)
    o_ref, l_ref = oracle.varlen(q, k, v, cu)
    qd, kd, vd = gpu(q, k, v)
    cud = torch.from_numpy(cu).to(DEV)
    L = pec.lib()
    ws = torch.empty(L.pec_varlen_workspace_bytes(len(lengths), t), dtype=torch.uint8, device=DEV)
    for max_seqlen in (1, 256, 0, max(lengths)):
        out = torch.full((t, hq, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
        lse = torch.full((hq, t), float("nan"), dtype=torch.float32, device=DEV)
        shp = pec.PecShape(hq, hkv, 128, pec.PEC_BF16, 0.0, 0)
        rc = L.pec_attn_varlen(ctypes.byref(shp), qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), cud.data_ptr(),
                               len(lengths), t, max_seqlen, 1, out.data_ptr(), lse.data_ptr(), ws.data_ptr(),
                               ws.numel(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        assert_close(out, lse, o_ref, l_ref, "varlen with max_seqlen = %d" % max_seqlen)


def _colocated_case(len_q, len_k, hq, hkv, seed, causal=True, out_dtype=torch.float32):
    cq, ck = synth.cu_seqlens_of(len_q), synth.cu_seqlens_of(len_k)
    tq, tk = int(cq[-1]), int(ck[-1])
    q, _, _ = synth.qkv(seed, tq, 1, hq, hkv)
    _, k, v = synth.qkv(seed + 1, 1, tk, hq, hkv)
    o_ref, l_ref = oracle.colocated(q, k, v, cq, ck, causal=causal)
    qd, kd, vd = gpu(q, k, v)
    cqd, ckd = torch.from_numpy(cq).to(DEV), torch.from_numpy(ck).to(DEV)
    out = torch.full((tq, hq, 128), float("nan"), dtype=out_dtype, device=DEV)     # every row must be written
    lse = torch.full((hq, tq), float("nan"), dtype=torch.float32, device=DEV)
    pec.pec_attn_colocated(qd, kd, vd, cqd, ckd, causal, out_dtype=out_dtype, out=out, lse=lse)
    return (qd, kd, vd, cqd, ckd), (out, lse), (o_ref, l_ref)


def test_colocated_batch_matches_oracle():
    """Short prefills, decode steps of long requests (split into key ranges inside the same launch) and
    chunks of new tokens behind a cached prefix, in one pec_attn_colocated call."""
    len_q = [300, 1, 0, 17, 1, 257, 1, 1, 2, 1, 64]
    len_k = [300, 9000, 40, 500, 1, 257, 4096, 4097, 1, 70000, 64]
    # prompt | decode over 3 ranges | no query | chunk after a prefix | first token | prompt | decode with exactly one
    # range (not split) | decode with a 1-key second range | more queries than keys | long decode | prompt
    # (16 and 24 KV heads: an XCD's share of the work order then spans several KV heads, or cuts through one)
    for hq, hkv in ((8, 2), (4, 4), (16, 16), (24, 24)):
        for out_dtype in (torch.float32, torch.bfloat16):
            if hkv > 8 and out_dtype == torch.float32:
                continue
            _, (out, lse), (o_ref, l_ref) = _colocated_case(len_q, len_k, hq, hkv, 301 + hq, out_dtype=out_dtype)
            assert_close(out, lse, o_ref, l_ref, "colocated %dq/%dkv %s" % (hq, hkv, out_dtype))
    # non-causal: every query of a sequence sees all its keys
    _, (out, lse), (o_ref, l_ref) = _colocated_case([5, 1, 130], [40, 6000, 77], 8, 2, 311, causal=False)
    assert_close(out, lse, o_ref, l_ref, "colocated non-causal")


def test_colocated_batch_is_leak_free_and_reduces_to_the_packed_batch():
    len_q = [200, 1, 33, 1, 0, 1]
    len_k = [200, 10000, 700, 5000, 3, 8200]
    (qd, kd, vd, cqd, ckd), _, _ = _colocated_case(len_q, len_k, 8, 2, 321)
    # Q = 0: LSE = ln(number of visible keys), exactly the count Eq. 3 sums over, for every row of every sequence
    _, lse0 = pec.pec_attn_colocated(torch.zeros_like(qd), kd, vd, cqd, ckd, True)
    want = np.concatenate([np.clip(nk - nq + np.arange(nq) + 1, 0, nk) for nq, nk in zip(len_q, len_k)])
    got = np.rint(np.exp(lse0.cpu().numpy().astype(np.float64))).astype(np.int64)
    assert np.array_equal(got, np.tile(want, (8, 1)))
    # equal query and key offsets: bit-identical to pec_attn_varlen (same kernel, same work items)
    lengths = [5, 0, 1, 300, 257, 0, 64, 700, 256]
    cu = torch.from_numpy(synth.cu_seqlens_of(lengths)).to(DEV)
    q, k, v = gpu(*synth.qkv(331, sum(lengths), sum(lengths), 8, 2))
    o_c, l_c = pec.pec_attn_colocated(q, k, v, cu, cu, True)
    o_v, l_v = pec.pec_attn_varlen(q, k, v, cu, max(lengths), True)
    assert torch.equal(o_c, o_v) and torch.equal(l_c, l_v)
    # a decode step alone: same as pec_decode_splitkv up to where the bf16 rounding of the weights falls
    # (different key ranges, hence different softmax references)
    q1, k1, v1 = gpu(*synth.qkv(341, 1, 20000, 32, 8))
    one = torch.tensor([0, 1], dtype=torch.int32, device=DEV)
    kk = torch.tensor([0, 20000], dtype=torch.int32, device=DEV)
    o_c, l_c = pec.pec_attn_colocated(q1, k1, v1, one, kk, True, out_dtype=torch.float32)
    o_d, l_d = pec.pec_decode_splitkv(q1, k1, v1, out_dtype=torch.float32)
    assert (o_c - o_d).abs().max().item() <= 1e-3 and (l_c[:, 0] - l_d).abs().max().item() <= 1e-4


def test_full_size_colocated_decode_with_short_prefills_sampled_rows():
    """The paper's colocation case at full size: 256 log-normal short prompts batched with the decode step of
    a long request whose cache holds 524,288 tokens (32 query / 8 KV heads), one launch."""
    hq, hkv = 32, 8
    short = synth.lognormal_lengths(synth.VARLEN_SEED, synth.VARLEN_N_SHORT)
    len_q = np.concatenate([short[:100], [1], short[100:]])
    len_k = np.concatenate([short[:100], [524288], short[100:]])
    cq, ck = synth.cu_seqlens_of(len_q), synth.cu_seqlens_of(len_k)
    tq, tk = int(cq[-1]), int(ck[-1])
    q, _, _ = synth.qkv(351, tq, 1, hq, hkv, device=DEV)
    _, k, v = synth.qkv(352, 1, tk, hq, hkv, device=DEV)
    out, lse = pec.pec_attn_colocated(q, k, v, torch.from_numpy(cq).to(DEV), torch.from_numpy(ck).to(DEV), True)
    # the decode row, all heads
    b = 100
    q0, k0 = int(cq[b]), int(ck[b])
    o_ref, l_ref = oracle.attention(q[q0:q0 + 1].cpu(), k[k0:k0 + 524288].cpu(), v[k0:k0 + 524288].cpu(), causal=False)
    assert_close(out[q0:q0 + 1], lse[:, q0:q0 + 1], o_ref, l_ref, "colocated decode row")
    # sampled rows of a few short prompts next to it and elsewhere
    for b in (99, 101, 3, 255):
        q0, k0, n = int(cq[b]), int(ck[b]), int(len_q[b])
        rows = synth.sample_rows(b, n, boundaries=(256,) if n > 300 else (), n_random=6, edge=2)
        _sampled_check(q[q0:q0 + n], k[k0:k0 + n], v[k0:k0 + n], out[q0:q0 + n], lse[:, q0:q0 + n], 0, rows,
                       heads=b % hkv, what="colocated short prompt %d (len %d)" % (b, n))


def test_many_sequences_fill_the_work_lists_without_gaps_or_leaks():
    """More sequences than the work-list builders have threads (1024), many of them empty or one token long:
    the Q = 0 count of visible keys must be right for every row of every sequence (a dropped, duplicated or
    misplaced work item shows as a wrong or unwritten count), packed and colocated."""
    rng = np.random.default_rng(77)
    n = 2600
    lens = rng.integers(0, 40, size=n)
    lens[rng.integers(0, n, size=40)] = rng.integers(250, 600, size=40)       # some spill into a second / third query tile
    cu = synth.cu_seqlens_of(lens)
    t, hq, hkv = int(cu[-1]), 4, 2
    _, k, v = synth.qkv(401, 1, t, hq, hkv)
    q0 = torch.zeros(t, hq, 128, dtype=torch.bfloat16, device=DEV)
    cud = torch.from_numpy(cu).to(DEV)
    lse = torch.full((hq, t), float("nan"), dtype=torch.float32, device=DEV)
    pec.pec_attn_varlen(q0, k.to(DEV), v.to(DEV), cud, int(lens.max()), True, lse=lse)
    pos = np.concatenate([np.arange(m) for m in lens])
    got = np.rint(np.exp(lse.cpu().numpy().astype(np.float64))).astype(np.int64)
    assert np.array_equal(got, np.tile(pos + 1, (hq, 1)))
    # colocated: the same prompts, every fifth sequence replaced by a decode step over a cache of its own
    len_q, len_k = lens.copy(), lens.copy()
    dec = np.arange(0, n, 5)
    len_q[dec] = 1
    len_k[dec] = rng.integers(1, 9000, size=dec.size)
    cq, ck = synth.cu_seqlens_of(len_q), synth.cu_seqlens_of(len_k)
    tq, tk = int(cq[-1]), int(ck[-1])
    _, k2, v2 = synth.qkv(402, 1, tk, hq, hkv)
    q0 = torch.zeros(tq, hq, 128, dtype=torch.bfloat16, device=DEV)
    lse = torch.full((hq, tq), float("nan"), dtype=torch.float32, device=DEV)
    pec.pec_attn_colocated(q0, k2.to(DEV), v2.to(DEV), torch.from_numpy(cq).to(DEV), torch.from_numpy(ck).to(DEV), True,
                           lse=lse)
    want = np.concatenate([np.clip(nk - nq + np.arange(nq) + 1, 0, nk) for nq, nk in zip(len_q, len_k)])
    got = np.rint(np.exp(lse.cpu().numpy().astype(np.float64))).astype(np.int64)
    assert np.array_equal(got, np.tile(want, (hq, 1)))


def _sampled_check(qd, kd, vd, out, lse, q_off, rows, heads=None, what=""):
    """Oracle on sampled rows against the full key range (rows are independent in Eq. 2-3)."""
    g = qd.shape[1] // kd.shape[1]
    rows_t = torch.from_numpy(rows).to(qd.device)
    if heads is None:
        qs, k_h, v_h = qd[rows_t].cpu(), kd.cpu(), vd.cpu()
        o_s, l_s = out[rows_t], lse[:, rows_t]
    else:                                             # one KV head and its query group
        kvh = heads
        hs = slice(kvh * g, (kvh + 1) * g)
        qs, k_h, v_h = qd[rows_t][:, hs].cpu().contiguous(), kd[:, kvh:kvh + 1].cpu().contiguous(), \
            vd[:, kvh:kvh + 1].cpu().contiguous()
        o_s, l_s = out[rows_t][:, hs], lse[hs][:, rows_t]
    o_ref, l_ref = oracle.attention(qs, k_h, v_h, q_pos=q_off + rows, kv_off=0, causal=True)
    assert_close(o_s, l_s, o_ref, l_ref, what)


def test_full_size_gqa_32k_last_member_sampled_rows():
    """32 query / 8 KV heads, seq 32768 in 8 segments of 4096: the last ring member's share."""
    w = synth.WORKLOADS["c2_gqa_32k"]
    q_off = w.seq - w.chunk
    q, k, v = synth.qkv(w.seed, w.chunk, w.seq, w.n_q_heads, w.n_kv_heads, device=DEV)
    rows = synth.sample_rows(w.seed, w.chunk, boundaries=(256, 2048), n_random=24)
    for mode in (0, pec.PEC_FLAG_SP_STEP_LAUNCHES):
        out, lse = pec.pec_sp_prefill(q, k, v, q_off, w.chunk, True, flags=mode)
        _sampled_check(q, k, v, out, lse, q_off, rows, what="c2 mode %d" % mode)


def _bench_sweep(q, k, v, q_off, chunk):
    """One ring member's prefill the way bench.py launches it: the stoppable sweep with a stop word that stays clear."""
    out = torch.empty_like(q)
    lse = torch.empty((q.shape[1], q.shape[0]), dtype=torch.float32, device=DEV)
    ws = torch.empty(pec.pec_sp_resumable_workspace_bytes(q, k), dtype=torch.uint8, device=DEV)
    stop = torch.zeros(1, dtype=torch.int32, device=DEV)
    pending = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    pec.pec_sp_prefill_resumable(q, k, v, q_off, chunk, out, lse, ws, pending, stop=stop)
    assert int(pending.item()) == 0
    return out, lse


def _edge_rows(n_rows, edges, seed, n_random):
    """Rows 0, +-1, +-2 around every edge, both ends of the segment, and seeded-random rows."""
    rows = {0, 1, n_rows - 2, n_rows - 1}
    for e in edges:
        rows |= {e - 2, e - 1, e, e + 1, e + 2}
    rows |= set(int(x) for x in np.random.default_rng(seed).integers(0, n_rows, size=n_random))
    return np.array(sorted(r for r in rows if 0 <= r < n_rows), dtype=np.int64)


def test_full_size_gqa_128k_sampled_rows():
    """The headline shape: seq 131072 in 16 segments of 8192, launch configuration of the benchmark (one
    stoppable sweep per ring member; members 15 and 6 also with one launch per ring step).  Every ring member is checked on one KV head (so every KV
    head is covered twice), on rows around a 256-row workgroup edge, a 32-row wavefront edge, both ends of
    the segment and random rows; members 15, 6 and 0 additionally on a second KV head."""
    w = synth.WORKLOADS["c3_gqa_128k"]
    q_all, k, v = synth.qkv(w.seed, w.seq, w.seq, w.n_q_heads, w.n_kv_heads, device=DEV)
    n_members = w.seq // w.chunk
    for r in range(n_members):
        q_off = r * w.chunk
        q = q_all[q_off:q_off + w.chunk]
        out, lse = _bench_sweep(q, k, v, q_off, w.chunk)
        if r in (15, 6):
            out_s, lse_s = pec.pec_sp_prefill(q, k, v, q_off, w.chunk, True, flags=pec.PEC_FLAG_SP_STEP_LAUNCHES)
            assert (out_s.float() - out.float()).abs().max().item() <= 2.0 ** -7
            assert torch.allclose(lse_s, lse, rtol=1e-5, atol=1e-5)
        if r == 15:     # the same member cut at every segment boundary (stop word set throughout), then continued
            raised = torch.ones(1, dtype=torch.int32, device=DEV)
            out_c, lse_c, calls, hist = _resumable_run(q, k, v, q_off, w.chunk, True, raised)
            assert calls >= 16 and all(a >= b for a, b in zip(hist, hist[1:])), (calls, hist[:8])
            assert torch.equal(out_c, out) and torch.equal(lse_c, lse)
        wg_edge = 256 * (1 + (5 * r) % 31)            # a workgroup (256-row) edge, different for every member
        wave_edge = wg_edge + 32 * (1 + r % 7)        # a wavefront (32-row) edge inside the next workgroup
        rows = _edge_rows(w.chunk, (wg_edge, wave_edge), w.seed + r, 4)
        heads = [r % w.n_kv_heads] + ([(r + 3) % w.n_kv_heads] if r in (15, 6, 0) else [])
        for kvh in heads:
            _sampled_check(q, k, v, out, lse, q_off, rows, heads=kvh, what="c3 member %d kv head %d" % (r, kvh))


def test_full_size_colocated_varlen_batch_sampled_rows():
    """256 log-normal short prompts + one 65,536-token prompt, packed; the long prompt first, in the
    middle and last.  Sampled rows of the long prompt and of a few short ones against the oracle."""
    hq, hkv = 32, 8
    for where in ("last", "first", "middle"):
        lengths = synth.varlen_lengths(long_at=where)
        cu = synth.cu_seqlens_of(lengths)
        total = int(cu[-1])
        q, k, v = synth.qkv(synth.VARLEN_SEED, total, total, hq, hkv, device=DEV)
        out, lse = pec.pec_attn_varlen(q, k, v, torch.from_numpy(cu).to(DEV), int(lengths.max()), True)
        b_long = int(np.argmax(lengths))
        picks = [b_long] + [int(b) for b in np.random.default_rng(5).choice(len(lengths), size=4, replace=False)]
        for b in picks:
            lo, n = int(cu[b]), int(lengths[b])
            rows = synth.sample_rows(b, n, boundaries=(256,) if n > 300 else (), n_random=8, edge=2)
            kvh = b % hkv
            _sampled_check(q[lo:lo + n], k[lo:lo + n], v[lo:lo + n], out[lo:lo + n], lse[:, lo:lo + n], 0, rows,
                           heads=kvh, what="c4 %s seq %d (len %d)" % (where, b, n))
        del q, k, v, out, lse


def test_full_size_gqa_512k_last_member_sampled_rows():
    """64 query / 8 KV heads, seq 524288 in 32 segments of 16384: the last ring member's share
    (16384 query rows against 2.1 GB of K/V)."""
    w = synth.WORKLOADS["c5_gqa_512k"]
    q_off = w.seq - w.chunk
    q, k, v = synth.qkv(w.seed, w.chunk, w.seq, w.n_q_heads, w.n_kv_heads, device=DEV)
    out, lse = _bench_sweep(q, k, v, q_off, w.chunk)
    for kvh, wg_edge, wave_edge in ((3, 256 * 17, 256 * 40 + 96), (0, 256 * 1, 256 * 63 + 32), (6, 256 * 50, 256 * 9 + 224)):
        rows = _edge_rows(w.chunk, (wg_edge, wave_edge), w.seed + kvh, 2)
        _sampled_check(q, k, v, out, lse, q_off, rows, heads=kvh, what="c5 last member kv head %d" % kvh)


def test_resumable_prefill_states_match_oracle_and_survive_preemption():
    """pec_sp_prefill_step: the running (O, LSE) after every ring step against the oracle's, and a
    prefill that is paused after every step -- other work runs on the GPU, the state is swapped
    out to the host and back -- ends bit-identical to the uninterrupted pec_sp_prefill."""
    s, hq, hkv, chunk = 1500, 8, 2, 256                       # 6 segments, the last one short
    q_all, k, v = synth.qkv(23, s, s, hq, hkv)
    qd_all, kd, vd = gpu(q_all, k, v)
    lengths = [300, 64, 700]
    cu = torch.from_numpy(synth.cu_seqlens_of(lengths)).to(DEV)
    qs, ks, vs = gpu(*synth.qkv(24, sum(lengths), sum(lengths), hq, hkv))
    for r in (5, 3, 0):
        lo, hi = r * chunk, min(s, (r + 1) * chunk)
        qd = qd_all[lo:hi].contiguous()
        n = pec.pec_sp_prefill_num_steps(qd, kd, lo, chunk)
        assert n == r + 1
        states = oracle.sp_prefill_states(q_all[lo:hi], k, v, q_off=lo, chunk=chunk, causal=True)
        ref_out, ref_lse = pec.pec_sp_prefill(qd, kd, vd, lo, chunk, True, flags=pec.PEC_FLAG_SP_STEP_LAUNCHES)
        o_acc = torch.full((hi - lo, hq, 128), float("nan"), dtype=torch.float32, device=DEV)   # step 0 must not read it
        l_acc = torch.full((hq, hi - lo), float("nan"), dtype=torch.float32, device=DEV)
        out = torch.empty((hi - lo, hq, 128), dtype=torch.bfloat16, device=DEV)
        for t in range(n):
            pec.pec_sp_prefill_step(qd, kd, vd, lo, chunk, t, o_acc, l_acc, True, out_final=out if t == n - 1 else None)
            if t < n - 1:
                assert_close(o_acc, l_acc, states[t][0], states[t][1], "member %d state after step %d" % (r, t))
                # preempted: a batch of short prompts runs, the state leaves the GPU and comes back
                pec.pec_attn_varlen(qs, ks, vs, cu, max(lengths), True)
                o_host, l_host = o_acc.cpu(), l_acc.cpu()
                o_acc.fill_(float("nan"))
                l_acc.fill_(float("nan"))
                o_acc.copy_(o_host)
                l_acc.copy_(l_host)
        assert_close(out, l_acc, states[-1][0], states[-1][1], "member %d final" % r)
        assert torch.equal(out, ref_out) and torch.equal(l_acc, ref_lse)
    # a member that sees nothing (its segment lies before kv position 0 is impossible; use s_kv = 0)
    qd = qd_all[:100].contiguous()
    assert pec.pec_sp_prefill_num_steps(qd, kd[:0], 0, chunk) == 0
    o_acc = torch.full((100, hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    l_acc = torch.full((hq, 100), float("nan"), dtype=torch.float32, device=DEV)
    out = torch.empty((100, hq, 128), dtype=torch.bfloat16, device=DEV)
    pec.pec_sp_prefill_step(qd, kd[:0], vd[:0], 0, chunk, 0, o_acc, l_acc, True, out_final=out)
    assert torch.all(o_acc == 0) and torch.all(out == 0) and torch.all(l_acc == -math.inf)
    with pytest.raises(pec.PecError):
        pec.pec_sp_prefill_step(qd, kd, vd, 0, chunk, 7, o_acc, l_acc, True)


@pytest.mark.parametrize("sk,hq,hkv,n_splits", [(1, 8, 8, 0), (63, 8, 2, 1), (64, 4, 4, 3), (700, 32, 8, 0),
                                                (5000, 64, 8, 7), (70000, 32, 8, 0), (0, 8, 2, 0),
                                                (33, 12, 3, 0),        # three KV heads: a workgroup with an idle wavefront
                                                (3000, 40, 5, 300),    # more ranges than tiles: most ranges are empty
                                                (2100, 64, 1, 3),      # 64 heads on one KV head: the wide-group path
                                                (4097, 32, 1, 0)])     # 32 heads on one KV head: every query column in use
def test_decode_splitkv_matches_oracle(sk, hq, hkv, n_splits):
    """One new token against a KV-cache shard (long-request decode colocated with short prefills)."""
    q, k, v = synth.qkv(31 + sk, 1, sk, hq, hkv)
    o_ref, l_ref = oracle.attention(q, k, v, causal=False)
    for out_dtype in (torch.float32, torch.bfloat16):
        out, lse = pec.pec_decode_splitkv(*gpu(q, k, v), n_splits=n_splits, out_dtype=out_dtype)
        assert_close(out, lse.reshape(hq, 1), o_ref, l_ref, "decode sk=%d %s" % (sk, out_dtype))


def test_decode_with_late_jumps_of_the_maximum():
    # keys far above the bulk late in the cache, in different key ranges
    sk, hq, hkv = 6000, 16, 4
    q, k, v = synth.qkv_with_outlier_keys(4545, 1, sk, hq, hkv, [(100, 0, 1), (2500, 0, 4), (5990, 0, 8)])
    o_ref, l_ref = oracle.attention(q, k, v, causal=False)
    for n_splits in (0, 1, 5):
        out, lse = pec.pec_decode_splitkv(*gpu(q, k, v), n_splits=n_splits, out_dtype=torch.float32)
        assert_close(out, lse.reshape(hq, 1), o_ref, l_ref, "decode with outlier keys, %d ranges" % n_splits)


def test_decode_over_two_shards_merges_like_the_two_gpu_example():
    """The long request's KV cache lives on two GPUs; each computes its partial, the partials are
    merged (here: both shards on the one GPU, merged with pec_attn_merge)."""
    sk, hq, hkv = 9000, 32, 8
    q, k, v = synth.qkv(37, 1, sk, hq, hkv)
    o_ref, l_ref = oracle.attention(q, k, v, causal=False)
    qd, kd, vd = gpu(q, k, v)
    cut = 5123
    o1, l1 = pec.pec_decode_splitkv(qd, kd[:cut], vd[:cut], out_dtype=torch.float32)
    o2, l2 = pec.pec_decode_splitkv(qd, kd[cut:], vd[cut:], out_dtype=torch.float32)
    o, lse = pec.pec_attn_merge(o1, l1.reshape(hq, 1).contiguous(), o2, l2.reshape(hq, 1).contiguous())
    assert_close(o, lse, o_ref, l_ref, "two-shard decode")
    # all keys identical, Q = 0: every key weighs 1/sk, LSE = ln sk exactly
    _, l0 = pec.pec_decode_splitkv(torch.zeros_like(qd), kd, vd)
    assert np.all(np.rint(np.exp(l0.cpu().numpy().astype(np.float64))) == sk)


@pytest.mark.parametrize("s,h,g", [(1, 8, 8), (333, 32, 4), (1000, 40, 8), (77, 64, 1), (0, 8, 2)])
def test_ulysses_layout_is_bit_exact(s, h, g):
    x = synth.randn_bf16((s, h, 128), 41 + s)
    bits = x.view(torch.int16).numpy()
    want = oracle.ulysses_to_messages(bits, g)
    y = pec.pec_ulysses_layout(x.to(DEV), g, True)
    assert y.shape == (g, s, h // g, 128)
    assert np.array_equal(y.cpu().view(torch.int16).numpy(), want)
    back = pec.pec_ulysses_layout(y, g, False)
    assert np.array_equal(back.cpu().view(torch.int16).numpy(), oracle.ulysses_from_messages(want))
    assert torch.equal(back.cpu(), x)
