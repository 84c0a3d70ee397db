"""Strategy selector of fast SP: the oracle's cost model against hand-evaluated values and limiting
cases, and the library's host function against the oracle (no GPU involved)."""
import itertools
import os
import random

import pytest

from oracle import sp_cost
from paper_2409_15104_amd import binding as pec

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sp_cost_example.txt")


def golden_cases():
    cases, cur = [], None
    for ln in open(GOLDEN):
        if not ln.strip() or ln[0] == "#":
            continue
        key, *vals = ln.split()
        if key == "case":
            cur = {"name": vals[0]}
            cases.append(cur)
        else:
            cur[key] = [int(x) for x in vals]
    return cases


def test_volumes_match_the_hand_evaluated_examples():
    cases = golden_cases()
    assert len(cases) == 3
    for vals in cases:
        v = sp_cost.volumes(*vals["params"])
        for key in ("attn_comm", "attn_compute", "mlp_comm", "mlp_compute"):
            assert [int(x) for x in v[key]] == vals[key] and all(x.denominator == 1 for x in v[key]), (vals["name"], key)


def test_time_estimates_match_the_hand_evaluated_examples():
    """The seconds of every combination, exactly, for stated element size, bandwidth and flop rate (section
    "Fast Sequence Parallelism for Long-Request Prefill"; communication and computation time are added).
    Dropping the element size, or swapping bandwidth and flop rate, changes every one of these values;
    cases B and C differ only in the element size and choose differently."""
    bests = {}
    for vals in golden_cases():
        _, sec, best = sp_cost.select(*vals["params"], *vals["rates"])
        flat = [sec[0][0], sec[0][1], sec[1][0], sec[1][1]]
        assert all(x.denominator == 1 for x in flat) and [int(x) for x in flat] == vals["seconds"], vals["name"]
        assert list(best) == vals["best"], vals["name"]
        bests[vals["name"]] = best
    assert bests["B"] != bests["C"]


def test_limiting_cases():
    base = dict(d=4096, n_h=32, n_kv=8, d_h=128, s=8192)
    v = sp_cost.volumes(T=1, G=8, **base)                # no tensor parallelism: nothing to gather, no parameters to move
    assert v["attn_comm"][0] == 0 and v["mlp_comm"] == [0, 0]
    assert v["attn_comm"][1] == 2 * 8192 * 40 * 128 * 7
    v = sp_cost.volumes(T=1, G=1, **base)                # one GPU: no communication at all, both strategies do the same work
    assert v["attn_comm"] == [0, 0] and v["attn_compute"][0] == v["attn_compute"][1]
    # doubling the segment: the attention term 4 (s T)^2 d / T is the only quadratic one, so
    # compute(2s) - 2 compute(s) = 2 * that term; everything in the MLP stage is linear or constant
    v1 = sp_cost.volumes(T=4, G=8, **base)
    v2 = sp_cost.volumes(T=4, G=8, **dict(base, s=2 * 8192))
    assert v2["attn_compute"][0] - 2 * v1["attn_compute"][0] == 2 * 4 * (8192 * 4) ** 2 * 4096 // 4
    assert v2["attn_compute"][1] - 2 * v1["attn_compute"][1] == 2 * 4 * (8192 * 8) ** 2 * 4096 // 8
    assert v2["mlp_compute"][0] == 2 * v1["mlp_compute"][0] and v2["mlp_comm"][1] == v1["mlp_comm"][1]


def test_selection_is_the_argmin_and_moves_with_the_inputs():
    # slow links, short segment, TP 4: moving parameters (Ulysses MLP) costs more than moving activations
    _, sec, best = sp_cost.select(4096, 32, 8, 128, 512, 4, 8, 2, 1e11, 1e15)
    assert best == min(itertools.product((0, 1), (0, 1)), key=lambda am: (sec[am[0]][am[1]], am))
    assert best[1] == sp_cost.MEGATRON
    # very long segment: activations dominate, parameters are cheap -> Ulysses MLP
    _, sec, best = sp_cost.select(4096, 32, 8, 128, 1 << 20, 4, 8, 2, 1e11, 1e15)
    assert best[1] == sp_cost.ULYSSES


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pec.LIB_PATH):
        from paper_2409_15104_amd import build

        build.build()
    return pec.lib()


def test_library_matches_the_oracle(lib):
    rng = random.Random(7)
    for _ in range(200):
        T = rng.choice([1, 2, 4, 8])
        G = rng.choice([1, 2, 4, 8])
        n_kv = rng.choice([1, 2, 4, 8])
        n_h = n_kv * rng.choice([1, 2, 4, 8])
        d_h = rng.choice([64, 128])
        args = (n_h * d_h, n_h, n_kv, d_h, rng.choice([128, 1000, 8192, 65536, 500000]), T, G,
                2, rng.choice([5e10, 4e11, 1e12]), rng.choice([2e14, 1e15, 2.5e15]))
        v, sec, best = sp_cost.select(*args)
        got = pec.pec_sp_select_strategy(*args)
        for key in ("attn_comm", "attn_compute", "mlp_comm", "mlp_compute"):
            for i in range(2):
                assert abs(got[key][i] - float(v[key][i])) <= 1e-12 * max(1.0, float(v[key][i])), (key, args)
        flat = sorted(float(sec[a][m]) for a in (0, 1) for m in (0, 1))
        for a in (0, 1):
            for m in (0, 1):
                assert abs(got["seconds"][a][m] - float(sec[a][m])) <= 1e-12 * float(sec[a][m])
        if flat[1] - flat[0] > 1e-9 * flat[0]:          # a clear winner: the choices must agree
            assert got["best"] == best, args


def test_library_matches_the_hand_evaluated_examples(lib):
    for vals in golden_cases():
        got = pec.pec_sp_select_strategy(*vals["params"], *vals["rates"])
        assert [got["seconds"][0][0], got["seconds"][0][1], got["seconds"][1][0], got["seconds"][1][1]] == \
            [float(x) for x in vals["seconds"]], vals["name"]
        assert list(got["best"]) == vals["best"], vals["name"]


def test_library_rejects_bad_models(lib):
    m = pec.PecSpModel(0, 32, 8, 128, 8192, 4, 8, 2.0, 1e11, 1e15)
    import ctypes

    assert lib.pec_sp_select_strategy(ctypes.byref(m), ctypes.byref(pec.PecSpChoice())) == -1
    assert lib.pec_sp_select_strategy(None, None) == -1
