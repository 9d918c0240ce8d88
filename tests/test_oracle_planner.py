"""Pins for oracle/planner.py: the paper's worked partition example (Sec. 4.2: L = 20, N = 4,
P = (5, 10, 15); 3^3 = 27 candidates for r = 1, N = 4), hand-worked Eq. 4 / Eq. 5 values, the
exhaustive optimum on small cases, and closed forms of the Step-4 arithmetic (Sec. 4.3)."""
import itertools
import os
import random

import pytest

from oracle import planner as pl


def _paper_example():
    """The values the paper prints for its worked partition example (tests/golden/paper_bmp_example.txt)."""
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_bmp_example.txt")) as f:
        for ln in f:
            if ln.strip() and not ln.startswith("#"):
                key, val = [c.strip() for c in ln.split(";")]
                rows[key] = [int(v) for v in val.split()]
    return rows


def test_paper_partition_example():
    # "The first partition consists of layers l1 .. l4 since P0 = 1, P1 = 5"
    ex = _paper_example()
    L, N, P = ex["L"][0], ex["N"][0], tuple(ex["P"])
    assert (L, N, P) == (20, 4, (5, 10, 15))
    st = pl.stages(P, L)
    assert len(st) == N and st[0] == ex["first_stage_layers"]
    assert [len(s) for s in st] == [4, 5, 5, 6]
    assert sorted(sum(st, [])) == list(range(1, L + 1))
    assert pl.is_valid(P, L) and not pl.is_valid((5, 5, 15), L)
    assert not pl.is_valid((1, 10, 15), L) and not pl.is_valid((5, 10, 21), L)


def test_candidate_count_r1_n4_is_27():
    ex = _paper_example()
    L, N, r, n_cand = ex["L"][0], ex["N"][0], ex["r"][0], ex["n_candidates"][0]
    a = pl.anchor([1.0] * L, N)
    assert a == (6, 11, 16)                       # uniform layers: the equal split
    cands = pl.candidates(a, L, r)
    assert n_cand == 27 and len(cands) == n_cand and len(set(cands)) == n_cand
    assert len(pl.candidates(tuple(ex["P"]), L, r)) == n_cand      # around the printed partition too
    assert all(max(abs(p - q) for p, q in zip(P, a)) <= 1 for P in cands)
    # candidates that fall off an end or collide are dropped
    assert len(pl.candidates((2, 3, 4), 20, 1)) < 27


def test_metrics_hand_worked():
    fwd, activ = [1.0, 2.0, 3.0, 4.0], [10.0, 20.0, 30.0, 40.0]
    assert pl.stage_times((3,), fwd) == [3.0, 7.0]
    assert pl.var_fwd_time((3,), fwd) == 8.0          # (3-5)^2 + (7-5)^2, no 1/N (Eq. 4 as printed)
    assert pl.sum_comm((3,), activ) == 20.0           # output of layer 2, the last layer of stage 1
    assert pl.sum_comm((2, 4), activ) == 10.0 + 30.0
    ranked, n = pl.search(fwd, activ, 2, 3, comm_weight=0.0, top_k=10)
    assert n == 3 and ranked[0] == (0.0 + (6 - 5) ** 2 + (4 - 5) ** 2, (4,))   # [1,2,3] vs [4]: 6, 4


def test_anchor_tracks_the_running_time():
    rng = random.Random(1)
    for _ in range(50):
        N = rng.randint(2, 5)
        L = rng.randint(3 * N, 40)
        fwd = [rng.uniform(1.0, 2.0) for _ in range(L)]
        P = pl.anchor(fwd, N)
        assert pl.is_valid(P, L) and len(P) == N - 1
        total, big = sum(fwd), max(fwd)
        for i, p in enumerate(P, 1):
            assert abs(sum(fwd[:p - 1]) - total * i / N) <= big / 2 + 1e-12
        assert max(pl.stage_times(P, fwd)) <= total / N + big + 1e-12


def test_heterogeneous_stack_gets_unequal_layer_counts():
    # a ViT-like prefix of slow layers followed by fast ones: equal layer counts would be unbalanced
    fwd = [4.0] * 8 + [1.0] * 32
    P = pl.anchor(fwd, 4)
    t = pl.stage_times(P, fwd)
    assert max(t) - min(t) <= 4.0
    equal = pl.stage_times((11, 21, 31), fwd)
    assert pl.var_fwd_time(P, fwd) < pl.var_fwd_time((11, 21, 31), fwd) and max(equal) > max(t)


def test_search_with_large_radius_finds_the_global_optimum():
    rng = random.Random(7)
    for _ in range(20):
        N = rng.randint(2, 4)
        L = rng.randint(N, 9)
        fwd = [float(rng.randint(1, 9)) for _ in range(L)]
        activ = [float(rng.randint(0, 5)) for _ in range(L)]
        w = rng.choice([0.0, 0.5, 2.0])
        ranked, n = pl.search(fwd, activ, N, L, comm_weight=w, top_k=1)
        every = [tuple(c) for c in itertools.combinations(range(2, L + 1), N - 1)]
        assert n == len(every)
        best = min(pl.var_fwd_time(P, fwd) + w * pl.sum_comm(P, activ) for P in every)
        assert ranked[0][0] == best


def test_search_ranking_is_sorted_and_contains_the_anchor():
    rng = random.Random(3)
    fwd = [rng.uniform(0.5, 3.0) for _ in range(30)]
    activ = [rng.uniform(0.0, 1.0) for _ in range(30)]
    ranked, n = pl.search(fwd, activ, 4, 2, top_k=1000)
    assert n == len(ranked) <= 125
    assert [s for s, _ in ranked] == sorted(s for s, _ in ranked)
    assert pl.anchor(fwd, 4) in [P for _, P in ranked]


@pytest.mark.parametrize("free,n,b,expect", [(0, 5, 10, 0), (9, 5, 10, 0), (10, 5, 10, 1), (49, 5, 10, 4),
                                             (50, 5, 10, 5), (10 ** 9, 5, 10, 5)])
def test_recompute_plan_single_kind_is_floor_division(free, n, b, expect):
    assert pl.recompute_plan(free, 0, 1, 1.0, n, b, 2.0) == (0, expect)
    assert pl.recompute_plan(free, n, b, 2.0, 0, 1, 1.0) == (expect, 0)


def test_recompute_plan_properties():
    rng = random.Random(11)
    for _ in range(200):
        nv, nt = rng.randint(0, 6), rng.randint(0, 6)
        bv, bt = rng.randint(1, 20), rng.randint(1, 20)
        mv, mt = rng.uniform(0.1, 5.0), rng.uniform(0.1, 5.0)
        free = rng.randint(0, 150)
        kv, kt = pl.recompute_plan(free, nv, bv, mv, nt, bt, mt)
        assert 0 <= kv <= nv and 0 <= kt <= nt and kv * bv + kt * bt <= free
        # maximal: no layer of either kind can be added
        assert kv == nv or (kv + 1) * bv + kt * bt > free
        assert kt == nt or kv * bv + (kt + 1) * bt > free
        # more memory never saves less time
        kv2, kt2 = pl.recompute_plan(free + rng.randint(0, 30), nv, bv, mv, nt, bt, mt)
        assert kv2 * mv + kt2 * mt >= kv * mv + kt * mt - 1e-12
        # each failed trial gives one kept layer up
        e = rng.randint(0, 4)
        kv3, kt3 = pl.recompute_plan(free, nv, bv, mv, nt, bt, mt, extra=e)
        assert kv3 + kt3 == max(0, kv + kt - e) and kv3 <= kv and kt3 <= kt


def test_recompute_plan_prefers_the_better_time_per_byte():
    # 100 bytes: either 1 ViT layer (100 B, saves 3 ms) or 2 LLM layers (50 B each, 2 ms each)
    assert pl.recompute_plan(100, 4, 100, 3.0, 4, 50, 2.0) == (0, 2)
    assert pl.recompute_plan(100, 4, 100, 5.0, 4, 50, 2.0) == (1, 0)
    # after a failed trial the larger footprint goes first
    assert pl.recompute_plan(250, 4, 100, 5.0, 4, 50, 2.0) == (2, 1)
    assert pl.recompute_plan(250, 4, 100, 5.0, 4, 50, 2.0, extra=1) == (1, 1)
