"""Pins for oracle/packer.py: paper-printed values, hand-worked examples, invariants."""
import os
from itertools import permutations

import numpy as np
import pytest

import synth_inputs as si
from oracle import packer as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def test_splitmix64_published_vectors():
    ref = [int(r) for r in _rows("splitmix64_seed1234567.txt")]
    rng = op.SplitMix64(1234567)
    assert [rng.next() for _ in ref] == ref


def test_randperm_is_a_uniform_looking_permutation():
    p = op.randperm(1000, 7)
    assert sorted(p) == list(range(1000))
    assert p != list(range(1000)) and op.randperm(1000, 7) == p and op.randperm(1000, 8) != p
    assert op.randperm(1, 3) == [0] and op.randperm(0, 3) == []
    # every one of the 3! orders of 3 items turns up with frequency near 1/6
    counts = {q: 0 for q in permutations(range(3))}
    for s in range(3000):
        counts[tuple(op.randperm(3, s))] += 1
    assert min(counts.values()) > 400 and max(counts.values()) < 600


def test_paper_fig2_std_is_population_std_and_totals():
    for row in _rows("paper_fig2_stage_times.txt"):
        label, times, total, std = [c.strip() for c in row.split(";")]
        t = [float(a) for a in times.split()]
        if total != "-":
            assert sum(t) == float(total)
        if std != "-":
            # printed value is the truncated/rounded population std; the sample std is far off
            assert abs(op.population_std(t) - float(std)) < 1.0
            assert abs(np.std(t, ddof=1) - float(std)) > 20.0


def test_pad_and_dist_ratio_hand_vectors():
    assert op.pad_ratio([2, 4]) == 0.25              # (2 + 0) / (4 * 2)
    assert op.pad_ratio([5, 5, 5]) == 0.0
    assert op.pad_ratio([1, 2, 3, 6]) == pytest.approx((5 + 4 + 3) / 24)
    assert op.dist_ratio([100, 50]) == 0.25
    assert op.dist_ratio([7]) == 0.0
    s = op.spread_stats([1.0, 1.0, 1.0, 1.0])
    assert s["cv"] == 0.0 and s["range_over_mean"] == 0.0 and s["dist_ratio"] == 0.0
    s = op.spread_stats([1.0, 3.0])
    assert s["cv"] == 0.5 and s["range_over_mean"] == 1.0 and s["dist_ratio"] == pytest.approx(1 / 3)


def test_sampling_stage_hand_worked_example():
    # six samples walked in order 0..5, budgets Qv = 4 images, Qt = 10 tokens
    img = [1, 2, 1, 3, 1, 1]
    tok = [4, 3, 5, 2, 8, 2]
    # 0: G=[0] (1,4); 1: (3,7) ok; 2: tokens 12 > 10 -> close [0,1], G=[2] (1,5);
    # 3: (4,7) ok -- reaches Qv exactly, stays open; 4: images 5 > 4 -> close [2,3], G=[4] (1,8);
    # 5: (2,10) ok -- reaches Qt exactly; end of data -> last open group is a candidate too.
    groups = op.isf_sampling(range(6), img, tok, 4, 10)
    assert groups == [[0, 1], [2, 3], [4, 5]]
    # filter with Q'v = 4, Q't = 8: [0,1] has (3,7) -> dropped; [2,3] has (4,7) -> kept by
    # images; [4,5] has (2,10) -> kept by tokens
    assert op.isf_filtering(groups, img, tok, 4, 8) == [[2, 3], [4, 5]]
    with pytest.raises(ValueError):
        op.isf_sampling(range(6), img, tok, 2, 10)       # sample 3 alone has 3 > 2 images


def _check_invariants(img, tok, Qv, Qt, Qvm, Qtm, P, left):
    seen = [i for G in P for i in G]
    assert len(seen) == len(set(seen))
    assert sorted(seen + list(left)) == list(range(len(img)))
    for G in P:
        Iv, It = sum(img[i] for i in G), sum(tok[i] for i in G)
        assert len(G) > 0 and Iv <= Qv and It <= Qt and (Iv >= Qvm or It >= Qtm)


def test_isf_invariants_on_random_tiny_datasets():
    rng = np.random.default_rng(0)
    for trial in range(40):
        n = int(rng.integers(1, 60))
        img = rng.integers(1, 5, n).tolist()
        tok = rng.integers(1, 40, n).tolist()
        Qv, Qt = int(rng.integers(4, 12)), int(rng.integers(40, 120))
        Qvm, Qtm = Qv - int(rng.integers(0, 2)), Qt - int(rng.integers(0, 16))
        P, left, per_iter = op.isf(img, tok, Qv, Qt, Qvm, Qtm, 5, trial)
        _check_invariants(img, tok, Qv, Qt, Qvm, Qtm, P, left)
        assert sum(per_iter) == len(P) and left == sorted(left)


def test_sampling_groups_are_maximal_prefix_runs():
    # brute force: within the walk order, no closed group could have taken its successor
    rng = np.random.default_rng(1)
    img = rng.integers(1, 4, 200).tolist()
    tok = rng.integers(1, 30, 200).tolist()
    order = op.randperm(200, 5)
    groups = op.isf_sampling(order, img, tok, 6, 64)
    assert [i for G in groups for i in G] == order
    for G, nxt in zip(groups[:-1], groups[1:]):
        Iv, It = sum(img[i] for i in G), sum(tok[i] for i in G)
        assert Iv + img[nxt[0]] > 6 or It + tok[nxt[0]] > 64


def test_isf_on_the_synthetic_dataset_matches_the_papers_qualitative_claims():
    tiles, tokens = si.synthetic_dataset(4000, seed=0)
    assert tiles.min() >= 1 and tiles.max() <= 12 and tokens.max() <= 12 * 256 + 4096
    frac_1_to_4 = np.mean(tiles <= 4)
    assert 0.68 < frac_1_to_4 < 0.76
    Qt = 16384
    Qv = op.choose_qv(tiles, tokens, Qt)
    # token-bound grouping (Qv out of the way): every accepted group within 128 tokens of Qt
    P, left, per_iter = op.isf(tiles, tokens, 10 ** 9, Qt, 10 ** 9, Qt - 128, 10, 0)
    _check_invariants(tiles.tolist(), tokens.tolist(), 10 ** 9, Qt, 10 ** 9, Qt - 128, P, left)
    totals = [sum(int(tokens[i]) for i in G) for G in P]
    assert min(totals) >= Qt - 128 and max(totals) <= Qt
    assert op.dist_ratio(totals) < 0.01
    # App. G: the first iteration finds the most groups, later ones add fewer and fewer
    assert per_iter[0] == max(per_iter) and per_iter[0] > per_iter[-1]
    assert len(left) < 0.5 * len(tiles)
    # random fixed-size grouping of the same data is far less balanced (Table 3, row 1 vs 4)
    B = max(1, round(np.mean([len(G) for G in P])))
    R, _ = op.random_groups(len(tiles), B, 0)
    r_totals = [sum(int(tokens[i]) for i in G) for G in R]
    assert op.dist_ratio(r_totals) > 10 * op.dist_ratio(totals)


def test_budget_rule_hand_worked_and_the_papers_own_pair():
    """Sec. 5.2: the image budget follows from the token budget through the dataset's tokens per image
    (and the other way round).  Hand-worked: 6 images over 600 tokens is 100 tokens per image."""
    img, tok = [1, 2, 3], [100, 200, 300]
    assert op.choose_qv(img, tok, 1000) == 10                 # 1000 / 100
    assert op.choose_qv(img, tok, 1050) == 11                 # 10.5 rounds half up
    assert op.choose_qv(img, tok, 1049) == 10                 # 10.49 rounds down
    assert op.choose_qv(img, tok, 10) == 1                    # 0.1 images: never below one
    assert op.choose_qt(img, tok, 10) == 1000                 # 10 images x 100 tokens
    assert op.choose_qt(img, tok, 1) == 100
    assert op.choose_qt([3], [10], 1) == 3                    # 3.33 rounds down
    assert op.choose_qt([2], [5], 1) == 3                     # 2.5 rounds half up
    # a transposed ratio (tokens over images where images over tokens belongs) would give 100000 here
    assert op.choose_qv(img, tok, 1000) != 100000
    # the pair the paper prints for its own data (Sec. 5.2: Q_t = 4K, Q_v = 9): a dataset with 455 tokens
    # per image maps one onto the other, both ways
    img, tok = [1, 1, 2], [455, 455, 910]
    assert op.choose_qv(img, tok, 4096) == 9
    assert abs(op.choose_qt(img, tok, 9) - 4096) <= 1


def test_cu_seqlens_builders():
    assert op.cu_seqlens_llm([2, 0], [5, 9, 7]) == [0, 7, 12]
    assert op.cu_seqlens_vit(3, 1025) == [0, 1025, 2050, 3075]


def test_random_groups():
    G, left = op.random_groups(10, 3, 1)
    assert len(G) == 3 and all(len(g) == 3 for g in G) and len(left) == 1
    assert sorted([i for g in G for i in g] + left) == list(range(10))


# ---- the other grouping arms of Sec. 5.4 (readings: see the oracle's docstrings) ---------------

def test_length_groups_are_runs_of_the_sorted_order():
    tiles, tok = si.synthetic_dataset(1000, 5)
    B = 7
    groups, left = op.length_groups(tok, B, seed=3)
    assert len(groups) == 1000 // B and len(left) == 1000 % B
    assert sorted(sum(groups, []) + left) == list(range(1000))
    spans = sorted((min(int(tok[i]) for i in g), max(int(tok[i]) for i in g)) for g in groups)
    assert all(spans[k][1] <= spans[k + 1][0] for k in range(len(spans) - 1))   # runs do not interleave
    # similar sizes inside a mini-batch: far less padding than random mini-batches of the same size
    rgroups, _ = op.random_groups(1000, B, seed=3)
    pad = lambda gs: sum(op.pad_ratio([int(tok[i]) for i in g]) for g in gs) / len(gs)
    assert pad(groups) < 0.25 * pad(rgroups)
    # but the mini-batches of one step differ in size more than the random arm's do
    step = lambda gs: [sum(int(tok[i]) for i in g) for g in gs[:8]]
    assert op.dist_ratio(step(groups)) > op.dist_ratio(step(rgroups))


def test_device_groups_reorder_the_random_arm_by_total():
    tiles, tok = si.synthetic_dataset(1000, 6)
    B = 5
    groups, left = op.device_groups(tok, B, seed=9)
    rgroups, rleft = op.random_groups(1000, B, seed=9)
    assert sorted(map(tuple, groups)) == sorted(map(tuple, rgroups)) and left == rleft
    totals = [sum(int(tok[i]) for i in g) for g in groups]
    assert totals == sorted(totals)
    # consecutive mini-batches (one step's devices) are close in size; padding inside is untouched
    d = [op.dist_ratio(totals[k:k + 8]) for k in range(0, len(totals) - 8, 8)]
    rt = [sum(int(tok[i]) for i in g) for g in rgroups]
    rd = [op.dist_ratio(rt[k:k + 8]) for k in range(0, len(rt) - 8, 8)]
    assert sum(d) / len(d) < 0.2 * sum(rd) / len(rd)
