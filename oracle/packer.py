"""Oracle: the paper's balanced dynamic mini-batch grouping (Alg. 1, ISF) and its metrics.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Pure-Python loops, written independently of
the library's C++ packer; the two must agree bit for bit.

Follows Alg. 1 (sampling stage, filtering stage), Sec. 4.1 (outer iteration, Eq. 1 PadRatio,
Eq. 2 DistRatio) and Sec. 5.2 (Q' rule).  Readings taken where the paper is silent:
  * the group budget test is "adding the next sample would exceed Q" (Alg. 1 uses >), so a group
    may reach Q exactly;
  * the group still open when the sampling loop ends is also a candidate;
  * empty groups are never produced; a sample that alone exceeds a budget is an input error;
  * |y_i| is the LLM-side token count of the sample (visual tokens + text);
  * samples left in D after the last iteration are returned as leftover;
  * randperm is Fisher-Yates driven by splitmix64 seeded with seed + iteration.
"""
from __future__ import annotations

import math

_M64 = (1 << 64) - 1


class SplitMix64:
    """splitmix64 (Steele, Lea, Flood 2014; public-domain reference by Vigna)."""

    def __init__(self, seed: int):
        self.s = seed & _M64

    def next(self) -> int:
        self.s = (self.s + 0x9E3779B97F4A7C15) & _M64
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
        return z ^ (z >> 31)

    def below(self, n: int) -> int:
        """uniform integer in [0, n) without modulo bias (reject the top partial range)."""
        limit = (1 << 64) - ((1 << 64) % n)
        while True:
            r = self.next()
            if r < limit:
                return r % n


def randperm(n: int, seed: int):
    """Fisher-Yates: for i = n-1 .. 1 swap p[i] with p[j], j uniform in [0, i]."""
    rng = SplitMix64(seed)
    p = list(range(n))
    for i in range(n - 1, 0, -1):
        j = rng.below(i + 1)
        p[i], p[j] = p[j], p[i]
    return p


# ------------------------------------------------------------------------------------------
# Alg. 1
# ------------------------------------------------------------------------------------------

def isf_sampling(order, n_img, n_tok, Qv, Qt):
    """Sampling stage: walk the samples in `order`; append to the open group until the image
    total would exceed Qv or the token total would exceed Qt; then close it and start a new
    group with that sample."""
    groups, G, Iv, It = [], [], 0, 0
    for i in order:
        xi, yi = int(n_img[i]), int(n_tok[i])
        if xi > Qv or yi > Qt:
            raise ValueError(f"sample {i} alone exceeds the budget")
        if G and (Iv + xi > Qv or It + yi > Qt):
            groups.append(G)
            G, Iv, It = [], 0, 0
        G.append(int(i))
        Iv += xi
        It += yi
    if G:
        groups.append(G)
    return groups


def isf_filtering(groups, n_img, n_tok, Qv_min, Qt_min):
    """Filtering stage: keep a group iff Iv >= Q'v or It >= Q't."""
    kept = []
    for G in groups:
        Iv = sum(int(n_img[i]) for i in G)
        It = sum(int(n_tok[i]) for i in G)
        if Iv >= Qv_min or It >= Qt_min:
            kept.append(G)
    return kept


def isf(n_img, n_tok, Qv, Qt, Qv_min, Qt_min, iters, seed):
    """Alternate sampling and filtering up to `iters` times on the not-yet-grouped samples.

    returns (accepted groups in acceptance order, leftover sample ids ascending,
             per-iteration count of accepted groups)
    """
    D = list(range(len(n_img)))
    P, per_iter = [], []
    for it in range(iters):
        if not D:
            break
        perm = randperm(len(D), seed + it)
        order = [D[p] for p in perm]
        kept = isf_filtering(isf_sampling(order, n_img, n_tok, Qv, Qt), n_img, n_tok,
                             Qv_min, Qt_min)
        P.extend(kept)
        per_iter.append(len(kept))
        gone = set(i for G in kept for i in G)
        D = [i for i in D if i not in gone]
    return P, D, per_iter


def random_groups(n_samples, B, seed):
    """The baseline arm: consecutive runs of B samples of one random permutation; the last
    partial run is left over."""
    perm = randperm(n_samples, seed)
    n_full = n_samples // B
    groups = [perm[g * B:(g + 1) * B] for g in range(n_full)]
    return groups, sorted(perm[n_full * B:])


def length_groups(n_tok, B, seed):
    """Sec. 5.4 method 2 (Length-Group), reading: sort by token count (ties by id), cut into runs of
    B, then put the mini-batches in a random order; the last partial run is left over."""
    n = len(n_tok)
    order = sorted(range(n), key=lambda i: (int(n_tok[i]), i))
    n_full = n // B
    batch_order = randperm(n_full, seed)
    groups = [order[b * B:(b + 1) * B] for b in batch_order]
    return groups, sorted(order[n_full * B:])


def device_groups(n_tok, B, seed):
    """Sec. 5.4 method 3 (Device-Group), reading: the random arm's mini-batches ordered by their
    token totals (ties keep the random order)."""
    groups, left = random_groups(len(n_tok), B, seed)
    totals = [sum(int(n_tok[i]) for i in g) for g in groups]
    idx = sorted(range(len(groups)), key=lambda g: (totals[g], g))
    return [groups[g] for g in idx], left


def choose_qv(n_img, n_tok, Qt):
    """Sec. 5.2: Qv from the dataset's image-to-token ratio at the token budget Qt."""
    return max(1, int(math.floor(Qt * sum(int(a) for a in n_img)
                                 / sum(int(b) for b in n_tok) + 0.5)))


def choose_qt(n_img, n_tok, Qv):
    return max(1, int(math.floor(Qv * sum(int(b) for b in n_tok)
                                 / sum(int(a) for a in n_img) + 0.5)))


# ------------------------------------------------------------------------------------------
# segment offsets of one packed mini-batch
# ------------------------------------------------------------------------------------------

def cu_seqlens_llm(group, n_tok):
    """One segment per sample, in group order."""
    cu = [0]
    for i in group:
        cu.append(cu[-1] + int(n_tok[i]))
    return cu


def cu_seqlens_vit(total_tiles, tile_len):
    """One segment of tile_len tokens per image tile."""
    return [j * tile_len for j in range(total_tiles + 1)]


# ------------------------------------------------------------------------------------------
# metrics
# ------------------------------------------------------------------------------------------

def pad_ratio(t):
    """Eq. 1: sum_i (t_max - t_i) / (t_max * B) over the B samples of one mini-batch."""
    tmax = max(t)
    return sum(tmax - ti for ti in t) / (tmax * len(t))


def dist_ratio(Ts):
    """Eq. 2: sum_i (T_max - T_i) / (T_max * N) over the N devices' mini-batch token counts."""
    Tmax = max(Ts)
    return sum(Tmax - Ti for Ti in Ts) / (Tmax * len(Ts))


def population_std(v):
    """The paper's STD (Fig. 2 numbers): divide by N, not N-1."""
    m = sum(v) / len(v)
    return math.sqrt(sum((a - m) ** 2 for a in v) / len(v))


def spread_stats(times):
    """Three readings of the step-time spread: population CV, (max-min)/mean, Eq.-2 form."""
    m = sum(times) / len(times)
    return dict(cv=population_std(times) / m, range_over_mean=(max(times) - min(times)) / m,
                dist_ratio=dist_ratio(times))
