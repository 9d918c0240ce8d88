"""Oracle (test infrastructure only) for the two host-side planning steps that sit next to the hot
path.  Plain Python, brute force where the method is a search.

* Balanced model partitioning, Sec. 4.2: layers 1..L, pipeline size N, a partition
  P = (P1 < ... < P(N-1)) with P0 = 1 and PN = L + 1; stage i holds the layers P(i-1) <= l < P(i).
  Anchor = greedy cuts that make the stage times close; candidates = the anchor jittered within a
  radius r; ranking by VAR(fwd_time) (Eq. 4, as printed: a sum of squared deviations, no 1/N) plus
  SUM(comm) (Eq. 5: the activation count of the last layer of every stage but the last).
* Adaptive re-computation, Sec. 4.3 Step 4: how many layers can keep their activations in the
  memory that is left when re-computation is on everywhere.

Pins: tests/test_oracle_planner.py (the paper's L = 20, N = 4, P = (5, 10, 15) example and its
3^3 = 27 candidates for r = 1, N = 4; exhaustive optimum on small cases; closed forms).
"""
import itertools


def stages(P, L):
    """Layer lists (1-based) of the N stages of partition P."""
    cuts = [1] + list(P) + [L + 1]
    return [list(range(cuts[i], cuts[i + 1])) for i in range(len(cuts) - 1)]


def is_valid(P, L):
    cuts = [1] + list(P) + [L + 1]
    return all(cuts[i] < cuts[i + 1] for i in range(len(cuts) - 1))


def stage_times(P, fwd):
    return [sum(fwd[l - 1] for l in st) for st in stages(P, len(fwd))]


def var_fwd_time(P, fwd):
    """Eq. 4 as printed: sum over stages of (FWD(S_i) - mean)^2."""
    t = stage_times(P, fwd)
    m = sum(t) / len(t)
    return sum((a - m) ** 2 for a in t)


def sum_comm(P, activ):
    """Eq. 5: activation count of the last layer of each of the first N-1 stages."""
    return sum(activ[p - 2] for p in P)      # last layer of the stage that ends before P(i) is P(i) - 1


def anchor(fwd, N):
    """Greedy anchor: cut i is put where the running time is closest to i/N of the total, among the
    positions that leave every stage (before and after) at least one layer; ties take the earlier."""
    L = len(fwd)
    total = sum(fwd)
    P, prev = [], 1
    for i in range(1, N):
        target = total * i / N
        best, best_d = None, None
        for p in range(prev + 1, L + 1 - (N - i) + 1):
            run = 0.0
            for l in range(1, p):
                run += fwd[l - 1]
            dist = abs(run - target)
            if best is None or dist < best_d:
                best, best_d = p, dist
        P.append(best)
        prev = best
    return tuple(P)


def candidates(P_anchor, L, r):
    out = []
    for offs in itertools.product(range(-r, r + 1), repeat=len(P_anchor)):
        P = tuple(a + o for a, o in zip(P_anchor, offs))
        if is_valid(P, L):
            out.append(P)
    return out


def search(fwd, activ, N, r, comm_weight=1.0, top_k=10):
    """Ranked candidates [(score, P)], ascending score, ties in lexicographic order of P."""
    L = len(fwd)
    cands = candidates(anchor(fwd, N), L, r)
    scored = sorted((var_fwd_time(P, fwd) + comm_weight * sum_comm(P, activ), P) for P in cands)
    return scored[:top_k], len(cands)


def recompute_plan(free_bytes, n_vit, bytes_vit, ms_vit, n_llm, bytes_llm, ms_llm, extra=0):
    """Sec. 4.3 Step 4 by exhaustive search over (keep_vit, keep_llm): most replay time saved within
    the budget; ties: fewer bytes, then fewer ViT layers.  Each failed trial (`extra`) gives up one
    kept layer, the kind with the larger footprint first (ties: the one that saves less time)."""
    best = None
    for kv in range(n_vit + 1):
        for kt in range(n_llm + 1):
            used = kv * bytes_vit + kt * bytes_llm
            if used > free_bytes:
                continue
            key = (-(kv * ms_vit + kt * ms_llm), used, kv)
            if best is None or key < best[0]:
                best = (key, kv, kt)
    _, kv, kt = best
    for _ in range(extra):
        if kv + kt == 0:
            break
        drop_vit = kv > 0 and (kt == 0 or bytes_vit > bytes_llm or (bytes_vit == bytes_llm and ms_vit <= ms_llm))
        if drop_vit:
            kv -= 1
        else:
            kt -= 1
    return kv, kt
