"""TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT PATH.

Plain Python statement of the paper's control-plane formulas, in double
precision, sharing no code with the library: the corrective seasonal predictor
(Sec. 3.1, Eq. 1-3), the prewarming scores (App. B.1) and the placement
algorithm (Sec. 3.2 Alg. 1; App. B.2).  Loops in the paper's order and
notation; sums use math.fsum (correctly rounded).

Readings where the paper is silent or at odds with itself:
  * Eq. 2 weights the error of window i-w by 2^(w-1); the sentence after it says
    recent errors count more, which the printed weights do not do.  The printed
    equation is followed.
  * Delta is 0 for the first window of a day (min(i, N) = 0 gives 0/0).
  * A burst score with L_A = 0 is +infinity.
  * GPU groups are the aligned runs of D GPUs inside one server: any two such
    groups are disjoint or nested, which is the paper's placement guideline.
  * "Share GPUs with group g" = placed on at least one GPU of g; an untouched
    group has H = -infinity, R = 0.  Ties go to the lowest GPU index; replicas
    with equal score keep model order, then replica order.

Pins: tests/test_control.py (closed forms, hand-worked cases, invariants).
"""
from __future__ import annotations

import math


def seasonal(history, k, i, D):
    """Eq. 1: P(k,i) = (1/D) sum_{d=1..D} L(k-d, i)."""
    return math.fsum(history[k - d][i] for d in range(1, D + 1)) / D


def corrective(history, k, i, D, N):
    """Eq. 2: weighted deviation of today's last min(i,N) windows from their seasonal terms."""
    m = min(i, N)
    if m == 0:
        return 0.0
    terms = [(history[k][i - w] - seasonal(history, k, i - w, D)) * 2.0 ** (w - 1) for w in range(1, m + 1)]
    return math.fsum(terms) / (2.0 ** m - 1.0)


def predict(history, k, i, D=7, N=10):
    """Eq. 3."""
    return seasonal(history, k, i, D) + corrective(history, k, i, D, N)


def replica_counts(L_A, L_P, B, K):
    n_basic = max(math.ceil(L_A / B) - K, 0)
    n_burst = max(math.ceil(L_P / B) - n_basic - K, 0)
    return n_basic, n_burst


def replica_scores(L_A, L_P, B, K, T_c):
    """App. B.1: (n_basic, n_burst, [basic scores..., burst scores...])."""
    n_basic, n_burst = replica_counts(L_A, L_P, B, K)
    total = n_basic + n_burst
    scores = [math.exp(-i / total) * T_c for i in range(n_basic)]
    burstiness = math.inf if L_A == 0 else (L_P - L_A) / L_A
    scores += [math.exp(-(n_basic + i) / total) * T_c * burstiness for i in range(n_burst)]
    return n_basic, n_burst, scores


def place(models, gpu_free, gpus_per_server):
    """Alg. 1.  models: list of dicts with S, D, B, K, L_A, L_P, T_c.  gpu_free: list, updated in
    place.  Returns [(model, replica, first_gpu, is_burst, score)] in placement order."""
    replicas = []
    for i, m in enumerate(models):
        n_basic, n_burst, scores = replica_scores(m["L_A"], m["L_P"], m["B"], m["K"], m["T_c"])
        for r, sc in enumerate(scores):
            replicas.append((1 if r >= n_basic else 0, -sc, i, r))
    replicas.sort()                       # basic first, then score descending, then model, then replica
    on_gpu = [[] for _ in gpu_free]       # indices into `placed` of the replicas on each GPU
    placed = []
    for is_burst, neg_score, i, r in replicas:
        score = -neg_score
        m = models[i]
        D = m["D"]
        need = math.ceil(m["S"] / D)
        candidates = []
        for server in range(len(gpu_free) // gpus_per_server):
            for slot in range(gpus_per_server // D):
                g = server * gpus_per_server + slot * D
                gpus = range(g, g + D)
                if all(gpu_free[j] >= need for j in gpus):
                    sharing = sorted({q for j in gpus for q in on_gpu[j]})
                    H = max((placed[q][4] for q in sharing), default=-math.inf)
                    R = math.fsum(placed[q][4] for q in sharing) if all(math.isfinite(placed[q][4]) for q in sharing) \
                        else math.inf
                    candidates.append((g, H, R))
        if not candidates:
            continue
        isolated = [c for c in candidates if c[1] < score]
        pool = isolated if isolated else candidates
        g = min(pool, key=lambda c: (c[2], c[0]))[0]
        for j in range(g, g + D):
            gpu_free[j] -= need
            on_gpu[j].append(len(placed))
        placed.append((i, r, g, is_burst, score))
    return placed
