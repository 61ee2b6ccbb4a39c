"""Brute-force checker for tiny shapes: pure Python loops and math.exp, written straight from
Eq. 4 / Eq. 5 / Algorithm 1 of the paper.  Independent of the oracle package (imports nothing
from it) so that it can pin the oracle; far too slow for anything but tiny inputs."""
from __future__ import annotations

import math


def brute_scores(q, k, Hq, Hkv, Lq, L, d, scale, mode="sum"):
    """q[h][i][c], k[g][t][c] nested lists of Python floats -> score[t]."""
    G = Hq // Hkv
    score = [0.0] * L
    for h in range(Hq):
        g = h // G
        for i in range(Lq):
            logit = []
            for t in range(L):
                s = 0.0
                for c in range(d):
                    s += q[h][i][c] * k[g][t][c]
                logit.append(s * scale)
            m = max(logit)
            e = [math.exp(x - m) for x in logit]
            z = math.fsum(e)
            for t in range(L):
                p = e[t] / z
                if mode == "sum":
                    score[t] += p
                else:
                    score[t] = max(score[t], p)
    return score


def brute_pool(score, w):
    L = len(score)
    r = (w - 1) // 2
    return [max(score[u] for u in range(max(0, t - r), min(L, t + r + 1))) for t in range(L)]


def brute_allocate(score, kernels, budget, sink=0):
    """Algorithm 1, stride-1 max-pool reading: the sink tokens are in I from the start and the pooling
    never sees them; every other token is walked in rank order per kernel size."""
    L = len(score)
    n = len(kernels)
    shares = [budget // n + (1 if j < budget % n else 0) for j in range(n)]
    chosen = set(range(sink))
    for w, share in zip(kernels, shares):
        pooled = [None] * sink + brute_pool(score[sink:], w)
        ranked = sorted(range(sink, L), key=lambda t: (-pooled[t], t))
        got = 0
        for t in ranked:
            if got >= share:
                break
            if t not in chosen:
                chosen.add(t)
                got += 1
    return sorted(chosen)


def brute_allocate_max_avg(score, max_kernels, avg_kernels, budget, sink=0):
    """Algorithm 1 with strided max pooling then average pooling, cell by cell, on numpy float32 scalars
    (the precision the decisions are taken in).  Same readings as the oracle states."""
    import numpy as np
    body = [np.float32(x) for x in score[sink:]]
    Lb = len(body)
    ncombo = len(max_kernels) * len(avg_kernels)
    shares = [budget // ncombo + (1 if c < budget % ncombo else 0) for c in range(ncombo)]
    chosen = set()
    combo = 0
    for m in max_kernels:
        ncell = Lb // m
        cells = [max(body[p * m:p * m + m]) for p in range(ncell)]
        k_m = budget // m + 1
        for n in avg_kernels:
            pooled = []
            for p in range(ncell):
                acc = np.float32(0)
                for q in range(p - (n - 1) // 2, p + n // 2 + 1):
                    acc = np.float32(acc + (cells[q] if 0 <= q < ncell else np.float32(0)))
                pooled.append(np.float32(acc / np.float32(n)))
            ranked = sorted(range(ncell), key=lambda p: (-float(pooled[p]), p))[:k_m]
            added = 0
            for p in ranked:
                for t in range(p * m, p * m + m):
                    if added < shares[combo] and t not in chosen:
                        chosen.add(t)
                        added += 1
            combo += 1
    return list(range(sink)) + [sink + t for t in sorted(chosen)]
