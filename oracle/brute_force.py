"""Scalar-loop causal GQA attention for tiny inputs (TEST INFRASTRUCTURE ONLY).

Every score, mask decision, exponential and weighted sum is an explicit Python
loop over (head, query, key, channel); the N x N score matrix is materialised
with an explicit visibility mask.  It is used to pin the vectorised oracle and
is far too slow for anything beyond a few dozen tokens.
"""
from __future__ import annotations

import math
from typing import List


def attention_loops(q, k, v, n_prior: int = 0):
    """q[T][Hq][d], k[P+T][Hkv][d], v[P+T][Hkv][d] (nested lists or arrays) -> out[T][Hq][d], probs[Hq][T][P+T].

    Query row t (absolute position n_prior + t) may see key m iff m <= n_prior + t.
    """
    t_rows = len(q)
    hq = len(q[0])
    d = len(q[0][0])
    n_keys = len(k)
    hkv = len(k[0])
    group = hq // hkv
    inv_sqrt_d = 1.0 / math.sqrt(d)
    out: List = [[[0.0] * d for _ in range(hq)] for _ in range(t_rows)]
    probs: List = [[[0.0] * n_keys for _ in range(t_rows)] for _ in range(hq)]
    for h in range(hq):
        c = h // group
        for t in range(t_rows):
            scores = []
            for m in range(n_keys):
                visible = m <= n_prior + t
                if visible:
                    dot = 0.0
                    for j in range(d):
                        dot += float(q[t][h][j]) * float(k[m][c][j])
                    scores.append(dot * inv_sqrt_d)
                else:
                    scores.append(-math.inf)
            top = max(scores)
            exps = [math.exp(s - top) if s != -math.inf else 0.0 for s in scores]
            z = math.fsum(exps)
            for m in range(n_keys):
                probs[h][t][m] = exps[m] / z
            for j in range(d):
                acc = 0.0
                for m in range(n_keys):
                    acc += probs[h][t][m] * float(v[m][c][j])
                out[t][h][j] = acc
    return out, probs
