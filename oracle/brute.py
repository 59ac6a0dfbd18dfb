"""Pure-Python brute force for tiny inputs — TEST INFRASTRUCTURE used to pin ``fastav_oracle``.

Everything here is written as scalar loops straight from the definitions, with no NumPy arithmetic, so
that a vectorisation mistake in the oracle (a transposed operand, a wrong axis, an off-by-one in the
causal mask) cannot be shared.  Only usable at sizes of a few dozen tokens.
"""
from __future__ import annotations

import math
from typing import List, Sequence


def attention_map(q, k, head: int, group: int) -> List[List[float]]:
    """Full causal attention map of one query head: A[i][j] = softmax_j(q_i . k_j / sqrt(dh)), j <= i.

    q[n][Hq][dh], k[n][Hkv][dh] nested sequences; KV head = head // group."""
    n, dh = len(q), len(q[0][0])
    kv = head // group
    A = [[0.0] * n for _ in range(n)]
    for i in range(n):
        z = []
        for j in range(i + 1):
            acc = 0.0
            for c in range(dh):
                acc += float(q[i][head][c]) * float(k[j][kv][c])
            z.append(acc / math.sqrt(dh))
        zmax = max(z)
        e = [math.exp(t - zmax) for t in z]
        tot = sum(e)
        for j in range(i + 1):
            A[i][j] = e[j] / tot
    return A


def attention_output(q, k, v, group: int) -> List[List[List[float]]]:
    """out[i][h][c] = sum_j A_h[i][j] v[j][h // group][c]."""
    n, Hq, dh = len(q), len(q[0]), len(q[0][0])
    out = [[[0.0] * dh for _ in range(Hq)] for _ in range(n)]
    for h in range(Hq):
        A = attention_map(q, k, h, group)
        for i in range(n):
            for c in range(dh):
                acc = 0.0
                for j in range(i + 1):
                    acc += A[i][j] * float(v[j][h // group][c])
                out[i][h][c] = acc
    return out


def head_mean_last_rows(q, k, group: int, n_last: int = 1) -> List[float]:
    """Section 2.2: the head-averaged attention matrix A (mean over heads of the per-head maps), from
    which Eq. 4 reads the last query's row; for n_last > 1 the last rows are averaged."""
    n, Hq = len(q), len(q[0])
    maps = [attention_map(q, k, h, group) for h in range(Hq)]
    rows = list(range(max(0, n - n_last), n))
    s = [0.0] * n
    for j in range(n):
        acc = 0.0
        for r in rows:
            for h in range(Hq):
                acc += maps[h][r][j]
        s[j] = acc / (Hq * len(rows))
    return s


def topk_by_full_sort(scores: Sequence[float], prot: Sequence[bool], k: int) -> List[int]:
    """Keep every protected index plus the best k - n_prot others: full sort by (score desc, index asc);
    NaN ranks as -inf."""
    def val(x):
        x = float(x)
        return -math.inf if math.isnan(x) else x
    cand = [j for j in range(len(scores)) if not prot[j]]
    cand.sort(key=lambda j: (-val(scores[j]), j))
    n_prot = sum(1 for p in prot if p)
    keep = [j for j in range(len(scores)) if prot[j]] + cand[: k - n_prot]
    return sorted(keep)


def rmsnorm_row(x: Sequence[float], g: Sequence[float], eps: float) -> List[float]:
    ms = sum(float(t) * float(t) for t in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [float(t) * r * float(gg) for t, gg in zip(x, g)]


def rope_vec(x: Sequence[float], pos: int, base: float) -> List[float]:
    dh = len(x)
    half = dh // 2
    out = [0.0] * dh
    for i in range(half):
        ang = pos * (base ** (-2.0 * i / dh))
        c, s = math.cos(ang), math.sin(ang)
        out[i] = float(x[i]) * c - float(x[i + half]) * s
        out[i + half] = float(x[i + half]) * c + float(x[i]) * s
    return out
