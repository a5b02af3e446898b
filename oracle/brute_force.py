"""Pure-Python brute force of the SpecKV path for tiny inputs.

TEST INFRASTRUCTURE ONLY: scalar loops and ``math.exp`` / ``math.fsum``, no
numpy arithmetic, so that a mistake in the vectorised oracle (a dropped term, a
transposed operand, an off-by-one in the mask or the pooling window) does not
repeat here.  Same definition and the same readings as ``speckv_oracle``:
Eq. 1 softmax importance; Alg. 1 row set (window rows, then lookahead rows),
reduce, pool, select-with-window, gather; GQA groups summed (App. C.2).
"""
from __future__ import annotations

import itertools
import math
from typing import List, Sequence


def raw_scores(q, k, n_window: int, sm_scale: float, reduce: str = "sum") -> List[List[float]]:
    """q[i][h][c], k[j][g][c] nested sequences -> raw[g][j]."""
    R, Hq, d = len(q), len(q[0]), len(q[0][0])
    n, Hkv = len(k), len(k[0])
    G = Hq // Hkv
    m = n - n_window
    raw = [[0.0] * n for _ in range(Hkv)]
    if reduce == "max":
        # per query head: largest probability any observation row gives the key; heads of a group summed
        for h in range(Hq):
            g = h // G
            best = [0.0] * n
            for i in range(R):
                last = m + i if i < n_window else n - 1
                logits = [sm_scale * sum(float(q[i][h][c]) * float(k[j][g][c]) for c in range(d))
                          for j in range(last + 1)]
                top = max(logits)
                exps = [math.exp(x - top) for x in logits]
                denom = math.fsum(exps)
                for j in range(last + 1):
                    best[j] = max(best[j], exps[j] / denom)
            for j in range(n):
                raw[g][j] += best[j]
        return raw
    contrib = [[[] for _ in range(n)] for _ in range(Hkv)]
    for h in range(Hq):
        g = h // G
        for i in range(R):
            last = m + i if i < n_window else n - 1       # last visible key (lookahead rows see all)
            logits = []
            for j in range(last + 1):
                acc = 0.0
                for c in range(d):
                    acc += float(q[i][h][c]) * float(k[j][g][c])
                logits.append(sm_scale * acc)
            top = max(logits)
            exps = [math.exp(x - top) for x in logits]
            denom = math.fsum(exps)
            for j in range(last + 1):
                contrib[g][j].append(exps[j] / denom)
    for g in range(Hkv):
        for j in range(n):
            raw[g][j] = math.fsum(contrib[g][j])
    return raw


def max_pool(row: Sequence[float], pool_k: int) -> List[float]:
    """Window j - k//2 .. j + (k-1)//2 (symmetric for odd k; for even k one position more before j
    than after it), clipped to the row."""
    m = len(row)
    out = []
    for j in range(m):
        best = None
        for t in range(j - pool_k // 2, j - pool_k // 2 + pool_k):      # the k positions of the window
            if 0 <= t < m and (best is None or row[t] > best):
                best = row[t]
        out.append(best)
    return out


def avg_pool(row: Sequence[float], pool_k: int) -> List[float]:
    """Mean over the same k positions with zeros outside the row."""
    m = len(row)
    out = []
    for j in range(m):
        out.append(math.fsum(row[t] for t in range(j - pool_k // 2, j - pool_k // 2 + pool_k) if 0 <= t < m)
                   / pool_k)
    return out


def select_top(pooled: Sequence[float], count: int) -> List[int]:
    order = sorted(range(len(pooled)), key=lambda j: (-pooled[j], j))
    return sorted(order[:count])


def keep_indices(pooled: Sequence[float], n_in: int, n_window: int, c_max: int) -> List[int]:
    m = n_in - n_window
    return select_top(pooled, min(c_max, m)) + list(range(m, n_in))


def best_subset_exhaustive(pooled: Sequence[float], count: int) -> List[int]:
    """Among all `count`-subsets: maximal score sum, then lexicographically smallest."""
    best_key, best = None, None
    for comb in itertools.combinations(range(len(pooled)), count):
        key = (-math.fsum(pooled[j] for j in comb), comb)
        if best_key is None or key < best_key:
            best_key, best = key, comb
    return list(best)


def ada_head_counts(pooled: Sequence[Sequence[float]], count: int, floor: int) -> List[int]:
    """Shared layer budget: each head's best min(floor, count) first, then the best of the rest
    of the layer by (-value, head, index) until Hkv * count are kept."""
    H, m = len(pooled), len(pooled[0])
    f = min(floor, count)
    taken = set()
    for h in range(H):
        for j in sorted(range(m), key=lambda j: (-pooled[h][j], j))[:f]:
            taken.add((h, j))
    rest = sorted(((h, j) for h in range(H) for j in range(m) if (h, j) not in taken),
                  key=lambda hj: (-pooled[hj[0]][hj[1]], hj[0], hj[1]))[:H * (count - f)]
    counts = [f] * H
    for h, _ in rest:
        counts[h] += 1
    return counts


def best_allocation_exhaustive(pooled: Sequence[Sequence[float]], count: int, floor: int) -> float:
    """Largest total score any allocation (n_0..n_{H-1}), n_h >= min(floor, count), sum = H * count,
    can keep when head h keeps its n_h best candidates."""
    H, m = len(pooled), len(pooled[0])
    f = min(floor, count)
    ranked = [sorted(row, reverse=True) for row in pooled]
    best = -math.inf
    for alloc in itertools.product(range(f, m + 1), repeat=H):
        if sum(alloc) != H * count:
            continue
        best = max(best, math.fsum(math.fsum(ranked[h][:alloc[h]]) for h in range(H)))
    return best


def speckv_layer(q, k, v, n_window: int, pool_k: int, c_max: int, sm_scale: float,
                 reduce: str = "sum", pool: str = "max"):
    n, Hkv = len(k), len(k[0])
    m = n - n_window
    raw = raw_scores(q, k, n_window, sm_scale, reduce)
    pool_fn = max_pool if pool == "max" else avg_pool
    pooled = [pool_fn(raw[g][:m], pool_k) for g in range(Hkv)]
    idx = [keep_indices(pooled[g], n, n_window, c_max) for g in range(Hkv)]
    k_out = [[list(k[j][g]) for j in idx[g]] for g in range(Hkv)]
    v_out = [[list(v[j][g]) for j in idx[g]] for g in range(Hkv)]
    return {"raw": raw, "pooled": pooled, "idx": idx, "k_out": k_out, "v_out": v_out}


def compact_ragged(x, idx: Sequence[Sequence[int]]):
    """x[j][g][c], idx[g] of any length -> rows x[idx[g][r]][g] of head 0, 1, ... one after another
    (Alg. 1 last step, with a different number of kept rows per head)."""
    rows = []
    for g in range(len(idx)):
        for j in idx[g]:
            rows.append([float(c) for c in x[j][g]])
    return rows


def speckv_layer_ada(q, k, v, n_window: int, pool_k: int, c_max: int, floor: int, sm_scale: float,
                     reduce: str = "sum", pool: str = "max"):
    """One (sequence, layer) with the layer's budget shared across its KV heads, loops only:
    scores -> pooled -> per-head counts (ada_head_counts) -> each head's best n_h candidates
    ascending, then the window -> head offsets -> gathered K and V rows."""
    n, Hkv = len(k), len(k[0])
    m = n - n_window
    raw = raw_scores(q, k, n_window, sm_scale, reduce)
    pool_fn = max_pool if pool == "max" else avg_pool
    pooled = [pool_fn(raw[g][:m], pool_k) for g in range(Hkv)]
    counts = ada_head_counts(pooled, min(c_max, m), floor)
    idx = [select_top(pooled[g], counts[g]) + list(range(m, n)) for g in range(Hkv)]
    head_off = [0]
    for g in range(Hkv):
        head_off.append(head_off[-1] + len(idx[g]))
    return {"raw": raw, "pooled": pooled, "idx": idx, "head_off": head_off,
            "k_out": compact_ragged(k, idx), "v_out": compact_ragged(v, idx)}
