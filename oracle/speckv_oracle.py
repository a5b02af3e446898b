"""CPU float64 oracle for SpecKV importance scoring, selection and cache compaction.

TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the HIP
library computes, written from the paper; it is slow on purpose and is never on
the product path.  Only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it.  It shares no code with the HIP path.

What it follows (paper notation: n_in prompt tokens, n_window, n_lookahead,
pool kernel k, budget C_max, m = n_in - n_window):

* importance of a key = attention probability it receives from the observation
  queries, softmax of scaled dot products (Sec. 3.1, Eq. 1);
* observation queries = the last n_window prompt rows stacked over the
  n_lookahead draft rows (Alg. 1, the step that sets m and the CrossAttention
  step; Sec. 4.1);
* reduce over queries (Alg. 1 reduce step), local pooling with kernel k
  (Alg. 1 pooling step; hyper-parameter table: Pool = Max, k = 7);
* keep the top-scoring non-window keys plus the whole window (Alg. 1 "Select
  KVs" step; Fig. 2 caption), then cache <- K[i_cache], V[i_cache]
  (Alg. 1 last step);
* grouped-query attention: the scores of the query heads that share a KV head
  are combined into one score per KV head (App. C.2, the GQA note).

Readings taken where the paper is silent or at odds with itself:

* by default the reduction over queries and over the heads of a group is a SUM
  (Eq. 1's mean times a constant); with reduce="max" (Alg. 1 MaxReduce step;
  hyper-parameter table "Reduction = Max") it is the maximum over the observation
  rows of each query head, and the per-head maxima of a GQA group are summed
  (the group is averaged as in App. C.2, times a constant);
* by default pooling is MAX pooling (hyper-parameter table), stride 1, same
  length, the neighbourhood clipped at both ends of the candidate range [0, m);
  an even kernel k (the table's SpecPC column: 64 / 32) covers k // 2 positions
  before j and k // 2 - 1 after it (the library call with padding k // 2, first m
  outputs kept);
  with pool="avg" (Alg. 1 AvgPool1D step) it is the mean over the k positions of
  the window with zeros outside [0, m) (the usual library convention: padding
  k//2, padded zeros counted in the divisor);
* a window row at prompt position p sees keys j <= p (causal); a lookahead row
  sees every prompt key; the softmax denominator runs over the visible prompt
  keys only (lookahead keys are not inputs);
* the budget ``c_max`` counts NON-window keys: C = min(c_max, m) are selected
  and all n_window window keys are appended, so C + n_window are kept;
* equal pooled scores at the boundary: the smaller index wins;
* kept indices are emitted in ascending order (window last);
* per-head budgets (App. "Integration and Comparison with the AdaKV Baseline"
  only says that a different budget per attention head is applied to SpecKV as
  that baseline does; no formula): per (sequence, layer) every KV head first
  keeps its own best min(floor, C) candidates, then the remaining
  Hkv*C - Hkv*min(floor, C) slots go to the best remaining candidates of the
  whole layer whatever their head (ties: smaller head, then smaller index).
  The layer keeps Hkv*C non-window keys in total, as with equal budgets.  The
  exact safeguard the authors used is UNPINNED.

Parity with the authors' own implementation is UNPINNED: the paper prints no
numeric example for this path.  The functions below are pinned instead by
closed forms, invariants, brute force and library compositions in the CPU tests.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------- #
# Scoring (Eq. 1; Alg. 1 CrossAttention + reduce)
# --------------------------------------------------------------------------- #
def observation_positions(n_in: int, n_window: int, n_lookahead: int) -> np.ndarray:
    """Sequence position of each observation row (window rows first).

    Window row i is prompt token m + i; lookahead row t sits after the prompt at
    n_in + t (Alg. 1: Q from [X_{m:}; Y]).
    """
    m = n_in - n_window
    return np.concatenate([m + np.arange(n_window), n_in + np.arange(n_lookahead)]).astype(np.int64)


def row_lse(q_rows: np.ndarray, k_head: np.ndarray, pos: np.ndarray, sm_scale: float) -> np.ndarray:
    """Natural-log normaliser of every row: log sum over visible keys of exp(sm_scale * q.k)."""
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k_head = np.asarray(k_head, dtype=np.float64)
    logits = sm_scale * (q_rows @ k_head.T)
    visible = np.arange(k_head.shape[0])[None, :] <= np.asarray(pos)[:, None]
    logits = np.where(visible, logits, -np.inf)
    top = logits.max(axis=1)
    return top + np.log(np.exp(logits - top[:, None]).sum(axis=1))


def attention_probs(q_rows: np.ndarray, k_head: np.ndarray, pos: np.ndarray,
                    sm_scale: float, lse: Optional[np.ndarray] = None) -> np.ndarray:
    """Row softmax of sm_scale * q k^T over the causally visible prompt keys.

    q_rows [R, d], k_head [n, d], pos [R] -> P [R, n]; P[i, j] = 0 for j > pos[i].
    With `lse` [R] the rows are normalised by exp(lse) supplied by the caller (for example the
    log-sum-exp of the real forward pass, which also counts the draft keys) instead of by
    their own sum over the prompt keys.
    """
    if lse is not None:
        q_rows = np.asarray(q_rows, dtype=np.float64)
        k_head = np.asarray(k_head, dtype=np.float64)
        logits = sm_scale * (q_rows @ k_head.T)
        visible = np.arange(k_head.shape[0])[None, :] <= np.asarray(pos)[:, None]
        return np.where(visible, np.exp(logits - np.asarray(lse, dtype=np.float64)[:, None]), 0.0)
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k_head = np.asarray(k_head, dtype=np.float64)
    n = k_head.shape[0]
    logits = sm_scale * (q_rows @ k_head.T)                       # [R, n]
    visible = np.arange(n)[None, :] <= np.asarray(pos)[:, None]   # [R, n]
    logits = np.where(visible, logits, -np.inf)
    row_max = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - row_max)                                  # exp(-inf) = 0
    return e / e.sum(axis=1, keepdims=True)


def raw_scores(q: np.ndarray, k: np.ndarray, n_window: int, sm_scale: float,
               reduce: str = "sum", row_weights: Optional[np.ndarray] = None,
               head_reduce: str = "sum", lse_in: Optional[np.ndarray] = None) -> np.ndarray:
    """Importance of every prompt key for every KV head, before pooling.

    q [R, Hq, d] (window rows first), k [n, Hkv, d] -> raw [Hkv, n].  Per query head h the
    probabilities P_h[i, j] (optionally scaled by row_weights[i]) are reduced over the rows i
    with `reduce` ("sum" or "max"); the G heads of a group are combined with `head_reduce`.
    `lse_in` [R, Hq], when given, replaces the rows' own normalisers (see attention_probs).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    R, Hq, _ = q.shape
    n, Hkv, _ = k.shape
    if Hq % Hkv:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    if reduce not in ("sum", "max") or head_reduce not in ("sum", "max"):
        raise ValueError("reduce / head_reduce must be 'sum' or 'max'")
    G = Hq // Hkv
    pos = observation_positions(n, n_window, R - n_window)
    raw = np.zeros((Hkv, n), dtype=np.float64)
    for g in range(Hkv):
        for h in range(g * G, (g + 1) * G):
            P = attention_probs(q[:, h, :], k[:, g, :], pos, sm_scale,
                                None if lse_in is None else np.asarray(lse_in)[:, h])
            if row_weights is not None:
                P = P * np.asarray(row_weights, dtype=np.float64)[:, None]
            per_head = P.sum(axis=0) if reduce == "sum" else P.max(axis=0)
            raw[g] = raw[g] + per_head if head_reduce == "sum" else np.maximum(raw[g], per_head)
    return raw


# --------------------------------------------------------------------------- #
# Pooling (Alg. 1 pooling step; table: Max, k = 7)
# --------------------------------------------------------------------------- #
def pool_window(pool_k: int):
    """Positions a pooling kernel covers around j: j - before .. j + after.

    Odd k: the symmetric window.  Even k (the hyper-parameter table's SpecPC column uses 64 and
    32): the window of the usual library call with padding k // 2, whose first m outputs are
    kept, i.e. k // 2 positions before j and k // 2 - 1 after it.  One formula covers both.
    """
    if pool_k < 1:
        raise ValueError("pool_k must be >= 1")
    return pool_k // 2, (pool_k - 1) // 2


def max_pool_1d(x: np.ndarray, pool_k: int) -> np.ndarray:
    """Same-length max pooling along the last axis, window (see pool_window) clipped at the ends."""
    before, after = pool_window(pool_k)
    x = np.asarray(x, dtype=np.float64)
    m = x.shape[-1]
    out = x.copy()
    for t in range(1, before + 1):
        if t >= m:
            break
        out[..., t:] = np.maximum(out[..., t:], x[..., :-t])      # neighbour j - t
    for t in range(1, after + 1):
        if t >= m:
            break
        out[..., :-t] = np.maximum(out[..., :-t], x[..., t:])     # neighbour j + t
    return out


def avg_pool_1d(x: np.ndarray, pool_k: int) -> np.ndarray:
    """Same-length mean over the k positions of pool_window along the last axis, zeros outside the
    array (the divisor is always k)."""
    before, after = pool_window(pool_k)
    x = np.asarray(x, dtype=np.float64)
    m = x.shape[-1]
    out = x.copy()
    for t in range(1, before + 1):
        if t >= m:
            break
        out[..., t:] += x[..., :-t]
    for t in range(1, after + 1):
        if t >= m:
            break
        out[..., :-t] += x[..., t:]
    return out / pool_k


def pooled_scores(raw: np.ndarray, n_window: int, pool_k: int, pool: str = "max") -> np.ndarray:
    """Pool the non-window candidates raw[..., :m]; returns [..., m]."""
    m = raw.shape[-1] - n_window
    if pool == "max":
        return max_pool_1d(raw[..., :m], pool_k)
    if pool == "avg":
        return avg_pool_1d(raw[..., :m], pool_k)
    raise ValueError("pool must be 'max' or 'avg'")


# --------------------------------------------------------------------------- #
# Selection (Alg. 1 "Select KVs")
# --------------------------------------------------------------------------- #
def select_top(pooled_row: np.ndarray, count: int) -> np.ndarray:
    """Indices of the `count` largest entries, ties to the smaller index, ascending."""
    pooled_row = np.asarray(pooled_row)
    order = np.argsort(-pooled_row, kind="stable")                # stable: ties keep index order
    return np.sort(order[:count]).astype(np.int64)


def keep_indices(pooled_row: np.ndarray, n_in: int, n_window: int, c_max: int) -> np.ndarray:
    """i_cache for one KV head: top C = min(c_max, m) candidates, then the window."""
    m = n_in - n_window
    if pooled_row.shape[-1] != m:
        raise ValueError("pooled_row must hold the m non-window candidates")
    C = min(c_max, m)
    return np.concatenate([select_top(pooled_row, C), np.arange(m, n_in, dtype=np.int64)])


def ada_head_counts(pooled: np.ndarray, count: int, floor: int) -> np.ndarray:
    """Non-window keys kept per KV head when a layer shares its budget across heads.

    pooled [Hkv, m]; `count` = C, the per-head budget if it were equal; every head
    keeps at least min(floor, C).  Returns n[Hkv] with sum Hkv * C.
    (App. "Integration and Comparison with the AdaKV Baseline"; rule: see header.)
    """
    pooled = np.asarray(pooled, dtype=np.float64)
    Hkv, m = pooled.shape
    f = min(floor, count)
    guaranteed = np.zeros((Hkv, m), dtype=bool)
    for g in range(Hkv):
        guaranteed[g, select_top(pooled[g], f)] = True
    heads, cols = np.nonzero(~guaranteed)                     # head-major, index ascending
    order = np.argsort(-pooled[heads, cols], kind="stable")   # ties keep (head, index) order
    extra = heads[order[:Hkv * (count - f)]]
    return f + np.bincount(extra, minlength=Hkv).astype(np.int64)


def ada_keep_indices(pooled: np.ndarray, n_in: int, n_window: int, c_max: int,
                     floor: int) -> List[np.ndarray]:
    """i_cache per KV head with shared budget: head g keeps its top n[g], then the window."""
    m = n_in - n_window
    if pooled.shape[-1] != m:
        raise ValueError("pooled must hold the m non-window candidates")
    counts = ada_head_counts(pooled, min(c_max, m), floor)
    window = np.arange(m, n_in, dtype=np.int64)
    return [np.concatenate([select_top(pooled[g], int(counts[g])), window]) for g in range(pooled.shape[0])]


# --------------------------------------------------------------------------- #
# Compaction (Alg. 1 last step)
# --------------------------------------------------------------------------- #
def compact_ragged(x: np.ndarray, idx: Sequence[np.ndarray]) -> np.ndarray:
    """x [n, Hkv, d], idx[g] of any length -> rows x[idx[g], g, :] of head 0, 1, ... stacked."""
    return np.concatenate([x[idx[g], g, :] for g in range(x.shape[1])], axis=0)


def compact(x: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """x [n, Hkv, d], idx [Hkv, n_keep] -> out [Hkv, n_keep, d] = x[idx[g, r], g, :]."""
    Hkv = x.shape[1]
    return np.stack([x[idx[g], g, :] for g in range(Hkv)], axis=0)


# --------------------------------------------------------------------------- #
# Whole path
# --------------------------------------------------------------------------- #
def speckv_layer(q: np.ndarray, k: np.ndarray, v: Optional[np.ndarray], n_window: int,
                 pool_k: int, c_max: int, sm_scale: float, reduce: str = "sum",
                 pool: str = "max", lse_in: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """One (sequence, layer): scores -> pooled -> indices -> compacted K/V."""
    n = k.shape[0]
    if n < n_window:
        raise ValueError("n_in must be at least n_window")
    raw = raw_scores(q, k, n_window, sm_scale, reduce=reduce, lse_in=lse_in)
    pooled = pooled_scores(raw, n_window, pool_k, pool=pool)
    idx = np.stack([keep_indices(pooled[g], n, n_window, c_max) for g in range(k.shape[1])])
    out = {"raw": raw, "pooled": pooled, "idx": idx, "k_out": compact(k, idx)}
    if v is not None:
        out["v_out"] = compact(v, idx)
    return out


def speckv_layer_ada(q: np.ndarray, k: np.ndarray, v: Optional[np.ndarray], n_window: int,
                     pool_k: int, c_max: int, floor: int, sm_scale: float, reduce: str = "sum",
                     pool: str = "max") -> Dict[str, object]:
    """One (sequence, layer) with the layer's budget shared across its KV heads."""
    n = k.shape[0]
    raw = raw_scores(q, k, n_window, sm_scale, reduce=reduce)
    pooled = pooled_scores(raw, n_window, pool_k, pool=pool)
    idx = ada_keep_indices(pooled, n, n_window, c_max, floor)
    head_off = np.concatenate([[0], np.cumsum([len(i) for i in idx])]).astype(np.int64)
    out = {"raw": raw, "pooled": pooled, "idx": idx, "head_off": head_off, "k_out": compact_ragged(k, idx)}
    if v is not None:
        out["v_out"] = compact_ragged(v, idx)
    return out


def speckv_batch(q: np.ndarray, k: np.ndarray, v: Optional[np.ndarray],
                 cu_seqlens: Sequence[int], n_window: int, pool_k: int, c_max: int,
                 sm_scale: float, reduce: str = "sum",
                 pool: str = "max") -> List[List[Dict[str, np.ndarray]]]:
    """Every (layer, sequence) of a packed ragged batch.

    q [L, S, R, Hq, d], k/v [L, T, Hkv, d]; returns result[layer][seq] dicts with
    sequence-local indices.
    """
    L, S = q.shape[0], q.shape[1]
    out = []
    for layer in range(L):
        row = []
        for s in range(S):
            a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
            row.append(speckv_layer(q[layer, s], k[layer, a:b],
                                    None if v is None else v[layer, a:b],
                                    n_window, pool_k, c_max, sm_scale, reduce=reduce, pool=pool))
        out.append(row)
    return out


# --------------------------------------------------------------------------- #
# Prompt-token selection from draft attention (Sec. 4.2 / Alg. 2, simplified)
# --------------------------------------------------------------------------- #
def specpc_scores(q: np.ndarray, k: np.ndarray, n_window: int, sm_scale: float) -> np.ndarray:
    """One score per prompt token: probabilities summed over layers, heads, rows.

    q [L, R, Hq, d] (here R = n_window: the last prompt rows only), k [L, n, Hkv, d].
    """
    total = np.zeros(k.shape[1], dtype=np.float64)
    for layer in range(q.shape[0]):
        total += raw_scores(q[layer], k[layer], n_window, sm_scale).sum(axis=0)
    return total


def expand_neighbors(sel: np.ndarray, n_in: int, n_window: int, n_neighbor: int) -> np.ndarray:
    """Union of [t - nb, t + nb] for t in sel (clipped to the prompt) and the window."""
    keep = np.zeros(n_in, dtype=bool)
    for t in np.asarray(sel, dtype=np.int64):
        keep[max(0, t - n_neighbor): min(n_in - 1, t + n_neighbor) + 1] = True
    keep[n_in - n_window:] = True
    return np.nonzero(keep)[0].astype(np.int64)


def specpc_select_tokens(q: np.ndarray, k: np.ndarray, token_ids: np.ndarray, n_window: int,
                         pool_k: int, top_k: int, n_neighbor: int,
                         sm_scale: float) -> Dict[str, np.ndarray]:
    """Cross-layer token selection: sum, max-pool, top-k, +-neighbours, window, gather ids."""
    n = k.shape[1]
    m = n - n_window
    raw = specpc_scores(q, k, n_window, sm_scale)
    pooled = max_pool_1d(raw[:m], pool_k)
    sel = select_top(pooled, min(top_k, m))
    idx = expand_neighbors(sel, n, n_window, n_neighbor)
    return {"raw": raw, "pooled": pooled, "sel": sel, "idx": idx,
            "ids": np.asarray(token_ids)[idx], "count": np.int64(idx.shape[0])}


def specpc_window_weights(n_window: int, n_rows: int) -> np.ndarray:
    """Row weights of Alg. 2: the j-th window row (1-based) gets j / n_window, later rows 1."""
    wts = np.ones(n_rows, dtype=np.float64)
    wts[:n_window] = (np.arange(n_window) + 1.0) / n_window
    return wts


def specpc_compress_prompt(q: np.ndarray, k: np.ndarray, token_ids: np.ndarray, n_window: int,
                           pool_k: int, n_neighbor: int, c_max: int, l_skip: int,
                           sm_scale: float) -> Dict[str, np.ndarray]:
    """Prompt compression of Sec. 4.2 / Alg. 2 on draft-model queries and keys.

    q [L, R, Hq, d] (window rows first, then the lookahead rows), k [L, n, Hkv, d].  The first
    l_skip layers are ignored; window row j is weighted j / n_window; the weighted probabilities
    are max-reduced over layers, heads and rows; AvgPool1D(pool_k) then MaxPool1D(n_neighbor)
    (zero / clipped padding and the window of pool_window for even kernels); the top c_max
    non-window tokens plus the window are kept, ascending.
    """
    n = k.shape[1]
    m = n - n_window
    wts = specpc_window_weights(n_window, q.shape[1])
    raw = np.zeros(n, dtype=np.float64)
    for layer in range(l_skip, q.shape[0]):
        per_head = raw_scores(q[layer], k[layer], n_window, sm_scale, reduce="max", row_weights=wts,
                              head_reduce="max")
        raw = np.maximum(raw, per_head.max(axis=0))
    smooth = avg_pool_1d(raw[:m], pool_k)
    spread = max_pool_1d(smooth, n_neighbor)
    sel = select_top(spread, min(c_max, m))
    idx = np.concatenate([sel, np.arange(m, n, dtype=np.int64)])
    return {"raw": raw, "smooth": smooth, "pooled": spread, "sel": sel, "idx": idx,
            "ids": np.asarray(token_ids)[idx], "count": np.int64(idx.shape[0])}
