"""Pins for the CPU oracle: closed forms, invariants, library compositions, brute force.

None of these tests re-types the oracle's own formula.  Each one fixes a part of
the definition through something the paper or the mathematics determines
independently (a closed form, a conservation law, Lemma 1, a library routine of
different provenance, exhaustive enumeration on tiny inputs).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads
from oracle import brute_force as bf
from oracle import speckv_oracle as orc


def _rand_case(rng, R, w, Hq, Hkv, d, n, scale=1.0):
    q = rng.standard_normal((R, Hq, d)) * scale
    k = rng.standard_normal((n, Hkv, d))
    v = rng.standard_normal((n, Hkv, d))
    return q, k, v


# ------------------------------------------------------------------ softmax / mass
@pytest.mark.parametrize("w,a,G", [(4, 3, 2), (0, 5, 1), (6, 0, 3), (1, 1, 4)])
def test_rows_sum_to_one_and_mass_conservation(w, a, G):
    rng = np.random.default_rng(10 + w + a)
    Hkv, d, n = 2, 8, 37
    q, k, _ = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n)
    pos = orc.observation_positions(n, w, a)
    P = orc.attention_probs(q[:, 0], k[:, 0], pos, 0.3)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    raw = orc.raw_scores(q, k, w, 0.3)
    # every one of the R*G rows of a group distributes exactly one unit of probability
    np.testing.assert_allclose(raw.sum(axis=1), (w + a) * G, rtol=1e-12)
    assert (raw >= 0).all()


def test_causal_mask_closed_form_zero_queries():
    """Q = 0: every visible key of a row gets 1/(#visible).  Harmonic closed form."""
    w, a, G, Hkv, d, n = 5, 3, 2, 2, 4, 23
    m = n - w
    rng = np.random.default_rng(3)
    k = rng.standard_normal((n, Hkv, d))
    q = np.zeros((w + a, G * Hkv, d))
    raw = orc.raw_scores(q, k, w, 1.0)
    for g in range(Hkv):
        for j in range(n):
            first_window_row = max(0, j - m)   # window row i sees j iff j <= m + i
            want = G * (a / n + sum(1.0 / (m + i + 1) for i in range(first_window_row, w)))
            assert raw[g, j] == pytest.approx(want, rel=1e-13)


def test_window_rows_never_see_later_keys():
    """A huge key placed after a window row's position must not change that row."""
    w, a, n, d = 4, 0, 16, 4
    m = n - w
    rng = np.random.default_rng(5)
    q = rng.standard_normal((w, 1, d))
    k = rng.standard_normal((n, 1, d))
    pos = orc.observation_positions(n, w, a)
    P0 = orc.attention_probs(q[:, 0], k[:, 0], pos, 1.0)
    k2 = k.copy()
    k2[n - 1, 0] = 50.0 * q[w - 1, 0]               # last key: only the last window row may see it
    P1 = orc.attention_probs(q[:, 0], k2[:, 0], pos, 1.0)
    np.testing.assert_array_equal(P0[: w - 1], P1[: w - 1])
    assert P1[w - 1, n - 1] > 0.5
    assert pos.tolist() == [m, m + 1, m + 2, m + 3]


def test_lookahead_rows_see_whole_prompt():
    w, a, n, d = 2, 3, 11, 4
    rng = np.random.default_rng(6)
    q = rng.standard_normal((w + a, 1, d))
    k = rng.standard_normal((n, 1, d))
    pos = orc.observation_positions(n, w, a)
    P = orc.attention_probs(q[:, 0], k[:, 0], pos, 1.0)
    assert (P[w:] > 0).all()
    assert P[0, n - 1] == 0.0 and P[1, n - 1] > 0.0


def test_scores_match_torch_softmax_composition():
    """Independent library route: masked logits -> torch.softmax(float64) -> sums."""
    rng = np.random.default_rng(7)
    w, a, G, Hkv, d, n = 6, 5, 3, 2, 16, 97
    q, k, _ = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n, scale=0.7)
    sm = 1.0 / math.sqrt(d)
    raw = orc.raw_scores(q, k, w, sm)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    m = n - w
    want = torch.zeros(Hkv, n, dtype=torch.float64)
    for h in range(G * Hkv):
        g = h // G
        logits = torch.einsum("id,jd->ij", tq[:, h], tk[:, g]) * sm
        for i in range(w):
            logits[i, m + i + 1:] = float("-inf")
        want[g] += torch.softmax(logits, dim=1).sum(0)
    np.testing.assert_allclose(raw, want.numpy(), rtol=1e-12, atol=1e-15)


def test_softmax_lipschitz_lemma():
    """Lemma 1 / Theorem 1: logits moved by at most eps move the mean score by <= eps in l2.

    A perturbation of the queries q -> q + dq changes every logit by at most
    sm_scale * ||dq||_2 * max_j ||k_j||_2.
    """
    rng = np.random.default_rng(8)
    a, d, n = 7, 8, 64
    q = rng.standard_normal((a, 1, d))
    k = rng.standard_normal((n, 1, d))
    dq = 1e-2 * rng.standard_normal((a, 1, d))
    s0 = orc.raw_scores(q, k, 0, 0.5)[0] / a
    s1 = orc.raw_scores(q + dq, k, 0, 0.5)[0] / a
    eps = 0.5 * np.linalg.norm(dq, axis=-1).max() * np.linalg.norm(k, axis=-1).max()
    assert np.linalg.norm(s0 - s1) <= eps
    assert np.linalg.norm(s0 - s1) > 0


def test_oracle_matches_brute_force_end_to_end():
    for seed in range(6):
        rng = np.random.default_rng(100 + seed)
        w = int(rng.integers(0, 4))
        a = int(rng.integers(1 if w == 0 else 0, 4))
        G = int(rng.integers(1, 4))
        Hkv = int(rng.integers(1, 3))
        d = int(rng.integers(1, 5))
        n = int(rng.integers(max(w, 1) + 1, 20))
        pool_k = int(rng.choice([1, 3, 5, 7]))
        c_max = int(rng.integers(0, n + 2))
        q, k, v = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n, scale=1.5)
        got = orc.speckv_layer(q, k, v, w, pool_k, c_max, 0.8)
        want = bf.speckv_layer(q.tolist(), k.tolist(), v.tolist(), w, pool_k, c_max, 0.8)
        np.testing.assert_allclose(got["raw"], np.array(want["raw"]), rtol=1e-11, atol=1e-15)
        np.testing.assert_allclose(got["pooled"], np.array(want["pooled"]).reshape(Hkv, n - w),
                                   rtol=1e-11, atol=1e-15)
        assert got["idx"].tolist() == want["idx"]
        np.testing.assert_array_equal(got["k_out"], np.array(want["k_out"]).reshape(got["k_out"].shape))
        np.testing.assert_array_equal(got["v_out"], np.array(want["v_out"]).reshape(got["v_out"].shape))


# ------------------------------------------------------------------ pooling
@pytest.mark.parametrize("pool_k", [1, 2, 3, 4, 7, 8, 9, 64])
@pytest.mark.parametrize("m", [1, 2, 5, 64, 100])
def test_max_pool_matches_library_and_loop(pool_k, m):
    """Odd and even kernels: the library call with padding k // 2 (an even kernel yields m + 1
    outputs, of which the first m are the same-length result) and a scalar loop."""
    rng = np.random.default_rng(pool_k * 100 + m)
    x = rng.random((3, m))
    got = orc.max_pool_1d(x, pool_k)
    lib = F.max_pool1d(torch.from_numpy(x)[None], pool_k, stride=1, padding=pool_k // 2)[0].numpy()[:, :m]
    np.testing.assert_array_equal(got, lib)
    for r in range(3):
        assert got[r].tolist() == bf.max_pool(x[r].tolist(), pool_k)
    assert (got >= x).all()
    if pool_k == 1:
        np.testing.assert_array_equal(got, x)


def test_pooling_never_reads_window_columns():
    """Candidates are [0, m): a huge window-column score must not leak into m-1, m-2, ..."""
    raw = np.zeros((1, 20))
    raw[0, 16] = 9.0          # first window column with n_window = 4
    raw[0, 3] = 1.0
    pooled = orc.pooled_scores(raw, 4, 7)
    assert pooled.shape == (1, 16)
    assert pooled[0, 15] == 0.0 and pooled[0, 13] == 0.0
    assert pooled[0, :7].tolist() == [1.0] * 7 and pooled[0, 7] == 0.0


# ------------------------------------------------------------------ selection
def test_select_matches_exhaustive_subsets_with_ties():
    rng = np.random.default_rng(11)
    for trial in range(30):
        m = int(rng.integers(1, 11))
        base = rng.integers(0, 4, size=m).astype(np.float64)      # many exact ties
        pooled = orc.max_pool_1d(base, 3)
        count = int(rng.integers(0, m + 1))
        got = orc.select_top(pooled, count).tolist()
        assert got == bf.best_subset_exhaustive(pooled.tolist(), count)
        assert got == bf.select_top(pooled.tolist(), count)


def test_select_matches_library_stable_sort_and_is_optimal():
    rng = np.random.default_rng(12)
    x = np.round(rng.random(500), 2)                               # ties guaranteed
    for count in [0, 1, 17, 250, 499, 500]:
        got = orc.select_top(x, count)
        order = torch.sort(torch.from_numpy(x), descending=True, stable=True).indices[:count]
        assert got.tolist() == sorted(order.tolist())
        rest = np.setdiff1d(np.arange(500), got)
        if count and rest.size:
            assert x[got].min() >= x[rest].max()
        assert len(set(got.tolist())) == count


def test_boundary_tie_takes_smaller_index():
    pooled = np.array([1.0, 5.0, 5.0, 5.0, 2.0, 5.0])
    assert orc.select_top(pooled, 2).tolist() == [1, 2]
    assert orc.select_top(pooled, 4).tolist() == [1, 2, 3, 5]
    assert orc.keep_indices(pooled, 8, 2, 3).tolist() == [1, 2, 3, 6, 7]
    # budget larger than the candidates: keep everything, still ascending
    assert orc.keep_indices(pooled, 8, 2, 100).tolist() == list(range(8))


# ------------------------------------------------------------------ structure on the workloads
def _structure_checks(w, res, n, planted):
    m = n - w.n_window
    C = min(w.c_max, m)
    idx = res["idx"]
    assert idx.shape == (w.n_kv_heads, C + w.n_window)
    for g in range(w.n_kv_heads):
        row = idx[g]
        assert (np.diff(row) > 0).all()                            # ascending => unique
        assert row[0] >= 0 and row[-1] == n - 1
        assert row[C:].tolist() == list(range(m, n))               # window always kept, last
        assert (row[:C] < m).all()
        sel = set(row[:C].tolist())
        assert set(planted[g].tolist()) <= sel                     # planted heavy hitters survive
        rest = np.setdiff1d(np.arange(m), row[:C])
        if rest.size:
            assert res["pooled"][g][row[:C]].min() >= res["pooled"][g][rest].max()
    np.testing.assert_allclose(res["raw"].sum(axis=1), w.n_rows * w.group, rtol=1e-10)


def test_tiny_fp32_workload_structure_and_planted_keys():
    w = workloads.tiny_fp32()
    t = workloads.generate(w)
    q, k, v = (workloads.to_float64(t[x][0]) for x in ("q", "k", "v"))
    res = orc.speckv_layer(q[0], k, v, w.n_window, w.pool_k, w.c_max, w.sm_scale)
    _structure_checks(w, res, w.seq_lens[0], t["planted"][0, 0].numpy())
    # compaction is a bit copy of the float32 inputs
    for g in range(w.n_kv_heads):
        np.testing.assert_array_equal(res["k_out"][g], k[res["idx"][g], g])
        np.testing.assert_array_equal(res["v_out"][g], v[res["idx"][g], g])


def test_llama_shaped_workload_structure_small():
    w = workloads.llama8b_layer(n_in=2048, c_max=256, name="c2_small")
    t = workloads.generate(w)
    q, k, v = (workloads.to_float64(t[x][0]) for x in ("q", "k", "v"))
    res = orc.speckv_layer(q[0], k, v, w.n_window, w.pool_k, w.c_max, w.sm_scale)
    _structure_checks(w, res, 2048, t["planted"][0, 0].numpy())


def test_identity_compaction_when_budget_covers_prompt():
    rng = np.random.default_rng(13)
    q, k, v = _rand_case(rng, 5, 2, 2, 2, 4, 12)
    res = orc.speckv_layer(q, k, v, 2, 7, 1000, 1.0)
    for g in range(2):
        assert res["idx"][g].tolist() == list(range(12))
        np.testing.assert_array_equal(res["k_out"][g], k[:, g])
        np.testing.assert_array_equal(res["v_out"][g], v[:, g])


def test_ragged_batch_equals_per_sequence_calls():
    w = workloads.ragged_batch(n_layers=2, lo=70, hi=200, n_seqs=3, seed=4, name="c4_tiny")
    t = workloads.generate(w)
    q, k, v = (workloads.to_float64(t[x]) for x in ("q", "k", "v"))
    cu = w.cu_seqlens
    res = orc.speckv_batch(q, k, v, cu, w.n_window, w.pool_k, 16, w.sm_scale)
    for layer in range(2):
        for s in range(3):
            one = orc.speckv_layer(q[layer, s], k[layer, cu[s]:cu[s + 1]], v[layer, cu[s]:cu[s + 1]],
                                   w.n_window, w.pool_k, 16, w.sm_scale)
            assert res[layer][s]["idx"].tolist() == one["idx"].tolist()
            assert res[layer][s]["idx"].max() == w.seq_lens[s] - 1  # sequence-local indices


# ------------------------------------------------------------------ prompt-token selection
def test_specpc_expand_matches_set_arithmetic():
    rng = np.random.default_rng(14)
    for _ in range(20):
        n = int(rng.integers(5, 80))
        w = int(rng.integers(0, min(n, 6)))
        nb = int(rng.integers(0, 5))
        sel = np.sort(rng.choice(n - w, size=int(rng.integers(0, n - w)), replace=False))
        want = set(range(n - w, n))
        for t in sel.tolist():
            want |= {j for j in range(t - nb, t + nb + 1) if 0 <= j < n}
        got = orc.expand_neighbors(sel, n, w, nb)
        assert got.tolist() == sorted(want)


def test_specpc_sums_over_layers_and_heads_and_gathers_ids():
    w = workloads.specpc_draft(n_in=512, n_layers=3, name="c5_tiny")
    t = workloads.generate(w)
    ids = workloads.generate_token_ids(w, vocab=1000)
    q, k = workloads.to_float64(t["q"][:, 0]), workloads.to_float64(t["k"])
    res = orc.specpc_select_tokens(q, k, ids.numpy(), w.n_window, w.pool_k, 32, 2, w.sm_scale)
    per_layer = sum(orc.raw_scores(q[l], k[l], w.n_window, w.sm_scale).sum(0) for l in range(3))
    np.testing.assert_allclose(res["raw"], per_layer, rtol=1e-12)
    np.testing.assert_allclose(res["raw"].sum(), 3 * w.n_q_heads * w.n_window, rtol=1e-10)
    assert res["count"] == len(res["idx"]) and (np.diff(res["idx"]) > 0).all()
    assert res["idx"][-w.n_window:].tolist() == list(range(512 - w.n_window, 512))
    np.testing.assert_array_equal(res["ids"], ids.numpy()[res["idx"]])
    assert set(res["sel"].tolist()) <= set(res["idx"].tolist())
    assert res["ids"].dtype == np.int32


# ------------------------------------------------------------------ planted mistakes are caught
def test_pins_catch_planted_mistakes(monkeypatch):
    """Plant plausible mistakes into the oracle (on the CPU): a pin must fail for each."""
    w, a, G, Hkv, d, n = 5, 3, 2, 2, 4, 23

    def closed_form_ok():
        q = np.zeros((w + a, G * Hkv, d))
        k = np.random.default_rng(3).standard_normal((n, Hkv, d))
        raw = orc.raw_scores(q, k, w, 1.0)
        m = n - w
        want = G * (a / n + sum(1.0 / (m + i + 1) for i in range(w)))
        return abs(raw[0, 0] - want) < 1e-12 and abs(raw.sum() - Hkv * G * (w + a)) < 1e-9

    def brute_force_ok():
        rng = np.random.default_rng(21)
        q, k, v = _rand_case(rng, 4, 2, 4, 2, 3, 9)
        got = orc.raw_scores(q, k, 2, 0.9)
        return np.allclose(got, np.array(bf.raw_scores(q.tolist(), k.tolist(), 2, 0.9)), rtol=1e-11)

    assert closed_form_ok() and brute_force_ok()

    real_pos = orc.observation_positions
    monkeypatch.setattr(orc, "observation_positions", lambda *x: real_pos(*x) - 1)   # mask off by one
    assert not closed_form_ok()
    monkeypatch.setattr(orc, "observation_positions", real_pos)

    real_probs = orc.attention_probs
    monkeypatch.setattr(orc, "attention_probs",                                      # scale dropped
                        lambda q_, k_, pos, sm, lse=None: real_probs(q_, k_, pos, 1.0, lse))
    assert closed_form_ok() and not brute_force_ok()
    monkeypatch.setattr(orc, "attention_probs",                                      # keys reversed
                        lambda q_, k_, pos, sm, lse=None: real_probs(q_, k_[::-1], pos, sm, lse))
    assert not brute_force_ok()
    monkeypatch.setattr(orc, "attention_probs", real_probs)

    flipped = lambda p, c: np.sort(len(p) - 1 - np.argsort(-np.asarray(p)[::-1], kind="stable")[:c])
    assert flipped(np.array([1.0, 5.0, 5.0, 5.0]), 2).tolist() == [2, 3]            # larger index wins
    assert flipped(np.array([1.0, 5.0, 5.0, 5.0]), 2).tolist() != bf.best_subset_exhaustive([1.0, 5.0, 5.0, 5.0], 2)


# ------------------------------------------------------------------ golden facts from the paper
def test_golden_kv_cache_size(repo_root):
    """Sec. 1: 128K tokens of Llama-3.1-8B take over 16 GB of KV cache (16-bit)."""
    import os
    lines = [l for l in open(os.path.join(repo_root, "tests", "golden", "kv_cache_size.txt"))
             if l.strip() and not l.startswith("#")]
    fields = dict(l.split("=") for l in lines[0].split())
    w = workloads.llama8b_full_128k()
    size = 2 * w.seq_lens[0] * w.n_layers * w.n_kv_heads * w.head_dim * 2
    assert w.seq_lens[0] == int(fields["tokens"]) and size == int(fields["bytes"])
    assert size > 16e9


def test_stored_c1_expectation_is_current(repo_root):
    """The oracle still produces what tests/golden/make_c1_expected.py stored."""
    import importlib.util
    import os
    path = os.path.join(repo_root, "tests", "golden", "make_c1_expected.py")
    spec = importlib.util.spec_from_file_location("make_c1_expected", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(repo_root, "tests", "golden", "c1_expected.txt")).read().splitlines()
    now = mod.expected_lines()
    assert len(stored) == len(now)
    for a, b in zip(stored[1:], now[1:]):
        fa, fb = dict(x.split("=") for x in a.split()), dict(x.split("=") for x in b.split())
        assert fa["idx_sha"] == fb["idx_sha"] and fa["n_keep"] == fb["n_keep"]
        assert float(fa["pooled_sum"]) == pytest.approx(float(fb["pooled_sum"]), rel=1e-9)


# ------------------------------------------------------------------ max reduction / average pooling
def test_max_reduce_matches_library_and_brute_force():
    rng = np.random.default_rng(41)
    w, a, G, Hkv, d, n = 3, 4, 2, 2, 5, 29
    q, k, _ = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n, scale=1.3)
    got = orc.raw_scores(q, k, w, 0.7, reduce="max")
    m = n - w
    want = torch.zeros(Hkv, n, dtype=torch.float64)
    for h in range(G * Hkv):
        logits = torch.einsum("id,jd->ij", torch.from_numpy(q[:, h]), torch.from_numpy(k[:, h // G])) * 0.7
        for i in range(w):
            logits[i, m + i + 1:] = float("-inf")
        want[h // G] += torch.softmax(logits, dim=1).amax(dim=0)        # library route
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(got, np.array(bf.raw_scores(q.tolist(), k.tolist(), w, 0.7, "max")),
                               rtol=1e-11, atol=1e-15)
    total = orc.raw_scores(q, k, w, 0.7, reduce="sum")
    assert (got <= total + 1e-15).all() and (got * (w + a) >= total - 1e-12).all()   # max <= sum <= R * max


def test_max_reduce_closed_form_and_single_row():
    """Q = 0: a key's best row is the one that sees the fewest keys."""
    w, a, G, Hkv, d, n = 4, 2, 3, 1, 2, 17
    m = n - w
    k = np.random.default_rng(42).standard_normal((n, Hkv, d))
    raw = orc.raw_scores(np.zeros((w + a, G * Hkv, d)), k, w, 1.0, reduce="max")
    for j in range(n):
        first = max(0, j - m)                                   # first window row that sees key j
        assert raw[0, j] == pytest.approx(G * max(1.0 / n, 1.0 / (m + first + 1)), rel=1e-13)
    # a single observation row: max and sum coincide
    q1 = np.random.default_rng(43).standard_normal((1, G, d))
    np.testing.assert_allclose(orc.raw_scores(q1, k, 0, 1.0, reduce="max"),
                               orc.raw_scores(q1, k, 0, 1.0, reduce="sum"), rtol=1e-14)


def test_row_weights_and_head_max():
    rng = np.random.default_rng(44)
    w, a, G, Hkv, d, n = 4, 1, 2, 2, 3, 15
    q, k, _ = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n)
    wts = np.array([0.25, 0.5, 0.75, 1.0, 1.0])
    got = orc.raw_scores(q, k, w, 1.0, reduce="max", row_weights=wts, head_reduce="max")
    pos = orc.observation_positions(n, w, a)
    for g in range(Hkv):
        stack = np.stack([orc.attention_probs(q[:, h], k[:, g], pos, 1.0) * wts[:, None]
                          for h in range(g * G, (g + 1) * G)])
        np.testing.assert_allclose(got[g], stack.max(axis=(0, 1)), rtol=1e-14)


@pytest.mark.parametrize("pool_k", [1, 2, 3, 4, 7, 32, 64])
@pytest.mark.parametrize("m", [1, 4, 50, 130])
def test_avg_pool_matches_library_and_loop(pool_k, m):
    x = np.random.default_rng(pool_k + m).random((2, m))
    got = orc.avg_pool_1d(x, pool_k)
    lib = F.avg_pool1d(torch.from_numpy(x)[None], pool_k, stride=1, padding=pool_k // 2,
                       count_include_pad=True)[0].numpy()[:, :m]
    np.testing.assert_allclose(got, lib, rtol=1e-13, atol=1e-16)
    for r in range(2):
        np.testing.assert_allclose(got[r], bf.avg_pool(x[r].tolist(), pool_k), rtol=1e-13)
    # mass identity: x[j] is counted once by every output whose window holds j, i.e. by the
    # outputs j - (k-1)//2 .. j + k//2 that exist
    covers = [min(m - 1, j + pool_k // 2) - max(0, j - (pool_k - 1) // 2) + 1 for j in range(m)]
    np.testing.assert_allclose(got.sum(), sum(x[:, j].sum() * covers[j] for j in range(m)) / pool_k, rtol=1e-12)


def test_even_pooling_kernels_on_a_hand_worked_row():
    """k = 2 looks one position back, k = 4 two back and one ahead (hyper-parameter table, SpecPC
    column: kernel sizes 64 / 32).  The mirrored convention (more positions ahead than back) gives
    different numbers, so a flipped window cannot pass."""
    x = np.array([1.0, 2.0, 3.0, 4.0])
    assert orc.pool_window(2) == (1, 0) and orc.pool_window(4) == (2, 1) and orc.pool_window(7) == (3, 3)
    assert orc.max_pool_1d(x, 2).tolist() == [1.0, 2.0, 3.0, 4.0]
    assert orc.avg_pool_1d(x, 2).tolist() == [0.5, 1.5, 2.5, 3.5]
    assert orc.max_pool_1d(x, 4).tolist() == [2.0, 3.0, 4.0, 4.0]
    assert orc.avg_pool_1d(x, 4).tolist() == [0.75, 1.5, 2.5, 2.25]
    mirrored_max_k2 = [max(x[j:j + 2]) for j in range(4)]              # j .. j + 1
    assert mirrored_max_k2 != orc.max_pool_1d(x, 2).tolist()
    assert bf.max_pool(x.tolist(), 4) == [2.0, 3.0, 4.0, 4.0] and bf.avg_pool(x.tolist(), 2) == [0.5, 1.5, 2.5, 3.5]


def test_paper_setting_end_to_end_vs_brute_force():
    """Max reduction + average pooling (the Alg. 1 listing) through the whole path."""
    for seed in range(4):
        rng = np.random.default_rng(200 + seed)
        w, a, G, Hkv, d = int(rng.integers(0, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 3)), 2, 3
        n = int(rng.integers(w + 2, 16))
        q, k, v = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n, scale=1.5)
        for reduce, pool in (("max", "avg"), ("max", "max"), ("sum", "avg")):
            got = orc.speckv_layer(q, k, v, w, 5, 4, 0.9, reduce=reduce, pool=pool)
            want = bf.speckv_layer(q.tolist(), k.tolist(), v.tolist(), w, 5, 4, 0.9, reduce, pool)
            np.testing.assert_allclose(got["pooled"], np.array(want["pooled"]).reshape(Hkv, n - w), rtol=1e-11, atol=1e-15)
            assert got["idx"].tolist() == want["idx"]


# ------------------------------------------------------------------ prompt compression (Alg. 2)
@pytest.mark.parametrize("pk,nn", [(5, 9), (6, 8), (64, 32)])
def test_specpc_alg2_matches_library_composition(pk, nn):
    w = workloads.specpc_draft(n_in=300, n_layers=4, name="c5_alg2")
    w = workloads.SpecKVWorkload(**{**w.__dict__, "n_lookahead": 2})
    t = workloads.generate(w)
    ids = workloads.generate_token_ids(w, vocab=5000)
    q, k = workloads.to_float64(t["q"][:, 0]), workloads.to_float64(t["k"])
    n, nw, l_skip, cm = 300, w.n_window, 1, 40
    res = orc.specpc_compress_prompt(q, k, ids.numpy(), nw, pk, nn, cm, l_skip, w.sm_scale)
    # library route: stack the weighted probabilities and take one amax over layers, heads, rows
    m = n - nw
    G = w.group
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    wts = torch.ones(w.n_rows, dtype=torch.float64)
    wts[:nw] = (torch.arange(nw, dtype=torch.float64) + 1) / nw          # j / n_window, j = 1..n_window
    best = torch.zeros(n, dtype=torch.float64)
    for layer in range(l_skip, w.n_layers):
        for h in range(w.n_q_heads):
            logits = torch.einsum("id,jd->ij", tq[layer, :, h], tk[layer, :, h // G]) * w.sm_scale
            for i in range(nw):
                logits[i, m + i + 1:] = float("-inf")
            best = torch.maximum(best, (torch.softmax(logits, 1) * wts[:, None]).amax(0))
    np.testing.assert_allclose(res["raw"], best.numpy(), rtol=1e-12)
    s1 = F.avg_pool1d(best[None, None, :m], pk, stride=1, padding=pk // 2)[..., :m]
    s2 = F.max_pool1d(s1, nn, stride=1, padding=nn // 2)[0, 0, :m]
    np.testing.assert_allclose(res["pooled"], s2.numpy(), rtol=1e-12)
    order = torch.sort(s2, descending=True, stable=True).indices[:cm]
    assert res["sel"].tolist() == sorted(order.tolist())
    assert res["idx"].tolist() == sorted(order.tolist()) + list(range(m, n))
    np.testing.assert_array_equal(res["ids"], ids.numpy()[res["idx"]])
    # layers below l_skip must not matter
    q2 = q.copy()
    q2[0] *= 3.0
    np.testing.assert_array_equal(orc.specpc_compress_prompt(q2, k, ids.numpy(), nw, pk, nn, cm, l_skip,
                                                             w.sm_scale)["idx"], res["idx"])
    assert orc.specpc_window_weights(4, 6).tolist() == [0.25, 0.5, 0.75, 1.0, 1.0, 1.0]


# ------------------------------------------------------------------ caller-supplied normalisers
def test_supplied_lse_reduces_to_the_default_and_scales():
    rng = np.random.default_rng(51)
    w, a, G, Hkv, d, n = 3, 2, 2, 2, 4, 21
    q, k, _ = _rand_case(rng, w + a, w, G * Hkv, Hkv, d, n, scale=1.2)
    pos = orc.observation_positions(n, w, a)
    lse = np.stack([orc.row_lse(q[:, h], k[:, h // G], pos, 0.6) for h in range(G * Hkv)], axis=1)   # [R, Hq]
    # independent check of row_lse against the library
    for h in range(G * Hkv):
        logits = torch.from_numpy(0.6 * q[:, h] @ k[:, h // G].T)
        for i in range(w + a):
            logits[i, pos[i] + 1:] = float("-inf")
        np.testing.assert_allclose(lse[:, h], torch.logsumexp(logits, dim=1).numpy(), rtol=1e-13)
    base = orc.raw_scores(q, k, w, 0.6)
    np.testing.assert_allclose(orc.raw_scores(q, k, w, 0.6, lse_in=lse), base, rtol=1e-12)
    # a normaliser larger by ln 2 (half the mass elsewhere) halves every score
    np.testing.assert_allclose(orc.raw_scores(q, k, w, 0.6, lse_in=lse + math.log(2.0)), base / 2, rtol=1e-12)
    # masked entries stay zero with a supplied normaliser
    P = orc.attention_probs(q[:, 0], k[:, 0], pos, 0.6, lse[:, 0])
    assert P[0, n - 1] == 0.0 and P[w, n - 1] > 0.0


# --------------------------------------------------------------------------- #
# Shared layer budget across KV heads (App. "Integration and Comparison with the AdaKV Baseline")
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("seed", range(6))
def test_ada_counts_match_brute_force_and_invariants(seed):
    rng = np.random.default_rng(seed)
    H, m = int(rng.integers(1, 5)), int(rng.integers(4, 40))
    count = int(rng.integers(0, m + 1))
    floor = int(rng.integers(0, count + 3))
    levels = int(rng.choice([3, 10, 10 ** 6]))                    # heavy ties included
    pooled = rng.integers(0, levels, size=(H, m)).astype(np.float64) / levels
    got = orc.ada_head_counts(pooled, count, floor)
    assert got.tolist() == bf.ada_head_counts(pooled.tolist(), count, floor)
    assert got.sum() == H * count
    assert got.min() >= min(floor, count) and got.max() <= m


@pytest.mark.parametrize("seed", range(5))
def test_ada_allocation_keeps_the_largest_total_score(seed):
    """The rule is the allocation that maximises the retained pooled mass under the floor:
    checked against every allocation on small inputs."""
    rng = np.random.default_rng(100 + seed)
    H, m = 3, 7
    count = int(rng.integers(1, 6))
    floor = int(rng.integers(0, count + 1))
    pooled = rng.random((H, m))
    counts = orc.ada_head_counts(pooled, count, floor)
    kept = sum(np.sort(pooled[h])[::-1][:counts[h]].sum() for h in range(H))
    assert kept == pytest.approx(bf.best_allocation_exhaustive(pooled.tolist(), count, floor), rel=1e-12)


def test_ada_floor_extremes_reduce_to_plain_selections():
    rng = np.random.default_rng(7)
    H, m, count, w = 4, 50, 9, 3
    pooled = rng.random((H, m))
    # floor = C: equal budgets, the ordinary per-head selection
    idx = orc.ada_keep_indices(pooled, m + w, w, count, floor=count)
    for g in range(H):
        assert idx[g].tolist() == orc.keep_indices(pooled[g], m + w, w, count).tolist()
    # floor = 0: the H*C largest entries of the layer (library sort of the flattened scores)
    idx0 = orc.ada_keep_indices(pooled, m + w, w, count, floor=0)
    flat_top = np.argsort(-pooled.reshape(-1), kind="stable")[:H * count]
    want = sorted((int(t) // m, int(t) % m) for t in flat_top)
    got = sorted((g, int(j)) for g in range(H) for j in idx0[g][:-w])
    assert got == want


def test_ada_tie_rule_prefers_smaller_head_then_index():
    pooled = np.array([[1.0, 0.5, 0.5, 0.0], [0.5, 0.5, 0.9, 0.0]])
    # C = 2 per head, floor 1: floors are (0,0) and (1,2); two more slots among the 0.5 ties
    counts = orc.ada_head_counts(pooled, 2, 1)
    assert counts.tolist() == [3, 1]
    idx = orc.ada_keep_indices(pooled, 4, 0, 2, 1)
    assert idx[0].tolist() == [0, 1, 2] and idx[1].tolist() == [2]


def _ada_tiny():
    w = workloads.SpecKVWorkload(name="ada_tiny", n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=8,
                                 seq_lens=(40,), n_window=4, n_lookahead=3, pool_k=3, c_max=6,
                                 dtype="f32", sm_scale=0.5, n_planted=2)
    t = workloads.generate(w)
    q, k, v = (workloads.to_float64(t[x][0]) for x in ("q", "k", "v"))
    return q[0], k, v


@pytest.mark.parametrize("floor", [0, 2, 6, 9])
def test_ada_layer_end_to_end_against_brute_force(floor):
    """speckv_layer_ada and compact_ragged against the loops-only brute force of the same path:
    indices, head offsets and the gathered K and V rows."""
    q, k, v = _ada_tiny()
    out = orc.speckv_layer_ada(q, k, v, 4, 3, 6, floor, 0.5)
    ref = bf.speckv_layer_ada(q.tolist(), k.tolist(), v.tolist(), 4, 3, 6, floor, 0.5)
    assert [i.tolist() for i in out["idx"]] == ref["idx"]
    assert out["head_off"].tolist() == ref["head_off"]
    assert out["head_off"][-1] == 2 * (6 + 4)                      # the layer total never moves
    assert out["k_out"].shape == (ref["head_off"][-1], 8)
    assert out["k_out"].tolist() == ref["k_out"]
    assert out["v_out"].tolist() == ref["v_out"]
    # K and V differ, so a swap of the two tensors could not pass
    assert out["k_out"].tolist() != out["v_out"].tolist()


def test_compact_ragged_against_hand_written_rows():
    """Two heads with different counts on a tensor whose entries name their own position."""
    n, H, d = 6, 2, 3
    x = np.array([[[100 * j + 10 * g + c for c in range(d)] for g in range(H)] for j in range(n)], dtype=np.float64)
    idx = [np.array([4, 1]), np.array([0, 2, 5])]
    want = [[400, 401, 402], [100, 101, 102], [10, 11, 12], [210, 211, 212], [510, 511, 512]]
    assert orc.compact_ragged(x, idx).tolist() == want
    assert bf.compact_ragged(x.tolist(), [i.tolist() for i in idx]) == want


def test_planted_wrong_head_in_the_ragged_gather_is_caught():
    """A gather that reads every row from head 0 (a dropped head index) must fail the pin."""
    q, k, v = _ada_tiny()
    ref = bf.speckv_layer_ada(q.tolist(), k.tolist(), v.tolist(), 4, 3, 6, 2, 0.5)
    wrong = np.concatenate([k[np.asarray(ref["idx"][g]), 0, :] for g in range(2)], axis=0)
    assert wrong.tolist() != ref["k_out"]
    shifted = np.concatenate([k[np.asarray(ref["idx"][g]), (g + 1) % 2, :] for g in range(2)], axis=0)
    assert shifted.tolist() != ref["k_out"]
