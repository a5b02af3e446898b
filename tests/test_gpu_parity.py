"""GPU parity: the HIP library (through its C ABI) against the CPU float64 oracle.

Inputs are seeded and synthetic (module `workloads`); both sides consume the same
bits.  Bars: scores within 2e-3 relative (plus a 1e-6 * row-max absolute floor);
index sets exact except where the oracle's own score gap at the budget boundary is
below that tolerance; selection on given scores and compaction on given indices
bit-exact.
"""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import speckv_oracle as orc

pytestmark = pytest.mark.gpu

REL_TOL = 2e-3
ABS_FLOOR = 1e-6


@pytest.fixture(scope="module")
def S():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_08373_amd as lib
    lib.load_library()            # raises if the HIP library is missing: no fallback
    return lib


def make_params(S, w, c_max=None, pool_k=None, q=None, k=None, reduce="sum", pool="max"):
    if q is not None:
        return S.SpecKVParams.for_tensors(q, k, seq_lens=w.seq_lens, n_window=w.n_window,
                                          pool_k=w.pool_k if pool_k is None else pool_k,
                                          c_max=w.c_max if c_max is None else c_max,
                                          sm_scale=w.sm_scale, reduce=reduce, pool=pool)
    return S.SpecKVParams(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                          head_dim=w.head_dim, seq_lens=w.seq_lens, n_window=w.n_window,
                          n_lookahead=w.n_lookahead, pool_k=w.pool_k if pool_k is None else pool_k,
                          c_max=w.c_max if c_max is None else c_max, sm_scale=w.sm_scale,
                          dtype=w.torch_dtype, reduce=reduce, pool=pool)


def alloc_ws(S, p):
    return torch.empty(max(S.workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")


def oracle_batch(w, t, c_max=None, pool_k=None, reduce="sum", pool="max"):
    q, k, v = (workloads.to_float64(t[x]) for x in ("q", "k", "v"))
    return orc.speckv_batch(q, k, v, w.cu_seqlens, w.n_window,
                            w.pool_k if pool_k is None else pool_k,
                            w.c_max if c_max is None else c_max, w.sm_scale, reduce=reduce, pool=pool)


def split_scores(w, flat, layer, s):
    """[L, Hkv*T] flat scores -> [Hkv, n_s] view of one (layer, sequence)."""
    cu = w.cu_seqlens
    n = w.seq_lens[s]
    a = w.n_kv_heads * cu[s]
    return flat[layer, a:a + w.n_kv_heads * n].reshape(w.n_kv_heads, n)


def split_keep(w, flat, layer, s, c_max, trailing=()):
    keeps = [min(c_max, n - w.n_window) + w.n_window for n in w.seq_lens]
    ck = np.concatenate([[0], np.cumsum(keeps)])
    a = w.n_kv_heads * ck[s]
    return flat[layer, a:a + w.n_kv_heads * keeps[s]].reshape((w.n_kv_heads, keeps[s]) + tuple(trailing))


def assert_scores_close(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == want.shape, what
    if want.size == 0:
        return
    tol = REL_TOL * np.abs(want) + ABS_FLOOR * np.abs(want).max(axis=-1, keepdims=True)
    bad = np.abs(got - want) > tol
    assert not bad.any(), "%s: %d entries off, worst rel err %.3e" % (
        what, bad.sum(), (np.abs(got - want) / np.maximum(np.abs(want), 1e-300)).max())


def assert_indices_valid(idx_row, pooled_ref_row, n, w_, c_max, what):
    """Exact where the oracle's decision is unambiguous; any choice inside the tolerance band."""
    m = n - w_
    C = min(c_max, m)
    idx_row = np.asarray(idx_row, dtype=np.int64)
    assert idx_row.shape == (C + w_,), what
    assert (np.diff(idx_row) > 0).all(), what + ": not strictly ascending"
    assert idx_row[C:].tolist() == list(range(m, n)), what + ": window not kept last"
    if C == 0:
        return True
    sel = idx_row[:C]
    assert sel.min() >= 0 and sel.max() < m, what
    want = orc.select_top(pooled_ref_row, C)
    if np.array_equal(sel, want):
        return True
    tau = np.sort(pooled_ref_row)[m - C]                 # C-th largest oracle score
    band = REL_TOL * abs(tau) + ABS_FLOOR * np.abs(pooled_ref_row).max()
    must = np.nonzero(pooled_ref_row > tau + band)[0]
    never = np.nonzero(pooled_ref_row < tau - band)[0]
    assert np.isin(must, sel).all(), what + ": a clearly better key was dropped"
    assert not np.isin(never, sel).any(), what + ": a clearly worse key was kept"
    return False


def assert_ada_indices_in_band(got_rows, pooled_ref, want_rows, w_, f, what):
    """Shared layer budget: index-by-index check against the oracle's pooled scores.  The layer-wide
    threshold tau is the smallest score the oracle keeps; a head whose floor reaches below tau has
    its own f-th largest score as threshold.  Outside the tolerance band around its threshold every
    key of a head must be decided as the oracle decides it."""
    H, m = pooled_ref.shape
    kept = np.concatenate([pooled_ref[g][np.asarray(want_rows[g][:len(want_rows[g]) - w_], dtype=np.int64)]
                           for g in range(H)])
    if kept.size == 0:
        return
    tau = kept.min()
    band = REL_TOL * abs(tau) + ABS_FLOOR * np.abs(pooled_ref).max()
    for g in range(H):
        sel = np.asarray(got_rows[g][:len(got_rows[g]) - w_], dtype=np.int64)
        thr = tau if f == 0 else min(tau, np.sort(pooled_ref[g])[m - f])
        must = np.nonzero(pooled_ref[g] > thr + band)[0]
        never = np.nonzero(pooled_ref[g] < thr - band)[0]
        assert np.isin(must, sel).all(), what + " head %d: a clearly better key was dropped" % g
        assert not np.isin(never, sel).any(), what + " head %d: a clearly worse key was kept" % g


def run_compress(S, w, t_gpu, c_max=None, pool_k=None, reduce="sum", pool="max"):
    p = make_params(S, w, c_max=c_max, pool_k=pool_k, reduce=reduce, pool=pool)
    KT = S.total_keep(p)
    L, H, d = w.n_layers, w.n_kv_heads, w.head_dim
    idx = torch.full((L, H * KT), -7, dtype=torch.int32, device="cuda")
    k_out = torch.zeros((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
    v_out = torch.zeros_like(k_out)
    ws = alloc_ws(S, p)
    S.speckv_compress(p, t_gpu["q"], t_gpu["k"], t_gpu["v"], idx, k_out, v_out, ws)
    torch.cuda.synchronize()
    return p, idx.cpu().numpy(), k_out.cpu(), v_out.cpu()


def check_full_path(S, w, c_max=None, pool_k=None, expect_exact=None, reduce="sum", pool="max"):
    c_eff = w.c_max if c_max is None else c_max
    t = workloads.generate(w)
    tg = {x: t[x].cuda() for x in ("q", "k", "v")}
    ref = oracle_batch(w, t, c_max=c_max, pool_k=pool_k, reduce=reduce, pool=pool)

    # --- scores
    p = make_params(S, w, c_max=c_max, pool_k=pool_k, reduce=reduce, pool=pool)
    L, H, T = w.n_layers, w.n_kv_heads, w.total_tokens
    pooled = torch.full((L, H * T), -1.0, dtype=torch.float32, device="cuda")
    raw = torch.full((L, H * T), -1.0, dtype=torch.float32, device="cuda")
    ws = alloc_ws(S, p)
    S.speckv_score(p, tg["q"], tg["k"], pooled, raw, ws)
    torch.cuda.synchronize()
    pooled_h, raw_h = pooled.cpu().numpy(), raw.cpu().numpy()
    for layer in range(L):
        for s in range(w.n_seqs):
            n = w.seq_lens[s]
            m = n - w.n_window
            r = ref[layer][s]
            assert_scores_close(split_scores(w, raw_h, layer, s), r["raw"], "raw l%d s%d" % (layer, s))
            got_p = split_scores(w, pooled_h, layer, s)
            assert_scores_close(got_p[:, :m], r["pooled"], "pooled l%d s%d" % (layer, s))
            assert (got_p[:, m:] == 0).all()

    # --- fused path: indices and compacted cache
    _, idx_h, k_out, v_out = run_compress(S, w, tg, c_max=c_max, pool_k=pool_k, reduce=reduce, pool=pool)
    exact = 0
    total = 0
    cu = w.cu_seqlens
    for layer in range(L):
        for s in range(w.n_seqs):
            n = w.seq_lens[s]
            r = ref[layer][s]
            idx_ls = split_keep(w, idx_h, layer, s, c_eff)
            ko = split_keep(w, k_out.view(torch.int16 if w.dtype != "f32" else torch.int32).numpy(),
                            layer, s, c_eff, trailing=(w.head_dim,))
            vo = split_keep(w, v_out.view(torch.int16 if w.dtype != "f32" else torch.int32).numpy(),
                            layer, s, c_eff, trailing=(w.head_dim,))
            kin = t["k"][layer, cu[s]:cu[s + 1]].view(torch.int16 if w.dtype != "f32" else torch.int32).numpy()
            vin = t["v"][layer, cu[s]:cu[s + 1]].view(torch.int16 if w.dtype != "f32" else torch.int32).numpy()
            for g in range(H):
                total += 1
                exact += assert_indices_valid(idx_ls[g], r["pooled"][g], n, w.n_window, c_eff,
                                              "idx l%d s%d g%d" % (layer, s, g))
                # gathered rows are bit copies of the rows the library itself selected
                np.testing.assert_array_equal(ko[g], kin[idx_ls[g], g])
                np.testing.assert_array_equal(vo[g], vin[idx_ls[g], g])
                # selection is exact integer work on the library's own fp32 scores
                m = n - w.n_window
                got_p = split_scores(w, pooled_h, layer, s)[g, :m]
                assert idx_ls[g][:min(c_eff, m)].tolist() == orc.select_top(got_p, min(c_eff, m)).tolist()
    if expect_exact is not None:
        assert exact >= expect_exact * total, "only %d of %d index rows equal the oracle's" % (exact, total)
    return exact, total


# ------------------------------------------------------------------ whole path
def test_tiny_fp32_workload(S):
    exact, total = check_full_path(S, workloads.tiny_fp32(), expect_exact=1.0)
    assert total == 2


def test_llama8b_single_layer_4k(S):
    check_full_path(S, workloads.llama8b_layer(n_in=4096 + 77, c_max=512, name="c2_4k"), expect_exact=0.5)


def test_llama8b_two_layers_ragged_tail(S):
    # spans several LDS tiles and chunks, ends in a ragged tile, two layers
    check_full_path(S, workloads.llama8b_layer(n_in=3000, c_max=300, n_layers=2, name="c2_3000"))


def test_ragged_batch_gqa7(S):
    w = workloads.ragged_batch(n_layers=2, lo=200, hi=2500, n_seqs=4, seed=4, name="c4_small")
    check_full_path(S, w, c_max=128)


def test_head_dim_64_bf16(S):
    w = workloads.specpc_draft(n_in=2048 + 5, n_layers=2, name="c5_shape_as_speckv")
    check_full_path(S, w, c_max=100)


@pytest.mark.parametrize("n_in,c_max,n_window,n_lookahead,pool_k", [
    (64, 1000, 64, 3, 7),      # m = 0: only the window survives
    (65, 0, 64, 64, 7),        # zero budget
    (130, 10_000, 2, 1, 1),    # budget above m, pool_k = 1, a single lookahead row
    (33, 5, 0, 16, 3),         # no window at all
    (129, 17, 16, 0, 255),     # window rows only, widest pool
    (1, 1, 0, 1, 7),           # a single key
])
def test_degenerate_shapes(S, n_in, c_max, n_window, n_lookahead, pool_k):
    w = workloads.SpecKVWorkload(
        name="edge", n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=64, seq_lens=(n_in,),
        n_window=n_window, n_lookahead=n_lookahead, pool_k=pool_k, c_max=c_max, dtype="bf16",
        sm_scale=0.125, n_planted=0, channel_scale=(0.5, 4.0), seed=21)
    check_full_path(S, w)


def test_fp32_head_dim_128_and_group_1(S):
    w = workloads.SpecKVWorkload(
        name="f32_d128", n_layers=1, n_q_heads=2, n_kv_heads=2, head_dim=128, seq_lens=(700,),
        n_window=8, n_lookahead=24, pool_k=5, c_max=64, dtype="f32", sm_scale=1 / math.sqrt(128),
        n_planted=4, channel_scale=None, seed=22)
    check_full_path(S, w, expect_exact=1.0)


# ------------------------------------------------------------------ the listing's setting
@pytest.mark.parametrize("reduce,pool", [("max", "max"), ("max", "avg"), ("sum", "avg")])
def test_max_reduction_and_average_pooling_llama_shape(S, reduce, pool):
    """Alg. 1 as printed: max over the observation rows of a head, average pooling."""
    w = workloads.llama8b_layer(n_in=4096 + 300, c_max=512, name="c2_maxavg")
    check_full_path(S, w, reduce=reduce, pool=pool)


@pytest.mark.parametrize("pool_k,pool", [(2, "max"), (8, "avg"), (64, "max")])
def test_even_pooling_kernels(S, pool_k, pool):
    """Even kernels look one position further back than ahead (window j - k/2 .. j + k/2 - 1)."""
    w = workloads.llama8b_layer(n_in=3000 + 41, c_max=300, name="even_pool")
    check_full_path(S, w, pool_k=pool_k, pool=pool)


def test_max_reduction_ragged_gqa7_and_tiny(S):
    w = workloads.ragged_batch(n_layers=2, lo=150, hi=1500, n_seqs=3, seed=9, name="c4_max")
    check_full_path(S, w, c_max=100, reduce="max", pool="avg")
    check_full_path(S, workloads.tiny_fp32(), reduce="max", pool="max")


@pytest.mark.parametrize("n_window,n_lookahead,G", [
    (32, 64, 4),      # the paper's window with 64 draft tokens: 96 rows per head
    (5, 8, 3),        # rows per head far from a multiple of 32
    (64, 500, 2),     # a head larger than one workgroup's 512 rows
    (0, 1, 8),        # a single row per head
])
@pytest.mark.parametrize("reduce", ["sum", "max"])
def test_row_layouts(S, n_window, n_lookahead, G, reduce):
    w = workloads.SpecKVWorkload(
        name="rows", n_layers=1, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, seq_lens=(777,),
        n_window=n_window, n_lookahead=n_lookahead, pool_k=7, c_max=60, dtype="bf16",
        sm_scale=1 / math.sqrt(128), n_planted=4, channel_scale=(0.5, 4.0), seed=23)
    check_full_path(S, w, reduce=reduce)


def test_strided_inputs(S):
    """q and k/v views with non-contiguous strides (fused QKV-style buffers)."""
    w = workloads.llama8b_layer(n_in=1500, c_max=200, name="strided")
    t = workloads.generate(w)
    L, T, H, d = t["k"].shape
    big = torch.zeros(L, T, 3, H, d, dtype=t["k"].dtype, device="cuda")
    big[:, :, 1] = t["k"].cuda()
    big[:, :, 2] = t["v"].cuda()
    kview, vview = big[:, :, 1], big[:, :, 2]
    qbig = torch.zeros(L, 1, w.n_rows, w.n_q_heads, 2 * d, dtype=t["q"].dtype, device="cuda")
    qbig[..., :d] = t["q"].cuda()
    qview = qbig[..., :d]
    p = S.SpecKVParams.for_tensors(qview, kview, seq_lens=w.seq_lens, n_window=w.n_window,
                                   pool_k=w.pool_k, c_max=w.c_max, sm_scale=w.sm_scale)
    KT = S.total_keep(p)
    idx = torch.empty((L, H * KT), dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
    v_out = torch.empty_like(k_out)
    ws = alloc_ws(S, p)
    S.speckv_compress(p, qview, kview, vview, idx, k_out, v_out, ws)
    p2, idx2, k2, v2 = run_compress(S, w, {x: t[x].cuda() for x in ("q", "k", "v")})
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), idx2)
    assert torch.equal(k_out.cpu(), k2) and torch.equal(v_out.cpu(), v2)


def test_bitwise_reproducible(S):
    w = workloads.llama8b_layer(n_in=5000, c_max=400, name="repro")
    t = workloads.generate(w)
    tg = {x: t[x].cuda() for x in ("q", "k", "v")}
    a = run_compress(S, w, tg)
    b = run_compress(S, w, tg)
    np.testing.assert_array_equal(a[1], b[1])
    assert torch.equal(a[2], b[2]) and torch.equal(a[3], b[3])


# ------------------------------------------------------------------ stages on given inputs
def test_select_on_given_scores_is_bit_exact(S):
    """Plateaus from max-pooling make boundary ties the norm; both sides decide in fp32."""
    rng = np.random.default_rng(31)
    w = workloads.SpecKVWorkload(
        name="sel", n_layers=2, n_q_heads=4, n_kv_heads=4, head_dim=64, seq_lens=(5000, 37, 12345),
        n_window=32, n_lookahead=1, pool_k=7, c_max=777, dtype="bf16", sm_scale=1.0)
    p = make_params(S, w)
    L, H, T = 2, 4, w.total_tokens
    base = np.round(rng.random((L, H * T)) * 50).astype(np.float32) / 8      # heavy ties
    base[0, :100] = -base[0, :100]                                            # negative scores too
    base[1, 5:9] = 0.0
    base[1, 6] = -0.0
    pooled = torch.from_numpy(base).cuda()
    KT = S.total_keep(p)
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    S.speckv_select(p, pooled, idx)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    for layer in range(L):
        for s in range(3):
            n = w.seq_lens[s]
            rows = split_scores(w, base, layer, s)
            got = split_keep(w, idx_h, layer, s, w.c_max)
            for g in range(H):
                want = orc.keep_indices(rows[g, :n - 32].astype(np.float64), n, 32, w.c_max)
                assert got[g].tolist() == want.tolist()


def test_compact_on_given_indices_is_bit_exact(S):
    w = workloads.SpecKVWorkload(
        name="cmp", n_layers=3, n_q_heads=4, n_kv_heads=2, head_dim=128, seq_lens=(300, 41),
        n_window=8, n_lookahead=1, pool_k=7, c_max=50, dtype="bf16", sm_scale=1.0)
    t = workloads.generate(w)
    p = make_params(S, w)
    KT = S.total_keep(p)
    rng = np.random.default_rng(32)
    idx_h = np.zeros((3, 2 * KT), dtype=np.int32)
    for layer in range(3):
        for s in range(2):
            view = split_keep(w, idx_h, layer, s, w.c_max)
            view[...] = rng.integers(0, w.seq_lens[s], size=view.shape)       # arbitrary, repeated, unsorted
    idx_h[0, 3] = -5                                                          # out of range -> zero row
    idx_h[1, 7] = 10 ** 6
    idx = torch.from_numpy(idx_h).cuda()
    k_out = torch.full((3, 2 * KT, 128), 9.0, dtype=torch.bfloat16, device="cuda")
    v_out = torch.full_like(k_out, 9.0)
    S.speckv_compact(p, t["k"].cuda(), t["v"].cuda(), idx, k_out, v_out)
    k_only = torch.full_like(k_out, 9.0)
    S.speckv_compact(p, t["k"].cuda(), None, idx, k_only, None)
    torch.cuda.synchronize()
    cu = w.cu_seqlens
    for name, out, src in (("k", k_out, t["k"]), ("v", v_out, t["v"]), ("k_only", k_only, t["k"])):
        out_h = out.cpu().view(torch.int16).numpy()
        for layer in range(3):
            for s in range(2):
                rows = split_keep(w, out_h, layer, s, w.c_max, trailing=(128,))
                ids = split_keep(w, idx_h, layer, s, w.c_max)
                sin = src[layer, cu[s]:cu[s + 1]].view(torch.int16).numpy()
                for g in range(2):
                    ok = (ids[g] >= 0) & (ids[g] < w.seq_lens[s])
                    np.testing.assert_array_equal(rows[g][ok], sin[ids[g][ok], g])
                    assert (rows[g][~ok] == 0).all()


# ------------------------------------------------------------------ prompt-token selection
@pytest.mark.parametrize("n_in,top_k,nb", [(3000, 200, 8), (700, 5000, 0), (257, 1, 300)])
def test_specpc_select_tokens(S, n_in, top_k, nb):
    w = workloads.specpc_draft(n_in=n_in, n_layers=3, name="c5_small")
    t = workloads.generate(w)
    ids = workloads.generate_token_ids(w)
    ref = orc.specpc_select_tokens(workloads.to_float64(t["q"][:, 0]), workloads.to_float64(t["k"]),
                                   ids.numpy(), w.n_window, w.pool_k, top_k, nb, w.sm_scale)
    p = make_params(S, w)
    ws = torch.empty(S.specpc_workspace_bytes(p, top_k), dtype=torch.uint8, device="cuda")
    idx_out = torch.full((n_in,), -1, dtype=torch.int32, device="cuda")
    ids_out = torch.full((n_in,), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    S.specpc_select_tokens(p, top_k, nb, t["q"].cuda(), t["k"].cuda(), ids.cuda(), idx_out, ids_out,
                           count, ws)
    torch.cuda.synchronize()
    c = int(count.item())
    got_idx = idx_out.cpu().numpy()[:c]
    assert (np.diff(got_idx) > 0).all() and (idx_out.cpu().numpy()[c:] == -1).all()
    np.testing.assert_array_equal(ids_out.cpu().numpy()[:c], ids.numpy()[got_idx])
    m = n_in - w.n_window
    assert got_idx[-w.n_window:].tolist() == list(range(m, n_in))
    if np.array_equal(got_idx, ref["idx"]):
        return
    # boundary ambiguity only: rebuild the expected set from any valid top-k choice
    C = min(top_k, m)
    tau = np.sort(ref["pooled"])[m - C]
    band = REL_TOL * tau + ABS_FLOOR * ref["pooled"].max()
    sure = np.nonzero(ref["pooled"] > tau + band)[0]
    maybe = np.nonzero(ref["pooled"] >= tau - band)[0]
    lo = orc.expand_neighbors(sure, n_in, w.n_window, nb)
    hi = orc.expand_neighbors(maybe, n_in, w.n_window, nb)
    assert np.isin(lo, got_idx).all() and np.isin(got_idx, hi).all()


@pytest.mark.parametrize("n_in,n_layers,l_skip,n_lookahead,pool_k,n_neighbor,c_max", [
    (3000, 4, 1, 1, 7, 9, 300),
    (900, 3, 0, 3, 63, 31, 5000),       # budget above m, wide pools
    (1500, 10, 8, 1, 1, 1, 100),        # the paper's l_skip; pools of one
    (2500, 10, 8, 1, 64, 64, 400),      # the hyper-parameter table's SpecPC column: even kernels of 64
    (1200, 3, 1, 1, 32, 32, 150),       # ... and of 32 (the smaller draft)
    (700, 2, 0, 2, 2, 4, 90),           # the smallest even kernels
    (1800, 3, 1, 64, 7, 9, 200),        # 128 rows per head: full row super-blocks, head maxima merged in pairs
])
def test_specpc_compress_prompt_alg2(S, n_in, n_layers, l_skip, n_lookahead, pool_k, n_neighbor, c_max):
    base = workloads.specpc_draft(n_in=n_in, n_layers=n_layers, name="c5_alg2")
    w = workloads.SpecKVWorkload(**{**base.__dict__, "n_lookahead": n_lookahead, "pool_k": pool_k,
                                    "c_max": c_max})
    t = workloads.generate(w)
    ids = workloads.generate_token_ids(w)
    ref = orc.specpc_compress_prompt(workloads.to_float64(t["q"][:, 0]), workloads.to_float64(t["k"]),
                                     ids.numpy(), w.n_window, pool_k, n_neighbor, c_max, l_skip, w.sm_scale)
    p = make_params(S, w)
    ws = torch.empty(S.specpc_compress_workspace_bytes(p, l_skip), dtype=torch.uint8, device="cuda")
    m = n_in - w.n_window
    cap = min(c_max, m) + w.n_window
    idx_out = torch.full((cap + 3,), -1, dtype=torch.int32, device="cuda")
    ids_out = torch.full((cap + 3,), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    S.specpc_compress_prompt(p, l_skip, n_neighbor, t["q"].cuda(), t["k"].cuda(), ids.cuda(), idx_out,
                             ids_out, count, ws)
    torch.cuda.synchronize()
    assert int(count.item()) == cap and (idx_out.cpu().numpy()[cap:] == -1).all()
    got = idx_out.cpu().numpy()[:cap].astype(np.int64)
    np.testing.assert_array_equal(ids_out.cpu().numpy()[:cap], ids.numpy()[got])
    assert_indices_valid(got, ref["pooled"], n_in, w.n_window, c_max, "alg2")


@pytest.mark.parametrize("shift", [0.0, 0.37])
def test_scores_with_supplied_row_normalisers(S, shift):
    """One sweep with caller-supplied log-sum-exps: equals the two-sweep path when they are the
    rows' own normalisers, and the oracle with any other value."""
    w = workloads.ragged_batch(n_layers=2, lo=300, hi=1800, n_seqs=2, seed=11, name="c4_lse")
    t = workloads.generate(w)
    q64, k64 = workloads.to_float64(t["q"]), workloads.to_float64(t["k"])
    cu, G = w.cu_seqlens, w.group
    L, Sn, R, Hq = w.n_layers, w.n_seqs, w.n_rows, w.n_q_heads
    lse = np.zeros((L, Sn, R, Hq))
    for layer in range(L):
        for s in range(Sn):
            pos = orc.observation_positions(w.seq_lens[s], w.n_window, w.n_lookahead)
            for h in range(Hq):
                lse[layer, s, :, h] = orc.row_lse(q64[layer, s, :, h], k64[layer, cu[s]:cu[s + 1], h // G],
                                                  pos, w.sm_scale) + shift * (1 + h % 3)
    p = make_params(S, w)
    H, T = w.n_kv_heads, w.total_tokens
    pooled = torch.empty((L, H * T), dtype=torch.float32, device="cuda")
    raw = torch.empty_like(pooled)
    ws = alloc_ws(S, p)
    S.speckv_score_lse(p, t["q"].cuda(), t["k"].cuda(), torch.from_numpy(lse).float().cuda(), pooled, raw, ws)
    torch.cuda.synchronize()
    raw_h = raw.cpu().numpy()
    lse32 = lse.astype(np.float32).astype(np.float64)              # the library sees the fp32 rounding
    for layer in range(L):
        for s in range(Sn):
            want = orc.raw_scores(q64[layer, s], k64[layer, cu[s]:cu[s + 1]], w.n_window, w.sm_scale,
                                  lse_in=lse32[layer, s])
            assert_scores_close(split_scores(w, raw_h, layer, s), want, "raw with lse l%d s%d" % (layer, s))
    if shift == 0.0:
        pooled2 = torch.empty_like(pooled)
        S.speckv_score(p, t["q"].cuda(), t["k"].cuda(), pooled2, None, ws)
        torch.cuda.synchronize()
        np.testing.assert_allclose(pooled.cpu().numpy(), pooled2.cpu().numpy(), rtol=1e-4, atol=1e-9)
    # fused variant runs and selects from the same scores
    KT = S.total_keep(p)
    idx = torch.empty((L, H * KT), dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, w.head_dim), dtype=w.torch_dtype, device="cuda")
    v_out = torch.empty_like(k_out)
    S.speckv_compress_lse(p, t["q"].cuda(), t["k"].cuda(), t["v"].cuda(), torch.from_numpy(lse).float().cuda(),
                          idx, k_out, v_out, ws)
    idx2 = torch.empty_like(idx)
    S.speckv_select(p, pooled, idx2)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2)


def test_many_short_sequences(S):
    """The maximum of 128 sequences in one call, most of them shorter than one key tile."""
    rng = np.random.default_rng(61)
    lens = tuple(int(x) for x in rng.integers(40, 400, size=128))
    w = workloads.SpecKVWorkload(
        name="many", n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=64, seq_lens=lens, n_window=8,
        n_lookahead=8, pool_k=7, c_max=20, dtype="bf16", sm_scale=0.125, n_planted=2,
        channel_scale=(0.5, 4.0), seed=62)
    check_full_path(S, w)


def test_largest_row_group(S):
    """G * R at the documented limit of 4096 rows per KV head (8 row super-blocks)."""
    w = workloads.SpecKVWorkload(
        name="rows4096", n_layers=1, n_q_heads=16, n_kv_heads=1, head_dim=128, seq_lens=(600,),
        n_window=100, n_lookahead=156, pool_k=7, c_max=50, dtype="bf16", sm_scale=1 / math.sqrt(128),
        n_planted=4, channel_scale=(0.5, 4.0), seed=63)
    check_full_path(S, w)
    check_full_path(S, w, reduce="max", pool="avg")


def test_graph_capture_and_replay(S):
    """The fused call records into a HIP graph (no allocation, no memset, no sync inside) and
    every replay reproduces the eager result, also after the inputs changed in place."""
    w = workloads.llama8b_layer(n_in=3000, c_max=256, name="graph")
    t = workloads.generate(w)
    q, k, v = (t[x].cuda() for x in ("q", "k", "v"))
    p = make_params(S, w)
    KT, H, d = S.total_keep(p), w.n_kv_heads, w.head_dim
    idx = torch.zeros((1, H * KT), dtype=torch.int32, device="cuda")
    k_out = torch.zeros((1, H * KT, d), dtype=w.torch_dtype, device="cuda")
    v_out = torch.zeros_like(k_out)
    ws = alloc_ws(S, p)
    S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)          # eager warm-up (module load)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)
    for trial in range(3):
        if trial:                                                   # new inputs, same buffers
            t2 = workloads.generate(workloads.llama8b_layer(n_in=3000, c_max=256, seed=70 + trial, name="graph"))
            q.copy_(t2["q"].cuda()); k.copy_(t2["k"].cuda()); v.copy_(t2["v"].cuda())
        idx.fill_(-1); k_out.zero_(); v_out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (idx.clone(), k_out.clone(), v_out.clone())
        idx.fill_(-1); k_out.zero_(); v_out.zero_()
        S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)
        torch.cuda.synchronize()
        assert torch.equal(got[0], idx) and torch.equal(got[1], k_out) and torch.equal(got[2], v_out)
        assert int(idx.min()) >= 0


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_fuzz_bit_exact(S, seed):
    """Random ragged rows with heavy ties, negative and zero scores, budgets from 0 to beyond m:
    selection on given fp32 scores is integer work and must equal the oracle exactly."""
    rng = np.random.default_rng(1000 + seed)
    n_seqs = 24
    n_window = int(rng.integers(0, 40))
    lens = tuple(int(x) for x in np.concatenate([rng.integers(max(1, n_window), 300, size=16),
                                                 rng.integers(3000, 70000, size=n_seqs - 16)]))
    c_max = int(rng.choice([0, 1, 7, 500, 4096, 100000]))
    w = workloads.SpecKVWorkload(
        name="fuzz", n_layers=2, n_q_heads=3, n_kv_heads=3, head_dim=64, seq_lens=lens,
        n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
    p = make_params(S, w)
    L, H, T = 2, 3, w.total_tokens
    levels = int(rng.choice([2, 17, 1000, 10 ** 6]))
    base = (rng.integers(0, levels, size=(L, H * T)).astype(np.float32) - levels // 3) / np.float32(levels)
    pooled = torch.from_numpy(base).cuda()
    KT = S.total_keep(p)
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    S.speckv_select(p, pooled, idx)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    for layer in range(L):
        for s in range(n_seqs):
            n = lens[s]
            rows = split_scores(w, base, layer, s)
            got = split_keep(w, idx_h, layer, s, c_max)
            for g in range(H):
                want = orc.keep_indices(rows[g, :n - n_window].astype(np.float64), n, n_window, c_max)
                assert got[g].tolist() == want.tolist(), (seed, layer, s, g)


def test_second_index_set_from_the_same_scores(S):
    """Alg. 1 also takes i_vert = topk(s, n_vert) from the same pooled scores: scoring once and
    selecting twice with different budgets gives both sets; the larger contains the smaller."""
    w = workloads.llama8b_layer(n_in=6000, c_max=256, name="ivert")
    t = workloads.generate(w)
    p_cache = make_params(S, w, c_max=256)
    p_vert = make_params(S, w, c_max=2048)
    H, T = w.n_kv_heads, w.total_tokens
    pooled = torch.empty((1, H * T), dtype=torch.float32, device="cuda")
    S.speckv_score(p_cache, t["q"].cuda(), t["k"].cuda(), pooled, None, alloc_ws(S, p_cache))
    idx_c = torch.empty((1, H * S.total_keep(p_cache)), dtype=torch.int32, device="cuda")
    idx_v = torch.empty((1, H * S.total_keep(p_vert)), dtype=torch.int32, device="cuda")
    S.speckv_select(p_cache, pooled, idx_c)
    S.speckv_select(p_vert, pooled, idx_v)
    torch.cuda.synchronize()
    ic = idx_c.cpu().numpy().reshape(H, -1)
    iv = idx_v.cpu().numpy().reshape(H, -1)
    m = 6000 - w.n_window
    pooled_h = pooled.cpu().numpy().reshape(H, 6000)
    for g in range(H):
        assert set(ic[g].tolist()) <= set(iv[g].tolist())
        assert iv[g][:2048].tolist() == orc.select_top(pooled_h[g, :m], 2048).tolist()    # i_vert itself


# --------------------------------------------------------------------------- #
# Layer budget shared across KV heads (App. "Integration and Comparison with the AdaKV Baseline")
# --------------------------------------------------------------------------- #
def ada_block(w, flat, layer, s, c_max, trailing=()):
    """All Hkv*n_keep_s rows of one (layer, sequence) block of an idx / k_out style tensor."""
    keeps = [min(c_max, n - w.n_window) + w.n_window for n in w.seq_lens]
    ck = np.concatenate([[0], np.cumsum(keeps)])
    a = w.n_kv_heads * ck[s]
    return flat[layer, a:a + w.n_kv_heads * keeps[s]]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_select_ada_fuzz_bit_exact(S, seed):
    """Selection with a shared layer budget on given fp32 scores is integer work: head offsets and
    indices must equal the oracle's exactly (ties, negative scores, floors from 0 to beyond C)."""
    rng = np.random.default_rng(2000 + seed)
    n_seqs, H, L = 6, (40 if seed == 3 else int(rng.choice([1, 3, 8]))), 2
    n_window = int(rng.integers(0, 20))
    lens = tuple(int(x) for x in np.concatenate([rng.integers(max(1, n_window), 200, size=3),
                                                 rng.integers(2000, 40000, size=n_seqs - 3)]))
    c_max = int(rng.choice([0, 5, 300, 2048, 50000]))
    c_floor = int(rng.choice([0, 1, c_max // 5, c_max, c_max + 7]))
    w = workloads.SpecKVWorkload(
        name="ada_fuzz", n_layers=L, n_q_heads=H, n_kv_heads=H, head_dim=64, seq_lens=lens,
        n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
    p = make_params(S, w)
    T = w.total_tokens
    levels = int(rng.choice([3, 50, 10 ** 6]))
    base = (rng.integers(0, levels, size=(L, H * T)).astype(np.float32) - levels // 4) / np.float32(levels)
    # heads of very different sharpness so that the budgets really move between heads
    for layer in range(L):
        for s in range(n_seqs):
            split_scores(w, base, layer, s)[...] *= np.float32(2.0) ** rng.integers(-3, 4, size=(H, 1))
    pooled = torch.from_numpy(base).cuda()
    KT = S.total_keep(p)
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    head_off = torch.full((L, n_seqs, H + 1), -1, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(S.ada_workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")
    S.speckv_select_ada(p, c_floor, pooled, idx, head_off, ws)
    torch.cuda.synchronize()
    idx_h, off_h = idx.cpu().numpy(), head_off.cpu().numpy()
    for layer in range(L):
        for s in range(n_seqs):
            n = lens[s]
            rows = split_scores(w, base, layer, s)[:, :n - n_window].astype(np.float64)
            want = orc.ada_keep_indices(rows, n, n_window, c_max, c_floor)
            want_off = np.concatenate([[0], np.cumsum([len(x) for x in want])])
            assert off_h[layer, s].tolist() == want_off.tolist(), (seed, layer, s)
            got = ada_block(w, idx_h, layer, s, c_max)
            assert got.tolist() == np.concatenate(want).tolist(), (seed, layer, s)


def test_compress_ada_full_path(S):
    """score -> shared-budget select -> compact in one call, against the oracle; the floor equal to
    the budget reproduces the equal-budget call bit for bit."""
    w = workloads.SpecKVWorkload(
        name="ada_path", n_layers=2, n_q_heads=8, n_kv_heads=4, head_dim=128, seq_lens=(3000, 700, 5121),
        n_window=16, n_lookahead=8, pool_k=7, c_max=256, dtype="bf16", sm_scale=1.0 / math.sqrt(128.0),
        n_planted=16, seed=11)
    t = workloads.generate(w)
    q, k, v = (t[x].cuda() for x in ("q", "k", "v"))
    p = make_params(S, w)
    L, H, KT, d = w.n_layers, w.n_kv_heads, S.total_keep(p), w.head_dim
    ws = torch.empty(S.ada_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    q64, k64, v64 = (workloads.to_float64(t[x]) for x in ("q", "k", "v"))
    for c_floor in (51, 256):
        idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
        head_off = torch.full((L, len(w.seq_lens), H + 1), -1, dtype=torch.int32, device="cuda")
        k_out = torch.zeros((L, H * KT, d), dtype=torch.bfloat16, device="cuda")
        v_out = torch.zeros_like(k_out)
        S.speckv_compress_ada(p, c_floor, q, k, v, idx, head_off, k_out, v_out, ws)
        torch.cuda.synchronize()
        idx_h, off_h = idx.cpu().numpy(), head_off.cpu().numpy()
        ko, vo = k_out.cpu().float().numpy(), v_out.cpu().float().numpy()
        for layer in range(L):
            for s, n in enumerate(w.seq_lens):
                a, b = w.cu_seqlens[s], w.cu_seqlens[s + 1]
                ref = orc.speckv_layer_ada(q64[layer, s], k64[layer, a:b], v64[layer, a:b], w.n_window,
                                           w.pool_k, w.c_max, c_floor, w.sm_scale)
                got_off = off_h[layer, s]
                got = ada_block(w, idx_h, layer, s, w.c_max)
                # structure: every head ascending, window last, floor respected, layer total fixed
                assert got_off[0] == 0 and got_off[-1] == H * (min(w.c_max, n - w.n_window) + w.n_window)
                for g in range(H):
                    rows = got[got_off[g]:got_off[g + 1]]
                    assert (np.diff(rows) > 0).all() and rows[-w.n_window:].tolist() == list(range(n - w.n_window, n))
                    assert len(rows) - w.n_window >= min(c_floor, w.c_max, n - w.n_window)
                # the sets match the oracle wherever its own score gaps exceed the tolerance: per head,
                # every key clearly above the head's threshold (the layer-wide one, or the head's own
                # floor threshold when that is lower) is kept and every key clearly below it is not
                if not (got_off.tolist() == ref["head_off"].tolist()
                        and got.tolist() == np.concatenate(ref["idx"]).tolist()):
                    assert_ada_indices_in_band([got[got_off[g]:got_off[g + 1]] for g in range(H)], ref["pooled"],
                                               ref["idx"], w.n_window, min(c_floor, w.c_max, n - w.n_window),
                                               "ada (l%d,s%d,floor %d)" % (layer, s, c_floor))
                # gathered rows are bit copies of the rows the returned indices name
                kb = ada_block(w, ko, layer, s, w.c_max)
                vb = ada_block(w, vo, layer, s, w.c_max)
                for g in range(H):
                    rows = got[got_off[g]:got_off[g + 1]]
                    assert np.array_equal(kb[got_off[g]:got_off[g + 1]], k64[layer, a:b][rows, g, :])
                    assert np.array_equal(vb[got_off[g]:got_off[g + 1]], v64[layer, a:b][rows, g, :])
        if c_floor == 256:
            idx_u = torch.empty_like(idx); k_u = torch.empty_like(k_out); v_u = torch.empty_like(v_out)
            S.speckv_compress(p, q, k, v, idx_u, k_u, v_u, ws)
            torch.cuda.synchronize()
            assert torch.equal(idx_u, idx) and torch.equal(k_u, k_out) and torch.equal(v_u, v_out)


def test_cascade_prompt_compression_then_cache_compression(S):
    """SpecKV-PC (Sec. "SpecKV-PC: Cascaded Compression"): Alg. 2 shortens the prompt from the draft
    model's attention, the target model is prefilled on the kept tokens, Alg. 1 compresses that
    cache.  The target prefill is outside this library; its K/V of the kept tokens are stood in
    for by the rows of a synthetic target tensor at the kept positions (a torch gather here, the
    same gather in numpy for the oracle).  Both stages run on one stream, the second sized by the
    count the first returns."""
    n_in, l_skip, n_neighbor, keep_tokens = 6000, 2, 9, 1500
    base = workloads.specpc_draft(n_in=n_in, n_layers=5, name="pc_draft")
    wd = workloads.SpecKVWorkload(**{**base.__dict__, "n_lookahead": 4, "pool_k": 5, "c_max": keep_tokens})
    td = workloads.generate(wd)
    ids = workloads.generate_token_ids(wd)
    wt = workloads.llama8b_layer(n_in=n_in, c_max=200, n_layers=2, seed=23, name="pc_target")
    tt = workloads.generate(wt)

    # oracle: stage 1, gather, stage 2
    ref1 = orc.specpc_compress_prompt(workloads.to_float64(td["q"][:, 0]), workloads.to_float64(td["k"]),
                                      ids.numpy(), wd.n_window, wd.pool_k, n_neighbor, keep_tokens, l_skip,
                                      wd.sm_scale)
    kept = ref1["idx"]
    assert kept[-wt.n_window:].tolist() == list(range(n_in - wt.n_window, n_in))   # target's window rows survive
    q64, k64, v64 = (workloads.to_float64(tt[x]) for x in ("q", "k", "v"))
    ref2 = [orc.speckv_layer(q64[layer, 0], k64[layer][kept], v64[layer][kept], wt.n_window, wt.pool_k,
                             wt.c_max, wt.sm_scale) for layer in range(wt.n_layers)]

    # library: stage 1
    p1 = make_params(S, wd)
    ws1 = torch.empty(S.specpc_compress_workspace_bytes(p1, l_skip), dtype=torch.uint8, device="cuda")
    cap = keep_tokens + wd.n_window
    idx_out = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    ids_out = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    S.specpc_compress_prompt(p1, l_skip, n_neighbor, td["q"].cuda(), td["k"].cuda(), ids.cuda(), idx_out,
                             ids_out, count, ws1)
    n2 = int(count.item())                                            # the one host round trip of the cascade
    got_kept = idx_out[:n2].cpu().numpy().astype(np.int64)
    assert_indices_valid(got_kept, ref1["pooled"], n_in, wd.n_window, keep_tokens, "cascade stage 1")
    assert np.array_equal(got_kept, kept), "stage 1 differs inside its tolerance band: pick another seed"
    np.testing.assert_array_equal(ids_out[:n2].cpu().numpy(), ids.numpy()[kept])

    # stand-in for the target prefill on the kept tokens
    k2 = tt["k"].cuda().index_select(1, idx_out[:n2].long()).contiguous()
    v2 = tt["v"].cuda().index_select(1, idx_out[:n2].long()).contiguous()
    q2 = tt["q"].cuda()

    # library: stage 2 on the shortened prompt
    w2 = workloads.SpecKVWorkload(**{**wt.__dict__, "seq_lens": (n2,)})
    p2 = make_params(S, w2)
    KT = S.total_keep(p2)
    H, d, L = wt.n_kv_heads, wt.head_dim, wt.n_layers
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    S.speckv_compress(p2, q2, k2, v2, idx, k_out, v_out, alloc_ws(S, p2))
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy().reshape(L, H, KT)
    ko = k_out.cpu().float().numpy().reshape(L, H, KT, d)
    vo = v_out.cpu().float().numpy().reshape(L, H, KT, d)
    for layer in range(L):
        for g in range(H):
            assert_indices_valid(idx_h[layer, g], ref2[layer]["pooled"][g], n2, wt.n_window, wt.c_max,
                                 "cascade stage 2 l%d g%d" % (layer, g))
            # rows of the final cache are rows of the ORIGINAL prompt: kept[idx] names them
            orig = kept[idx_h[layer, g]]
            assert np.array_equal(ko[layer, g], k64[layer][orig, g, :])
            assert np.array_equal(vo[layer, g], v64[layer][orig, g, :])


@pytest.mark.parametrize("shape", ["8b_d128", "draft_d64"])
@pytest.mark.parametrize("n_live", [7000, 4097, 3968, 1100, 300, 64])
def test_device_side_token_count_equals_a_host_length_call(S, n_live, shape):
    """`n_in_dev`: the kernels read the number of live prompt tokens from device memory; the host
    length is only an upper bound.  Scores, indices and the compacted cache must equal those of a
    call whose host length is the live length (on the same first n_live tokens), with zeros / -1 in
    the slots a shorter prompt leaves unused."""
    n_cap = 7000
    if shape == "8b_d128":
        w = workloads.llama8b_layer(n_in=n_cap, c_max=512, n_layers=2, name="devlen")
    else:       # d = 64, 8 row blocks per group: the row-statistics sweep runs in the Q-stationary kernel
        base = workloads.specpc_draft(n_in=n_cap, n_layers=2, name="devlen64")
        w = workloads.SpecKVWorkload(**{**base.__dict__, "c_max": 512, "n_lookahead": 64})
    t = workloads.generate(w)
    q, k, v = (t[x].cuda() for x in ("q", "k", "v"))
    # the window rows of the live prompt are its last n_window tokens: only the key/value prefix matters
    n_dev = torch.tensor([n_live], dtype=torch.int32, device="cuda")
    p_dev = S.SpecKVParams.for_tensors(q, k, seq_lens=(n_cap,), n_window=w.n_window, pool_k=w.pool_k,
                                       c_max=w.c_max, sm_scale=w.sm_scale, n_in_dev=n_dev)
    k_live, v_live = k[:, :n_live].contiguous(), v[:, :n_live].contiguous()
    p_host = S.SpecKVParams.for_tensors(q, k_live, seq_lens=(n_live,), n_window=w.n_window, pool_k=w.pool_k,
                                        c_max=w.c_max, sm_scale=w.sm_scale)
    L, H, d = w.n_layers, w.n_kv_heads, w.head_dim
    outs = {}
    for name, p, kk, vv, n in (("dev", p_dev, k, v, n_cap), ("host", p_host, k_live, v_live, n_live)):
        KT = S.total_keep(p)
        pooled = torch.full((L, H * n), -1.0, dtype=torch.float32, device="cuda")
        raw = torch.full((L, H * n), -1.0, dtype=torch.float32, device="cuda")
        idx = torch.full((L, H * KT), -7, dtype=torch.int32, device="cuda")
        k_out = torch.full((L, H * KT, d), 3.0, dtype=torch.bfloat16, device="cuda")
        v_out = torch.full((L, H * KT, d), 3.0, dtype=torch.bfloat16, device="cuda")
        ws = alloc_ws(S, p)
        if shape == "draft_d64" and name == "dev":
            assert S.plan_info(p)["q_stationary"] == 1
        S.speckv_score(p, q, kk, pooled, raw, ws)
        S.speckv_compress(p, q, kk, vv, idx, k_out, v_out, ws)
        torch.cuda.synchronize()
        outs[name] = (pooled.view(L, H, n), raw.view(L, H, n), idx.view(L, H, KT), k_out.view(L, H, KT, d),
                      v_out.view(L, H, KT, d))
    pd, rd, idd, kd, vd = outs["dev"]
    ph, rh, idh, kh, vh = outs["host"]
    assert torch.equal(pd[..., :n_live], ph) and torch.equal(rd[..., :n_live], rh)
    assert bool((pd[..., n_live:] == 0).all()) and bool((rd[..., n_live:] == 0).all())
    keep_live = idh.shape[-1]
    assert torch.equal(idd[..., :keep_live], idh)
    assert bool((idd[..., keep_live:] == -1).all())
    assert torch.equal(kd[..., :keep_live, :], kh) and torch.equal(vd[..., :keep_live, :], vh)
    assert bool((kd[..., keep_live:, :] == 0).all()) and bool((vd[..., keep_live:, :] == 0).all())


@pytest.mark.parametrize("n_live", [6000, 3000, 700, 130])
def test_shared_budget_with_device_side_token_count(S, n_live):
    """Per-head budgets with `n_in_dev`: head offsets, indices and the compacted cache equal those of
    a call whose host length is the live length; the slots a shorter prompt leaves behind the last
    head hold -1 / zero rows."""
    n_cap, c_floor = 7000, 100
    w = workloads.llama8b_layer(n_in=n_cap, c_max=512, n_layers=2, name="devlen_ada")
    t = workloads.generate(w)
    q, k, v = (t[x].cuda() for x in ("q", "k", "v"))
    n_dev = torch.tensor([n_live], dtype=torch.int32, device="cuda")
    p_dev = S.SpecKVParams.for_tensors(q, k, seq_lens=(n_cap,), n_window=w.n_window, pool_k=w.pool_k,
                                       c_max=w.c_max, sm_scale=w.sm_scale, n_in_dev=n_dev)
    k_live, v_live = k[:, :n_live].contiguous(), v[:, :n_live].contiguous()
    p_host = S.SpecKVParams.for_tensors(q, k_live, seq_lens=(n_live,), n_window=w.n_window, pool_k=w.pool_k,
                                        c_max=w.c_max, sm_scale=w.sm_scale)
    L, H, d = w.n_layers, w.n_kv_heads, w.head_dim
    outs = {}
    for name, p, kk, vv in (("dev", p_dev, k, v), ("host", p_host, k_live, v_live)):
        KT = S.total_keep(p)
        idx = torch.full((L, H * KT), -7, dtype=torch.int32, device="cuda")
        head_off = torch.full((L, 1, H + 1), -7, dtype=torch.int32, device="cuda")
        k_out = torch.full((L, H * KT, d), 3.0, dtype=torch.bfloat16, device="cuda")
        v_out = torch.full((L, H * KT, d), 3.0, dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(S.ada_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        S.speckv_compress_ada(p, c_floor, q, kk, vv, idx, head_off, k_out, v_out, ws)
        torch.cuda.synchronize()
        outs[name] = (idx, head_off, k_out, v_out)
    idd, hod, kd, vd = outs["dev"]
    idh, hoh, kh, vh = outs["host"]
    assert torch.equal(hod, hoh)
    used = idh.shape[1]                                   # H * (min(c_max, m_live) + n_window)
    assert int(hoh[0, 0, H]) == used
    assert torch.equal(idd[:, :used], idh) and bool((idd[:, used:] == -1).all())
    assert torch.equal(kd[:, :used], kh) and torch.equal(vd[:, :used], vh)
    assert bool((kd[:, used:] == 0).all()) and bool((vd[:, used:] == 0).all())


def test_cascade_on_the_device_in_one_graph(S):
    """SpecKV-PC (Sec. "SpecKV-PC: Cascaded Compression") without a host round trip: the prompt-token
    selection leaves its data-dependent count on the device, the gather that stands in for the
    target prefill and the cache compression follow on the same stream, the latter reading the count
    through `n_in_dev`.  The three steps are captured into one HIP graph; every replay (also after
    the draft inputs, and with them the count, changed) equals the eager run, and the eager run
    equals the oracle's composition."""
    n_in, top_k, nb = 6000, 300, 5
    wd = workloads.specpc_draft(n_in=n_in, n_layers=3, name="pc_draft_dev")
    wt = workloads.llama8b_layer(n_in=n_in, c_max=200, n_layers=2, seed=23, name="pc_target_dev")
    tt = workloads.generate(wt)
    qt, kt, vt = (tt[x].cuda() for x in ("q", "k", "v"))
    td = workloads.generate(wd)
    qd, kd = td["q"].cuda(), td["k"].cuda()
    ids = workloads.generate_token_ids(wd).cuda()
    L, H, d = wt.n_layers, wt.n_kv_heads, wt.head_dim

    p1 = make_params(S, wd)
    ws1 = torch.empty(S.specpc_workspace_bytes(p1, top_k), dtype=torch.uint8, device="cuda")
    idx_out = torch.empty(n_in, dtype=torch.int32, device="cuda")
    ids_out = torch.empty(n_in, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    k2, v2 = torch.empty_like(kt), torch.empty_like(vt)             # capacity: the whole prompt
    p2 = S.SpecKVParams.for_tensors(qt, k2, seq_lens=(n_in,), n_window=wt.n_window, pool_k=wt.pool_k,
                                    c_max=wt.c_max, sm_scale=wt.sm_scale, n_in_dev=count)
    KT = S.total_keep(p2)
    idx = torch.empty((L, H * KT), dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    ws2 = alloc_ws(S, p2)

    def cascade():
        idx_out.fill_(-1)
        S.specpc_select_tokens(p1, top_k, nb, qd, kd, ids, idx_out, ids_out, count, ws1)
        kept = idx_out.clamp(min=0).long()                            # slots past the count are never read
        torch.index_select(kt, 1, kept, out=k2)
        torch.index_select(vt, 1, kept, out=v2)
        S.speckv_compress(p2, qt, k2, v2, idx, k_out, v_out, ws2)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                     # warm-up outside the capture
        cascade()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cascade()

    counts = []
    for trial in range(3):
        if trial:                                                     # other draft inputs: another count
            t2 = workloads.generate(workloads.specpc_draft(n_in=n_in, n_layers=3, seed=80 + trial, name="pc_draft_dev"))
            qd.copy_(t2["q"].cuda()); kd.copy_(t2["k"].cuda())
        for x in (idx, k_out, v_out):
            x.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (idx.clone(), k_out.clone(), v_out.clone(), idx_out.clone(), count.clone())
        for x in (idx, k_out, v_out):
            x.fill_(-5)
        cascade()
        torch.cuda.synchronize()
        assert torch.equal(got[4], count) and torch.equal(got[3], idx_out)
        assert torch.equal(got[0], idx) and torch.equal(got[1], k_out) and torch.equal(got[2], v_out)
        counts.append(int(count.item()))
        if trial == 0:
            # the eager run against the oracle: stage 1, gather, stage 2
            ref1 = orc.specpc_select_tokens(workloads.to_float64(td["q"][:, 0]), workloads.to_float64(td["k"]),
                                            ids.cpu().numpy(), wd.n_window, wd.pool_k, top_k, nb, wd.sm_scale)
            kept = ref1["idx"]
            n2 = counts[0]
            assert n2 == len(kept) and np.array_equal(idx_out[:n2].cpu().numpy(), kept), \
                "stage 1 differs inside its tolerance band: pick another seed"
            assert n2 < n_in and n2 - wt.n_window > wt.c_max
            q64, k64, v64 = (workloads.to_float64(tt[x]) for x in ("q", "k", "v"))
            idx_h = idx.cpu().numpy().reshape(L, H, KT)
            ko = k_out.cpu().float().numpy().reshape(L, H, KT, d)
            for layer in range(L):
                ref2 = orc.speckv_layer(q64[layer, 0], k64[layer][kept], v64[layer][kept], wt.n_window, wt.pool_k,
                                        wt.c_max, wt.sm_scale)
                for g in range(H):
                    assert_indices_valid(idx_h[layer, g], ref2["pooled"][g], n2, wt.n_window, wt.c_max,
                                         "device cascade l%d g%d" % (layer, g))
                    assert np.array_equal(ko[layer, g], k64[layer][kept[idx_h[layer, g]], g, :])
    assert len(set(counts)) > 1, "the count never changed between replays: nothing was tested"


def test_select_signed_zeros_denormals_and_negative_rows(S):
    """-0 and +0 tie (smaller index first), denormal scores keep their order, rows that are all
    negative or mixed select from the right end of the order."""
    n_window, H = 2, 6
    m = 5003
    n = m + n_window
    rng = np.random.default_rng(5)
    rows = np.zeros((H, n), dtype=np.float32)
    rows[0, :m] = np.where(rng.random(m) < 0.5, np.float32(0.0), np.float32(-0.0))          # only zeros
    rows[1, :m] = (rng.integers(-3, 4, size=m) * np.float32(1e-42)).astype(np.float32)       # denormals, zeros
    rows[1, ::7] = np.float32(-0.0)
    rows[2, :m] = -np.abs(rng.standard_normal(m)).astype(np.float32) - 1                     # all negative
    rows[3, :m] = rng.standard_normal(m).astype(np.float32) * np.float32(1e-30)              # mixed signs, tiny
    rows[4, :m] = rng.integers(-2, 3, size=m).astype(np.float32)                             # few levels around 0
    rows[5, :m] = np.float32(3.0e38) * rng.choice([-1, 1], size=m).astype(np.float32)        # extremes
    for c_max in (1, 700, 2600, m):
        w = workloads.SpecKVWorkload(
            name="zeros", n_layers=1, n_q_heads=H, n_kv_heads=H, head_dim=64, seq_lens=(n,),
            n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
        p = make_params(S, w)
        idx = torch.full((1, H * S.total_keep(p)), -1, dtype=torch.int32, device="cuda")
        S.speckv_select(p, torch.from_numpy(rows.reshape(1, -1)).cuda(), idx)
        torch.cuda.synchronize()
        got = idx.cpu().numpy().reshape(H, -1)
        for g in range(H):
            want = orc.keep_indices(rows[g, :m].astype(np.float64), n, n_window, c_max)
            assert got[g].tolist() == want.tolist(), (c_max, g)


@pytest.mark.parametrize("seed", range(12))
def test_random_configurations(S, seed):
    """Seeded random shapes: group size, rows per head, head dimension, number type, ragged lengths,
    window, lookahead, pooling width, budget, reduction and pooling options, all drawn together so
    that combinations no hand-written case names are exercised too."""
    rng = np.random.default_rng(7000 + seed)
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
    Hkv = int(rng.choice([1, 2, 3]))
    d = int(rng.choice([64, 128]))
    dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    n_window = int(rng.choice([0, 1, 7, 16, 33, 64]))
    n_lookahead = int(rng.choice([0, 1, 5, 32, 70])) if n_window > 0 else int(rng.choice([1, 5, 32, 70]))
    n_seqs = int(rng.choice([1, 2, 4]))
    lens = tuple(int(x) for x in rng.integers(max(1, n_window), 2600, size=n_seqs))
    w = workloads.SpecKVWorkload(
        name="rand%d" % seed, n_layers=int(rng.choice([1, 2])), n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d,
        seq_lens=lens, n_window=n_window, n_lookahead=n_lookahead, pool_k=int(rng.choice([1, 3, 7, 13])),
        c_max=int(rng.choice([0, 1, 50, 400, 5000])), dtype=dtype, sm_scale=float(1.0 / math.sqrt(d)),
        n_planted=int(rng.choice([0, 3])) if min(lens) - n_window > 8 else 0,
        channel_scale=(0.5, 4.0) if rng.random() < 0.5 else None, seed=300 + seed)
    check_full_path(S, w, reduce=str(rng.choice(["sum", "sum", "max"])), pool=str(rng.choice(["max", "max", "avg"])))


def test_select_on_a_three_million_key_row(S):
    """A row far longer than any benchmark row (many emission tiles, counts above 16 bits)."""
    n, n_window, c_max = 3_000_001, 5, 200_000
    rng = np.random.default_rng(9)
    rows = rng.standard_normal((2, n)).astype(np.float32)
    rows[1] = np.round(rows[1] * 50) / 50                     # heavy ties
    w = workloads.SpecKVWorkload(
        name="long_row", n_layers=1, n_q_heads=2, n_kv_heads=2, head_dim=64, seq_lens=(n,),
        n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
    p = make_params(S, w)
    pooled = torch.from_numpy(rows.reshape(1, -1)).cuda()
    want = [orc.keep_indices(rows[g, :n - n_window].astype(np.float64), n, n_window, c_max) for g in range(2)]
    # without a workspace one workgroup ranks each row; with it the rows are split over many
    assert 0 < S.select_workspace_bytes(p) < 64 << 20
    for ws in (None, torch.empty(S.select_workspace_bytes(p), dtype=torch.uint8, device="cuda")):
        idx = torch.full((1, 2 * S.total_keep(p)), -1, dtype=torch.int32, device="cuda")
        S.speckv_select(p, pooled, idx, ws)
        torch.cuda.synchronize()
        got = idx.cpu().numpy().reshape(2, -1)
        for g in range(2):
            assert np.array_equal(got[g], want[g]), (g, ws is None)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_random_rows_distributions_and_budgets(S, seed):
    """Selection on given scores over random row lengths (1 to 300 000 and the tile boundaries of the
    kernel), value distributions (smooth, heavy-tailed, few levels, constant, runs of equal values as
    max pooling leaves them, signed zeros and denormals), row alignments and budgets from 0 to beyond
    the row: every row equal to the oracle's."""
    rng = np.random.default_rng(7000 + seed)
    for case in range(40):
        H = int(rng.choice([1, 2, 3, 5]))
        n_window = int(rng.choice([0, 1, 2, 3, 5, 64]))
        kind = rng.choice(["tiny", "small", "mid", "big", "edge"])
        m = {"tiny": lambda: rng.integers(1, 40), "small": lambda: rng.integers(40, 5000),
             "mid": lambda: rng.integers(5000, 70000), "big": lambda: rng.integers(70000, 300000),
             "edge": lambda: rng.choice([1023, 1024, 1025, 16383, 16384, 16385, 65536, 65537, 229375, 229376,
                                         229377, 229380])}[kind]()
        m = int(m)
        n = m + n_window
        dist = rng.choice(["normal", "lognormal", "levels", "const", "softmaxlike", "runs", "zeros"])
        rows = np.zeros((H, n), dtype=np.float32)
        for g in range(H):
            if dist == "normal":
                r = rng.standard_normal(n)
            elif dist == "lognormal":
                r = np.exp(3 * rng.standard_normal(n))
            elif dist == "levels":
                r = rng.integers(0, int(rng.choice([2, 5, 100, 5000])), size=n) / 7.0
            elif dist == "const":
                r = np.full(n, rng.choice([0.0, 1.5, -2.0]))
            elif dist == "softmaxlike":
                z = rng.standard_normal(n) * rng.choice([0.2, 1.0, 4.0])
                r = np.exp(z - z.max())
                r /= r.sum()
            elif dist == "runs":
                r = np.repeat(rng.random((n + 6) // 7), 7)[:n]
            else:
                r = rng.choice([0.0, -0.0, 1e-40, -1e-40, 1e-3, -1e-3], size=n)
            rows[g] = r.astype(np.float32)
        c_max = int(rng.choice([0, 1, 2, 17, 128, 1024, 2048, 5000, m // 2 + 1, max(m - 1, 0), m, m + 5]))
        if n_window == 0 and c_max == 0:
            c_max = 1                                    # nothing to keep is not a call
        w = workloads.SpecKVWorkload(
            name="random_rows", n_layers=1, n_q_heads=H, n_kv_heads=H, head_dim=64, seq_lens=(n,),
            n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
        p = make_params(S, w)
        idx = torch.full((1, H * S.total_keep(p)), -7, dtype=torch.int32, device="cuda")
        S.speckv_select(p, torch.from_numpy(rows.reshape(1, -1)).cuda(), idx)
        torch.cuda.synchronize()
        got = idx.cpu().numpy().reshape(H, -1)
        for g in range(H):
            want = orc.keep_indices(rows[g, :m].astype(np.float64), n, n_window, c_max)
            assert np.array_equal(got[g], want), (seed, case, g, m, n_window, str(dist), c_max)


@pytest.mark.parametrize("m,in_bin", [(20000, 4096), (20000, 4097), (20000, 40), (229376, 300), (229379, 300),
                                      (229381, 300), (131072, 4000)])
def test_select_around_the_limits_of_the_one_read_path(S, m, in_bin):
    """The one-workgroup selection reads a row once more after the first radix digit when the row is
    short enough (229376 entries plus up to three unaligned ones at either end) and the
    threshold's first-digit bin holds at most 4096 entries; otherwise it runs all three digits.
    Both sides of both limits, with runs of equal values and several budgets, against the oracle.
    [1, 1.25) is one first-digit bin (sign, exponent and two mantissa bits)."""
    n_window, H = 3, 3                        # odd row length: the rows start at different alignments
    n = m + n_window
    rng = np.random.default_rng(m + in_bin)
    rows = np.empty((H, n), dtype=np.float32)
    n_above = 700
    for g in range(H):
        r = (rng.random(n) * 0.5).astype(np.float32)                            # below the bin
        pos = rng.permutation(m)[:in_bin + n_above]
        r[pos[:in_bin]] = (1.0 + 0.25 * rng.random(in_bin)).astype(np.float32)   # the bin [1, 1.25)
        r[pos[in_bin:]] = (2.0 + rng.random(n_above)).astype(np.float32)         # above it
        if g == 1:                                                              # runs of equal values inside the bin
            r[pos[:in_bin]] = np.float32(1.0) + np.float32(0.25 / 8) * rng.integers(0, 8, size=in_bin).astype(np.float32)
        rows[g] = r
    pooled = torch.from_numpy(rows.reshape(1, -1)).cuda()
    for c_max in (n_above + 1, n_above + in_bin // 2, n_above + in_bin):         # threshold inside the bin
        w = workloads.SpecKVWorkload(
            name="limits", n_layers=1, n_q_heads=H, n_kv_heads=H, head_dim=64, seq_lens=(n,),
            n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
        p = make_params(S, w)
        idx = torch.full((1, H * S.total_keep(p)), -1, dtype=torch.int32, device="cuda")
        S.speckv_select(p, pooled, idx)
        torch.cuda.synchronize()
        got = idx.cpu().numpy().reshape(H, -1)
        for g in range(H):
            want = orc.keep_indices(rows[g, :m].astype(np.float64), n, n_window, c_max)
            assert np.array_equal(got[g], want), (c_max, g)


@pytest.mark.parametrize("seed", [0, 1])
def test_split_row_selection_ragged(S, seed):
    """Few long ragged rows (split over workgroups, parts past a short row's end are empty) with
    heavy ties, against the oracle and against the one-workgroup path."""
    rng = np.random.default_rng(3000 + seed)
    n_window = int(rng.choice([0, 3, 64]))
    lens = (int(rng.integers(262144 + 70, 600000)), int(rng.integers(max(1, n_window), 5000)), 300001)
    H, L = 2, 1
    c_max = int(rng.choice([1, 4096, 250000]))
    w = workloads.SpecKVWorkload(
        name="split", n_layers=L, n_q_heads=H, n_kv_heads=H, head_dim=64, seq_lens=lens,
        n_window=n_window, n_lookahead=1, pool_k=7, c_max=c_max, dtype="bf16", sm_scale=1.0)
    p = make_params(S, w)
    T = w.total_tokens
    levels = int(rng.choice([4, 1000, 10 ** 7]))
    base = (rng.integers(0, levels, size=(L, H * T)).astype(np.float32) - levels // 5) / np.float32(levels)
    pooled = torch.from_numpy(base).cuda()
    outs = []
    assert S.plan_info(p)["select_parts"] > 1 and S.select_workspace_bytes(p) > 0
    for ws in (None, torch.empty(S.select_workspace_bytes(p), dtype=torch.uint8, device="cuda")):
        idx = torch.full((L, H * S.total_keep(p)), -1, dtype=torch.int32, device="cuda")
        S.speckv_select(p, pooled, idx, ws)
        torch.cuda.synchronize()
        outs.append(idx.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    for s in range(len(lens)):
        rows = split_scores(w, base, 0, s)
        got = split_keep(w, outs[1], 0, s, c_max)
        for g in range(H):
            want = orc.keep_indices(rows[g, :lens[s] - n_window].astype(np.float64), lens[s], n_window, c_max)
            assert np.array_equal(got[g], want), (seed, s, g)


def test_two_streams_with_their_own_workspaces(S):
    """The library keeps no state: calls enqueued on two streams at once, each with its own
    workspace and outputs, give the results of the same calls made one after the other."""
    wa = workloads.llama8b_layer(n_in=9000, c_max=300, n_layers=2, seed=41, name="stream_a")
    wb = workloads.ragged_batch(n_layers=2, lo=500, hi=4000, n_seqs=3, seed=42, name="stream_b")
    jobs = []
    for w in (wa, wb):
        t = workloads.generate(w)
        tg = {x: t[x].cuda() for x in ("q", "k", "v")}
        p = make_params(S, w)
        KT, L, H, d = S.total_keep(p), w.n_layers, w.n_kv_heads, w.head_dim
        outs = [(torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda"),
                 torch.zeros((L, H * KT, d), dtype=w.torch_dtype, device="cuda"),
                 torch.zeros((L, H * KT, d), dtype=w.torch_dtype, device="cuda")) for _ in range(2)]
        jobs.append((p, tg, outs, alloc_ws(S, p)))
    torch.cuda.synchronize()
    for p, tg, outs, ws in jobs:                                   # reference: one after the other
        S.speckv_compress(p, tg["q"], tg["k"], tg["v"], *outs[0], ws)
        torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for _ in range(3):                                             # interleaved on two streams
        for (p, tg, outs, ws), st in zip(jobs, streams):
            with torch.cuda.stream(st):
                S.speckv_compress(p, tg["q"], tg["k"], tg["v"], *outs[1], ws)
    torch.cuda.synchronize()
    for p, tg, outs, ws in jobs:
        for a, b in zip(outs[0], outs[1]):
            assert torch.equal(a, b)


@pytest.mark.parametrize("head_dim,group", [(128, 4), (64, 3)])
def test_half_precision_inputs(S, head_dim, group):
    """fp16 Q/K/V (the number type of the GPTQ/AWQ-quantised targets): same path, f16 MFMA."""
    w = workloads.SpecKVWorkload(
        name="f16", n_layers=2, n_q_heads=2 * group, n_kv_heads=2, head_dim=head_dim, seq_lens=(2500, 700),
        n_window=16, n_lookahead=24, pool_k=7, c_max=200, dtype="f16", sm_scale=1.0 / math.sqrt(head_dim),
        n_planted=4, channel_scale=(0.5, 4.0), seed=51)
    check_full_path(S, w)


def test_sharp_softmax_large_logits(S):
    """Logits with a standard deviation of tens of nats (max far above 100): rows are nearly one-hot,
    most probabilities underflow; no overflow, no NaN, and the scores still match the oracle."""
    w = workloads.SpecKVWorkload(
        name="sharp", n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_lens=(3000, 1500),
        n_window=32, n_lookahead=32, pool_k=7, c_max=300, dtype="bf16", sm_scale=1.0 / math.sqrt(128.0),
        q_gain=8.0, n_planted=4, channel_scale=(0.5, 4.0), seed=61)
    t = workloads.generate(w)
    logits = (t["q"][0, 0, :, 0].float() @ t["k"][0, :3000, 0].float().T) * w.sm_scale
    assert float(logits.std()) > 20 and float(logits.max()) > 100        # the case is what it claims to be
    check_full_path(S, w)


@pytest.mark.parametrize("dtype,n_planted", [("bf16", 6), ("f32", 512)])
def test_row_statistics_repair_launch(S, dtype, n_planted):
    """Sweeps of several rounds of workgroups take the row statistics against fixed reference exponents
    and leave overflowed segments to a repair launch.  Outliers hundreds of nats above the rest force
    that: a few per head (bf16: segments listed one by one, in the middle of 4096-key chunks), and one
    every 64 keys in fp32 (64-key tiles: every segment of a chunk overflows, far more than a
    wavefront lists, so the list's "every segment from here on" form is taken)."""
    w = workloads.SpecKVWorkload(
        name="repair_" + dtype, n_layers=8, n_q_heads=16, n_kv_heads=8, head_dim=128, seq_lens=(33000,),
        n_window=32, n_lookahead=32, pool_k=7, c_max=300, dtype=dtype, sm_scale=1.0 / math.sqrt(128.0),
        q_gain=8.0, n_planted=n_planted, channel_scale=(0.5, 4.0), seed=66)
    info = S.plan_info(make_params(S, w))
    assert info["fixed_reference_rows"] == 1 and info["chunk_keys"] == 4096
    assert info["tile_keys"] == (64 if dtype == "f32" else 128)
    check_full_path(S, w)


def test_row_statistics_modes_on_small_shapes(S, monkeypatch):
    """SPECKV_ROW_STATISTICS=fixed forces the fixed-reference sweep and its repair launch onto calls
    that would take the online step (one round of workgroups): ragged tails, partly filled row
    super-blocks, fp32 and fp16 tiles, chunks of one segment, outliers in a chunk's first tile.
    Both modes must match the oracle."""
    import dataclasses
    shapes = [workloads.llama8b_layer(n_in=4096 + 300, c_max=512, name="modes_8b"),
              workloads.ragged_batch(n_layers=2, lo=200, hi=2500, n_seqs=4, seed=4, name="modes_ragged"),
              workloads.tiny_fp32(),
              workloads.SpecKVWorkload(name="modes_sharp", n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128,
                                       seq_lens=(3000, 1500), n_window=32, n_lookahead=32, pool_k=7, c_max=300,
                                       dtype="bf16", sm_scale=1.0 / math.sqrt(128.0), q_gain=8.0, n_planted=4,
                                       channel_scale=(0.5, 4.0), seed=61),
              workloads.SpecKVWorkload(name="modes_f16", n_layers=2, n_q_heads=6, n_kv_heads=2, head_dim=128,
                                       seq_lens=(1700,), n_window=16, n_lookahead=24, pool_k=7, c_max=200,
                                       dtype="f16", sm_scale=1.0 / math.sqrt(128.0), n_planted=4,
                                       channel_scale=(0.5, 4.0), seed=51)]
    for mode in ("fixed", "online"):
        monkeypatch.setenv("SPECKV_ROW_STATISTICS", mode)
        for w in shapes:
            info = S.plan_info(make_params(S, w))
            if info["q_stationary"] & 1 == 0 and info["n_chunks"] > 0:
                assert info["fixed_reference_rows"] == (1 if mode == "fixed" else 0), w.name
            check_full_path(S, w)


def test_q_stationary_kernel_against_oracle_and_tile_kernel(S, monkeypatch):
    """The alternative scoring dataflow (query rows stationary in LDS, SPECKV_SCORE_KERNEL=qs)
    against the oracle on sum and max reduction, G = 4 and G = 7, d = 128 and d = 64, and
    its index sets against the default kernel's."""
    cases = [
        (workloads.llama8b_layer(n_in=9000 + 77, c_max=512, n_layers=2, name="qs_8b"), "sum"),
        (workloads.llama8b_layer(n_in=5000, c_max=300, name="qs_8b_max"), "max"),
        (workloads.ragged_batch(n_layers=2, lo=600, hi=6000, n_seqs=3, seed=12, name="qs_gqa7"), "sum"),
        (workloads.specpc_draft(n_in=8192 + 300, n_layers=2, name="qs_d64"), "sum"),
    ]
    for w, reduce in cases:
        t = workloads.generate(w)
        tg = {x: t[x].cuda() for x in ("q", "k", "v")}
        c_max = min(w.c_max, 256)
        monkeypatch.setenv("SPECKV_SCORE_KERNEL", "tile")
        p = make_params(S, w, c_max=c_max, reduce=reduce)
        assert S.plan_info(p)["q_stationary"] == 0
        _, idx_tile, _, _ = run_compress(S, w, tg, c_max=c_max, reduce=reduce)
        monkeypatch.delenv("SPECKV_SCORE_KERNEL", raising=False)
        # default: only the row-statistics sweep at d = 64 keeps the query rows stationary
        assert S.plan_info(p)["q_stationary"] == (1 if w.head_dim == 64 else 0)
        monkeypatch.setenv("SPECKV_SCORE_KERNEL", "qs")
        assert S.plan_info(p)["q_stationary"] == 3, "the geometry of %s should be supported" % w.name
        check_full_path(S, w, c_max=c_max, reduce=reduce)
        _, idx_qs, _, _ = run_compress(S, w, tg, c_max=c_max, reduce=reduce)
        monkeypatch.delenv("SPECKV_SCORE_KERNEL", raising=False)
        # the two kernels sum in different orders: rows may differ only inside the tolerance band,
        # which check_full_path has verified against the oracle; most rows agree exactly
        same = (idx_tile == idx_qs).all(axis=-1).mean() if idx_tile.ndim > 1 else float((idx_tile == idx_qs).all())
        assert (idx_tile == idx_qs).mean() > 0.98, (w.name, same)


def test_token_selection_with_stage_events_matches_the_plain_call(S):
    """`specpc_select_tokens_events` (the benchmark's timing variant) records its seven marks on the
    launch stream and returns exactly what `specpc_select_tokens` returns."""
    import ctypes
    w = workloads.specpc_draft(n_in=5000, n_layers=3, name="pc_events")
    t = workloads.generate(w)
    q, k = t["q"].cuda(), t["k"].cuda()
    ids = workloads.generate_token_ids(w).cuda()
    p = make_params(S, w)
    top_k, nb, n = 300, 4, w.seq_lens[0]
    ws = torch.empty(S.specpc_workspace_bytes(p, top_k), dtype=torch.uint8, device="cuda")
    outs = []
    events = [torch.cuda.Event(enable_timing=True) for _ in range(S.N_STAGE_EVENTS)]
    for e in events:
        e.record()                                   # creates the underlying HIP events
    arr = (ctypes.c_void_p * S.N_STAGE_EVENTS)(*[e.cuda_event for e in events])
    for timed in (False, True):
        idx_out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        ids_out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        count = torch.zeros(1, dtype=torch.int32, device="cuda")
        if timed:
            S.specpc_select_tokens_events(p, top_k, nb, q, k, ids, idx_out, ids_out, count, ws, arr)
        else:
            S.specpc_select_tokens(p, top_k, nb, q, k, ids, idx_out, ids_out, count, ws)
        torch.cuda.synchronize()
        outs.append((idx_out, ids_out, count))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert int(outs[0][2].item()) > top_k
    stage_ms = [events[i].elapsed_time(events[i + 1]) for i in range(S.N_STAGE_EVENTS - 1)]
    assert all(ms >= 0.0 for ms in stage_ms) and sum(stage_ms) > 0.0


def test_ceiling_probe_runs_and_reports_its_flops(S):
    """The diagnostic loops behind `bench.py --ceilings` launch, finish and report the flops of the
    launch: 256 workgroups x 8 waves x iters x 8 MFMAs of 32x32x16."""
    ops = torch.randn(1 << 16, device="cuda").to(torch.bfloat16)
    out = torch.full((256 * 512,), float("nan"), dtype=torch.float32, device="cuda")
    for kind in (0, 1, 2):
        flops = S.probe_ceiling(kind, 10, ops, out)
        torch.cuda.synchronize()
        assert flops == 256 * 8 * 10 * 8 * 32768
        assert not bool(torch.isnan(out).any())


def test_token_selection_ignores_the_reduction_and_pooling_options(S):
    """`specpc_select_tokens` is defined as sum aggregation with max pooling: parameters that ask for
    max reduction or average pooling give the same tokens (rows above one workgroup's 512 rows, so
    that a head spans several partial planes, the case where mixing the two would show)."""
    base = workloads.specpc_draft(n_in=3000, n_layers=2, name="pc_ops")
    w = workloads.SpecKVWorkload(**{**base.__dict__, "n_q_heads": 4, "n_kv_heads": 2, "n_window": 64,
                                    "n_lookahead": 500})
    t = workloads.generate(w)
    q, k = t["q"].cuda(), t["k"].cuda()
    ids = workloads.generate_token_ids(w).cuda()
    top_k, nb, n = 200, 3, w.seq_lens[0]
    outs = []
    for reduce, pool in (("sum", "max"), ("max", "avg")):
        p = make_params(S, w, reduce=reduce, pool=pool)
        ws = torch.empty(S.specpc_workspace_bytes(p, top_k), dtype=torch.uint8, device="cuda")
        idx_out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        ids_out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        count = torch.zeros(1, dtype=torch.int32, device="cuda")
        S.specpc_select_tokens(p, top_k, nb, q, k, ids, idx_out, ids_out, count, ws)
        torch.cuda.synchronize()
        outs.append((idx_out, ids_out, count))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    ref = orc.specpc_select_tokens(workloads.to_float64(t["q"][:, 0]), workloads.to_float64(t["k"]),
                                   ids.cpu().numpy(), w.n_window, w.pool_k, top_k, nb, w.sm_scale)
    c = int(outs[0][2].item())
    got = outs[0][0][:c].cpu().numpy().astype(np.int64)
    m = n - w.n_window
    if not np.array_equal(got, ref["idx"]):
        tau = np.sort(ref["pooled"])[m - top_k]
        band = REL_TOL * tau + ABS_FLOOR * ref["pooled"].max()
        lo = orc.expand_neighbors(np.nonzero(ref["pooled"] > tau + band)[0], n, w.n_window, nb)
        hi = orc.expand_neighbors(np.nonzero(ref["pooled"] >= tau - band)[0], n, w.n_window, nb)
        assert np.isin(lo, got).all() and np.isin(got, hi).all()


def test_more_than_65535_layer_head_units(S):
    """Many layers times many KV heads: the launch grids put (layer, head) on the x dimension, which
    has no 65535 limit."""
    w = workloads.SpecKVWorkload(
        name="many_units", n_layers=1100, n_q_heads=64, n_kv_heads=64, head_dim=64, seq_lens=(300,),
        n_window=8, n_lookahead=8, pool_k=7, c_max=32, dtype="bf16", sm_scale=0.125, n_planted=2,
        channel_scale=(0.5, 4.0), seed=41)
    assert w.n_layers * w.n_kv_heads > 65535
    t = workloads.generate(w, layers=range(3))                       # three distinct layers, tiled
    reps = (w.n_layers + 2) // 3
    q = t["q"].repeat(reps, 1, 1, 1, 1)[: w.n_layers].cuda()
    k = t["k"].repeat(reps, 1, 1, 1)[: w.n_layers].cuda()
    v = t["v"].repeat(reps, 1, 1, 1)[: w.n_layers].cuda()
    p = make_params(S, w)
    KT, L, H, d = S.total_keep(p), w.n_layers, w.n_kv_heads, w.head_dim
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    k_out = torch.zeros((L, H * KT, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.zeros_like(k_out)
    S.speckv_compress(p, q, k, v, idx, k_out, v_out, alloc_ws(S, p))
    torch.cuda.synchronize()
    # every third layer has the same inputs, so the same outputs; the first three against the oracle
    idx3 = idx.view(L, H, KT)
    for layer in range(3, L):
        if layer % 97 == 0 or layer >= L - 3:
            assert torch.equal(idx3[layer], idx3[layer % 3])
            assert torch.equal(k_out[layer], k_out[layer % 3])
    w3 = workloads.SpecKVWorkload(**{**w.__dict__, "n_layers": 3})
    ref = oracle_batch(w3, t)
    n = w.seq_lens[0]
    got = idx3[:3].cpu().numpy()
    for layer in range(3):
        for g in range(H):
            assert_indices_valid(got[layer, g], ref[layer][0]["pooled"][g], n, w.n_window, w.c_max,
                                 "many units l%d g%d" % (layer, g))
