"""GPU parity at the full sizes of the benchmark configurations.

The workloads are generated on the GPU (the tensors are too large to draw on the host
quickly); the oracle gets the same bits by downloading the sampled (layer, sequence)
slices.  Every layer, sequence and head is checked for the structural properties that
hold at any size; sampled heads are compared with the float64 oracle element by element.
The calls use the same launch configuration the benchmark times (one fused
`speckv_compress` over the whole workload).
"""
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
    lib.load_library()
    return lib


def run_workload(S, w, want_scores=True, reduce="sum"):
    data = workloads.generate(w, device="cuda")
    q, k, v = data["q"], data["k"], data["v"]
    p = S.SpecKVParams.for_tensors(q, k, seq_lens=w.seq_lens, n_window=w.n_window, pool_k=w.pool_k,
                                   c_max=w.c_max, sm_scale=w.sm_scale, reduce=reduce)
    KT, L, H, d = S.total_keep(p), w.n_layers, w.n_kv_heads, w.head_dim
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
    v_out = torch.empty_like(k_out)
    ws = torch.empty(S.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    pooled = None
    if want_scores:
        pooled = torch.empty((L, H * w.total_tokens), dtype=torch.float32, device="cuda")
        S.speckv_score(p, q, k, pooled, None, ws)
    S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)
    torch.cuda.synchronize()
    return data, p, idx, k_out, v_out, pooled


def keep_layout(w):
    keeps = [w.n_keep(s) for s in range(w.n_seqs)]
    return keeps, np.concatenate([[0], np.cumsum(keeps)])


def check_structure_everywhere(w, data, idx, k_out, v_out):
    """Properties that hold at any size, checked on the GPU for every (layer, seq, head)."""
    keeps, ck = keep_layout(w)
    cu = w.cu_seqlens
    H = w.n_kv_heads
    for s in range(w.n_seqs):
        n, m, nk = w.seq_lens[s], w.seq_lens[s] - w.n_window, keeps[s]
        C = nk - w.n_window
        rows = idx[:, H * ck[s]: H * ck[s + 1]].reshape(w.n_layers, H, nk).long()
        assert bool((rows[..., 1:] > rows[..., :-1]).all()), "indices not strictly ascending"
        assert bool((rows[..., 0] >= 0).all()) and bool((rows[..., :C] < m).all())
        win = torch.arange(m, n, device="cuda")
        assert bool((rows[..., C:] == win).all()), "window not kept last"
        planted = data["planted"][:, s]                                    # [L, H, P]
        hit = (rows[..., None, :C] == planted[..., :, None]).any(-1)       # [L, H, P]
        assert bool(hit.all()), "a planted heavy hitter was dropped"
        # compaction is a bit copy of the selected rows
        view = torch.int16 if w.dtype != "f32" else torch.int32
        ksrc = data["k"][:, cu[s]:cu[s + 1]].view(view)                    # [L, n, H, d]
        vsrc = data["v"][:, cu[s]:cu[s + 1]].view(view)
        ko = k_out[:, H * ck[s]: H * ck[s + 1]].view(view).reshape(w.n_layers, H, nk, w.head_dim)
        vo = v_out[:, H * ck[s]: H * ck[s + 1]].view(view).reshape(w.n_layers, H, nk, w.head_dim)
        for g in range(H):
            for layer in range(w.n_layers):
                assert torch.equal(ko[layer, g], ksrc[layer, rows[layer, g], g])
                assert torch.equal(vo[layer, g], vsrc[layer, rows[layer, g], g])


def check_sampled_heads(w, data, idx, pooled, samples, reduce="sum"):
    """Element-by-element comparison with the oracle on sampled (layer, seq, head) triples."""
    keeps, ck = keep_layout(w)
    cu = w.cu_seqlens
    H, G = w.n_kv_heads, w.group
    exact = 0
    for layer, s, g in samples:
        n, m = w.seq_lens[s], w.seq_lens[s] - w.n_window
        qh = workloads.to_float64(data["q"][layer, s, :, g * G:(g + 1) * G])
        kh = workloads.to_float64(data["k"][layer, cu[s]:cu[s + 1], g:g + 1])
        raw = orc.raw_scores(qh, kh, w.n_window, w.sm_scale, reduce=reduce)
        ref_pooled = orc.pooled_scores(raw, w.n_window, w.pool_k)[0]
        if reduce == "sum":
            assert abs(raw.sum() - w.n_rows * G) < 1e-6 * w.n_rows * G    # oracle sanity at this size
        a = H * cu[s] + g * n
        got = pooled[layer, a:a + m].double().cpu().numpy()
        tol = REL_TOL * np.abs(ref_pooled) + ABS_FLOOR * np.abs(ref_pooled).max()
        bad = np.abs(got - ref_pooled) > tol
        assert not bad.any(), "pooled scores off at (l%d,s%d,g%d): %d entries" % (layer, s, g, bad.sum())
        C = keeps[s] - w.n_window
        b = H * ck[s] + g * keeps[s]
        sel = idx[layer, b:b + C].cpu().numpy().astype(np.int64)
        want = orc.select_top(ref_pooled, C)
        if np.array_equal(sel, want):
            exact += 1
            continue
        tau = np.sort(ref_pooled)[m - C]
        band = REL_TOL * abs(tau) + ABS_FLOOR * np.abs(ref_pooled).max()
        assert np.isin(np.nonzero(ref_pooled > tau + band)[0], sel).all()
        assert not np.isin(np.nonzero(ref_pooled < tau - band)[0], sel).any()
    return exact


def test_llama8b_single_layer_32k_full_oracle(S):
    w = workloads.llama8b_layer()
    data, p, idx, k_out, v_out, pooled = run_workload(S, w)
    check_structure_everywhere(w, data, idx, k_out, v_out)
    exact = check_sampled_heads(w, data, idx, pooled, [(0, 0, g) for g in range(w.n_kv_heads)])
    assert exact >= w.n_kv_heads // 2


def test_llama8b_full_stack_128k(S):
    w = workloads.llama8b_full_128k()
    data, p, idx, k_out, v_out, pooled = run_workload(S, w)
    check_structure_everywhere(w, data, idx, k_out, v_out)
    # every KV head of the first, a middle and the last layer against the oracle
    check_sampled_heads(w, data, idx, pooled, [(layer, 0, g) for layer in (0, 15, 31) for g in range(w.n_kv_heads)])


def test_ragged_batch_full(S):
    w = workloads.ragged_batch()
    data, p, idx, k_out, v_out, pooled = run_workload(S, w)
    check_structure_everywhere(w, data, idx, k_out, v_out)
    # one head of every sequence (layers and heads rotate), plus the two extreme lengths on other layers
    longest = int(np.argmax(w.seq_lens))
    shortest = int(np.argmin(w.seq_lens))
    samples = [((5 * s) % w.n_layers, s, s % w.n_kv_heads) for s in range(w.n_seqs)]
    check_sampled_heads(w, data, idx, pooled, samples + [(0, shortest, 0), (27, longest, 3)])


def test_specpc_full(S):
    w = workloads.specpc_draft()
    top_k, nb = w.c_max, workloads.SPECPC_NEIGHBORS
    data = workloads.generate(w, device="cuda")
    ids = workloads.generate_token_ids(w, device="cuda")
    n = w.seq_lens[0]
    p = S.SpecKVParams.for_tensors(data["q"], data["k"], seq_lens=w.seq_lens, n_window=w.n_window,
                                   pool_k=w.pool_k, c_max=w.c_max, sm_scale=w.sm_scale)
    ws = torch.empty(S.specpc_workspace_bytes(p, top_k), dtype=torch.uint8, device="cuda")
    idx_out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    ids_out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    S.specpc_select_tokens(p, top_k, nb, data["q"], data["k"], ids, idx_out, ids_out, count, ws)
    torch.cuda.synchronize()
    c = int(count.item())
    got = idx_out[:c].cpu().numpy().astype(np.int64)
    assert (np.diff(got) > 0).all() and bool((idx_out[c:] == -1).all())
    assert torch.equal(ids_out[:c], ids[idx_out[:c].long()])
    m = n - w.n_window
    assert got[-w.n_window:].tolist() == list(range(m, n))
    ref = orc.specpc_select_tokens(workloads.to_float64(data["q"][:, 0]), workloads.to_float64(data["k"]),
                                   ids.cpu().numpy(), w.n_window, w.pool_k, top_k, nb, w.sm_scale)
    if np.array_equal(got, ref["idx"]):
        return
    tau = np.sort(ref["pooled"])[m - top_k]
    band = REL_TOL * tau + ABS_FLOOR * ref["pooled"].max()
    lo = orc.expand_neighbors(np.nonzero(ref["pooled"] > tau + band)[0], n, w.n_window, nb)
    hi = orc.expand_neighbors(np.nonzero(ref["pooled"] >= tau - band)[0], n, w.n_window, nb)
    assert np.isin(lo, got).all() and np.isin(got, hi).all()


def test_shared_layer_budget_128k(S):
    """Per-head budgets (App. "Integration and Comparison with the AdaKV Baseline") at the 128K
    shape: structure for every layer and head on the GPU, one whole layer against the oracle."""
    w = workloads.llama8b_layer(n_in=131072, c_max=2048, n_layers=2, name="ada_128k")
    c_floor = 410                                                         # a fifth of the budget
    data = workloads.generate(w, device="cuda")
    q, k, v = data["q"], data["k"], data["v"]
    p = S.SpecKVParams.for_tensors(q, k, seq_lens=w.seq_lens, n_window=w.n_window, pool_k=w.pool_k,
                                   c_max=w.c_max, sm_scale=w.sm_scale)
    KT, L, H, d, G = S.total_keep(p), w.n_layers, w.n_kv_heads, w.head_dim, w.group
    n, m = w.seq_lens[0], w.seq_lens[0] - w.n_window
    idx = torch.full((L, H * KT), -1, dtype=torch.int32, device="cuda")
    head_off = torch.full((L, 1, H + 1), -1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
    v_out = torch.empty_like(k_out)
    ws = torch.empty(S.ada_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    S.speckv_compress_ada(p, c_floor, q, k, v, idx, head_off, k_out, v_out, ws)
    torch.cuda.synchronize()
    off = head_off.cpu().numpy()[:, 0]
    assert (off[:, 0] == 0).all() and (off[:, -1] == H * KT).all()
    counts = np.diff(off, axis=1) - w.n_window
    assert (counts >= c_floor).all() and (counts.sum(axis=1) == H * w.c_max).all()
    assert (counts != w.c_max).any(), "the budgets did not move between heads: nothing was tested"
    win = torch.arange(m, n, device="cuda")
    for layer in range(L):
        for g in range(H):
            rows = idx[layer, off[layer, g]:off[layer, g + 1]].long()
            assert bool((rows[1:] > rows[:-1]).all()) and bool((rows[-w.n_window:] == win).all())
            planted = data["planted"][layer, 0, g]
            assert bool((rows[:-w.n_window, None] == planted[None, :]).any(0).all())
            assert torch.equal(k_out[layer, off[layer, g]:off[layer, g + 1]].view(torch.int16),
                               k[layer, rows, g].view(torch.int16))
            assert torch.equal(v_out[layer, off[layer, g]:off[layer, g + 1]].view(torch.int16),
                               v[layer, rows, g].view(torch.int16))
    # one whole layer through the oracle: the heads' scores, then the shared-budget rule
    layer = 1
    pooled = np.stack([
        orc.pooled_scores(orc.raw_scores(workloads.to_float64(q[layer, 0, :, g * G:(g + 1) * G]),
                                         workloads.to_float64(k[layer, :, g:g + 1]),
                                         w.n_window, w.sm_scale), w.n_window, w.pool_k)[0]
        for g in range(H)])
    want = orc.ada_keep_indices(pooled, n, w.n_window, w.c_max, c_floor)
    got = [idx[layer, off[layer, g]:off[layer, g + 1]].cpu().numpy().astype(np.int64) for g in range(H)]
    if all(np.array_equal(a, b) for a, b in zip(got, want)):
        return
    # scores within the tolerance of the layer-wide threshold may fall either way
    kept = np.concatenate([pooled[g][want[g][:-w.n_window]] for g in range(H)])
    tau = kept.min()
    band = REL_TOL * abs(tau) + ABS_FLOOR * pooled.max()
    for g in range(H):
        sel = got[g][:-w.n_window]
        floor_tau = np.sort(pooled[g])[m - c_floor]                       # the head's own floor threshold
        must = np.nonzero(pooled[g] > min(tau, floor_tau) + band)[0]
        never = np.nonzero(pooled[g] < min(tau, floor_tau) - band)[0]
        assert np.isin(must, sel).all() and not np.isin(never, sel).any()


def test_one_million_token_prompt(S):
    """Eight times the longest benchmark prompt, ragged end: 64-bit offsets, many chunks, and the
    fp32 column sums of 2^20 keys against the float64 oracle on one head."""
    base = workloads.llama8b_layer(n_in=(1 << 20) + 77, c_max=4096, n_layers=1, seed=31, name="one_million")
    w = workloads.SpecKVWorkload(**{**base.__dict__, "n_q_heads": 4, "n_kv_heads": 2})
    data, p, idx, k_out, v_out, pooled = run_workload(S, w)
    check_structure_everywhere(w, data, idx, k_out, v_out)
    check_sampled_heads(w, data, idx, pooled, [(0, 0, 1)])


def test_paper_evaluated_setting_128k(S):
    """The hyper-parameter table's SpecKV column at the 128K shape: Reduction = Max (Alg. 1
    MaxReduce), Pool = Max with k = 7, n_window = 32, 96 lookahead rows, budget C_max - n_window
    non-window keys.  Structure on every layer and head; every KV head of two layers against the
    oracle element by element."""
    import dataclasses
    base = workloads.llama8b_layer(n_in=131072, c_max=2048 - 32, n_layers=4, seed=7, name="paper_setting_128k")
    w = dataclasses.replace(base, n_window=32, n_lookahead=96, pool_k=7)
    data, p, idx, k_out, v_out, pooled = run_workload(S, w, reduce="max")
    assert S.plan_info(p)["reduce_max"] == 1
    check_structure_everywhere(w, data, idx, k_out, v_out)
    check_sampled_heads(w, data, idx, pooled, [(layer, 0, g) for layer in (0, 3) for g in range(w.n_kv_heads)],
                        reduce="max")


def test_specpc_table_setting_full(S):
    """Alg. 2 with the hyper-parameter table's SpecPC column on the draft-model shape: window 64,
    one lookahead row, l_skip = 8, average pooling with kernel 64, max pooling over 64 neighbours,
    2048 kept tokens, 64K prompt tokens, 16 layers."""
    import dataclasses
    base = workloads.specpc_draft()
    w = dataclasses.replace(base, n_lookahead=1, pool_k=64, c_max=2048, name="c5_table_setting")
    l_skip, n_neighbor = 8, 64
    data = workloads.generate(w, device="cuda")
    ids = workloads.generate_token_ids(w, device="cuda")
    n, m = w.seq_lens[0], w.seq_lens[0] - w.n_window
    p = S.SpecKVParams.for_tensors(data["q"], data["k"], seq_lens=w.seq_lens, n_window=w.n_window,
                                   pool_k=w.pool_k, c_max=w.c_max, sm_scale=w.sm_scale)
    ws = torch.empty(S.specpc_compress_workspace_bytes(p, l_skip), dtype=torch.uint8, device="cuda")
    cap = w.c_max + w.n_window
    idx_out = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    ids_out = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    S.specpc_compress_prompt(p, l_skip, n_neighbor, data["q"], data["k"], ids, idx_out, ids_out, count, ws)
    torch.cuda.synchronize()
    assert int(count.item()) == cap
    got = idx_out.cpu().numpy().astype(np.int64)
    assert (np.diff(got) > 0).all() and got[-w.n_window:].tolist() == list(range(m, n))
    assert torch.equal(ids_out, ids[idx_out.long()])
    ref = orc.specpc_compress_prompt(workloads.to_float64(data["q"][:, 0]), workloads.to_float64(data["k"]),
                                     ids.cpu().numpy(), w.n_window, w.pool_k, n_neighbor, w.c_max, l_skip,
                                     w.sm_scale)
    if np.array_equal(got, ref["idx"]):
        return
    pooled = ref["pooled"]
    tau = np.sort(pooled)[m - w.c_max]
    band = REL_TOL * abs(tau) + ABS_FLOOR * np.abs(pooled).max()
    sel = got[:w.c_max]
    assert np.isin(np.nonzero(pooled > tau + band)[0], sel).all()
    assert not np.isin(np.nonzero(pooled < tau - band)[0], sel).any()
