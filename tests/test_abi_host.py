"""Host-side checks that need no GPU: the library loads, exports its ABI, validates arguments."""
import ctypes
import os
import re

import pytest
import torch

import paper_2506_08373_amd as S
from paper_2506_08373_amd import binding


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(S.library_path()):
        from paper_2506_08373_amd import build
        build.build(verbose=False)
    return S.load_library()


PLAN_INFO_WORDS = 11     # SPECKV_PLAN_INFO_WORDS of include/speckv.h


def base_params(**kw):
    args = dict(n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=64, seq_lens=[300, 500], n_window=16,
                n_lookahead=16, pool_k=7, c_max=64, sm_scale=0.125, dtype=torch.bfloat16)
    args.update(kw)
    return S.SpecKVParams(**args)


def test_every_declared_symbol_is_exported(lib, repo_root):
    header = open(os.path.join(repo_root, "include", "speckv.h")).read()
    declared = set(re.findall(r"\b(speck?v?_[a-z_]+|specpc_[a-z_]+)\s*\(", header))
    declared = {d for d in declared if not d.endswith("_t")}
    assert {"speckv_score", "speckv_select", "speckv_compact", "speckv_compress",
            "specpc_select_tokens"} <= declared
    for name in declared:
        assert hasattr(lib, name), "header declares %s but the library does not export it" % name
    assert set(binding.EXPORTS) == declared


def test_plan_info_word_count_matches_the_header(repo_root):
    header = open(os.path.join(repo_root, "include", "speckv.h")).read()
    assert int(re.search(r"#define SPECKV_PLAN_INFO_WORDS (\d+)", header).group(1)) == PLAN_INFO_WORDS


def test_status_strings(lib):
    assert lib.speckv_status_string(0) == b"ok"
    assert b"workspace" in lib.speckv_status_string(-3)


def test_keep_counts_follow_the_budget_rule(lib):
    p = base_params(seq_lens=[300, 20, 500], c_max=64, n_window=16)
    assert [S.n_keep(p, s) for s in range(3)] == [80, 20, 80]     # min(c_max, m) + n_window
    assert S.total_keep(p) == 180
    assert S.n_keep(p, 3) == -1
    assert S.workspace_bytes(p) > 0 and S.workspace_bytes(p) % 256 == 0


@pytest.mark.parametrize("kw", [
    dict(n_q_heads=7),                       # not a multiple of n_kv_heads
    dict(pool_k=0),
    dict(c_max=-1),
    dict(sm_scale=0.0),
    dict(sm_scale=float("nan")),
    dict(n_window=0, n_lookahead=0),         # no observation rows
    dict(seq_lens=[300, 10]),                # shorter than the window
    dict(seq_lens=[300, 0]),
    dict(n_layers=0),
    dict(q_strides=(1, 1, 1, 3)),            # rows not 16-byte aligned
])
def test_invalid_arguments_are_rejected_before_any_launch(lib, kw):
    p = base_params(**kw)
    assert S.workspace_bytes(p) == 0
    # pointers are never touched when validation fails: dummy non-null values are safe here
    st = lib.speckv_compress(p.ref(), 256, 256, 256, 256, 256, 256, 256, 1 << 40, None)
    assert st == -1


@pytest.mark.parametrize("kw", [dict(head_dim=96), dict(pool_k=257), dict(seq_lens=[64] * 129),
                                dict(n_q_heads=64, n_kv_heads=1, n_lookahead=100)])
def test_unsupported_configurations(lib, kw):
    p = base_params(**kw)
    st = lib.speckv_compress(p.ref(), 256, 256, 256, 256, 256, 256, 256, 1 << 40, None)
    assert st == -2


def test_select_workspace_is_small_and_checked(lib):
    """Selection needs scratch only when few, very long rows are split over workgroups; the size is
    a few MiB, far below the scoring workspace, and a smaller buffer is refused before any launch."""
    short = base_params()
    assert S.select_workspace_bytes(short) == 0
    long_rows = base_params(n_layers=1, seq_lens=[600000], c_max=4096)
    need = S.select_workspace_bytes(long_rows)
    assert 0 < need < S.workspace_bytes(long_rows) and need % 256 == 0 and need < (16 << 20)
    assert S.plan_info(long_rows)["select_parts"] > 1
    assert lib.speckv_select(long_rows.ref(), 256, 256, 256, need - 1, None) == -3
    assert lib.speckv_select(long_rows.ref(), 256, 256, 257, need, None) == -3      # misaligned


def test_device_side_count_needs_one_sequence_and_supported_entry_points(lib):
    """n_in_dev is validated on the host like everything else (the pointer itself is never read
    there): one sequence only, 4-byte aligned, and not for the entry points that do not honour it."""
    p = base_params(seq_lens=[500])
    p.c.n_in_dev = 1024
    need = S.workspace_bytes(p)
    assert need > 0
    two = base_params()
    two.c.n_in_dev = 1024
    assert S.workspace_bytes(two) == 0
    assert lib.speckv_compress(two.ref(), 256, 256, 256, 256, 256, 256, 256, 1 << 40, None) == -2
    p.c.n_in_dev = 1026
    assert lib.speckv_compress(p.ref(), 256, 256, 256, 256, 256, 256, 256, 1 << 40, None) == -1
    p.c.n_in_dev = 1024
    assert lib.specpc_select_tokens(p.ref(), 10, 1, 256, 256, 256, 256, 256, 256, 256, 1 << 40, None) == -2


def test_null_misaligned_and_workspace_errors(lib):
    p = base_params()
    need = S.workspace_bytes(p)
    ok = 256
    assert lib.speckv_compress(p.ref(), None, ok, ok, ok, ok, ok, ok, need, None) == -1
    assert lib.speckv_compress(p.ref(), ok + 2, ok, ok, ok, ok, ok, ok, need, None) == -1     # q misaligned
    assert lib.speckv_compress(p.ref(), ok, ok, ok, ok, ok, None, ok, need, None) == -1       # v without v_out
    assert lib.speckv_compress(p.ref(), ok, ok, ok, ok, ok, ok, None, need, None) == -3
    assert lib.speckv_compress(p.ref(), ok, ok, ok, ok, ok, ok, ok, need - 1, None) == -3
    assert lib.speckv_compress(p.ref(), ok, ok, ok, ok, ok, ok, ok + 16, need, None) == -3    # ws misaligned
    assert lib.speckv_score(p.ref(), ok, ok, None, None, ok, need, None) == -1
    assert lib.speckv_select(p.ref(), None, ok, None, 0, None) == -1
    assert lib.speckv_compact(p.ref(), ok, ok, None, ok, ok, None) == -1
    assert lib.specpc_select_tokens(p.ref(), 10, 2, ok, ok, ok, ok, ok, ok, ok, 1 << 40, None) == -2  # 2 sequences
    one = base_params(seq_lens=[300])
    assert lib.specpc_select_tokens(one.ref(), -1, 2, ok, ok, ok, ok, ok, ok, ok, 1 << 40, None) == -1
    assert lib.specpc_select_tokens(one.ref(), 10, 2, ok, ok, ok, ok, ok, ok, ok, 16, None) == -3
    evs = (ctypes.c_void_p * 7)()
    assert lib.speckv_compress_events(p.ref(), ok, ok, ok, ok, ok, ok, ok, need, None, evs, 7) == -1  # null events
    assert lib.speckv_compress_events(p.ref(), ok, ok, ok, ok, ok, ok, ok, need, None, None, 7) == -1


def test_number_types(lib):
    for dt in (torch.bfloat16, torch.float16, torch.float32):
        assert S.workspace_bytes(base_params(dtype=dt)) > 0
    p = base_params()
    p.c.dtype = 3                                            # not a speckv_dtype
    assert S.workspace_bytes(p) == 0


def test_shared_budget_entry_points_validate(lib):
    p = base_params()
    ok = 256
    need = S.ada_workspace_bytes(p)
    assert need > S.workspace_bytes(p)
    assert lib.speckv_select_ada(p.ref(), -1, ok, ok, ok, ok, need, None) == -1           # negative floor
    assert lib.speckv_select_ada(p.ref(), 3, ok, ok, None, ok, need, None) == -1          # no head_off
    assert lib.speckv_select_ada(p.ref(), 3, ok, ok, ok, ok, need - 1, None) == -3
    assert lib.speckv_compact_ada(p.ref(), ok, ok, ok, None, ok, ok, None) == -1
    assert lib.speckv_compress_ada(p.ref(), 3, ok, ok, ok, ok, ok, ok, ok, None, need, None) == -3
    assert lib.speckv_compress_ada(p.ref(), 3, ok, ok, None, ok, ok, ok, ok, ok, need, None) == -1   # v_out without v
    many = base_params(n_q_heads=256, n_kv_heads=256)
    assert S.ada_workspace_bytes(many) == 0
    assert lib.speckv_select_ada(many.ref(), 3, ok, ok, ok, ok, 1 << 40, None) == -2


def test_binding_refuses_host_tensors(lib):
    p = base_params()
    x = torch.zeros(4)
    with pytest.raises(ValueError):
        S.speckv_select(p, x, x.to(torch.int32))


def test_bench_refuses_more_than_one_gpu(repo_root):
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


# --------------------------------------------------------------------------- #
# The host's launch plan (no GPU needed)
# --------------------------------------------------------------------------- #
def test_plan_of_the_benchmark_configurations(lib):
    import workloads
    def plan(w):
        return S.plan_info(S.SpecKVParams(
            n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
            seq_lens=list(w.seq_lens), n_window=w.n_window, n_lookahead=w.n_lookahead, pool_k=w.pool_k,
            c_max=w.c_max, sm_scale=w.sm_scale, dtype=w.torch_dtype))
    c3 = plan(workloads.llama8b_full_128k())
    # 512 rows per KV group: 8 waves x 2 blocks, one super-block; 4 equal chunks per (layer, head)
    # = 1024 identical workgroups = 4 whole rounds on 256 CUs
    assert (c3["waves"], c3["blocks_per_wave"], c3["row_super_blocks"]) == (8, 2, 1)
    assert c3["chunk_keys"] == 32768 and c3["n_chunks"] == 4 and c3["tile_keys"] == 128
    assert c3["select_parts"] == 1
    c4 = plan(workloads.ragged_batch())
    # G = 7: two super-blocks; ragged lengths: chunks shortened to balance the last round
    assert c4["row_super_blocks"] == 2 and c4["chunk_keys"] == 8192
    c5 = plan(workloads.specpc_draft())
    assert c5["tile_keys"] == 256 and (c5["waves"], c5["blocks_per_wave"]) == (8, 1)
    tiny = plan(workloads.tiny_fp32())
    assert (tiny["waves"], tiny["blocks_per_wave"]) == (4, 1) and tiny["tile_keys"] == 128
    # one layer of the 8B shape: the chunk workgroups and the 8 masked-tail workgroups of a sweep share
    # one launch and fit one round of the 256 CUs together (chunks a little longer than 1/32 of the prompt)
    for n_in in (32768, 131072):
        one = plan(workloads.llama8b_layer(n_in=n_in, n_layers=1))
        kc, kt = one["chunk_keys"], one["tile_keys"]
        unmasked = (n_in - 64 + 1) // kt * kt                       # keys every observation row may see, whole tiles
        assert kc % kt == 0 and one["n_chunks"] == -(-unmasked // kc)
        assert one["n_chunks"] * 8 + 8 <= 256 < -(-unmasked // (kc - kt)) * 8 + 8      # one tile shorter would not fit
        assert one["fixed_reference_rows"] == 0          # one round of workgroups: online step, no repair launch
    # sweeps of several rounds sum their row statistics against fixed references; the Q-stationary
    # kernel (row statistics at d = 64) has its own step
    assert c3["fixed_reference_rows"] == 1 and c4["fixed_reference_rows"] == 1
    assert c5["q_stationary"] & 1 and c5["fixed_reference_rows"] == 0 and tiny["fixed_reference_rows"] == 0


def test_row_statistics_mode_follows_the_environment(lib, monkeypatch):
    import workloads
    w = workloads.llama8b_layer(n_in=32768, n_layers=1)
    p = S.SpecKVParams(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                       seq_lens=list(w.seq_lens), n_window=w.n_window, n_lookahead=w.n_lookahead, pool_k=w.pool_k,
                       c_max=w.c_max, sm_scale=w.sm_scale, dtype=w.torch_dtype)
    assert S.plan_info(p)["fixed_reference_rows"] == 0
    monkeypatch.setenv("SPECKV_ROW_STATISTICS", "fixed")
    assert S.plan_info(p)["fixed_reference_rows"] == 1
    monkeypatch.setenv("SPECKV_ROW_STATISTICS", "online")
    full = workloads.llama8b_full_128k()
    pf = S.SpecKVParams(n_layers=full.n_layers, n_q_heads=full.n_q_heads, n_kv_heads=full.n_kv_heads,
                        head_dim=full.head_dim, seq_lens=list(full.seq_lens), n_window=full.n_window,
                        n_lookahead=full.n_lookahead, pool_k=full.pool_k, c_max=full.c_max, sm_scale=full.sm_scale,
                        dtype=full.torch_dtype)
    assert S.plan_info(pf)["fixed_reference_rows"] == 0


def test_plan_invariants_over_random_shapes(lib):
    import numpy as np
    rng = np.random.default_rng(0)
    for _ in range(300):
        G = int(rng.choice([1, 2, 4, 5, 7, 8, 16]))
        Hkv = int(rng.choice([1, 2, 4, 8]))
        d = int(rng.choice([64, 128]))
        dt = [torch.bfloat16, torch.float16, torch.float32][int(rng.integers(0, 3))]
        w_ = int(rng.choice([0, 16, 64]))
        a_ = int(rng.choice([1, 16, 64, 200]))
        n_seqs = int(rng.choice([1, 1, 3, 16]))
        lens = [int(x) for x in rng.integers(max(1, w_), int(rng.choice([2000, 70000, 1200000])), size=n_seqs)]
        L = int(rng.choice([1, 2, 32]))
        if sum(lens) * L * Hkv > 1 << 31:
            continue
        p = S.SpecKVParams(n_layers=L, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d, seq_lens=lens,
                           n_window=w_, n_lookahead=a_, pool_k=7, c_max=1024, sm_scale=0.1, dtype=dt)
        out = (ctypes.c_int64 * PLAN_INFO_WORDS)()
        st = lib.speckv_plan_info(p.ref(), out)
        if st == -2:
            continue                                           # outside the supported envelope
        assert st == 0
        info = S.plan_info(p)
        tile, kc = info["tile_keys"], info["chunk_keys"]
        assert kc % tile == 0 and kc >= 512
        rows_per_wg = info["waves"] * info["blocks_per_wave"] * 32
        rp = (w_ + a_ + 31) // 32 * 32
        assert info["row_super_blocks"] * rows_per_wg >= G * min(rp, rows_per_wg) or rp > rows_per_wg
        # the unmasked chunks cover exactly the whole tiles visible to every row
        want_chunks = 0
        for n in lens:
            visible = min(n, n - w_ + 1)
            want_chunks += -(-(visible // tile * tile) // kc)
        assert info["n_chunks"] == want_chunks
        # rows are split for selection only when they are long and few
        rows = L * n_seqs * Hkv
        if info["select_parts"] > 1:
            assert max(lens) - w_ >= 1 << 18 and rows * info["select_parts"] <= 512 + rows
            assert info["select_parts"] * info["select_part_keys"] >= max(lens) - w_
        assert S.workspace_bytes(p) > 0


def test_plain_c_caller(lib, repo_root, tmp_path):
    """The header and the library from a C99 program (host-side entry points only)."""
    import shutil
    import subprocess
    cc = shutil.which("gcc")
    if cc is None:
        pytest.skip("no C compiler")
    pkg = os.path.join(repo_root, "paper_2506_08373_amd")
    exe = str(tmp_path / "c_abi_check")
    subprocess.run([cc, "-std=c99", "-Wall", "-Werror", "-I", os.path.join(repo_root, "include"),
                    os.path.join(repo_root, "tests", "c_abi_check.c"), "-o", exe,
                    "-L", pkg, "-lspeckv", "-Wl,-rpath," + pkg, "-Wl,-rpath,/opt/rocm/lib",
                    "-L", "/opt/rocm/lib", "-lamdhip64"], check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr)
    assert "workspace" in r.stdout
