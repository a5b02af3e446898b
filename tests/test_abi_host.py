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
    dict(pool_k=4),                          # even pooling kernel
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
