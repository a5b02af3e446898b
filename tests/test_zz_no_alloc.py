"""The allocation-free entry point against the entry point it is a variant of.

`speckv_compress_static` runs the kernels of `speckv_compress` on a fixed scratch array inside
the library instead of a caller workspace.  Both are called through the C ABI on the same
inputs and must agree bit for bit (indices, compacted K and V): two calls in a row, the
second on a smaller input, so that whatever the first call left in the shared scratch is
there when the second runs.
"""
import ctypes
import math

import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_08373_amd as lib
    lib.load_library()
    return lib


def _both(S, w):
    lib = S.load_library()
    t = workloads.generate(w, device="cuda")
    q, k, v = t["q"], t["k"], t["v"]
    p = S.SpecKVParams.for_tensors(q, k, seq_lens=w.seq_lens, n_window=w.n_window, pool_k=w.pool_k,
                                   c_max=w.c_max, sm_scale=w.sm_scale)
    need = S.workspace_bytes(p)
    assert 0 < need <= S.STATIC_SCRATCH_BYTES, "test input must fit the fixed scratch"
    L, H, d, KT = w.n_layers, w.n_kv_heads, w.head_dim, S.total_keep(p)
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for static in (False, True):
        idx = torch.full((L, H * KT), -3, dtype=torch.int32, device="cuda")
        k_out = torch.zeros((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
        v_out = torch.zeros_like(k_out)
        if static:
            st = lib.speckv_compress_static(p.ref(), q.data_ptr(), k.data_ptr(), v.data_ptr(), idx.data_ptr(),
                                            k_out.data_ptr(), v_out.data_ptr(), stream)
        else:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            st = lib.speckv_compress(p.ref(), q.data_ptr(), k.data_ptr(), v.data_ptr(), idx.data_ptr(),
                                     k_out.data_ptr(), v_out.data_ptr(), ws.data_ptr(),
                                     ctypes.c_size_t(need), stream)
        assert st == 0, "status %d (static=%s)" % (st, static)
        torch.cuda.synchronize()
        out.append((idx, k_out, v_out))
    (i0, k0, v0), (i1, k1, v1) = out
    assert bool((i0 >= 0).all()), "the reference call left indices unwritten"
    assert torch.equal(i0, i1), "indices differ"
    assert torch.equal(k0.view(torch.int16), k1.view(torch.int16)), "compacted K differs"
    assert torch.equal(v0.view(torch.int16), v1.view(torch.int16)), "compacted V differs"


def test_static_scratch_matches_workspace_call_twice_second_smaller(S):
    big = workloads.SpecKVWorkload(
        name="static_big", n_layers=2, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_lens=(20000, 9001),
        n_window=64, n_lookahead=64, pool_k=7, c_max=1024, dtype="bf16", sm_scale=1.0 / math.sqrt(128.0),
        n_planted=16, channel_scale=(0.5, 4.0), seed=21)
    small = workloads.SpecKVWorkload(
        name="static_small", n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_lens=(1500,),
        n_window=16, n_lookahead=8, pool_k=7, c_max=128, dtype="bf16", sm_scale=1.0 / math.sqrt(128.0),
        n_planted=8, seed=22)
    _both(S, big)
    _both(S, small)


def test_static_scratch_rejects_what_does_not_fit(S):
    """A problem whose workspace exceeds the fixed array is refused before anything is launched."""
    lib = S.load_library()
    p = S.SpecKVParams(n_layers=32, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_lens=[131072], n_window=64,
                       n_lookahead=64, pool_k=7, c_max=2048, sm_scale=0.088, dtype=torch.bfloat16)
    assert S.workspace_bytes(p) > S.STATIC_SCRATCH_BYTES
    # validation fails before any pointer is used: dummy non-null values are safe
    st = lib.speckv_compress_static(p.ref(), 256, 256, 256, 256, 256, 256, None)
    assert st == -3
