"""ctypes binding of libspeckv.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks dtype /
device / contiguity of the innermost dimension, derives the element strides and
passes raw device pointers plus the current HIP stream through the C ABI.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libspeckv.so")
_lib = None

SPECKV_BF16, SPECKV_F32, SPECKV_F16 = 0, 1, 2
_STATUS = {0: "ok", -1: "invalid argument", -2: "unsupported configuration",
           -3: "workspace missing, misaligned or too small", -4: "HIP runtime error"}


class SpecKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__("%s failed: %s (%d)" % (where, _STATUS.get(status, "unknown"), status))
        self.status = status


class _CParams(ctypes.Structure):
    _fields_ = [
        ("n_seqs", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("n_window", ctypes.c_int32),
        ("n_lookahead", ctypes.c_int32), ("pool_k", ctypes.c_int32), ("c_max", ctypes.c_int32),
        ("sm_scale", ctypes.c_float), ("dtype", ctypes.c_int32),
        ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)), ("n_in", ctypes.c_int64),
        ("q_stride_layer", ctypes.c_int64), ("q_stride_seq", ctypes.c_int64),
        ("q_stride_row", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
        ("kv_stride_layer", ctypes.c_int64), ("kv_stride_token", ctypes.c_int64),
        ("kv_stride_head", ctypes.c_int64),
        ("reduce_op", ctypes.c_int32), ("pool_op", ctypes.c_int32),
        ("n_in_dev", ctypes.c_void_p),
    ]


EXPORTS = ("speckv_status_string", "speckv_n_keep", "speckv_total_keep", "speckv_workspace_bytes",
           "speckv_score", "speckv_select", "speckv_compact", "speckv_compress",
           "speckv_compress_events", "speckv_score_lse", "speckv_compress_lse",
           "specpc_workspace_bytes", "specpc_select_tokens", "specpc_compress_workspace_bytes",
           "specpc_compress_prompt", "speckv_ada_workspace_bytes", "speckv_select_ada",
           "speckv_compact_ada", "speckv_compress_ada", "speckv_plan_info", "speckv_compress_static",
           "specpc_select_tokens_events", "speckv_select_workspace_bytes", "speckv_probe_ceiling")


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads libspeckv.so once.  Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libspeckv.so is missing at %s; build it with "
                           "`python -m paper_2506_08373_amd.build` (needs hipcc)" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    P, vp, i32p, f32p = ctypes.POINTER(_CParams), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    lib.speckv_status_string.restype = ctypes.c_char_p
    lib.speckv_status_string.argtypes = [ctypes.c_int]
    lib.speckv_n_keep.restype = ctypes.c_int64
    lib.speckv_n_keep.argtypes = [P, ctypes.c_int32]
    lib.speckv_total_keep.restype = ctypes.c_int64
    lib.speckv_total_keep.argtypes = [P]
    lib.speckv_workspace_bytes.restype = ctypes.c_size_t
    lib.speckv_workspace_bytes.argtypes = [P]
    lib.speckv_select_workspace_bytes.restype = ctypes.c_size_t
    lib.speckv_select_workspace_bytes.argtypes = [P]
    lib.specpc_workspace_bytes.restype = ctypes.c_size_t
    lib.specpc_workspace_bytes.argtypes = [P, ctypes.c_int32]
    lib.speckv_score.restype = ctypes.c_int
    lib.speckv_score.argtypes = [P, vp, vp, f32p, f32p, vp, ctypes.c_size_t, vp]
    lib.speckv_score_lse.restype = ctypes.c_int
    lib.speckv_score_lse.argtypes = [P, vp, vp, f32p, f32p, f32p, vp, ctypes.c_size_t, vp]
    lib.speckv_compress_lse.restype = ctypes.c_int
    lib.speckv_compress_lse.argtypes = [P, vp, vp, vp, f32p, i32p, vp, vp, vp, ctypes.c_size_t, vp]
    lib.speckv_select.restype = ctypes.c_int
    lib.speckv_select.argtypes = [P, f32p, i32p, vp, ctypes.c_size_t, vp]
    lib.speckv_compact.restype = ctypes.c_int
    lib.speckv_compact.argtypes = [P, vp, vp, i32p, vp, vp, vp]
    lib.speckv_compress.restype = ctypes.c_int
    lib.speckv_compress.argtypes = [P, vp, vp, vp, i32p, vp, vp, vp, ctypes.c_size_t, vp]
    lib.speckv_compress_static.restype = ctypes.c_int
    lib.speckv_compress_static.argtypes = [P, vp, vp, vp, i32p, vp, vp, vp]
    lib.speckv_compress_events.restype = ctypes.c_int
    lib.speckv_compress_events.argtypes = [P, vp, vp, vp, i32p, vp, vp, vp, ctypes.c_size_t, vp,
                                           ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32]
    lib.speckv_plan_info.restype = ctypes.c_int
    lib.speckv_plan_info.argtypes = [P, ctypes.POINTER(ctypes.c_int64)]
    lib.speckv_ada_workspace_bytes.restype = ctypes.c_size_t
    lib.speckv_ada_workspace_bytes.argtypes = [P]
    lib.speckv_select_ada.restype = ctypes.c_int
    lib.speckv_select_ada.argtypes = [P, ctypes.c_int32, f32p, i32p, i32p, vp, ctypes.c_size_t, vp]
    lib.speckv_compact_ada.restype = ctypes.c_int
    lib.speckv_compact_ada.argtypes = [P, vp, vp, i32p, i32p, vp, vp, vp]
    lib.speckv_compress_ada.restype = ctypes.c_int
    lib.speckv_compress_ada.argtypes = [P, ctypes.c_int32, vp, vp, vp, i32p, i32p, vp, vp, vp,
                                        ctypes.c_size_t, vp]
    lib.specpc_select_tokens.restype = ctypes.c_int
    lib.specpc_select_tokens.argtypes = [P, ctypes.c_int32, ctypes.c_int32, vp, vp, i32p, i32p, i32p,
                                         i32p, vp, ctypes.c_size_t, vp]
    lib.specpc_select_tokens_events.restype = ctypes.c_int
    lib.specpc_select_tokens_events.argtypes = [P, ctypes.c_int32, ctypes.c_int32, vp, vp, i32p, i32p, i32p,
                                                i32p, vp, ctypes.c_size_t, vp,
                                                ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32]
    lib.specpc_compress_workspace_bytes.restype = ctypes.c_size_t
    lib.specpc_compress_workspace_bytes.argtypes = [P, ctypes.c_int32]
    lib.specpc_compress_prompt.restype = ctypes.c_int
    lib.specpc_compress_prompt.argtypes = [P, ctypes.c_int32, ctypes.c_int32, vp, vp, i32p, i32p, i32p,
                                           i32p, vp, ctypes.c_size_t, vp]
    lib.speckv_probe_ceiling.restype = ctypes.c_int
    lib.speckv_probe_ceiling.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp, vp, ctypes.POINTER(ctypes.c_int64)]
    _lib = lib
    return lib


class SpecKVParams:
    """Host-side description of one call (mirrors ``speckv_params``)."""

    def __init__(self, *, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 seq_lens: Sequence[int], n_window: int, n_lookahead: int, pool_k: int, c_max: int,
                 sm_scale: float, dtype: torch.dtype, reduce: str = "sum", pool: str = "max",
                 q_strides: Optional[Tuple[int, int, int, int]] = None,
                 kv_strides: Optional[Tuple[int, int, int]] = None,
                 n_in_dev: Optional[torch.Tensor] = None):
        self.seq_lens = [int(x) for x in seq_lens]
        S, R, T = len(self.seq_lens), n_window + n_lookahead, sum(self.seq_lens)
        if q_strides is None:        # contiguous [L, S, R, Hq, d]
            q_strides = (S * R * n_q_heads * head_dim, R * n_q_heads * head_dim,
                         n_q_heads * head_dim, head_dim)
        if kv_strides is None:       # contiguous [L, T, Hkv, d]
            kv_strides = (T * n_kv_heads * head_dim, n_kv_heads * head_dim, head_dim)
        cu = [0]
        for n in self.seq_lens:
            cu.append(cu[-1] + n)
        self._cu = (ctypes.c_int32 * (S + 1))(*cu)
        self.cu_seqlens = cu
        self.c = _CParams(
            n_seqs=S, n_layers=n_layers, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
            n_window=n_window, n_lookahead=n_lookahead, pool_k=pool_k, c_max=c_max, sm_scale=sm_scale,
            dtype={torch.bfloat16: SPECKV_BF16, torch.float32: SPECKV_F32, torch.float16: SPECKV_F16}[dtype],
            cu_seqlens=ctypes.cast(self._cu, ctypes.POINTER(ctypes.c_int32)), n_in=0,
            q_stride_layer=q_strides[0], q_stride_seq=q_strides[1], q_stride_row=q_strides[2],
            q_stride_head=q_strides[3], kv_stride_layer=kv_strides[0], kv_stride_token=kv_strides[1],
            kv_stride_head=kv_strides[2], reduce_op={"sum": 0, "max": 1}[reduce],
            pool_op={"max": 0, "avg": 1}[pool], n_in_dev=None)
        self.n_in_dev = n_in_dev            # keeps the tensor alive for as long as the parameters
        if n_in_dev is not None:
            if not n_in_dev.is_cuda or n_in_dev.dtype != torch.int32 or n_in_dev.numel() < 1:
                raise ValueError("n_in_dev must be a device int32 tensor")
            self.c.n_in_dev = n_in_dev.data_ptr()
        self.torch_dtype = dtype
        self.n_layers, self.n_kv_heads, self.head_dim = n_layers, n_kv_heads, head_dim
        self.n_window, self.total_tokens = n_window, T

    def ref(self):
        return ctypes.byref(self.c)

    @classmethod
    def for_tensors(cls, q: torch.Tensor, k: torch.Tensor, *, seq_lens, n_window, pool_k, c_max,
                    sm_scale, reduce: str = "sum", pool: str = "max",
                    n_in_dev: Optional[torch.Tensor] = None) -> "SpecKVParams":
        """q [L, S, R, Hq, d], k [L, T, Hkv, d] (any strides with d contiguous)."""
        if q.dim() != 5 or k.dim() != 4 or q.stride(-1) != 1 or k.stride(-1) != 1:
            raise ValueError("expected q [L,S,R,Hq,d] and k [L,T,Hkv,d] with contiguous d")
        L, S, R, Hq, d = q.shape
        return cls(n_layers=L, n_q_heads=Hq, n_kv_heads=k.shape[2], head_dim=d, seq_lens=seq_lens,
                   n_window=n_window, n_lookahead=R - n_window, pool_k=pool_k, c_max=c_max,
                   sm_scale=sm_scale, dtype=q.dtype, reduce=reduce, pool=pool,
                   q_strides=tuple(q.stride()[:4]),
                   kv_strides=tuple(k.stride()[:3]), n_in_dev=n_in_dev)


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libspeckv takes device tensors only")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SpecKVError(status, where)


def n_keep(p: SpecKVParams, seq: int) -> int:
    return int(load_library().speckv_n_keep(p.ref(), seq))


def total_keep(p: SpecKVParams) -> int:
    return int(load_library().speckv_total_keep(p.ref()))


def workspace_bytes(p: SpecKVParams) -> int:
    return int(load_library().speckv_workspace_bytes(p.ref()))


def select_workspace_bytes(p: SpecKVParams) -> int:
    return int(load_library().speckv_select_workspace_bytes(p.ref()))


def specpc_workspace_bytes(p: SpecKVParams, top_k: int) -> int:
    return int(load_library().specpc_workspace_bytes(p.ref(), top_k))


def _ws(ws: Optional[torch.Tensor]) -> Tuple[Optional[int], int]:
    if ws is None:
        return None, 0
    if not ws.is_cuda or not ws.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    return ws.data_ptr(), ws.numel() * ws.element_size()


def speckv_score(p: SpecKVParams, q, k, pooled, raw, workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().speckv_score(p.ref(), _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
                                       _ptr(pooled, torch.float32), _ptr(raw, torch.float32),
                                       wp, wb, _stream()), "speckv_score")


def speckv_score_lse(p: SpecKVParams, q, k, lse_in, pooled, raw, workspace) -> None:
    """lse_in: fp32 [L, S, R, Hq] natural-log row normalisers."""
    wp, wb = _ws(workspace)
    _check(load_library().speckv_score_lse(p.ref(), _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
                                           _ptr(lse_in, torch.float32), _ptr(pooled, torch.float32),
                                           _ptr(raw, torch.float32), wp, wb, _stream()), "speckv_score_lse")


def speckv_compress_lse(p: SpecKVParams, q, k, v, lse_in, idx, k_out, v_out, workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().speckv_compress_lse(
        p.ref(), _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype), _ptr(v, p.torch_dtype),
        _ptr(lse_in, torch.float32), _ptr(idx, torch.int32), _ptr(k_out, p.torch_dtype),
        _ptr(v_out, p.torch_dtype), wp, wb, _stream()), "speckv_compress_lse")


def speckv_select(p: SpecKVParams, pooled, idx, workspace=None) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().speckv_select(p.ref(), _ptr(pooled, torch.float32), _ptr(idx, torch.int32),
                                        wp, wb, _stream()), "speckv_select")


def speckv_compact(p: SpecKVParams, k, v, idx, k_out, v_out) -> None:
    _check(load_library().speckv_compact(p.ref(), _ptr(k, p.torch_dtype), _ptr(v, p.torch_dtype),
                                         _ptr(idx, torch.int32), _ptr(k_out, p.torch_dtype),
                                         _ptr(v_out, p.torch_dtype), _stream()), "speckv_compact")


def speckv_compress(p: SpecKVParams, q, k, v, idx, k_out, v_out, workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().speckv_compress(p.ref(), _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
                                          _ptr(v, p.torch_dtype), _ptr(idx, torch.int32),
                                          _ptr(k_out, p.torch_dtype), _ptr(v_out, p.torch_dtype),
                                          wp, wb, _stream()), "speckv_compress")


STATIC_SCRATCH_BYTES = 32 << 20


def speckv_compress_static(p: SpecKVParams, q, k, v, idx, k_out, v_out) -> None:
    """speckv_compress on the library's own fixed scratch: no workspace, no allocation."""
    _check(load_library().speckv_compress_static(p.ref(), _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
                                                 _ptr(v, p.torch_dtype), _ptr(idx, torch.int32),
                                                 _ptr(k_out, p.torch_dtype), _ptr(v_out, p.torch_dtype),
                                                 _stream()), "speckv_compress_static")


def plan_info(p: SpecKVParams) -> dict:
    """The host's launch plan for these parameters (diagnostics; needs no GPU)."""
    out = (ctypes.c_int64 * 11)()
    _check(load_library().speckv_plan_info(p.ref(), out), "speckv_plan_info")
    keys = ("waves", "blocks_per_wave", "row_super_blocks", "chunk_keys", "n_chunks", "tile_keys",
            "select_parts", "select_part_keys", "q_stationary", "reduce_max", "fixed_reference_rows")
    return dict(zip(keys, (int(x) for x in out)))


def ada_workspace_bytes(p: SpecKVParams) -> int:
    return int(load_library().speckv_ada_workspace_bytes(p.ref()))


def speckv_select_ada(p: SpecKVParams, c_floor: int, pooled, idx, head_off, workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().speckv_select_ada(p.ref(), int(c_floor), _ptr(pooled, torch.float32),
                                            _ptr(idx, torch.int32), _ptr(head_off, torch.int32),
                                            wp, wb, _stream()), "speckv_select_ada")


def speckv_compact_ada(p: SpecKVParams, k, v, idx, head_off, k_out, v_out) -> None:
    _check(load_library().speckv_compact_ada(p.ref(), _ptr(k, p.torch_dtype), _ptr(v, p.torch_dtype),
                                             _ptr(idx, torch.int32), _ptr(head_off, torch.int32),
                                             _ptr(k_out, p.torch_dtype), _ptr(v_out, p.torch_dtype),
                                             _stream()), "speckv_compact_ada")


def speckv_compress_ada(p: SpecKVParams, c_floor: int, q, k, v, idx, head_off, k_out, v_out,
                        workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().speckv_compress_ada(p.ref(), int(c_floor), _ptr(q, p.torch_dtype),
                                              _ptr(k, p.torch_dtype), _ptr(v, p.torch_dtype),
                                              _ptr(idx, torch.int32), _ptr(head_off, torch.int32),
                                              _ptr(k_out, p.torch_dtype), _ptr(v_out, p.torch_dtype),
                                              wp, wb, _stream()), "speckv_compress_ada")


N_STAGE_EVENTS = 7
STAGE_NAMES = ("score_pass1", "lse_merge", "score_pass2", "pool", "select", "compact")


def speckv_compress_events(p: SpecKVParams, q, k, v, idx, k_out, v_out, workspace, events) -> None:
    """`events`: ctypes array of N_STAGE_EVENTS raw hipEvent_t handles (c_void_p)."""
    wp, wb = _ws(workspace)
    _check(load_library().speckv_compress_events(
        p.ref(), _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype), _ptr(v, p.torch_dtype),
        _ptr(idx, torch.int32), _ptr(k_out, p.torch_dtype), _ptr(v_out, p.torch_dtype), wp, wb,
        _stream(), events, N_STAGE_EVENTS), "speckv_compress_events")


def specpc_select_tokens(p: SpecKVParams, top_k: int, n_neighbor: int, q, k, token_ids, idx_out,
                         ids_out, count_out, workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().specpc_select_tokens(
        p.ref(), top_k, n_neighbor, _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
        _ptr(token_ids, torch.int32), _ptr(idx_out, torch.int32), _ptr(ids_out, torch.int32),
        _ptr(count_out, torch.int32), wp, wb, _stream()), "specpc_select_tokens")


SPECPC_STAGE_NAMES = ("score_pass1", "lse_merge", "score_pass2", "pool", "select", "expand")


def specpc_select_tokens_events(p: SpecKVParams, top_k: int, n_neighbor: int, q, k, token_ids, idx_out,
                                ids_out, count_out, workspace, events) -> None:
    """`events`: ctypes array of N_STAGE_EVENTS raw hipEvent_t handles (c_void_p)."""
    wp, wb = _ws(workspace)
    _check(load_library().specpc_select_tokens_events(
        p.ref(), top_k, n_neighbor, _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
        _ptr(token_ids, torch.int32), _ptr(idx_out, torch.int32), _ptr(ids_out, torch.int32),
        _ptr(count_out, torch.int32), wp, wb, _stream(), events, N_STAGE_EVENTS), "specpc_select_tokens_events")


def specpc_compress_workspace_bytes(p: SpecKVParams, l_skip: int) -> int:
    return int(load_library().specpc_compress_workspace_bytes(p.ref(), l_skip))


def specpc_compress_prompt(p: SpecKVParams, l_skip: int, n_neighbor: int, q, k, token_ids, idx_out,
                           ids_out, count_out, workspace) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().specpc_compress_prompt(
        p.ref(), l_skip, n_neighbor, _ptr(q, p.torch_dtype), _ptr(k, p.torch_dtype),
        _ptr(token_ids, torch.int32), _ptr(idx_out, torch.int32), _ptr(ids_out, torch.int32),
        _ptr(count_out, torch.int32), wp, wb, _stream()), "specpc_compress_prompt")


def probe_ceiling(kind: int, iters: int, operands: torch.Tensor, out: torch.Tensor) -> int:
    """Launches one ceiling-probe loop on the current stream; returns the matrix flops it executes."""
    if operands.numel() * operands.element_size() < 65536 or out.numel() * out.element_size() < 512 * 1024:
        raise ValueError("operands needs 64 KiB, out 512 KiB")
    flops = ctypes.c_int64()
    _check(load_library().speckv_probe_ceiling(kind, iters, _ptr(operands), _ptr(out, torch.float32), _stream(),
                                               ctypes.byref(flops)), "speckv_probe_ceiling")
    return int(flops.value)
