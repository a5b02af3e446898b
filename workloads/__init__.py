"""Seeded synthetic inputs for the SpecKV scoring / selection / compaction path.

This module only draws random numbers and lays them out in memory.  It holds
none of the method's arithmetic (no softmax, no pooling, no selection): both the
CPU oracle and the HIP library consume the tensors it returns, so neither has to
know about the other.

The inputs stand in for the per-layer tensors a target-model prefill would hand
to SpecKV (Alg. 1, the loop over attention heads): the queries of the last
``n_window`` prompt positions and of the ``n_lookahead`` draft tokens, and the
keys / values of the whole prompt.  Long-context benchmark prompts are replaced
by random tensors of the same shapes; see ``SpecKVWorkload`` for the recipe.

Layouts (``d`` contiguous everywhere)::

    q  [n_layers, n_seqs, R, n_q_heads, d]        R = n_window + n_lookahead,
                                                   window rows first
    k  [n_layers, total_tokens, n_kv_heads, d]    sequences packed back to back
    v  [n_layers, total_tokens, n_kv_heads, d]
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class SpecKVWorkload:
    """Shape, distribution and seed of one synthetic workload.

    Value recipe, per (layer, sequence), drawn from one ``torch.Generator``
    seeded with ``seed * 1_000_003 + layer * 1009 + seq``:

    * ``scale[g, c]``: ``exp(U[ln lo, ln hi])`` per KV head and channel when
      ``channel_scale`` is set (mimics outlier channels), else 1.  The same scale
      multiplies K of that KV head and Q of the query heads in its group.
    * ``K = N(0,1) * scale``, ``V = N(0,1)``, ``Q = N(0,1) * scale * q_gain``.
    * ``n_planted`` heavy-hitter keys per KV head: one position drawn uniformly
      from each of ``n_planted`` equal strata of the non-window prompt
      ``[0, n_in - n_window)`` (distinct by construction); each is
      overwritten by ``3 * rho_g * q / ||q||`` for a random observation row ``q``
      of the group, ``rho_g`` being the RMS norm of that head's ordinary keys.
    * everything is rounded to ``dtype`` last.
    """

    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_lens: Tuple[int, ...]
    n_window: int
    n_lookahead: int
    pool_k: int
    c_max: int
    dtype: str  # "bf16", "f16" or "f32"
    sm_scale: float
    q_gain: float = 1.0
    n_planted: int = 0
    channel_scale: Optional[Tuple[float, float]] = None
    seed: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_rows(self) -> int:
        return self.n_window + self.n_lookahead

    @property
    def n_seqs(self) -> int:
        return len(self.seq_lens)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def cu_seqlens(self) -> List[int]:
        out = [0]
        for n in self.seq_lens:
            out.append(out[-1] + int(n))
        return out

    def n_keep(self, seq: int) -> int:
        """Rows of the compacted cache for one sequence (layout bookkeeping)."""
        n = self.seq_lens[seq]
        return min(self.c_max, n - self.n_window) + self.n_window

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[self.dtype]

    @property
    def key_units(self) -> int:
        """The metric's unit count: prompt keys x layers x KV heads."""
        return self.total_tokens * self.n_layers * self.n_kv_heads


def _ragged_lengths(seed: int, n_seqs: int, lo: int, hi: int) -> Tuple[int, ...]:
    rng = np.random.default_rng(seed)
    return tuple(int(x) for x in rng.integers(lo, hi + 1, size=n_seqs))


def tiny_fp32() -> SpecKVWorkload:
    """Single tiny fp32 layer; a CPU implementation finishes in seconds."""
    return SpecKVWorkload(
        name="c1_tiny_fp32", n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=64,
        seq_lens=(1024,), n_window=16, n_lookahead=16, pool_k=7, c_max=128,
        dtype="f32", sm_scale=1.0, q_gain=1.0 / math.sqrt(64.0), n_planted=8,
        channel_scale=None, seed=0)


def llama8b_layer(n_in: int = 32768, c_max: int = 1024, n_layers: int = 1,
                  seed: int = 1, name: str = "c2_llama8b_1layer_32k") -> SpecKVWorkload:
    """Llama-3.1-8B-shaped attention layer(s), bf16."""
    return SpecKVWorkload(
        name=name, n_layers=n_layers, n_q_heads=32, n_kv_heads=8, head_dim=128,
        seq_lens=(n_in,), n_window=64, n_lookahead=64, pool_k=7, c_max=c_max,
        dtype="bf16", sm_scale=1.0 / math.sqrt(128.0), n_planted=32,
        channel_scale=(0.5, 4.0), seed=seed)


def llama8b_full_128k() -> SpecKVWorkload:
    """Llama-3.1-8B-shaped full stack: 32 layers at 128K prompt tokens."""
    return llama8b_layer(n_in=131072, c_max=2048, n_layers=32, seed=3,
                         name="c3_llama8b_32layers_128k")


def ragged_batch(n_layers: int = 28, lo: int = 4096, hi: int = 65536,
                 n_seqs: int = 8, seed: int = 4,
                 name: str = "c4_ragged8_gqa7") -> SpecKVWorkload:
    """Ragged batch with a GQA group of 7 (28 query / 4 KV heads)."""
    return SpecKVWorkload(
        name=name, n_layers=n_layers, n_q_heads=28, n_kv_heads=4, head_dim=128,
        seq_lens=_ragged_lengths(seed, n_seqs, lo, hi), n_window=64, n_lookahead=64,
        pool_k=7, c_max=1024, dtype="bf16", sm_scale=1.0 / math.sqrt(128.0),
        n_planted=32, channel_scale=(0.5, 4.0), seed=seed)


def specpc_draft(n_in: int = 65536, n_layers: int = 16, seed: int = 5,
                 name: str = "c5_specpc_llama1b") -> SpecKVWorkload:
    """Llama-3.2-1B-shaped draft model, window queries only (prompt-token selection).

    ``c_max`` holds the number of top tokens (4096); the +-8 neighbour expansion
    and the vocabulary size for ``token_ids`` are passed separately.
    """
    return SpecKVWorkload(
        name=name, n_layers=n_layers, n_q_heads=32, n_kv_heads=8, head_dim=64,
        seq_lens=(n_in,), n_window=64, n_lookahead=0, pool_k=7, c_max=4096,
        dtype="bf16", sm_scale=1.0 / math.sqrt(64.0), n_planted=32,
        channel_scale=(0.5, 4.0), seed=seed)


SPECPC_NEIGHBORS = 8
SPECPC_VOCAB = 128256

PRESETS = {
    "c1": tiny_fp32,
    "c2": llama8b_layer,
    "c3": llama8b_full_128k,
    "c4": ragged_batch,
    "c5": specpc_draft,
}


def _layer_seq_seed(w: SpecKVWorkload, layer: int, seq: int) -> int:
    return w.seed * 1_000_003 + layer * 1009 + seq


def generate_layer_seq(w: SpecKVWorkload, layer: int, seq: int,
                       device: str = "cpu") -> Dict[str, torch.Tensor]:
    """Draw q [R, Hq, d], k [n, Hkv, d], v [n, Hkv, d] for one (layer, sequence).

    Returns tensors already rounded to ``w.torch_dtype`` on ``device`` plus
    ``planted`` (int64 [Hkv, n_planted], positions of the heavy hitters).
    The CPU and GPU generators produce different streams; a test must take both
    its oracle inputs and its library inputs from one call.
    """
    n = int(w.seq_lens[seq])
    m = n - w.n_window
    R, Hq, Hkv, d, G = w.n_rows, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    gen = torch.Generator(device=device)
    gen.manual_seed(_layer_seq_seed(w, layer, seq))

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

    def rand(*shape):
        return torch.rand(*shape, generator=gen, device=device, dtype=torch.float32)

    if w.channel_scale is not None:
        lo, hi = w.channel_scale
        scale = torch.exp(math.log(lo) + rand(Hkv, d) * (math.log(hi) - math.log(lo)))
    else:
        scale = torch.ones(Hkv, d, device=device)
    k = randn(n, Hkv, d) * scale[None]
    v = randn(n, Hkv, d)
    q = randn(R, Hq, d) * scale.repeat_interleave(G, dim=0)[None] * w.q_gain

    planted = torch.zeros(Hkv, w.n_planted, dtype=torch.int64, device=device)
    if w.n_planted > 0:
        if m < w.n_planted:
            raise ValueError("not enough non-window keys to plant heavy hitters")
        rho = k.pow(2).sum(-1).mean(0).sqrt()                     # [Hkv]
        for g in range(Hkv):
            # one position per stratum of [0, m): distinct by construction, no sort needed
            stride = m // w.n_planted
            pos = (torch.arange(w.n_planted, device=device) * stride +
                   torch.randint(0, stride, (w.n_planted,), generator=gen, device=device))
            rows = torch.randint(0, R, (w.n_planted,), generator=gen, device=device)
            heads = g * G + torch.randint(0, G, (w.n_planted,), generator=gen, device=device)
            qd = q[rows, heads]                                   # [P, d]
            qd = qd / qd.norm(dim=-1, keepdim=True)
            k[pos, g] = 3.0 * rho[g] * qd
            planted[g] = pos
    dt = w.torch_dtype
    return {"q": q.to(dt).contiguous(), "k": k.to(dt).contiguous(),
            "v": v.to(dt).contiguous(), "planted": planted}


def generate(w: SpecKVWorkload, device: str = "cpu",
             layers: Optional[Sequence[int]] = None) -> Dict[str, torch.Tensor]:
    """Draw the whole workload (or the listed layers) in the packed layouts.

    Returns ``q [L, S, R, Hq, d]``, ``k``/``v`` ``[L, T, Hkv, d]`` and ``planted``
    ``[L, S, Hkv, P]`` (sequence-local positions).
    """
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    L, S, T = len(layers), w.n_seqs, w.total_tokens
    dt = w.torch_dtype
    q = torch.empty(L, S, w.n_rows, w.n_q_heads, w.head_dim, dtype=dt, device=device)
    k = torch.empty(L, T, w.n_kv_heads, w.head_dim, dtype=dt, device=device)
    v = torch.empty_like(k)
    planted = torch.zeros(L, S, w.n_kv_heads, w.n_planted, dtype=torch.int64, device=device)
    cu = w.cu_seqlens
    for li, layer in enumerate(layers):
        for s in range(S):
            t = generate_layer_seq(w, layer, s, device)
            q[li, s] = t["q"]
            k[li, cu[s]:cu[s + 1]] = t["k"]
            v[li, cu[s]:cu[s + 1]] = t["v"]
            planted[li, s] = t["planted"]
            del t
    return {"q": q, "k": k, "v": v, "planted": planted}


def generate_token_ids(w: SpecKVWorkload, vocab: int = SPECPC_VOCAB,
                       device: str = "cpu") -> torch.Tensor:
    """int32 token ids, uniform in [0, vocab), one per prompt token."""
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed * 1_000_003 + 999_983)
    return torch.randint(0, vocab, (w.total_tokens,), generator=gen, device=device,
                         dtype=torch.int32)


def to_float64(t: torch.Tensor) -> np.ndarray:
    """Exact upcast of a bf16 / fp32 tensor to a float64 numpy array on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()
