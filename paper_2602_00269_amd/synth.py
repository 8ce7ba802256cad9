"""Seeded synthetic decode-step workloads.

This module only draws random numbers and deals block ids.  It contains none of
the arithmetic or index formulas of the decode step: pools are filled as opaque
``[P, Hkv, B*D]`` granules of i.i.d. values, so the same tensors can be handed
to the HIP library and (copied to the host) to the CPU oracle.

The paper evaluates on request traces (Poisson arrivals over LibriTTS /
VoiceBench prompts, Section 4.1); the decode step depends only on shapes and
context lengths, so the five presets below stand in for those traces: many
streams at unrelated progress points, freshly admitted short streams next to
long-running ones (startup vs steady-state phase, Section 3.2.1) and a
1000-request offline batch (Section 4.3.3).
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

BLOCK = 16
SEED_BASE = 0x5EED0000

# name, streams, q heads, kv heads, head dim, layers
_PRESETS = {
    1: ("cfg1_tiny_4x8q2kv64", 4, 8, 2, 64, 1),
    2: ("cfg2_64x24q8kv128", 64, 24, 8, 128, 1),
    3: ("cfg3_256x24q8kv128", 256, 24, 8, 128, 1),
    4: ("cfg4_512x24q8kv128_skew", 512, 24, 8, 128, 1),
    5: ("cfg5_1024x14q2kv64_28layers", 1024, 14, 2, 64, 28),
}


@dataclass
class Workload:
    """One decode step's inputs.  Per-layer tensors are lists of length ``layers``."""

    name: str
    cfg: int
    seed: int
    num_streams: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    num_blocks: int
    max_blocks_per_stream: int
    scale: float
    layers: int
    context_lens: np.ndarray  # int32 [S], counts the token appended this step
    block_tables: np.ndarray  # int32 [S, max_blocks_per_stream], -1 past the last block
    q: List[torch.Tensor] = field(default_factory=list)  # [S, Hq, D] bf16
    k_new: List[torch.Tensor] = field(default_factory=list)  # [S, Hkv, D] bf16
    v_new: List[torch.Tensor] = field(default_factory=list)
    k_pool: List[torch.Tensor] = field(default_factory=list)  # [P, Hkv, B*D] bf16 granules
    v_pool: List[torch.Tensor] = field(default_factory=list)

    @property
    def total_tokens(self) -> int:
        return int(self.context_lens.astype(np.int64).sum())

    @property
    def kv_bytes_per_token(self) -> int:
        # K and V rows of every kv head, bf16
        return 2 * self.num_kv_heads * self.head_dim * 2

    @property
    def kv_bytes_per_layer(self) -> int:
        return self.total_tokens * self.kv_bytes_per_token


def draw_context_lens(cfg: int, num_streams: int, rng: np.random.Generator) -> np.ndarray:
    """Context lengths (including the token appended this step) of preset ``cfg``."""
    s = num_streams
    if cfg == 1:
        lens = rng.integers(1, 257, size=s)
    elif cfg == 2:
        lens = rng.integers(200, 2001, size=s)
    elif cfg == 3:
        lens = rng.integers(500, 4001, size=s)
    elif cfg == 4:
        z = rng.standard_normal(s)
        lens = np.clip(np.rint(np.exp(math.log(1000.0) + 0.8 * z)), 1, 8192).astype(np.int64)
        fresh = rng.permutation(s)[: int(round(0.1 * s))]
        lens[fresh] = rng.integers(1, 33, size=fresh.size)
    elif cfg == 5:
        lens = rng.integers(64, 4097, size=s)
    else:
        raise ValueError(f"unknown preset {cfg}")
    return lens.astype(np.int32)


def deal_block_tables(lens: np.ndarray, num_blocks: int, rng: np.random.Generator,
                      max_blocks_per_stream: Optional[int] = None):
    """Deal a seeded permutation of ``[0, num_blocks)`` to the streams in order.

    Returns ``(tables, unused_ids)``; table entries past a stream's last block are -1.
    """
    nb = (lens.astype(np.int64) + BLOCK - 1) // BLOCK
    need = int(nb.sum())
    if need > num_blocks:
        raise ValueError(f"pool of {num_blocks} blocks cannot hold {need}")
    width = int(max(1, nb.max() if nb.size else 1))
    if max_blocks_per_stream is not None:
        if max_blocks_per_stream < width:
            raise ValueError("max_blocks_per_stream too small")
        width = max_blocks_per_stream
    perm = rng.permutation(num_blocks).astype(np.int32)
    tables = np.full((lens.size, width), -1, dtype=np.int32)
    pos = 0
    for s, n in enumerate(nb):
        n = int(n)
        tables[s, :n] = perm[pos:pos + n]
        pos += n
    return tables, perm[pos:].copy()


def pool_blocks_for(cfg: int, lens: np.ndarray) -> int:
    need = int(((lens.astype(np.int64) + BLOCK - 1) // BLOCK).sum())
    if cfg == 1:
        return 128
    if cfg == 2:
        return need  # shuffled, no slack
    return int(math.ceil(1.25 * need))  # fragmented pool with 25 % slack


def _randn_bf16(shape, gen: torch.Generator, device) -> torch.Tensor:
    # One fp32 draw rounded once (round-to-nearest-even) to bf16: the only rounding
    # the inputs ever see; both the library and the oracle consume these bits.
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)


def _fill_pool(num_blocks: int, hkv: int, granule: int, head_mul: Optional[torch.Tensor],
               unused: np.ndarray, gen: torch.Generator, device) -> torch.Tensor:
    pool = torch.empty((num_blocks, hkv, granule), dtype=torch.bfloat16, device=device)
    step = max(1, (1 << 26) // (hkv * granule))  # ~64 Mi values per draw
    for b0 in range(0, num_blocks, step):
        b1 = min(num_blocks, b0 + step)
        x = torch.randn((b1 - b0, hkv, granule), generator=gen, device=device, dtype=torch.float32)
        if head_mul is not None:
            x *= head_mul.view(1, hkv, 1)
        pool[b0:b1] = x.to(torch.bfloat16)
    if unused.size:
        idx = torch.from_numpy(unused.astype(np.int64)).to(device)
        pool[idx] = float("nan")  # blocks no stream owns must never be read
    return pool


def make_workload(cfg: int, seed: Optional[int] = None, device="cpu",
                  layers: Optional[int] = None, num_streams: Optional[int] = None) -> Workload:
    """Build preset ``cfg`` (1..5).  ``layers`` / ``num_streams`` shrink a preset for tests."""
    name, s, hq, hkv, d, nlayers = _PRESETS[cfg]
    if num_streams is not None:
        s = num_streams
    if layers is not None:
        nlayers = layers
    seed = SEED_BASE + cfg if seed is None else seed
    rng = np.random.default_rng(seed)
    lens = draw_context_lens(cfg, s, rng)
    p = pool_blocks_for(cfg, lens)
    tables, unused = deal_block_tables(lens, p, rng)
    w = Workload(name=name, cfg=cfg, seed=seed, num_streams=s, num_q_heads=hq, num_kv_heads=hkv,
                 head_dim=d, block_size=BLOCK, num_blocks=p, max_blocks_per_stream=tables.shape[1],
                 scale=1.0 / math.sqrt(d), layers=nlayers, context_lens=lens, block_tables=tables)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    k_mul = v_mul = None
    if cfg == 2:  # per-kv-head magnitude jitter U(0.5, 2), drawn once, K and V independently
        k_mul = torch.from_numpy(rng.uniform(0.5, 2.0, hkv).astype(np.float32)).to(dev)
        v_mul = torch.from_numpy(rng.uniform(0.5, 2.0, hkv).astype(np.float32)).to(dev)
    for _ in range(nlayers):
        w.q.append(_randn_bf16((s, hq, d), gen, dev))
        kn = torch.randn((s, hkv, d), generator=gen, device=dev, dtype=torch.float32)
        vn = torch.randn((s, hkv, d), generator=gen, device=dev, dtype=torch.float32)
        if k_mul is not None:
            kn *= k_mul.view(1, hkv, 1)
            vn *= v_mul.view(1, hkv, 1)
        w.k_new.append(kn.to(torch.bfloat16))
        w.v_new.append(vn.to(torch.bfloat16))
        w.k_pool.append(_fill_pool(p, hkv, BLOCK * d, k_mul, unused, gen, dev))
        w.v_pool.append(_fill_pool(p, hkv, BLOCK * d, v_mul, unused, gen, dev))
    return w


def make_custom(lens, num_q_heads: int, num_kv_heads: int, head_dim: int, seed: int,
                device="cpu", slack_blocks: int = 3, scale: Optional[float] = None,
                max_blocks_per_stream: Optional[int] = None) -> Workload:
    """A one-layer workload with explicit context lengths (zero = padded slot)."""
    lens = np.asarray(lens, dtype=np.int32)
    rng = np.random.default_rng(seed)
    need = int(((lens.astype(np.int64) + BLOCK - 1) // BLOCK).sum())
    p = max(1, need + slack_blocks)
    tables, unused = deal_block_tables(lens, p, rng, max_blocks_per_stream)
    s = int(lens.size)
    w = Workload(name=f"custom_{s}x{num_q_heads}q{num_kv_heads}kv{head_dim}", cfg=0, seed=seed,
                 num_streams=s, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                 head_dim=head_dim, block_size=BLOCK, num_blocks=p,
                 max_blocks_per_stream=tables.shape[1],
                 scale=(1.0 / math.sqrt(head_dim)) if scale is None else scale, layers=1,
                 context_lens=lens, block_tables=tables)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    w.q.append(_randn_bf16((s, num_q_heads, head_dim), gen, dev))
    w.k_new.append(_randn_bf16((s, num_kv_heads, head_dim), gen, dev))
    w.v_new.append(_randn_bf16((s, num_kv_heads, head_dim), gen, dev))
    w.k_pool.append(_fill_pool(p, num_kv_heads, BLOCK * head_dim, None, unused, gen, dev))
    w.v_pool.append(_fill_pool(p, num_kv_heads, BLOCK * head_dim, None, unused, gen, dev))
    return w


# ----------------------------------------------------------------------------------------------
# Multi-token steps: stream s brings n_s new tokens (a prompt, an admission chunk, a chunk of a
# stateful detokenizer whose self-attention cache lives in the same paged pools).  The paper
# fixes chunk sizes per model (Appendix A: 15, 25 and 28 tokens) and describes prompts only as
# text / reference-audio prompts of its request traces (Section 4.1); lengths below stand in.

@dataclass
class MultiWorkload:
    """Inputs of one multi-token step; ``base.context_lens`` already counts the new tokens."""

    name: str
    base: Workload
    new_tokens: np.ndarray  # int32 [S]
    q_offsets: np.ndarray   # int32 [S+1], exclusive prefix sums of new_tokens
    q: torch.Tensor         # [total_q, Hq, D] bf16
    k_new: torch.Tensor     # [total_q, Hkv, D] bf16
    v_new: torch.Tensor

    @property
    def total_q(self) -> int:
        return int(self.q_offsets[-1])


# name -> streams, q heads, kv heads, head dim
_MULTI_PRESETS = {
    "chunk15": ("chunk15_256x24q8kv128", 256, 24, 8, 128),
    "chunk25": ("chunk25_256x24q8kv128", 256, 24, 8, 128),
    "chunk28": ("chunk28_1024x14q2kv64", 1024, 14, 2, 64),
    "prefill": ("prefill_32x24q8kv128", 32, 24, 8, 128),
    "admit": ("admit_512x24q8kv128", 512, 24, 8, 128),
}
MULTI_NAMES = tuple(_MULTI_PRESETS)


def draw_multi_lens(kind: str, num_streams: int, rng: np.random.Generator):
    """(context lengths including the new tokens, new tokens per stream)."""
    s = num_streams
    if kind in ("chunk15", "chunk25"):  # detokenizer chunk on top of a cache of earlier chunks
        n = np.full(s, int(kind[5:]), dtype=np.int64)
        lens = np.maximum(rng.integers(500, 4001, size=s), n)
    elif kind == "chunk28":
        n = np.full(s, 28, dtype=np.int64)
        lens = np.maximum(rng.integers(64, 4097, size=s), n)
    elif kind == "prefill":  # whole prompts into empty caches
        lens = rng.integers(64, 513, size=s)
        n = lens.copy()
    elif kind == "admit":  # steady-state streams decode one token, one in ten is a new prompt
        lens = np.clip(np.rint(np.exp(math.log(1000.0) + 0.8 * rng.standard_normal(s))), 1, 8192)
        lens = lens.astype(np.int64)
        n = np.ones(s, dtype=np.int64)
        fresh = rng.permutation(s)[: max(1, s // 10)]
        lens[fresh] = rng.integers(32, 257, size=fresh.size)
        n[fresh] = lens[fresh]
    else:
        raise ValueError(f"unknown multi-token workload {kind!r}")
    return lens.astype(np.int32), n.astype(np.int32)


def make_multi_workload(kind: str, seed: Optional[int] = None, device="cpu",
                        num_streams: Optional[int] = None) -> MultiWorkload:
    name, s, hq, hkv, d = _MULTI_PRESETS[kind]
    if num_streams is not None:
        s = num_streams
    seed = SEED_BASE + 0x100 + MULTI_NAMES.index(kind) if seed is None else seed
    rng = np.random.default_rng(seed)
    lens, n = draw_multi_lens(kind, s, rng)
    base = make_custom(lens, hq, hkv, d, seed=seed, device=device,
                       slack_blocks=max(3, int(0.25 * ((lens.astype(np.int64) + 15) // 16).sum())))
    base.name = name
    qo = np.zeros(s + 1, dtype=np.int32)
    qo[1:] = np.cumsum(n)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed + 1)
    tq = int(qo[-1])
    return MultiWorkload(name=name, base=base, new_tokens=n, q_offsets=qo,
                         q=_randn_bf16((tq, hq, d), gen, dev),
                         k_new=_randn_bf16((tq, hkv, d), gen, dev),
                         v_new=_randn_bf16((tq, hkv, d), gen, dev))


# ----------------------------------------------------------------------------------------------
# Inputs of the fused RoPE + split + append step: the packed output rows of a layer's QKV
# projection and the caller's cos / sin tables.  Tables are evaluated in fp64 and rounded once.

def rope_tables(positions: int, head_dim: int, theta: float = 10000.0):
    """fp32 (cos, sin) of shape [positions, head_dim/2]; angle = pos * theta**(-2i/head_dim)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    ang = np.arange(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def make_qkv(w: Workload, seed: int, device="cpu", layers: Optional[int] = None) -> List[torch.Tensor]:
    """One packed [S, Hq + 2*Hkv, D] bf16 tensor of N(0,1) values per layer."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n = w.layers if layers is None else layers
    return [_randn_bf16((w.num_streams, w.num_q_heads + 2 * w.num_kv_heads, w.head_dim), gen, dev)
            for _ in range(n)]


# ----------------------------------------------------------------------------------------------
# Inputs of the sampling step: logits of a batch of streams, their recent tokens, uniforms.
# The paper gives the sampling settings per model (Appendix A) but no logits; a Zipf-like
# spectrum with Gaussian noise stands in for the output of an LM head: a few likely tokens, a
# long tail.

SAMPLING_PRESETS = {
    # name: (temperature, top_p, top_k, repetition_penalty): the settings of Appendix A
    "cosyvoice": (0.8, 0.95, 50, 1.1),
    "orpheus": (0.6, 0.8, 0, 1.3),
    "stepaudio": (0.7, 0.9, 0, 1.05),
}


def make_logits(num_streams: int, vocab: int, seed: int, device="cpu", spread: float = 2.0):
    """fp32 logits [S, V]: -1.2 * log(rank) over a per-stream random ranking + N(0, spread)."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    noise = torch.randn((num_streams, vocab), generator=gen, device=dev, dtype=torch.float32)
    ranks = torch.rand((num_streams, vocab), generator=gen, device=dev).argsort(dim=1).argsort(dim=1)
    return (-1.2 * torch.log(ranks.to(torch.float32) + 1.0) + spread * noise).contiguous()


def make_history(num_streams: int, vocab: int, window: int, seed: int):
    """int32 [S, window] recent tokens; a seeded fifth of the slots is empty (-1)."""
    rng = np.random.default_rng(seed)
    h = rng.integers(0, vocab, size=(num_streams, window)).astype(np.int32)
    h[rng.random((num_streams, window)) < 0.2] = -1
    return h


def make_uniforms(num_streams: int, seed: int):
    rng = np.random.default_rng(seed)
    return rng.random(num_streams, dtype=np.float32)
