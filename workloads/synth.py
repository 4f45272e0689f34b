"""Synthetic causal-prefill workloads with heterogeneous per-head sparsity.

The paper evaluates on long-context prompts pushed through Llama-3.1-8B / Qwen2.5
class models at up to 128K tokens (Section 5.1) and motivates the method with
per-head recovery-ratio heterogeneity (Section 2.4).  Neither the prompts nor the
weights are available, so these generators imitate the *shape* of one attention
layer (GQA, head_dim 128, 2K..128K tokens) and the *qualitative structure* the
paper describes: a few key positions carry most of a head's attention mass
(Section 2.3), initial and recent tokens matter (the StreamingLLM pattern of
Section 2.3), and the amount of concentration differs from head to head
(Section 2.4).

Recipe (all draws from Philox streams keyed by (seed, stream id)):
  * Q, K, V ~ N(0,1) in fp32, rounded to bf16 (round-to-nearest-even).
  * each query head h has a mean direction m_h = rho * u_h (rho = 4); the G
    sibling heads of one KV group get orthonormal u_h; Q[:, h, :] += m_h.
  * each (sequence, head) has a concentration c and two "heavy" key blocks drawn
    uniformly from [1, nb-2]; the keys of those blocks and of block 0 (the sink)
    in the head's KV group get += c * m_h before rounding.
  * budgets are drawn per head (per (sequence, head) for the varlen batch) as a
    fraction f of the sequence's block count: k = clamp(floor(f*nb + 0.5), 2, nb).

Nothing here pools, scores, selects, attends or partitions.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

RHO = 4.0
_CHUNK_TOKENS = 4096

# Stream ids for the Philox key (seed, stream).
_S_Q, _S_K, _S_V, _S_DIR, _S_CONC, _S_HEAVY, _S_BUDGET, _S_DENSE = range(1, 9)


CONFIGS: Dict[int, dict] = {
    0: dict(name="cfg0_mha8_2k_b64", seqlens=[2048], n_q_heads=8, n_kv_heads=8, block=64,
            c_range=(0.5, 4.0), budget=("choice", (2, 4, 8, 16)), n_parts=2),
    1: dict(name="cfg1_llama3_8b_32k", seqlens=[32768], n_q_heads=32, n_kv_heads=8, block=128,
            c_range=(0.25, 6.0), budget=("loguniform", 0.02, 0.5)),
    2: dict(name="cfg2_llama3_8b_128k", seqlens=[131072], n_q_heads=32, n_kv_heads=8, block=128,
            c_range=(0.25, 6.0), budget=("loguniform", 0.01, 0.3), dense_heads=4),
    3: dict(name="cfg3_share_of_64h_64k", seqlens=[65536], n_q_heads=64, n_kv_heads=16, block=128,
            c_range=(0.25, 6.0), budget=("bimodal", ((0.03, 0.7), (0.4, 0.3))),
            n_parts=8, groups_per_part=2),
    4: dict(name="cfg4_varlen_batch", seqlens=[8192, 24576, 65536, 131072], n_q_heads=32,
            n_kv_heads=8, block=128, c_range=(0.25, 6.0), budget=("loguniform", 0.01, 0.5),
            per_sequence_budgets=True),
}
HEAD_DIM = 128


@dataclass
class Workload:
    name: str
    seed: int
    cu_seqlens: np.ndarray          # int32 [n_seq+1]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block: int
    q: np.ndarray                   # uint16 (bf16 bits) [T, n_q_heads, head_dim]
    k: np.ndarray                   # uint16 (bf16 bits) [T, n_kv_heads, head_dim]
    v: np.ndarray                   # uint16 (bf16 bits) [T, n_kv_heads, head_dim]
    budgets: np.ndarray             # int32 [n_seq * n_q_heads], in key blocks
    meta: dict = field(default_factory=dict)
    kv_head_of: Optional[np.ndarray] = None   # int32 [n_q_heads]: KV head of each query head; None = equal groups

    @property
    def n_seq(self) -> int:
        return len(self.cu_seqlens) - 1

    @property
    def n_blocks(self) -> List[int]:
        s = np.diff(self.cu_seqlens)
        return [int((x + self.block - 1) // self.block) for x in s]


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def _head_directions(seed: int, n_q_heads: int, n_kv_heads: int, d: int) -> np.ndarray:
    """m_h = RHO * u_h with the sibling heads of one KV group mutually orthonormal."""
    g = n_q_heads // n_kv_heads
    rng = _rng(seed, _S_DIR)
    m = np.empty((n_q_heads, d), np.float64)
    for grp in range(n_kv_heads):
        a = rng.standard_normal((d, g))
        qmat, _ = np.linalg.qr(a)
        m[grp * g:(grp + 1) * g] = qmat.T[:g]
    return (RHO * m).astype(np.float32)


def _draw_fractions(rng: np.random.Generator, spec, n: int) -> np.ndarray:
    kind = spec[0]
    if kind == "loguniform":
        lo, hi = spec[1], spec[2]
        return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n))
    if kind == "bimodal":
        vals = np.array([p[0] for p in spec[1]])
        probs = np.array([p[1] for p in spec[1]])
        return vals[rng.choice(len(vals), size=n, p=probs / probs.sum())]
    raise ValueError(kind)


def _budget_from_fraction(f: np.ndarray, nb: int) -> np.ndarray:
    k = np.floor(f * nb + 0.5).astype(np.int64)
    return np.clip(k, 2, max(nb, 2)).astype(np.int32)


def layer_budgets(config: int, seqlens: Optional[Sequence[int]] = None,
                  seed: Optional[int] = None) -> dict:
    """Budget draw for the whole layer of a config: fractions f[n_seq, Hq] and
    budgets[n_seq, Hq] in blocks.  For config 3 this is what a caller partitions
    before materialising one part's heads."""
    cfg = CONFIGS[config]
    seed = 1000 * config if seed is None else seed
    seqlens = list(cfg["seqlens"] if seqlens is None else seqlens)
    hq, blk = cfg["n_q_heads"], cfg["block"]
    nbs = [(s + blk - 1) // blk for s in seqlens]
    rng = _rng(seed, _S_BUDGET)
    spec = cfg["budget"]
    n_seq = len(seqlens)
    if spec[0] == "choice":
        k_head = rng.choice(np.array(spec[1]), size=hq)
        budgets = np.stack([np.clip(k_head, 2, max(nb, 2)) for nb in nbs]).astype(np.int32)
        return dict(f=None, budgets=budgets, n_blocks=nbs)
    if cfg.get("per_sequence_budgets"):
        f = _draw_fractions(rng, spec, n_seq * hq).reshape(n_seq, hq)
    else:
        f = np.tile(_draw_fractions(rng, spec, hq), (n_seq, 1))
    nd = cfg.get("dense_heads", 0)
    if nd:
        dense = _rng(seed, _S_DENSE).choice(hq, size=nd, replace=False)
        f[:, dense] = 1.0
    budgets = np.stack([_budget_from_fraction(f[s], nbs[s]) for s in range(n_seq)])
    return dict(f=f, budgets=budgets, n_blocks=nbs)


def make_workload(config: int, seqlens: Optional[Sequence[int]] = None,
                  q_heads: Optional[Sequence[int]] = None,
                  seed: Optional[int] = None) -> Workload:
    """Materialise one of the five benchmark configurations.

    seqlens overrides the config's sequence lengths (scaled-down parity cases and
    ragged tails); q_heads picks a subset of the layer's query heads (whole KV
    groups, ascending) -- config 3 materialises only one partition's share.
    """
    cfg = CONFIGS[config]
    seed = 1000 * config if seed is None else seed
    seqlens = list(cfg["seqlens"] if seqlens is None else seqlens)
    lb = layer_budgets(config, seqlens, seed)
    hq_layer, hkv_layer = cfg["n_q_heads"], cfg["n_kv_heads"]
    g = hq_layer // hkv_layer
    if q_heads is None:
        q_heads = list(range(8)) if config == 3 else list(range(hq_layer))
    q_heads = [int(h) for h in q_heads]
    if len(q_heads) % g or any(q_heads[i * g + j] != q_heads[i * g] + j or q_heads[i * g] % g
                               for i in range(len(q_heads) // g) for j in range(g)):
        raise ValueError("q_heads must be whole KV groups in ascending order")
    budgets = lb["budgets"][:, q_heads]
    f = None if lb["f"] is None else lb["f"][:, q_heads]
    name = cfg["name"] if seqlens == list(cfg["seqlens"]) else cfg["name"] + "_S" + "_".join(map(str, seqlens))
    return _materialise(name, seed, seqlens, len(q_heads), len(q_heads) // g, cfg["block"],
                        cfg["c_range"], budgets, extra=dict(config=config, f=f, layer_heads=q_heads,
                                                            n_parts=cfg.get("n_parts")))


def make_custom(seqlens: Sequence[int], n_q_heads: int, n_kv_heads: int, block: int,
                budgets: Sequence[int], seed: int, c_range=(0.5, 4.0), name: str = "custom") -> Workload:
    """Free-form workload for edge cases (ragged tails, tiny sequences, explicit budgets).
    budgets: [n_seq * n_q_heads] or [n_q_heads] (repeated for every sequence)."""
    b = np.asarray(budgets, dtype=np.int32)
    if b.size == n_q_heads:
        b = np.tile(b, (len(seqlens), 1))
    b = b.reshape(len(seqlens), n_q_heads)
    return _materialise(name, seed, list(seqlens), n_q_heads, n_kv_heads, block, c_range, b,
                        extra=dict(config=None, f=None))


def _materialise(name, seed, seqlens, hq, hkv, blk, c_range, budgets, extra) -> Workload:
    d = HEAD_DIM
    g = hq // hkv
    n_seq = len(seqlens)
    cu = np.zeros(n_seq + 1, np.int32)
    cu[1:] = np.cumsum(seqlens)
    total = int(cu[-1])
    nbs = [(s + blk - 1) // blk for s in seqlens]

    m = _head_directions(seed, hq, hkv, d)                       # [hq, d] fp32
    conc = _rng(seed, _S_CONC).uniform(c_range[0], c_range[1], size=hq).astype(np.float32)
    rng_heavy = _rng(seed, _S_HEAVY)
    heavy = np.full((n_seq, hq, 2), -1, np.int32)
    for s in range(n_seq):
        for h in range(hq):
            if nbs[s] >= 4:
                heavy[s, h] = np.sort(rng_heavy.choice(np.arange(1, nbs[s] - 1), size=2, replace=False))

    # Q: noise + per-head mean direction.
    q = np.empty((total, hq, d), np.uint16)
    rq = _rng(seed, _S_Q)
    for t0 in range(0, total, _CHUNK_TOKENS):
        t1 = min(total, t0 + _CHUNK_TOKENS)
        x = rq.standard_normal((t1 - t0, hq, d), dtype=np.float32)
        x += m[None]
        q[t0:t1] = bf16_bits_from_f32(x)

    # V: noise only.
    v = np.empty((total, hkv, d), np.uint16)
    rv = _rng(seed, _S_V)
    for t0 in range(0, total, _CHUNK_TOKENS * 4):
        t1 = min(total, t0 + _CHUNK_TOKENS * 4)
        v[t0:t1] = bf16_bits_from_f32(rv.standard_normal((t1 - t0, hkv, d), dtype=np.float32))

    # K: noise, then the planted sink / heavy-block bias of every query head of the group.
    kf = _rng(seed, _S_K).standard_normal((total, hkv, d), dtype=np.float32)
    for s in range(n_seq):
        for h in range(hq):
            blocks = [0] + [int(b) for b in heavy[s, h] if b >= 0]
            for b in blocks:
                t0 = int(cu[s]) + b * blk
                t1 = min(int(cu[s + 1]), t0 + blk)
                kf[t0:t1, h // g, :] += conc[h] * m[h]
    k = bf16_bits_from_f32(kf)
    del kf

    meta = dict(extra)
    meta.update(mean_dir=m, conc=conc, heavy=heavy, n_blocks=nbs)
    return Workload(name=name, seed=seed, cu_seqlens=cu, n_q_heads=hq, n_kv_heads=hkv, head_dim=d,
                    block=blk, q=q, k=k, v=v, budgets=np.ascontiguousarray(budgets.reshape(-1), np.int32),
                    meta=meta)


def take_heads(wl: Workload, heads: Sequence[int]) -> Workload:
    """The share of a layer that a device holding the query heads `heads` works on: their Q
    columns and budgets, and the distinct KV heads they read (each once), with the map from
    the share's query heads to its KV heads.  Any subset in any order: the groups of a share
    need not be whole or of equal size.  Slicing only."""
    heads = [int(h) for h in heads]
    if wl.kv_head_of is None:
        g = wl.n_q_heads // wl.n_kv_heads
        kv_of_layer = [h // g for h in range(wl.n_q_heads)]
    else:
        kv_of_layer = [int(x) for x in wl.kv_head_of]
    kv = sorted({kv_of_layer[h] for h in heads})
    local = {x: n for n, x in enumerate(kv)}
    budgets = wl.budgets.reshape(wl.n_seq, wl.n_q_heads)[:, heads]
    meta = dict(layer_heads=heads, layer_kv_heads=kv)
    return Workload(name=wl.name + "_heads_" + "_".join(map(str, heads)), seed=wl.seed, cu_seqlens=wl.cu_seqlens,
                    n_q_heads=len(heads), n_kv_heads=len(kv), head_dim=wl.head_dim, block=wl.block,
                    q=np.ascontiguousarray(wl.q[:, heads]), k=np.ascontiguousarray(wl.k[:, kv]),
                    v=np.ascontiguousarray(wl.v[:, kv]), budgets=np.ascontiguousarray(budgets.reshape(-1)),
                    meta=meta, kv_head_of=np.asarray([local[kv_of_layer[h]] for h in heads], np.int32))


def one_kv_head_per_query_head(wl: Workload) -> Workload:
    """The same inputs with every query head given its own copy of the K/V head it reads (no
    sharing, no map): what a reference that only knows equal groups can be fed.  Slicing only."""
    if wl.kv_head_of is None:
        g = wl.n_q_heads // wl.n_kv_heads
        kv = [h // g for h in range(wl.n_q_heads)]
    else:
        kv = [int(x) for x in wl.kv_head_of]
    return Workload(name=wl.name + "_unshared", seed=wl.seed, cu_seqlens=wl.cu_seqlens, n_q_heads=wl.n_q_heads,
                    n_kv_heads=wl.n_q_heads, head_dim=wl.head_dim, block=wl.block, q=wl.q,
                    k=np.ascontiguousarray(wl.k[:, kv]), v=np.ascontiguousarray(wl.v[:, kv]), budgets=wl.budgets,
                    meta=dict(wl.meta))
