"""Seeded synthetic inputs for the five benchmark configurations.

This module only *generates inputs* (activations, gate weights, routing biases, expert
weights, balance plans).  It holds none of the layer's arithmetic and imports neither the
HIP binding nor the CPU oracle, so both can be fed from it.

The paper measured on prompt sets pushed through two production checkpoints; those are not
reproduced.  What is kept is their structure: softmax top-k gating over 8..256 experts,
Zipf-like expert popularity whose hot set moves abruptly, per-rank batches of 128 (decode)
to 16K (prefill chunk) tokens, and a handful of replicated hot experts per GPU (Sec. 2.1,
Sec. 5 and Sec. 6 of the paper).

Everything is numpy; bf16 tensors are ``uint16`` bit patterns.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    cid: int            # 1-based index into the list of benchmark configurations
    name: str
    T: int              # tokens
    H: int              # hidden size
    E: int              # routed experts
    k: int              # top-k
    F: int              # expert FFN width
    E_loc: int          # native experts on this GPU (experts 0..E_loc-1, slot = expert id)
    n_rep: int          # replica slots on this GPU
    zipf_s: float       # skew exponent
    chunk: int          # tokens per routing-bias group (0 = one bias row for the call)
    n_batches: int      # distinct batches the generator defines (hot set moves per batch)
    ep: int             # virtual expert-parallel ranks (E / E_loc)

    @property
    def S(self) -> int:
        return self.E_loc + self.n_rep

    @property
    def N(self) -> int:
        return self.T * self.k

    @property
    def G(self) -> int:
        return 1 if self.chunk == 0 else (self.T + self.chunk - 1) // self.chunk


CONFIGS = {
    1: LayerConfig(1, "tiny", 256, 512, 8, 2, 1024, 8, 1, 1.2, 0, 2, 1),
    2: LayerConfig(2, "mixtral-8x7b-shaped", 4096, 4096, 8, 2, 14336, 8, 2, 1.0, 512, 2, 1),
    3: LayerConfig(3, "deepseek-v3-shaped-shard", 8192, 7168, 256, 8, 2048, 32, 4, 1.1, 0, 8, 8),
    4: LayerConfig(4, "qwen3-moe-shaped-decode", 128, 4096, 128, 8, 1536, 16, 2, 1.1, 0, 16, 8),
    5: LayerConfig(5, "predictor-stress", 16384, 7168, 256, 8, 2048, 64, 0, 1.5, 1024, 2, 4),
    # beyond the five benchmark configurations: one rank's share (ep = 8, two replica slots) of the two
    # models the paper evaluates (Sec. 5), at a prefill chunk of 8192 tokens per rank; shapes only
    6: LayerConfig(6, "gpt-oss-120b-shaped-prefill", 8192, 2880, 128, 4, 2880, 16, 2, 1.1, 0, 8, 8),
    7: LayerConfig(7, "qwen3-moe-235b-shaped-prefill", 8192, 4096, 128, 8, 1536, 16, 2, 1.1, 0, 8, 8),
}
ROTATING_HOT_SET = (3, 6, 7)   # one base popularity order, rotated by E_loc experts per batch


def small_config(T=96, H=128, E=16, k=4, F=192, E_loc=4, n_rep=2, zipf_s=1.1, chunk=32,
                 ep=4, cid=90) -> LayerConfig:
    """A reduced configuration for fast tests (same generator, arbitrary small shape)."""
    return LayerConfig(cid, "small", T, H, E, k, F, E_loc, n_rep, zipf_s, chunk, 4, ep)


# ------------------------------------------------------------------ bf16 helpers

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(cfg: LayerConfig, *key) -> np.random.Generator:
    return np.random.default_rng([1000 + cfg.cid, *[int(v) for v in key]])


def _normal_bf16(rng, shape, scale) -> np.ndarray:
    """N(0, scale^2) drawn in fp32 and rounded to bf16, generated in row blocks."""
    out = np.empty(shape, np.uint16)
    rows = shape[0]
    step = max(1, (1 << 22) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = rng.standard_normal((r1 - r0,) + tuple(shape[1:]), dtype=np.float32)
        if scale != 1.0:
            blk *= np.float32(scale)
        out[r0:r1] = f32_to_bf16_bits(blk)
    return out


# ------------------------------------------------------------------ layer inputs

def activations(cfg: LayerConfig, batch: int = 0) -> np.ndarray:
    """x ~ N(0,1) rounded to bf16, [T,H] uint16."""
    return _normal_bf16(_rng(cfg, 1, batch), (cfg.T, cfg.H), 1.0)


def gate_weights(cfg: LayerConfig, layer: int = 0) -> np.ndarray:
    """Gate (or next-layer gate / predictor) weights ~ N(0, 0.02^2), fp32 [E,H]."""
    w = _rng(cfg, 2, layer).standard_normal((cfg.E, cfg.H), dtype=np.float32)
    return w * np.float32(0.02)


def zipf_bias(cfg: LayerConfig, batch: int = 0, layer: int = 0) -> np.ndarray:
    """Routing bias b[g,e] = -s * ln(rank_g(e)), fp32 [G,E]: softmax prior ~ rank^-s.

    The popularity order is a seeded permutation.  Configurations with ``chunk`` draw a fresh
    order per chunk of tokens (hot-spot migration inside one call).  Configuration 3 rotates
    one base order by E_loc experts per batch, so the hot set visits every virtual rank (so do 6 and 7).
    Configurations 1, 4 draw a fresh order per batch (per decode step)."""
    G, E = cfg.G, cfg.E
    b = np.empty((G, E), np.float32)
    for g in range(G):
        if cfg.cid in ROTATING_HOT_SET:
            base = _rng(cfg, 3, layer).permutation(E)
            order = np.roll(base, cfg.E_loc * batch)
        else:
            order = _rng(cfg, 3, layer, batch, g).permutation(E)
        rank = np.empty(E, np.int64)
        rank[order] = np.arange(1, E + 1)
        b[g] = (-cfg.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)
    return b


def tokens_per_group(cfg: LayerConfig) -> int:
    return cfg.chunk if cfg.chunk else cfg.T


def drifted_activations(cfg: LayerConfig, x_bits: np.ndarray, alpha: float, batch: int = 0) -> np.ndarray:
    """Next layer's hidden states h' = (h + alpha*eps)/sqrt(1+alpha^2), eps ~ N(0,1), bf16."""
    rng = _rng(cfg, 4, batch)
    out = np.empty_like(x_bits)
    step = max(1, (1 << 22) // cfg.H)
    inv = np.float32(1.0 / np.sqrt(1.0 + alpha * alpha))
    for r0 in range(0, cfg.T, step):
        r1 = min(cfg.T, r0 + step)
        eps = rng.standard_normal((r1 - r0, cfg.H), dtype=np.float32)
        out[r0:r1] = f32_to_bf16_bits((bf16_bits_to_f32(x_bits[r0:r1]) + np.float32(alpha) * eps) * inv)
    return out


def expert_weights(cfg: LayerConfig, expert: int, copy: int = 0):
    """One expert's SwiGLU weights ~ N(0, 0.02^2) in bf16.

    Returns (w13 [2F,H], w2 [H,F]) uint16; rows 0..F-1 of w13 are the gate projection W1 and
    rows F..2F-1 the up projection W3.  The draw depends on the expert id only: every replica
    of an expert holds the same values (in its own buffer)."""
    del copy
    w13 = _normal_bf16(_rng(cfg, 5, expert), (2 * cfg.F, cfg.H), 0.02)
    w2 = _normal_bf16(_rng(cfg, 6, expert), (cfg.H, cfg.F), 0.02)
    return w13, w2


def expert_weights_many(cfg: LayerConfig, experts, threads: int = 8):
    """Weights for a list of expert ids, drawn on a thread pool (numpy releases the GIL)."""
    experts = [int(e) for e in experts]
    uniq = sorted(set(experts))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        res = dict(zip(uniq, ex.map(lambda e: expert_weights(cfg, e), uniq)))
    return [res[e] for e in experts]


# ------------------------------------------------------------------ balance plan

def build_plan(cfg: LayerConfig, expert_counts: np.ndarray) -> dict:
    """Host-built balance plan for this GPU (virtual rank 0) from per-expert token counts.

    Returns rep_off [E+1], rep_slot [R], rep_weight [R] (all int32), num_slots and
    slot_expert [S] (which expert's weights each local slot holds).

    * Native experts 0..E_loc-1 sit in slots 0..E_loc-1.
    * When every expert is native (ep == 1), the n_rep most loaded experts get a second
      local slot and share their tokens 1:1 (plain round-robin).
    * Otherwise the n_rep most loaded *non-native* experts get a replica slot here next to
      their home copy (slot -1, another GPU).  The share moved here is the part of the home
      rank's load above the mean rank load, as a fraction of the expert's tokens, in
      sixteenths, at least 1/16 and at most 15/16 (one water-filling step at rank level).
    * Every other non-native expert has a single remote replica.
    Ties in load are broken toward the lower expert id."""
    E, E_loc, n_rep = cfg.E, cfg.E_loc, cfg.n_rep
    n = np.asarray(expert_counts, dtype=np.int64)
    assert n.shape == (E,)
    order = sorted(range(E), key=lambda e: (-int(n[e]), e))
    if cfg.ep == 1:
        hot = order[:n_rep]
    else:
        hot = [e for e in order if e >= E_loc][:n_rep]
    per_rank = E // cfg.ep
    rank_load = n.reshape(cfg.ep, per_rank).sum(axis=1) if cfg.ep > 1 else n.sum(keepdims=True)
    mean_load = float(rank_load.mean())
    rep_off, rep_slot, rep_weight = [0], [], []
    slot_expert = list(range(E_loc)) + [-1] * n_rep
    for e in range(E):
        native = e < E_loc
        if e in hot:
            slot = E_loc + hot.index(e)
            slot_expert[slot] = e
            if native:
                rep_slot += [e, slot]
                rep_weight += [1, 1]
            else:
                home = e // per_rank
                excess = max(0.0, float(rank_load[home]) - mean_load)
                q = int(round(16.0 * excess / max(1, int(n[e]))))
                q = min(15, max(1, q))
                rep_slot += [-1, slot]
                rep_weight += [16 - q, q]
        elif native:
            rep_slot.append(e)
            rep_weight.append(1)
        else:
            rep_slot.append(-1)
            rep_weight.append(1)
        rep_off.append(len(rep_slot))
    for s in range(E_loc, E_loc + n_rep):
        if slot_expert[s] < 0:          # fewer candidates than replica slots: idle slot
            slot_expert[s] = 0
    return dict(rep_off=np.asarray(rep_off, np.int32), rep_slot=np.asarray(rep_slot, np.int32),
                rep_weight=np.asarray(rep_weight, np.int32), num_slots=cfg.S,
                slot_expert=np.asarray(slot_expert, np.int32))


def no_replica_plan(cfg: LayerConfig) -> dict:
    """The baseline placement: native experts only, everything else remote."""
    E, E_loc = cfg.E, cfg.E_loc
    rep_slot = np.where(np.arange(E) < E_loc, np.arange(E), -1).astype(np.int32)
    return dict(rep_off=np.arange(E + 1, dtype=np.int32), rep_slot=rep_slot,
                rep_weight=np.ones(E, np.int32), num_slots=E_loc,
                slot_expert=np.arange(E_loc, dtype=np.int32))


def rank_loads(cfg: LayerConfig, expert_counts: np.ndarray) -> np.ndarray:
    """Token load per virtual rank under the static sharded placement."""
    n = np.asarray(expert_counts, dtype=np.float64)
    return n.reshape(cfg.ep, cfg.E // cfg.ep).sum(axis=1)
