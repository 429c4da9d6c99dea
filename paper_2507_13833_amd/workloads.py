"""Seeded synthetic GRPO rollout batches (inputs only).

This module draws the *inputs* of the Data Coordinator reshard path: sequence
lengths, prompt groups, rewards and per-token payload fields in the rollout
layout.  It contains none of the method's arithmetic (no partitioning, no
advantage, no offsets of the training layout), so the CPU oracle's tests and
the HIP path's tests can both be fed from it without sharing any computation.

The five workloads stand in for the paper's RL post-training batches (Sec. 7.1,
"Datasets": DeepScaleR / MM-Eureka prompts with a group of sampled responses
per prompt; App. B: GSM8K with 8 responses per prompt).  Those datasets are not
reproduced; only shape, length mix and value distributions are.

Recipe (all draws from ``numpy.random.default_rng(1000 + cfg)``, in the order
prompt lengths, response lengths, rewards, then per-field token payloads,
and for workload 5 the mask segmentation last):

* a prompt's length is drawn once and shared by the G responses of its group;
* a sequence is prompt tokens followed by response tokens, packed back to back
  in response order inside its rollout shard;
* ``mask`` is 0 on prompt tokens and 1 on response tokens (workload 5: a
  response is cut into 1..4 segments with alternating 1/0 runs, first run 1);
* bf16 payloads are carried as uint16 bit patterns (round-to-nearest-even of
  the fp32 draw).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np


@dataclass
class Field:
    """One per-token payload field in the rollout layout."""
    name: str
    elem_bytes: int                 # 1, 2 or 4
    shards: List[np.ndarray]        # one packed array per rollout shard


@dataclass
class Workload:
    name: str
    cfg: int
    n_seq: int                      # N
    group_size: int                 # G
    n_shards: int                   # P: training-layout shards (K of Alg. 1)
    token_budget: int
    eps: float
    ddof: int
    align_tokens: int
    seq_len: np.ndarray             # int32 [N]  prompt + response tokens
    prompt_len: np.ndarray          # int32 [N]
    group_off: np.ndarray           # int32 [n_groups + 1]  CSR over sequences
    reward: np.ndarray              # float32 [N]
    src_shard_seq_off: np.ndarray   # int32 [n_src + 1]
    src_tok_off: np.ndarray         # int64 [N]  element offset inside own rollout shard
    src_shard_tokens: np.ndarray    # int64 [n_src]
    fields: List[Field] = field(default_factory=list)

    @property
    def n_src_shards(self) -> int:
        return len(self.src_shard_tokens)

    @property
    def total_tokens(self) -> int:
        return int(self.src_shard_tokens.sum())

    @property
    def n_groups(self) -> int:
        return len(self.group_off) - 1

    def field_by_name(self, name: str) -> Field:
        for f in self.fields:
            if f.name == name:
                return f
        raise KeyError(name)

    @property
    def payload_bytes_per_token(self) -> int:
        return sum(f.elem_bytes for f in self.fields)


# name, prompts, G, prompt lo/hi, P, budget, rollout shards
_SHAPES: Dict[int, dict] = {
    1: dict(name="tiny", prompts=64, G=8, plo=64, phi=256, P=4, budget=8192, n_src=1),
    2: dict(name="mid", prompts=256, G=8, plo=128, phi=1024, P=8, budget=16384, n_src=1),
    3: dict(name="large", prompts=512, G=16, plo=256, phi=2048, P=32, budget=32768, n_src=1),
    4: dict(name="layout_change", prompts=512, G=16, plo=256, phi=2048, P=16, budget=65536, n_src=8),
    5: dict(name="long_tail", prompts=1024, G=16, plo=512, phi=4096, P=64, budget=131072, n_src=1),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def _response_len(cfg: int, rng: np.random.Generator, n: int) -> np.ndarray:
    if cfg == 1:
        return np.clip(np.rint(rng.lognormal(5.5, 0.8, n)), 16, 1024).astype(np.int32)
    if cfg == 2:
        return np.clip(np.rint(rng.lognormal(6.5, 1.0, n)), 32, 4096).astype(np.int32)
    if cfg in (3, 4):
        return np.clip(np.rint(rng.lognormal(7.0, 1.1, n)), 64, 8192).astype(np.int32)
    # classical Pareto(alpha=1.3, x_m=1): X = (1-U)^(-1/alpha) >= 1
    u = rng.random(n)
    x = (1.0 - u) ** (-1.0 / 1.3)
    return np.minimum(32768.0, np.floor(64.0 * x)).astype(np.int32)


def _reward(cfg: int, rng: np.random.Generator, n: int, G: int) -> np.ndarray:
    if cfg == 1:
        return (rng.random(n) < 0.4).astype(np.float32)
    if cfg == 2:
        return (np.rint(10.0 * rng.random(n)) / 10.0).astype(np.float32)
    if cfg == 3:
        return (rng.random(n) < 0.3).astype(np.float32)
    if cfg == 4:
        r = (rng.random(n) < 0.3).astype(np.float32).reshape(-1, G)
        same = (np.arange(r.shape[0]) % 8) < 3      # three of every eight groups
        r[same, :] = r[same, :1]
        return np.ascontiguousarray(r.reshape(-1))
    return rng.standard_normal(n).astype(np.float32)


def _neg_abs_normal(rng: np.random.Generator, n: int) -> np.ndarray:
    x = rng.standard_normal(n, dtype=np.float32)
    np.abs(x, out=x)
    np.negative(x, out=x)
    return x


def _basic_mask(prompt_len: np.ndarray, seq_len: np.ndarray, tok_off: np.ndarray, total: int) -> np.ndarray:
    """0 on prompt tokens, 1 on response tokens (packed order)."""
    m = np.ones(total, dtype=np.uint8)
    # mark prompt spans with a difference array
    d = np.zeros(total + 1, dtype=np.int32)
    np.add.at(d, tok_off, 1)
    np.add.at(d, tok_off + prompt_len, -1)
    m[np.cumsum(d[:-1]) > 0] = 0
    return m


def _multiturn_mask(rng: np.random.Generator, prompt_len, seq_len, tok_off, total) -> np.ndarray:
    m = _basic_mask(prompt_len, seq_len, tok_off, total)
    n = len(seq_len)
    n_seg = rng.integers(1, 5, n)
    for i in range(n):
        r = int(seq_len[i] - prompt_len[i])
        k = min(int(n_seg[i]), r)
        if k <= 1:
            continue
        cuts = np.sort(rng.choice(np.arange(1, r), size=k - 1, replace=False))
        base = int(tok_off[i] + prompt_len[i])
        bounds = [0, *cuts.tolist(), r]
        for s in range(1, k, 2):                      # odd segments: tool output, no loss
            m[base + bounds[s]: base + bounds[s + 1]] = 0
    return m


def sequence_lengths(cfg: int, n_seq: int, seed: int | None = None) -> np.ndarray:
    """Only the sequence lengths of workload ``cfg`` with ``n_seq`` sequences, a multiple of its group size (the
    first two draws of make_workload): for measurements of the balance alone at sizes whose payload is not needed."""
    sh = _SHAPES[cfg]
    if n_seq % sh["G"]:
        raise ValueError("sequence count must be a multiple of the group size")
    prompts = n_seq // sh["G"]
    rng = np.random.default_rng(1000 + cfg if seed is None else seed)
    p_len = np.repeat(rng.integers(sh["plo"], sh["phi"] + 1, prompts), sh["G"]).astype(np.int32)
    return (p_len + _response_len(cfg, rng, prompts * sh["G"])).astype(np.int32)


def make_workload(cfg: int, prompts: int | None = None, n_shards: int | None = None,
                  seed: int | None = None) -> Workload:
    """Draw workload ``cfg`` (1..5).  ``prompts`` shrinks the batch for quick tests
    while keeping every distribution; ``n_shards`` overrides P."""
    sh = _SHAPES[cfg]
    rng = np.random.default_rng(1000 + cfg if seed is None else seed)
    n_prompts = sh["prompts"] if prompts is None else prompts
    G = sh["G"]
    N = n_prompts * G
    P = sh["P"] if n_shards is None else n_shards
    n_src = sh["n_src"]
    if N % n_src:
        raise ValueError("sequence count must divide over the rollout shards")

    p_len = np.repeat(rng.integers(sh["plo"], sh["phi"] + 1, n_prompts), G).astype(np.int32)
    r_len = _response_len(cfg, rng, N)
    seq_len = (p_len + r_len).astype(np.int32)
    reward = _reward(cfg, rng, N, G)
    group_off = (np.arange(n_prompts + 1, dtype=np.int64) * G).astype(np.int32)

    per = N // n_src
    src_shard_seq_off = (np.arange(n_src + 1, dtype=np.int64) * per).astype(np.int32)
    src_tok_off = np.zeros(N, dtype=np.int64)
    src_shard_tokens = np.zeros(n_src, dtype=np.int64)
    for s in range(n_src):
        a, b = int(src_shard_seq_off[s]), int(src_shard_seq_off[s + 1])
        c = np.cumsum(seq_len[a:b].astype(np.int64))
        src_tok_off[a + 1:b] = c[:-1]
        src_shard_tokens[s] = c[-1] if b > a else 0

    vocab = 32000 if cfg == 1 else 152064
    spec = {
        1: [("token_id", "i32"), ("old_logprob", "f32")],
        2: [("token_id", "i32"), ("old_logprob", "bf16"), ("ref_logprob", "bf16")],
        3: [("token_id", "i32"), ("old_logprob", "f32"), ("ref_logprob", "f32"), ("value", "f32")],
        4: [("token_id", "i32"), ("old_logprob", "f32"), ("ref_logprob", "f32"), ("value", "f32")],
        5: [("token_id", "i32"), ("old_logprob", "f32"), ("ref_logprob", "f32"), ("value", "f32"),
            ("entropy", "bf16")],
    }[cfg]

    fields: List[Field] = []
    for name, kind in spec:
        shards = []
        for s in range(n_src):
            t = int(src_shard_tokens[s])
            if kind == "i32":
                arr = rng.integers(0, vocab, t, dtype=np.int32)
            elif name == "value":
                arr = rng.standard_normal(t, dtype=np.float32)
            elif name == "entropy":
                arr = f32_to_bf16_bits(np.abs(rng.standard_normal(t, dtype=np.float32)))
            elif kind == "bf16":
                arr = f32_to_bf16_bits(_neg_abs_normal(rng, t))
            else:
                arr = _neg_abs_normal(rng, t)
            shards.append(arr)
        fields.append(Field(name, {"i32": 4, "f32": 4, "bf16": 2}[kind], shards))

    masks = []
    for s in range(n_src):
        a, b = int(src_shard_seq_off[s]), int(src_shard_seq_off[s + 1])
        t = int(src_shard_tokens[s])
        if cfg == 5:
            masks.append(_multiturn_mask(rng, p_len[a:b], seq_len[a:b], src_tok_off[a:b], t))
        else:
            masks.append(_basic_mask(p_len[a:b], seq_len[a:b], src_tok_off[a:b], t))
    fields.append(Field("mask", 1, masks))

    return Workload(name=sh["name"], cfg=cfg, n_seq=N, group_size=G, n_shards=P,
                    token_budget=sh["budget"], eps=1e-6, ddof=1, align_tokens=1,
                    seq_len=seq_len, prompt_len=p_len, group_off=group_off, reward=reward,
                    src_shard_seq_off=src_shard_seq_off, src_tok_off=src_tok_off,
                    src_shard_tokens=src_shard_tokens, fields=fields)
