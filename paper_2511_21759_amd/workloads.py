"""Seeded synthetic inputs for the block-decode step and the cache-refresh prefill.

This module only draws token ids and mask patterns; it contains none of the
method's arithmetic and loads neither the HIP library nor the CPU oracle.
Tests and the benchmark hand its arrays to both sides.

The shapes follow the paper's set-up (ODB-dLLM, Sec. 4.2 and Sec. 5.1): blocks
of 32 tokens, block_0 plus 3 speculative blocks in the accept-jump stage and
8 blocks in the decoded-share stage, responses of up to 1024 positions behind
few-shot prompts.  The paper's prompts come from public benchmarks that are
not reproduced here: ids are uniform random and stand in for them.
"""
from __future__ import annotations

import dataclasses
from typing import Dict

import numpy as np

#: model shapes named by the workloads (field names match the C struct odb_config)
MODEL_SHAPES: Dict[str, Dict] = {
    "tiny": dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=768,
                 vocab=1024, rope_base=10000.0, rms_eps=1e-5, mask_id=1023),
    "8b": dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ff=12288,
               vocab=126464, rope_base=10000.0, rms_eps=1e-5, mask_id=126463),
}

WEIGHT_SEED = 20251121
WEIGHT_STD = 0.02


@dataclasses.dataclass
class DecodeWorkload:
    """tokens[B, L]: the sequence the cache is built from (prompt + response,
    undecoded response positions hold mask_id); drafts[B, S, b]: the S
    candidate versions of the block at positions block_off .. block_off+b-1."""
    tokens: np.ndarray
    drafts: np.ndarray
    block_off: int
    resp_off: int
    tau: float


def _speculative_sets(n_extra: int):
    """Which of the ranked candidates c0..c3 each extra draft unmasks.

    Mirrors the structure of Sec. 4.2.1 (B, D, B+D) and Sec. 4.2.2 (third,
    top three, fourth, top four); here the ranking is random since the
    candidates of a synthetic block carry no meaning.
    """
    table = [(0,), (1,), (0, 1), (2,), (0, 1, 2), (3,), (0, 1, 2, 3)]
    return [table[i % len(table)] for i in range(n_extra)]


def decode_workload(shape: Dict, prompt_len: int, resp_len: int, block: int,
                    n_drafts: int, seed: int, batch: int = 1,
                    p_unmasked: float = 0.5, block_index: int = 0,
                    tau: float = 0.9, all_masked: bool = False) -> DecodeWorkload:
    rng = np.random.default_rng(seed)
    V, mask_id = shape["vocab"], shape["mask_id"]
    L = prompt_len + resp_len
    tokens = np.empty((batch, L), np.int32)
    tokens[:, :prompt_len] = rng.integers(0, V, (batch, prompt_len))
    resp = rng.integers(0, V, (batch, resp_len))
    if all_masked:
        keep = np.zeros((batch, resp_len), bool)
    else:
        keep = rng.random((batch, resp_len)) < p_unmasked
    tokens[:, prompt_len:] = np.where(keep, resp, mask_id)
    block_off = prompt_len + block_index * block
    assert block_off + block <= L
    drafts = np.empty((batch, n_drafts, block), np.int32)
    sets = _speculative_sets(n_drafts - 1)
    for bi in range(batch):
        base = tokens[bi, block_off:block_off + block].copy()
        drafts[bi, 0] = base
        masked = np.flatnonzero(base == mask_id)
        cand = rng.permutation(masked)[:4]
        ids = rng.integers(0, V - 1, 4)      # never mask_id when mask_id = V-1
        for s, which in enumerate(sets, start=1):
            d = base.copy()
            for c in which:
                if c < len(cand):
                    d[cand[c]] = ids[c]
            drafts[bi, s] = d
    return DecodeWorkload(tokens, drafts, block_off, prompt_len, tau)


def prefill_workload(shape: Dict, prompt_len: int, resp_len: int, seed: int,
                     batch: int = 1) -> np.ndarray:
    """tokens[B, L]: uniform-random prompt followed by an all-MASK response."""
    rng = np.random.default_rng(seed)
    tokens = np.full((batch, prompt_len + resp_len), shape["mask_id"], np.int32)
    tokens[:, :prompt_len] = rng.integers(0, shape["vocab"], (batch, prompt_len))
    return tokens


# The five workloads of the measurement plan, by index.
def config0(seed: int = WEIGHT_SEED + 1) -> DecodeWorkload:
    """Tiny model: 128 prompt ids in [0,1023], 64 MASK, block of 16 at offset 0, S=1."""
    return decode_workload(MODEL_SHAPES["tiny"], 128, 64, 16, 1, seed, all_masked=True)


def config1(seed: int = WEIGHT_SEED + 1) -> DecodeWorkload:
    """8B shape, 256 prompt + 256 response (half unmasked), block of 32, S=1."""
    return decode_workload(MODEL_SHAPES["8b"], 256, 256, 32, 1, seed)


def config2(seed: int = WEIGHT_SEED + 1) -> DecodeWorkload:
    """As config1 with S=4 drafts sharing the cache (128 rows per weight read)."""
    return decode_workload(MODEL_SHAPES["8b"], 256, 256, 32, 4, seed)


def config3(resp_len: int, seed: int = WEIGHT_SEED + 1) -> np.ndarray:
    """Cache-refresh prefill: 512 prompt + {512,256,128} MASK positions."""
    return prefill_workload(MODEL_SHAPES["8b"], 512, resp_len, seed)


def config4(seed: int = WEIGHT_SEED + 1) -> DecodeWorkload:
    """Batch 4, 2048 prompt + 1024 response, block of 64, S=8 (2048 rows)."""
    return decode_workload(MODEL_SHAPES["8b"], 2048, 1024, 64, 8, seed, batch=4)


def config4_small(seed: int = WEIGHT_SEED + 4) -> DecodeWorkload:
    """Config 4's structure (batch 4, block of 64, S=8: 2048 rows) on a 256 + 256 context, second response block:
    small enough for the CPU oracle at the full 8B width with two layers (parity test, not a bench line)."""
    return decode_workload(MODEL_SHAPES["8b"], 256, 256, 64, 8, seed, batch=4, block_index=1)


def config2_shared(seed: int = WEIGHT_SEED + 1) -> DecodeWorkload:
    """Decoded-share stage (ODB-dLLM Sec. 4.2.2): config 1's cache, a block of 32 three quarters decoded, block_0
    plus seven speculative blocks (third, top three, fourth, top four candidates on top of B, D, B+D)."""
    return decode_workload(MODEL_SHAPES["8b"], 256, 256, 32, 8, seed, p_unmasked=0.75)
