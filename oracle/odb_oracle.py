"""CPU oracle for the ODB-dLLM model step.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition of what the two library calls compute.
It is imported only by tests, by the smoke check and by the benchmark's
cpu_baseline leg; the product path never calls it and shares no code with it.

What it follows (ODB-dLLM, arXiv 2511.21759):
  * Sec. 2.1 (block-wise generation with a dual cache): K/V of every token
    outside the current block are cached by a full-sequence forward and reused
    while the block is decoded; the forward is bidirectional (no causal mask).
    Once a block is filled the cache is refreshed for the next one: generate()
    is that loop, with Sec. 4.1 and Sec. 4.2 as options.
  * Sec. 4.1 (adaptive length prediction): the refresh computes every response
    position and yields a decoding attempt (confidence, token) for all of them;
    the attempt is scanned for a confident [EOS] and the response cut there.
  * Sec. 3, Observation 3: masked tokens of the block are decoded in parallel
    and accepted when their confidence exceeds a threshold.
  * Sec. 4.2 (jump-share speculative decoding): speculative copies of the block
    (drafts) see the cached context and themselves, never each other, and keep
    the position ids of the block they shadow (Fig. 8 caption).  Sec. 4.2.1
    (accept-jump): which draft's result a step adopts and how the next drafts
    are formed from its two most confident unaccepted positions.  Sec. 4.2.2
    (decoded-share): decoded positions of the block are computed once, in
    block_0, and their K/V shared by the speculative blocks, which shrink to
    the still-masked positions.
    That stage's eight blocks (four extra candidate sets) are
    SPEC_SETS; the paper gives the jump rule for two candidates only, and
    speculative_jump() carries it over to eight blocks (for four blocks it is
    the rule of Sec. 4.2.1, which a test checks against accept_jump()).

Arithmetic: float64 throughout, on weights whose values are exactly
representable in bfloat16 (they are stored as bf16 bit patterns).  The model
step is exact mathematics, so the oracle is the definition written out with
numpy matmul/einsum as the only library steps; no blocking, fusion or caching
tricks.  Architecture (pre-norm residual blocks, RMSNorm, rotate-half RoPE,
SwiGLU, untied LM head, no biases) is not given by the paper, which only names
the LLaDA models (Sec. 5.1); the choices are recorded as readings in the
design notes of this repository.

Parity against numbers printed in the paper: unpinned (the paper prints no
intermediate value of the forward).  Every function is instead pinned by
closed forms, invariants, brute force and library routines in tests/.
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
import math
import os
from typing import Dict, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------- config

#: tensor ids of the counter-based weight generator (shared *by definition*
#: with the library, which implements the same generator separately)
T_EMBED, T_WQ, T_WK, T_WV, T_WO, T_WG, T_WU, T_WD, T_LM, T_G1, T_G2, T_GF = range(12)

TENSOR_NAMES = ("embed", "wq", "wk", "wv", "wo", "wg", "wu", "wd", "lm",
                "g1", "g2", "gf")


@dataclasses.dataclass(frozen=True)
class Config:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    mask_id: int = -1          # -1 -> vocab - 1

    def __post_init__(self):
        if self.mask_id < 0:
            object.__setattr__(self, "mask_id", self.vocab - 1)
        assert self.n_heads * self.head_dim == self.d_model
        assert self.head_dim % 2 == 0

    def shape(self, tid: int) -> Tuple[int, ...]:
        d, f, v = self.d_model, self.d_ff, self.vocab
        return {T_EMBED: (v, d), T_WQ: (d, d), T_WK: (d, d), T_WV: (d, d),
                T_WO: (d, d), T_WG: (f, d), T_WU: (f, d), T_WD: (d, f),
                T_LM: (v, d), T_G1: (d,), T_G2: (d,), T_GF: (d,)}[tid]


# --------------------------------------------------------------------------- weight generator

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _finalise(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function (Steele, Lea & Flood 2014) on uint64 arrays."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def splitmix64_stream(state0: int, start: int, n: int) -> np.ndarray:
    """Outputs number start .. start+n-1 of SplitMix64 seeded with state0.

    Output i is finalise(state0 + (i+1)*GAMMA mod 2^64): the generator is
    counter based, so any slice can be produced without the ones before it.
    """
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + n + 1, dtype=np.uint64)
        return _finalise(np.uint64(state0 & _MASK64) + idx * _GAMMA)


def stream_key(seed: int, tensor_id: int, layer: int) -> int:
    """State of the SplitMix64 stream that generates one tensor.

    key = finalise(finalise(seed + GAMMA) + ((tensor_id << 32) | layer) + GAMMA)
    i.e. the first SplitMix64 output for `seed`, offset by the tensor's tag,
    pushed through one more SplitMix64 step.
    """
    a = int(splitmix64_stream(seed, 0, 1)[0])
    tag = ((tensor_id & 0xFFFFFFFF) << 32) | (layer & 0xFFFFFFFF)
    return int(splitmix64_stream((a + tag) & _MASK64, 0, 1)[0])


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16, nearest-even, returning the 16-bit patterns.

    bfloat16 is the upper half of an IEEE binary32; rounding adds 0x7FFF plus
    the lowest kept bit and truncates.  NaN is not produced by the generator
    and is not handled here.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def normal_bf16_bits(seed: int, tensor_id: int, layer: int, start: int, n: int,
                     std: float) -> np.ndarray:
    """Elements start..start+n-1 (row-major flat index) of one weight tensor.

    z_i   = SplitMix64 output i of the tensor's stream
    u1    = (high 32 bits of z_i + 0.5) / 2^32,  u2 = (low 32 bits + 0.5) / 2^32
    x_i   = sqrt(-2 ln u1) * cos(2 pi u2)              (Box-Muller, float64)
    w_i   = bf16_rne(float32(std * x_i))
    """
    z = splitmix64_stream(stream_key(seed, tensor_id, layer), start, n)
    two32 = 1.0 / 4294967296.0
    u1 = ((z >> np.uint64(32)).astype(np.float64) + 0.5) * two32
    u2 = ((z & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * two32
    x = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)
    return f32_to_bf16_bits((std * x).astype(np.float32))


class Weights:
    """Model weights as bf16 bit patterns, generated on demand and cached.

    `overrides[(tensor_id, layer)]` replaces a generated tensor (tests plant
    weights this way).  Gains (g1, g2, gf) default to 1.0.
    """

    def __init__(self, cfg: Config, seed: int, std: float = 0.02,
                 keep: bool = True, threads: Optional[int] = None):
        self.cfg, self.seed, self.std, self.keep = cfg, seed, std, keep
        self.threads = threads or min(16, os.cpu_count() or 1)
        self._bits: Dict[Tuple[int, int], np.ndarray] = {}
        self.overrides: Dict[Tuple[int, int], np.ndarray] = {}

    def set_bits(self, tensor_id: int, layer: int, bits: np.ndarray) -> None:
        shape = self.cfg.shape(tensor_id)
        self.overrides[(tensor_id, layer)] = np.asarray(bits, np.uint16).reshape(shape)

    def set_values(self, tensor_id: int, layer: int, values: np.ndarray) -> None:
        self.set_bits(tensor_id, layer,
                      f32_to_bf16_bits(np.asarray(values, np.float32)))

    def bits(self, tensor_id: int, layer: int = 0) -> np.ndarray:
        key = (tensor_id, layer)
        if key in self.overrides:
            return self.overrides[key]
        if key in self._bits:
            return self._bits[key]
        shape = self.cfg.shape(tensor_id)
        n = int(np.prod(shape))
        if tensor_id in (T_G1, T_G2, T_GF):
            out = np.full(shape, 0x3F80, np.uint16)          # 1.0
        else:
            out = np.empty(n, np.uint16)
            step = 1 << 21

            def fill(s):
                m = min(step, n - s)
                out[s:s + m] = normal_bf16_bits(self.seed, tensor_id, layer, s, m,
                                                self.std)

            # chunks are independent (counter-based generator); numpy releases
            # the GIL inside its loops, so threads only shorten the wait
            with concurrent.futures.ThreadPoolExecutor(self.threads) as ex:
                list(ex.map(fill, range(0, n, step)))
            out = out.reshape(shape)
        if self.keep:
            self._bits[key] = out
        return out

    def f64(self, tensor_id: int, layer: int = 0) -> np.ndarray:
        return bf16_bits_to_f64(self.bits(tensor_id, layer))

    def embed_rows(self, tokens: np.ndarray) -> np.ndarray:
        """Rows E[tok] of the embedding table (only those rows are generated when
        the table itself is neither planted nor cached)."""
        tokens = np.asarray(tokens, np.int64)
        key = (T_EMBED, 0)
        if key in self.overrides or key in self._bits:
            return bf16_bits_to_f64(self.bits(T_EMBED, 0)[tokens])
        d = self.cfg.d_model
        rows = [normal_bf16_bits(self.seed, T_EMBED, 0, int(t) * d, d, self.std) for t in tokens]
        return bf16_bits_to_f64(np.stack(rows))


# --------------------------------------------------------------------------- operators

def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing, on x[rows, H, dh] at pos[rows].

    Pair j couples channels j and j + dh/2 and turns by pos * base^(-2j/dh):
      y[j]        = x[j] cos - x[j+dh/2] sin
      y[j + dh/2] = x[j+dh/2] cos + x[j] sin
    """
    dh = x.shape[-1]
    half = dh // 2
    inv = base ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.asarray(pos, np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Bidirectional softmax attention: q[R,H,dh], k/v[J,H,dh] -> [R,H,dh].

    Every query row sees every one of the J keys (no mask): Sec. 2.1 of the
    paper (bidirectional attention).
    """
    dh = q.shape[-1]
    s = np.einsum("rhd,jhd->hrj", q, k) / math.sqrt(dh)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("hrj,jhd->rhd", p, v)


def confidence_argmax(z: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Greedy token and its softmax probability for logits z[rows, V].

    conf = max_j softmax(z)_j = 1 / sum_j exp(z_j - max z); ties -> lowest id.
    """
    zmax = z.max(axis=-1, keepdims=True)
    conf = 1.0 / np.exp(z - zmax).sum(axis=-1)
    return conf, np.argmax(z, axis=-1).astype(np.int32)


def threshold_unmask(tokens: np.ndarray, conf: np.ndarray, tau: float,
                     mask_id: int) -> np.ndarray:
    """Acceptance rule for one draft (Sec. 3, Observation 3, plus forced progress).

    A position is unmasked iff it currently holds MASK and either its
    confidence exceeds tau (strictly) or it is the most confident masked
    position (lowest index on ties).  A draft with no MASK yields all zeros.
    """
    masked = np.asarray(tokens) == mask_id
    out = np.zeros(masked.shape, np.uint8)
    if not masked.any():
        return out
    c = np.where(masked, conf, -np.inf)
    top = int(np.argmax(c))
    out[masked & (conf > tau)] = 1
    out[top] = 1
    return out


def predict_length(tokens: np.ndarray, conf: np.ndarray, argmax: np.ndarray, resp_off: int,
                   mask_id: int, eos_id: int, truncate_thr: float) -> int:
    """Adaptive length prediction after a cache refresh (Sec. 4.1).

    The refresh yields a decoding attempt (conf[i], argmax[i]) for every response
    position resp_off + i.  The response as the model currently drafts it holds the
    decoded token where one is decoded and the attempted token where the position is
    still MASK.  That draft is scanned from the front for [EOS]: an attempted [EOS]
    counts only if its confidence exceeds the truncate threshold (strictly), a
    decoded [EOS] counts as it stands.  The sequence is cut right after the earliest
    such position and its new length is returned; without one the length is unchanged.
    """
    tokens = np.asarray(tokens)
    L = tokens.shape[0]
    for pos in range(resp_off, L):
        i = pos - resp_off
        if tokens[pos] == mask_id:
            if int(argmax[i]) == eos_id and float(conf[i]) > truncate_thr:
                return pos + 1
        elif tokens[pos] == eos_id:
            return pos + 1
    return L


def speculative_candidates(block: np.ndarray, conf: np.ndarray, argmax: np.ndarray, mask_id: int,
                           k: int = 2) -> Tuple[np.ndarray, np.ndarray]:
    """The k most confident positions of a block that are still MASK (Sec. 4.2: the top-k tokens among
    those that fell below the acceptance threshold) and the tokens attempted there; lower index first on
    equal confidence; position -1 (token 0) where fewer than k remain."""
    pos = np.full(k, -1, np.int32)
    tok = np.zeros(k, np.int32)
    masked = [i for i in range(len(block)) if block[i] == mask_id]
    masked.sort(key=lambda i: (-float(conf[i]), i))
    for j, i in enumerate(masked[:k]):
        pos[j], tok[j] = i, int(argmax[i])
    return pos, tok


def accept_jump_drafts(block: np.ndarray, cand_pos: np.ndarray, cand_tok: np.ndarray) -> np.ndarray:
    """block_0 and the three speculative blocks of the accept-jump stage (Sec. 4.2.1): the block as it is,
    with candidate B unmasked, with candidate D unmasked, with both.  A missing candidate (-1) adds nothing."""
    drafts = np.stack([np.asarray(block, np.int32)] * 4)
    for s, which in ((1, (0,)), (2, (1,)), (3, (0, 1))):
        for c in which:
            if cand_pos[c] >= 0:
                drafts[s, cand_pos[c]] = cand_tok[c]
    return drafts


def accept_jump(drafts: np.ndarray, conf: np.ndarray, argmax: np.ndarray, unmask: np.ndarray,
                cand_pos: np.ndarray, cand_tok: np.ndarray, mask_id: int):
    """One controller step of the accept-jump strategy (Sec. 4.2.1) on the outputs of a 4-draft block step.

    drafts/conf/argmax/unmask are [4, b]: block_0 (the block as it stood), block_1 (candidate B unmasked
    beforehand), block_2 (D), block_3 (B and D).  A candidate counts as verified in a draft when that
    draft's step unmasks its position with the very token that was speculated.
      * B and D both verified in block_0          -> jump to block_3;
      * only B verified in block_0                -> go to block_1; if D is verified there jump to block_3,
                                                     otherwise adopt block_1;  (symmetrically for only D, block_2)
      * neither                                   -> block_0.
    Adopting a draft means taking its tokens plus every position its own step unmasked (with that step's
    greedy token).  From the adopted draft's outputs the two most confident still-masked positions become
    the next candidates and the next four drafts are built.

    Returns (chosen, new_block[b], new_cand_pos[2], new_cand_tok[2], new_drafts[4, b]).
    """
    def verified(s, c):
        p = int(cand_pos[c])
        return p >= 0 and drafts[s, p] == mask_id and bool(unmask[s, p]) and int(argmax[s, p]) == int(cand_tok[c])

    b0, d0 = verified(0, 0), verified(0, 1)
    if b0 and d0:
        chosen = 3
    elif b0:
        chosen = 3 if verified(1, 1) else 1
    elif d0:
        chosen = 3 if verified(2, 0) else 2
    else:
        chosen = 0
    new_block = np.where(np.asarray(unmask[chosen], bool), argmax[chosen], drafts[chosen]).astype(np.int32)
    pos, tok = speculative_candidates(new_block, conf[chosen], argmax[chosen], mask_id)
    return chosen, new_block, pos, tok, accept_jump_drafts(new_block, pos, tok)


# Candidate sets of the eight blocks of the decoded-share stage (Sec. 4.2.2), by rank of the candidate among the
# most confident positions below the threshold: block_0, B, D, B+D (Sec. 4.2.1), then the four extra ones - the
# third, the top three, the fourth, the top four.
SPEC_SETS = ((), (0,), (1,), (0, 1), (2,), (0, 1, 2), (3,), (0, 1, 2, 3))


def speculative_drafts(block: np.ndarray, cand_pos: np.ndarray, cand_tok: np.ndarray, n: int) -> np.ndarray:
    """block_0 and the n - 1 speculative blocks (n = 4: Sec. 4.2.1; n = 8: Sec. 4.2.2): the block with the
    candidates of SPEC_SETS[s] unmasked beforehand.  A missing candidate (-1) adds nothing."""
    drafts = np.stack([np.asarray(block, np.int32)] * n)
    for s in range(n):
        for c in SPEC_SETS[s]:
            if c < len(cand_pos) and cand_pos[c] >= 0:
                drafts[s, cand_pos[c]] = cand_tok[c]
    return drafts


def speculative_jump(drafts: np.ndarray, conf: np.ndarray, argmax: np.ndarray, unmask: np.ndarray,
                     cand_pos: np.ndarray, cand_tok: np.ndarray, mask_id: int, n_next: int):
    """The jump rule of Sec. 4.2.1 carried over to the S = 4 or 8 blocks of SPEC_SETS (the paper states it for B
    and D only; for two candidates this function is that rule).

    Start at block_0.  At the current block, whose candidate set is X, the verified set is X plus every other
    candidate that this block's own step unmasks with the speculated token.  If some block's set lies strictly
    between: X < set <= verified, jump to the one with the most candidates (lowest block number among equals)
    and look again from there; otherwise adopt the current block - its tokens plus every position its own step
    unmasked.  The n_next // 2 most confident still-masked positions of the adopted block are the next
    candidates and the next n_next blocks are built from them.

    Returns (chosen, new_block[b], new_cand_pos[k], new_cand_tok[k], new_drafts[n_next, b]), k = n_next // 2.
    """
    S = drafts.shape[0]
    n_cand = S // 2

    def verified(s, c):
        p = int(cand_pos[c])
        return p >= 0 and drafts[s, p] == mask_id and bool(unmask[s, p]) and int(argmax[s, p]) == int(cand_tok[c])

    cur = 0
    while True:
        X = set(SPEC_SETS[cur])
        V = X | {c for c in range(n_cand) if c not in X and verified(cur, c)}
        best = None
        for s in range(S):
            T = set(SPEC_SETS[s])
            if X < T <= V and (best is None or len(T) > len(SPEC_SETS[best])):
                best = s
        if best is None:
            break
        cur = best
    new_block = np.where(np.asarray(unmask[cur], bool), argmax[cur], drafts[cur]).astype(np.int32)
    pos, tok = speculative_candidates(new_block, conf[cur], argmax[cur], mask_id, k=n_next // 2)
    return cur, new_block, pos, tok, speculative_drafts(new_block, pos, tok, n_next)


# --------------------------------------------------------------------------- the two calls

@dataclasses.dataclass
class Cache:
    """K (after RoPE) and V of every position at every layer: [NL, L, H, dh]."""
    k: np.ndarray
    v: np.ndarray

    @property
    def length(self) -> int:
        return self.k.shape[1]


def _layer(cfg: Config, w: Weights, layer: int, h: np.ndarray, pos: np.ndarray,
           kv_of_rows, rows_group=None):
    """One pre-norm transformer block on rows h[R, d].

    kv_of_rows(k_new, v_new) -> list of (row_slice, K[J,H,dh], V[J,H,dh]):
    which keys/values each group of rows attends to, given the fresh K/V the
    rows themselves produced.  Returns the new h and the fresh (k, v).
    """
    H, dh = cfg.n_heads, cfg.head_dim
    a = rmsnorm(h, w.f64(T_G1, layer), cfg.rms_eps)
    q = (a @ w.f64(T_WQ, layer).T).reshape(-1, H, dh)
    k = (a @ w.f64(T_WK, layer).T).reshape(-1, H, dh)
    v = (a @ w.f64(T_WV, layer).T).reshape(-1, H, dh)
    q = rope(q, pos, cfg.rope_base)
    k = rope(k, pos, cfg.rope_base)
    o = np.empty_like(q)
    for rows, kk, vv in kv_of_rows(k, v):
        o[rows] = attention(q[rows], kk, vv)
    h = h + o.reshape(-1, H * dh) @ w.f64(T_WO, layer).T
    m = rmsnorm(h, w.f64(T_G2, layer), cfg.rms_eps)
    gate = m @ w.f64(T_WG, layer).T
    up = m @ w.f64(T_WU, layer).T
    h = h + (silu(gate) * up) @ w.f64(T_WD, layer).T
    return h, k, v


def _head(cfg: Config, w: Weights, h: np.ndarray) -> np.ndarray:
    return rmsnorm(h, w.f64(T_GF, 0), cfg.rms_eps) @ w.f64(T_LM, 0).T


def prefill(cfg: Config, w: Weights, tokens: np.ndarray, resp_off: int = 0,
            pos0: int = 0, return_logits: bool = False):
    """Cache-refresh forward over one whole sequence (Sec. 2.1; Sec. 4.1).

    tokens[L] -> (Cache over all L positions, conf[L-resp_off],
    argmax[L-resp_off][, logits]).  Positions are pos0 + i (pos0 is a test
    hook: RoPE makes the result independent of it).
    """
    tokens = np.asarray(tokens, np.int64)
    L = tokens.shape[0]
    pos = pos0 + np.arange(L)
    h = w.embed_rows(tokens)
    ks, vs = [], []
    for layer in range(cfg.n_layers):
        h, k, v = _layer(cfg, w, layer, h, pos,
                         lambda kn, vn: [(slice(0, L), kn, vn)])
        ks.append(k)
        vs.append(v)
    z = _head(cfg, w, h[resp_off:])
    conf, amax = confidence_argmax(z)
    out = (Cache(np.stack(ks), np.stack(vs)), conf, amax)
    return out + (z,) if return_logits else out


def block_step(cfg: Config, w: Weights, cache: Cache, drafts: np.ndarray,
               block_off: int, tau: float, pos0: int = 0,
               return_logits: bool = False):
    """One decode step of S drafts of one block against the cache (Sec. 4.2).

    drafts[S, b] token ids for positions block_off .. block_off+b-1 (every
    draft uses the same position ids).  Each draft is forwarded on its own;
    at every layer its rows attend to the cached K/V of all positions outside
    the block plus the draft's own fresh K/V.  The cache entries at the block's
    positions are ignored and the cache is not modified.
    Returns conf[S,b], argmax[S,b], unmask[S,b] (uint8) [, logits[S,b,V]].
    """
    drafts = np.asarray(drafts, np.int64)
    S, b = drafts.shape
    L = cache.length
    assert 0 <= block_off and block_off + b <= L
    pos = pos0 + block_off + np.arange(b)
    conf = np.empty((S, b))
    amax = np.empty((S, b), np.int32)
    unmask = np.empty((S, b), np.uint8)
    logits = []
    for s in range(S):
        h = w.embed_rows(drafts[s])
        for layer in range(cfg.n_layers):
            ck, cv = cache.k[layer], cache.v[layer]

            def kv(kn, vn, ck=ck, cv=cv):
                kk = np.concatenate([ck[:block_off], kn, ck[block_off + b:]])
                vv = np.concatenate([cv[:block_off], vn, cv[block_off + b:]])
                return [(slice(0, b), kk, vv)]

            h, _, _ = _layer(cfg, w, layer, h, pos, kv)
        z = _head(cfg, w, h)
        conf[s], amax[s] = confidence_argmax(z)
        unmask[s] = threshold_unmask(drafts[s], conf[s], tau, cfg.mask_id)
        if return_logits:
            logits.append(z)
    out = (conf, amax, unmask)
    return out + (np.stack(logits),) if return_logits else out


def block_step_shared(cfg: Config, w: Weights, cache: Cache, drafts: np.ndarray,
                      block_off: int, tau: float, pos0: int = 0,
                      return_logits: bool = False):
    """Decode step in the decoded-share stage (Sec. 4.2.2, Fig. 8 caption).

    drafts[S, b]: block_0 = drafts[0] is forwarded in full, exactly as in block_step.  The positions
    that block_0 has already decoded (tokens other than MASK) are identical in every draft; they are
    computed only in block_0, and their fresh K/V of every layer are shared: a speculative block
    s >= 1 consists of the still-masked positions of block_0 only (with their position ids kept),
    and at every layer its rows attend to the cached K/V outside the block, to block_0's fresh K/V
    of the decoded positions, and to their own fresh K/V.  Speculative blocks do not see each other
    nor block_0's rows at masked positions.

    Returns conf[S,b], argmax[S,b], unmask[S,b] as block_step does; for s >= 1 the entries at decoded
    positions are not computed and read conf 0, argmax = the token held there, unmask 0.
    With return_logits: also a list of S arrays, [b, V] for block_0 and [m, V] for the others
    (rows in increasing position order).
    """
    drafts = np.asarray(drafts, np.int64)
    S, b = drafts.shape
    L = cache.length
    assert 0 <= block_off and block_off + b <= L
    masked = drafts[0] == cfg.mask_id
    P, D = np.flatnonzero(masked), np.flatnonzero(~masked)
    assert np.array_equal(drafts[:, D], np.broadcast_to(drafts[0, D], (S, D.size))), "decoded positions differ"
    conf = np.zeros((S, b))
    amax = drafts.astype(np.int32).copy()
    unmask = np.zeros((S, b), np.uint8)
    logits = []

    # block_0: the whole block; its fresh K/V of every layer are kept
    pos = pos0 + block_off + np.arange(b)
    h = w.embed_rows(drafts[0])
    k0, v0 = [], []
    for layer in range(cfg.n_layers):
        ck, cv = cache.k[layer], cache.v[layer]

        def kv(kn, vn, ck=ck, cv=cv):
            return [(slice(0, b), np.concatenate([ck[:block_off], kn, ck[block_off + b:]]),
                     np.concatenate([cv[:block_off], vn, cv[block_off + b:]]))]

        h, k, v = _layer(cfg, w, layer, h, pos, kv)
        k0.append(k)
        v0.append(v)
    z = _head(cfg, w, h)
    conf[0], amax[0] = confidence_argmax(z)
    unmask[0] = threshold_unmask(drafts[0], conf[0], tau, cfg.mask_id)
    logits.append(z)

    # speculative blocks: the masked positions only, decoded K/V borrowed from block_0
    for s in range(1, S):
        if P.size == 0:
            logits.append(np.zeros((0, cfg.vocab)))
            continue
        h = w.embed_rows(drafts[s, P])
        for layer in range(cfg.n_layers):
            ck, cv = cache.k[layer], cache.v[layer]

            def kv(kn, vn, ck=ck, cv=cv, layer=layer):
                return [(slice(0, P.size),
                         np.concatenate([ck[:block_off], k0[layer][D], kn, ck[block_off + b:]]),
                         np.concatenate([cv[:block_off], v0[layer][D], vn, cv[block_off + b:]]))]

            h, _, _ = _layer(cfg, w, layer, h, pos[P], kv)
        z = _head(cfg, w, h)
        c, a = confidence_argmax(z)
        conf[s, P], amax[s, P] = c, a
        unmask[s, P] = threshold_unmask(drafts[s, P], c, tau, cfg.mask_id)
        logits.append(z)
    out = (conf, amax, unmask)
    return out + (logits,) if return_logits else out


# --------------------------------------------------------------------------- the generation loop

@dataclasses.dataclass(frozen=True)
class GenParams:
    """Knobs of the generation loop.  None of their values is printed in the paper."""
    block_len: int                      # positions per block (32 in the paper's runs)
    n_drafts: int = 1                   # 1: threshold decoding only; 4: accept-jump (Sec. 4.2.1); 8: accept-jump,
                                        # then eight blocks with four extra candidates in the decoded-share stage
    tau: float = 0.9                    # acceptance threshold
    eos_id: Optional[int] = None        # None: no length prediction
    truncate_thr: float = 0.9           # Sec. 4.1
    share_from: Optional[int] = None    # decoded positions of the block from which steps run in the
                                        # decoded-share stage (Sec. 4.2.2); None: never (n_drafts = 8 needs it)
    row_budget: Optional[int] = None    # n_drafts = 8: a decoded-share step forwards eight blocks only if its
                                        # b + 7 * masked rows fit the budget, else the four accept-jump blocks
                                        # (Sec. 4.2: the step has to stay in the memory-bound region; Sec. 4.2.2:
                                        # the shrinking blocks make room for the extra candidates); None: always eight


def truncate_cache(cache: Cache, new_len: int) -> Cache:
    """The cache of a sequence cut to new_len positions: the dropped positions' K/V are no longer keys."""
    return Cache(cache.k[:, :new_len], cache.v[:, :new_len])


def generate(cfg: Config, w: Weights, prompt: np.ndarray, resp_len: int, p: GenParams):
    """Block-wise generation of one response (Sec. 2.1, with Sec. 4.1 and Sec. 4.2 switched on by p).

    The response starts as resp_len MASK tokens behind the prompt and is decoded block by block, front
    to back.  Each block cycle opens with a refresh: a forward over the whole sequence that rebuilds
    the cache and attempts every response position.  Then, in this order:
      * length prediction (Sec. 4.1) scans the attempt and may cut the sequence; the cut takes effect
        at once - dropped positions leave the token sequence and stop being keys of this cycle's steps
        (the K/V of the kept positions stay as the refresh computed them);
      * the refresh's attempt at the positions of the current block is put through the acceptance
        rule, so the refresh is also the block's first decoding iteration (unmasking decisions of a
        refresh are restricted to the current block);
      * decode steps against the cache follow until the block holds no MASK.  With n_drafts = 1 a step
        forwards the block alone; with n_drafts = 4 it forwards the four accept-jump drafts and the
        controller adopts one (the first candidates are the two most confident positions the refresh
        left masked).  Once share_from positions of the block are decoded the step runs in the
        decoded-share stage, with the same four drafts; with n_drafts = 8 that stage forwards eight
        blocks (the four most confident positions left masked are the candidates, SPEC_SETS) and the
        jump rule runs over all of them (speculative_jump), the steps before it stay four-draft ones -
        and so do the steps of that stage whose eight blocks would exceed row_budget rows.
    The block's tokens are written back and the next block cycle begins; generation ends when the
    block start reaches the (possibly shortened) end of the sequence.

    Returns (tokens[final_len], stats, events).  stats: n_refresh, n_step, n_step_shared (of n_step),
    refresh_positions (sum of the refreshed lengths), step_rows (rows forwarded by the steps).
    events: one dict per forward, in order - kind ('refresh' | 'step' | 'shared'), L (length after the
    event), block_off, block_len, chosen, cand_pos, cand_tok, tokens (copy of the sequence after it).
    """
    mask_id, b = cfg.mask_id, p.block_len
    assert p.n_drafts in (1, 4, 8) and b >= 1 and resp_len >= 1
    assert p.n_drafts != 8 or p.share_from is not None
    n_cand = p.n_drafts // 2 if p.n_drafts > 1 else 2
    prompt = np.asarray(prompt, np.int32)
    P = prompt.shape[0]
    tokens = np.concatenate([prompt, np.full(resp_len, mask_id, np.int32)])
    L, off = tokens.shape[0], P
    stats = dict(n_refresh=0, n_step=0, n_step_shared=0, refresh_positions=0, step_rows=0)
    events = []

    def record(kind, bb, chosen, cp, ct):
        events.append(dict(kind=kind, L=L, block_off=off, block_len=bb, chosen=int(chosen),
                           cand_pos=np.array(cp, np.int32), cand_tok=np.array(ct, np.int32), tokens=tokens.copy()))

    while off < L:
        cache, conf, am = prefill(cfg, w, tokens, resp_off=P)
        stats["n_refresh"] += 1
        stats["refresh_positions"] += L
        if p.eos_id is not None:
            new_len = predict_length(tokens, conf, am, P, mask_id, p.eos_id, p.truncate_thr)
            if new_len < L:
                L = new_len
                tokens, cache = tokens[:L], truncate_cache(cache, L)
        if off >= L:                                    # the cut fell into what is already decoded
            record("refresh", 0, 0, (-1,) * n_cand, (0,) * n_cand)
            break
        bb = min(b, L - off)
        block = tokens[off:off + bb].copy()
        c_blk, a_blk = conf[off - P:off - P + bb], am[off - P:off - P + bb]
        um = threshold_unmask(block, c_blk, p.tau, mask_id)
        block = np.where(um.astype(bool), a_blk, block).astype(np.int32)
        cp, ct = speculative_candidates(block, c_blk, a_blk, mask_id, k=n_cand)
        tokens[off:off + bb] = block
        record("refresh", bb, 0, cp, ct)
        while (block == mask_id).any():
            if p.n_drafts == 1:
                conf_s, am_s, um_s = block_step(cfg, w, cache, block[None], off, p.tau)
                block = np.where(um_s[0].astype(bool), am_s[0], block).astype(np.int32)
                cp, ct = speculative_candidates(block, conf_s[0], am_s[0], mask_id)
                chosen, kind, rows = 0, "step", bb
            else:
                n_masked = int((block == mask_id).sum())
                if p.share_from is not None and bb - n_masked >= p.share_from:
                    S = p.n_drafts
                    if S == 8 and p.row_budget is not None and bb + 7 * n_masked > p.row_budget:
                        S = 4
                    drafts = speculative_drafts(block, cp, ct, S)
                    conf_s, am_s, um_s = block_step_shared(cfg, w, cache, drafts, off, p.tau)
                    kind, rows = "shared", bb + (S - 1) * n_masked
                    stats["n_step_shared"] += 1
                else:
                    drafts = speculative_drafts(block, cp, ct, 4)
                    conf_s, am_s, um_s = block_step(cfg, w, cache, drafts, off, p.tau)
                    kind, rows = "step", 4 * bb
                if p.n_drafts == 4:
                    chosen, block, cp, ct, _ = accept_jump(drafts, conf_s, am_s, um_s, cp, ct, mask_id)
                else:
                    chosen, block, cp, ct, _ = speculative_jump(drafts, conf_s, am_s, um_s, cp, ct, mask_id, 8)
            stats["n_step"] += 1
            stats["step_rows"] += rows
            if int((block == mask_id).sum()) >= int((tokens[off:off + bb] == mask_id).sum()):
                # forced progress always unmasks a position, but nothing stops an untrained model from
                # attempting the MASK token itself there; the paper's models never do, so this is an error
                raise RuntimeError("a step left the block's MASK count unchanged (the greedy token is MASK)")
            tokens[off:off + bb] = block
            record(kind, bb, chosen, cp, ct)
        off += bb
    stats["final_len"] = L
    return tokens, stats, events
