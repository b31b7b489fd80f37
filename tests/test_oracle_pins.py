"""Pins for the CPU oracle: each checks it against something other than itself.

The paper (ODB-dLLM) prints no intermediate value of the forward pass, so the
pins are closed forms, invariants, brute force, published test vectors of the
random generator, and PyTorch CPU library routines used as a second opinion.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import odb_oracle as o

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

MICRO = o.Config(n_layers=2, d_model=32, n_heads=2, head_dim=16, d_ff=48, vocab=64)
TINY = o.Config(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=768,
                vocab=1024, mask_id=1023)


def micro_weights(seed=7, std=0.25):
    return o.Weights(MICRO, seed, std)


# ------------------------------------------------------------------ generator

def test_splitmix64_published_vectors():
    """SplitMix64 outputs for seeds 0 and 1234567 (vectors in tests/golden)."""
    for line in open(os.path.join(GOLDEN, "splitmix64_vectors.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        seed, *vals = line.split()
        got = o.splitmix64_stream(int(seed, 0), 0, len(vals))
        assert [int(x) for x in got] == [int(v, 0) for v in vals]


def test_splitmix64_is_counter_based():
    a = o.splitmix64_stream(99, 0, 1000)
    b = o.splitmix64_stream(99, 500, 100)
    assert np.array_equal(a[500:600], b)


def test_bf16_round_to_nearest_even_bit_patterns():
    cases = [
        (0x3F800000, 0x3F80),  # 1.0 exact
        (0x3F808000, 0x3F80),  # tie, kept bit even -> down
        (0x3F818000, 0x3F82),  # tie, kept bit odd -> up
        (0x3F808001, 0x3F81),  # just above tie -> up
        (0x3F807FFF, 0x3F80),  # just below tie -> down
        (0xBF818000, 0xBF82),  # sign carried
        (0x00000000, 0x0000),
        (0x80000000, 0x8000),
        (0x00008000, 0x0000),  # subnormal tie -> even (zero)
        (0x00018000, 0x0002),  # subnormal tie -> up to even
        (0x3FFFFFFF, 0x4000),  # mantissa carry into exponent
    ]
    x = np.array([c[0] for c in cases], np.uint32).view(np.float32)
    assert list(o.f32_to_bf16_bits(x)) == [c[1] for c in cases]
    # widening is exact and inverse on representable values
    bits = np.arange(0, 0x7F80, 37, dtype=np.uint16)
    back = o.f32_to_bf16_bits(o.bf16_bits_to_f64(bits).astype(np.float32))
    assert np.array_equal(back, bits)


def test_bf16_rounding_agrees_with_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(o.f32_to_bf16_bits(x), ref)


def test_generator_moments_and_independence():
    n = 4_000_000
    w = o.bf16_bits_to_f64(o.normal_bf16_bits(5, o.T_WQ, 3, 0, n, 1.0))
    assert abs(w.mean()) < 4 / math.sqrt(n)
    assert abs(w.var() - 1.0) < 5e-3           # bf16 rounding adds ~1e-6 relative
    assert abs((w ** 4).mean() - 3.0) < 3e-2
    assert abs((w ** 3).mean()) < 2e-2
    # Box-Muller tail: P(|x|>3) = 2.6998e-3
    assert abs((np.abs(w) > 3).mean() - 2.6998e-3) < 2e-4
    # different tensors / layers / seeds decorrelate
    a = o.bf16_bits_to_f64(o.normal_bf16_bits(5, o.T_WQ, 4, 0, 100000, 1.0))
    b = o.bf16_bits_to_f64(o.normal_bf16_bits(5, o.T_WK, 3, 0, 100000, 1.0))
    c = o.bf16_bits_to_f64(o.normal_bf16_bits(6, o.T_WQ, 3, 0, 100000, 1.0))
    for other in (a, b, c):
        assert abs(np.corrcoef(w[:100000], other)[0, 1]) < 0.02
    # lag-1 autocorrelation
    assert abs(np.corrcoef(w[:-1][:1000000], w[1:][:1000000])[0, 1]) < 5e-3
    # scaling by std happens before rounding
    s = o.bf16_bits_to_f64(o.normal_bf16_bits(5, o.T_WQ, 3, 0, 1000, 0.02))
    assert np.allclose(s, 0.02 * w[:1000], rtol=2 ** -7)


def test_generator_slices_agree():
    full = o.normal_bf16_bits(1, o.T_WD, 2, 0, 5000, 0.02)
    part = o.normal_bf16_bits(1, o.T_WD, 2, 1234, 100, 0.02)
    assert np.array_equal(full[1234:1334], part)
    w = o.Weights(MICRO, 1)
    assert np.array_equal(w.bits(o.T_WD, 1).ravel(),
                          o.normal_bf16_bits(1, o.T_WD, 1, 0, 32 * 48, 0.02))
    assert np.all(w.f64(o.T_G1, 0) == 1.0)


# ------------------------------------------------------------------ operators

def test_attention_against_brute_force_loops():
    rng = np.random.default_rng(1)
    R, J, H, dh = 5, 9, 2, 4
    q = rng.standard_normal((R, H, dh)) * 3
    k = rng.standard_normal((J, H, dh)) * 3
    v = rng.standard_normal((J, H, dh))
    got = o.attention(q, k, v)
    for r in range(R):
        for h in range(H):
            sc = [sum(q[r, h, d] * k[j, h, d] for d in range(dh)) / math.sqrt(dh)
                  for j in range(J)]
            mx = max(sc)
            e = [math.exp(s - mx) for s in sc]
            z = sum(e)
            for d in range(dh):
                ref = sum(e[j] / z * v[j, h, d] for j in range(J))
                assert abs(got[r, h, d] - ref) < 1e-12
    # sharp softmax really is far from uniform here
    assert np.abs(got - v.mean(0)).max() > 0.1


def test_attention_against_torch_sdpa():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((7, 3, 8))
    k = rng.standard_normal((11, 3, 8))
    v = rng.standard_normal((11, 3, 8))
    t = lambda a: torch.from_numpy(a).permute(1, 0, 2)[None]
    ref = F.scaled_dot_product_attention(t(q), t(k), t(v))[0].permute(1, 0, 2).numpy()
    assert np.abs(o.attention(q, k, v) - ref).max() < 1e-12


def test_rope_closed_form_and_invariants():
    # dh = 2: a single pair turning by pos * base^0 = pos radians
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    y = o.rope(x, np.array([1, 2]), 10000.0)
    assert np.allclose(y[0, 0], [math.cos(1), math.sin(1)], atol=1e-15)
    assert np.allclose(y[1, 0], [-math.sin(2), math.cos(2)], atol=1e-15)
    # dh = 4: second pair turns by pos * base^(-1/2); pairing is (j, j + dh/2)
    x = np.zeros((1, 1, 4)); x[0, 0, 1] = 1.0
    y = o.rope(x, np.array([3]), 100.0)
    assert np.allclose(y[0, 0], [0, math.cos(0.3), 0, math.sin(0.3)], atol=1e-15)
    rng = np.random.default_rng(3)
    q = rng.standard_normal((6, 2, 16)); k = rng.standard_normal((6, 2, 16))
    pos = np.array([0, 1, 5, 17, 100, 1000])
    rq, rk = o.rope(q, pos, 1e4), o.rope(k, pos, 1e4)
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1))
    rq2, rk2 = o.rope(q, pos + 77, 1e4), o.rope(k, pos + 77, 1e4)
    assert np.allclose(np.einsum("ahd,bhd->hab", rq, rk),
                       np.einsum("ahd,bhd->hab", rq2, rk2), atol=1e-11)
    assert np.allclose(o.rope(q, np.zeros(6), 1e4), q)


def test_rmsnorm_and_silu_against_torch():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 32)) * 3
    g = rng.standard_normal(32)
    ref = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), 1e-5).numpy()
    assert np.abs(o.rmsnorm(x, g, 1e-5) - ref).max() < 1e-13
    y = o.rmsnorm(x, np.ones(32), 0.0)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0)
    assert np.allclose(o.rmsnorm(7.5 * x, g, 0.0), o.rmsnorm(x, g, 0.0))
    assert np.abs(o.silu(x) - F.silu(torch.from_numpy(x)).numpy()).max() < 1e-14


def test_confidence_argmax_definition():
    z = np.array([[0.0, math.log(3.0), 0.0, 0.0], [2.0, 2.0, 1.0, 2.0]])
    conf, am = o.confidence_argmax(z)
    assert np.allclose(conf, [3 / 6, math.e ** 2 / (3 * math.e ** 2 + math.e)])
    assert list(am) == [1, 0]                       # ties -> lowest id
    ref = F.softmax(torch.from_numpy(z), -1).max(-1).values.numpy()
    assert np.allclose(conf, ref)


def test_threshold_unmask_rules():
    M = 9
    tok = np.array([M, 1, M, M, 2, M])
    conf = np.array([0.5, 0.99, 0.95, 0.2, 0.99, 0.95])
    assert list(o.threshold_unmask(tok, conf, 0.9, M)) == [0, 0, 1, 0, 0, 1]
    # tau >= 1: only the forced top-1 masked position, lowest index on ties
    assert list(o.threshold_unmask(tok, conf, 1.0, M)) == [0, 0, 1, 0, 0, 0]
    # tau < 0: every masked position
    assert list(o.threshold_unmask(tok, conf, -1.0, M)) == [1, 0, 1, 1, 0, 1]
    # strict comparison
    assert list(o.threshold_unmask(np.array([M, M]), np.array([0.9, 0.95]), 0.9, M)) == [0, 1]
    # no masked position -> nothing
    assert list(o.threshold_unmask(np.array([1, 2]), np.array([0.99, 0.99]), 0.1, M)) == [0, 0]
    # top-1 is taken among masked positions only
    assert list(o.threshold_unmask(np.array([1, M]), np.array([0.8, 0.1]), 0.9, M)) == [0, 1]


# ------------------------------------------------------------------ whole forward, second opinion

def _torch_rope_complex(x, pos, base):
    """RoPE as a complex multiplication: (x_j + i x_{j+dh/2}) * exp(i pos w_j)."""
    half = x.shape[-1] // 2
    w = torch.tensor([base ** (-2.0 * j / x.shape[-1]) for j in range(half)],
                     dtype=torch.float64)
    zc = torch.complex(x[..., :half], x[..., half:])
    rot = torch.polar(torch.ones(len(pos), half, dtype=torch.float64),
                      pos.to(torch.float64)[:, None] * w[None])
    zc = zc * rot[:, None, :]
    return torch.cat([zc.real, zc.imag], -1)


def _torch_forward(cfg, w, tokens, pos, ctx_kv=None, block=None):
    """Plain PyTorch-CPU float64 forward built from torch.nn.functional calls.

    ctx_kv: per-layer (K, V) tensors [L,H,dh] of a cache, block=(off, b): rows
    replace cache entries off..off+b-1 by their own K/V.  Returns logits and
    the per-layer (k, v) of the rows.
    """
    T = lambda tid, layer=0: torch.from_numpy(w.f64(tid, layer))
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    h = F.embedding(torch.as_tensor(tokens, dtype=torch.long), T(o.T_EMBED))
    pos = torch.as_tensor(pos)
    kvs = []
    for l in range(cfg.n_layers):
        a = F.rms_norm(h, (d,), T(o.T_G1, l), cfg.rms_eps)
        q = _torch_rope_complex(F.linear(a, T(o.T_WQ, l)).view(-1, H, dh), pos, cfg.rope_base)
        k = _torch_rope_complex(F.linear(a, T(o.T_WK, l)).view(-1, H, dh), pos, cfg.rope_base)
        v = F.linear(a, T(o.T_WV, l)).view(-1, H, dh)
        kvs.append((k, v))
        if ctx_kv is not None:
            off, b = block
            K = torch.cat([ctx_kv[l][0][:off], k, ctx_kv[l][0][off + b:]])
            V = torch.cat([ctx_kv[l][1][:off], v, ctx_kv[l][1][off + b:]])
        else:
            K, V = k, v
        att = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], K.permute(1, 0, 2)[None],
                                             V.permute(1, 0, 2)[None])[0].permute(1, 0, 2)
        h = h + F.linear(att.reshape(-1, d), T(o.T_WO, l))
        m = F.rms_norm(h, (d,), T(o.T_G2, l), cfg.rms_eps)
        h = h + F.linear(F.silu(F.linear(m, T(o.T_WG, l))) * F.linear(m, T(o.T_WU, l)), T(o.T_WD, l))
    z = F.linear(F.rms_norm(h, (d,), T(o.T_GF), cfg.rms_eps), T(o.T_LM))
    return z.numpy(), kvs


def _random_gains(w, cfg, rng):
    for l in range(cfg.n_layers):
        w.set_values(o.T_G1, l, rng.uniform(0.5, 2.0, cfg.d_model))
        w.set_values(o.T_G2, l, rng.uniform(0.5, 2.0, cfg.d_model))
    w.set_values(o.T_GF, 0, rng.uniform(2.0, 6.0, cfg.d_model))


@pytest.mark.parametrize("cfg,std", [(MICRO, 0.25), (TINY, 0.05)])
def test_prefill_and_step_against_torch_functional(cfg, std):
    rng = np.random.default_rng(11)
    w = o.Weights(cfg, 3, std)
    _random_gains(w, cfg, rng)
    L, off, b, S = 40, 16, 8, 3
    tokens = rng.integers(0, cfg.vocab, L)
    cache, conf, am, z = o.prefill(cfg, w, tokens, resp_off=4, return_logits=True)
    zt, kvs = _torch_forward(cfg, w, tokens, np.arange(L))
    assert np.abs(z - zt[4:]).max() < 1e-9 * max(1.0, np.abs(zt).max())
    for l in range(cfg.n_layers):
        assert np.abs(cache.k[l] - kvs[l][0].numpy()).max() < 1e-10
        assert np.abs(cache.v[l] - kvs[l][1].numpy()).max() < 1e-10
    assert np.array_equal(am, zt[4:].argmax(-1))
    drafts = rng.integers(0, cfg.vocab, (S, b))
    drafts[:, ::2] = cfg.mask_id
    c2, a2, u2, z2 = o.block_step(cfg, w, cache, drafts, off, 0.3, return_logits=True)
    for s in range(S):
        zs, _ = _torch_forward(cfg, w, drafts[s], off + np.arange(b), ctx_kv=kvs, block=(off, b))
        assert np.abs(z2[s] - zs).max() < 1e-9 * max(1.0, np.abs(zs).max())
        p = F.softmax(torch.from_numpy(zs), -1).max(-1).values.numpy()
        assert np.allclose(c2[s], p, rtol=1e-10)
    assert c2.shape == (S, b) and a2.dtype == np.int32 and u2.dtype == np.uint8


def test_one_layer_against_naive_python_matmul():
    cfg = o.Config(n_layers=1, d_model=8, n_heads=2, head_dim=4, d_ff=12, vocab=16)
    w = o.Weights(cfg, 21, 0.5)
    tokens = [3, 9, 1]
    _, _, _, z = o.prefill(cfg, w, tokens, return_logits=True)

    def mm(x, W):  # x[R][K] * W[N][K]^T
        return [[sum(xr[k] * W[n][k] for k in range(len(xr))) for n in range(len(W))] for xr in x]

    def rms(x, eps):
        return [[v / math.sqrt(sum(u * u for u in r) / len(r) + eps) for v in r] for r in x]

    E = w.f64(o.T_EMBED).tolist()
    h = [E[t] for t in tokens]
    a = rms(h, cfg.rms_eps)
    q, k, v = (mm(a, w.f64(t).tolist()) for t in (o.T_WQ, o.T_WK, o.T_WV))

    def rot(x, p):
        out = [0.0] * 8
        for hd in range(2):
            for j in range(2):
                th = p * cfg.rope_base ** (-2.0 * j / 4)
                x1, x2 = x[hd * 4 + j], x[hd * 4 + j + 2]
                out[hd * 4 + j] = x1 * math.cos(th) - x2 * math.sin(th)
                out[hd * 4 + j + 2] = x2 * math.cos(th) + x1 * math.sin(th)
        return out

    q = [rot(q[i], i) for i in range(3)]
    k = [rot(k[i], i) for i in range(3)]
    att = [[0.0] * 8 for _ in range(3)]
    for i in range(3):
        for hd in range(2):
            sc = [sum(q[i][hd * 4 + d] * k[j][hd * 4 + d] for d in range(4)) / 2.0 for j in range(3)]
            e = [math.exp(s - max(sc)) for s in sc]
            for d in range(4):
                att[i][hd * 4 + d] = sum(e[j] / sum(e) * v[j][hd * 4 + d] for j in range(3))
    o_ = mm(att, w.f64(o.T_WO).tolist())
    h = [[h[i][c] + o_[i][c] for c in range(8)] for i in range(3)]
    m = rms(h, cfg.rms_eps)
    g, u = mm(m, w.f64(o.T_WG).tolist()), mm(m, w.f64(o.T_WU).tolist())
    act = [[g[i][c] / (1 + math.exp(-g[i][c])) * u[i][c] for c in range(12)] for i in range(3)]
    dn = mm(act, w.f64(o.T_WD).tolist())
    h = [[h[i][c] + dn[i][c] for c in range(8)] for i in range(3)]
    zz = mm(rms(h, cfg.rms_eps), w.f64(o.T_LM).tolist())
    assert np.abs(np.array(zz) - z).max() < 1e-12


# ------------------------------------------------------------------ structural properties from the paper

def _setup(seed=5, L=48, off=16, b=8, S=4, cfg=MICRO):
    rng = np.random.default_rng(seed)
    w = o.Weights(cfg, seed, 0.25)
    w.set_values(o.T_GF, 0, np.full(cfg.d_model, 4.0))
    tokens = rng.integers(0, cfg.vocab - 1, L)
    tokens[off + 2: off + b] = cfg.mask_id
    return rng, w, tokens


def test_cached_step_equals_full_recompute_on_unchanged_block():
    """Sec. 2.1: K/V outside the block are what the refresh computed, so a step
    on the block as it stood at the refresh reproduces the refresh's outputs."""
    _, w, tokens = _setup()
    cache, conf, am, z = o.prefill(MICRO, w, tokens, return_logits=True)
    c, a, u, zs = o.block_step(MICRO, w, cache, tokens[None, 16:24], 16, 0.5, return_logits=True)
    assert np.abs(zs[0] - z[16:24]).max() < 1e-11
    assert np.allclose(c[0], conf[16:24], rtol=1e-11) and np.array_equal(a[0], am[16:24])
    # ... and after a token of the block changed it differs (stale outside K/V aside)
    d = tokens[None, 16:24].copy(); d[0, 3] = 5
    assert np.abs(o.block_step(MICRO, w, cache, d, 16, 0.5, return_logits=True)[3][0] - z[16:24]).max() > 1e-3


def test_step_ignores_cache_entries_of_the_block_and_leaves_cache_alone():
    rng, w, tokens = _setup()
    cache, *_ = o.prefill(MICRO, w, tokens)
    drafts = rng.integers(0, MICRO.vocab, (2, 8))
    ref = o.block_step(MICRO, w, cache, drafts, 16, 0.5, return_logits=True)
    k0, v0 = cache.k.copy(), cache.v.copy()
    bad = o.Cache(cache.k.copy(), cache.v.copy())
    bad.k[:, 16:24] = 1e3; bad.v[:, 16:24] = -1e3
    got = o.block_step(MICRO, w, bad, drafts, 16, 0.5, return_logits=True)
    assert np.array_equal(ref[3], got[3])
    assert np.array_equal(cache.k, k0) and np.array_equal(cache.v, v0)
    # entries outside the block do matter
    bad.k[:, 30] += 1.0
    assert np.abs(o.block_step(MICRO, w, bad, drafts, 16, 0.5, return_logits=True)[3] - ref[3]).max() > 1e-6


def test_drafts_are_mutually_invisible():
    """Sec. 4.2: drafts see the cached context and themselves only."""
    rng, w, tokens = _setup()
    cache, *_ = o.prefill(MICRO, w, tokens)
    drafts = rng.integers(0, MICRO.vocab, (4, 8)); drafts[:, 5] = MICRO.mask_id
    c, a, u, z = o.block_step(MICRO, w, cache, drafts, 16, 0.2, return_logits=True)
    perm = [2, 0, 3, 1]
    cp, ap, up, zp = o.block_step(MICRO, w, cache, drafts[perm], 16, 0.2, return_logits=True)
    assert np.array_equal(zp, z[perm]) and np.array_equal(cp, c[perm])
    assert np.array_equal(ap, a[perm]) and np.array_equal(up, u[perm])
    for s in range(4):
        c1, a1, u1, z1 = o.block_step(MICRO, w, cache, drafts[s:s + 1], 16, 0.2, return_logits=True)
        assert np.array_equal(z1[0], z[s])
    dup = np.stack([drafts[1]] * 3)
    zd = o.block_step(MICRO, w, cache, dup, 16, 0.2, return_logits=True)[3]
    assert np.array_equal(zd[0], zd[1]) and np.array_equal(zd[0], z[1])


def test_attention_is_bidirectional():
    _, w, tokens = _setup()
    z = o.prefill(MICRO, w, tokens, return_logits=True)[3]
    t2 = tokens.copy(); t2[-1] = (t2[-1] + 1) % 60
    z2 = o.prefill(MICRO, w, t2, return_logits=True)[3]
    assert np.abs(z2[0] - z[0]).max() > 1e-6      # row 0 depends on the last token


def test_prefill_invariant_to_position_offset():
    _, w, tokens = _setup()
    z = o.prefill(MICRO, w, tokens, return_logits=True)[3]
    z2 = o.prefill(MICRO, w, tokens, pos0=123, return_logits=True)[3]
    assert np.abs(z - z2).max() < 1e-9
    cache = o.prefill(MICRO, w, tokens, pos0=123)[0]
    d = tokens[None, 16:24]
    a = o.block_step(MICRO, w, cache, d, 16, 0.5, pos0=123, return_logits=True)[3]
    assert np.abs(a[0] - z[16:24]).max() < 1e-9


def test_zero_lm_head_gives_uniform_confidence():
    _, w, tokens = _setup()
    w.set_values(o.T_LM, 0, np.zeros((MICRO.vocab, MICRO.d_model)))
    _, conf, am = o.prefill(MICRO, w, tokens)
    assert np.all(conf == 1.0 / MICRO.vocab) and np.all(am == 0)


def test_zero_output_projections_closed_form():
    """With Wo = Wd = 0 the residual stream is the embedding: logits are
    rmsnorm(E[tok]) . W_lm^T, and a planted LM row gives a closed-form confidence."""
    _, w, tokens = _setup()
    for l in range(MICRO.n_layers):
        w.set_values(o.T_WO, l, np.zeros((32, 32)))
        w.set_values(o.T_WD, l, np.zeros((32, 48)))
    lm = np.zeros((MICRO.vocab, 32)); lm[7, 0] = 2.0
    w.set_values(o.T_LM, 0, lm)
    w.set_values(o.T_GF, 0, np.ones(32))
    emb = np.zeros((MICRO.vocab, 32)); emb[:, 0] = 3.0; emb[:, 1] = 4.0   # rms = sqrt(25/32)
    w.set_values(o.T_EMBED, 0, emb)
    _, conf, am, z = o.prefill(MICRO, w, tokens, return_logits=True)
    x0 = 3.0 / math.sqrt(25.0 / 32 + MICRO.rms_eps)
    assert np.allclose(z[:, 7], 2.0 * x0, rtol=1e-12) and np.all(am == 7)
    assert np.allclose(conf, 1.0 / (1.0 + (MICRO.vocab - 1) * math.exp(-2.0 * x0)), rtol=1e-12)
    cache = o.prefill(MICRO, w, tokens)[0]
    c, a, u = o.block_step(MICRO, w, cache, tokens[None, 16:24], 16, 0.5)
    assert np.allclose(c, conf[16:24]) and np.all(a == 7)
    assert np.array_equal(u[0], (tokens[16:24] == MICRO.mask_id).astype(np.uint8))


def test_step_unmask_uses_draft_tokens_and_tau():
    rng, w, tokens = _setup()
    cache, *_ = o.prefill(MICRO, w, tokens)
    drafts = np.stack([tokens[16:24], tokens[16:24]]); drafts[1, :] = 3
    c, a, u = o.block_step(MICRO, w, cache, drafts, 16, 1.0)
    assert u[0].sum() == 1 and u[1].sum() == 0
    masked = drafts[0] == MICRO.mask_id
    assert u[0][np.argmax(np.where(masked, c[0], -1))] == 1
    c, a, u = o.block_step(MICRO, w, cache, drafts, 16, -1.0)
    assert np.array_equal(u[0], masked.astype(np.uint8))


# ------------------------------------------------------------------ adaptive length prediction (Sec. 4.1)

def _alp_case(L=20, resp_off=8, mask_id=99, eos=7):
    tokens = np.arange(L, dtype=np.int32) % 5 + 10           # no MASK, no EOS anywhere
    tokens[resp_off:] = mask_id
    conf = np.full(L - resp_off, 0.5)
    am = np.full(L - resp_off, 3, np.int32)
    return tokens, conf, am


def test_length_prediction_cases_constructed_by_hand():
    """Each case is built so that the answer is known by construction (Sec. 4.1: no [EOS] or none above the
    threshold keeps the length; a confident [EOS] cuts right after itself; the earliest one wins)."""
    mask_id, eos, ro = 99, 7, 8
    t, c, a = _alp_case()
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == 20             # no [EOS] attempted
    a[5] = eos
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == 20             # attempted, confidence 0.5 <= 0.9
    c[5] = 0.9
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == 20             # "exceeds" is strict
    c[5] = np.nextafter(0.9, 1.0)
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 5 + 1     # cut right after position 13
    a[9], c[9] = eos, 0.99
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 5 + 1     # a later one does not matter
    a[2], c[2] = eos, 0.3
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 5 + 1     # an earlier unconfident one neither
    c[2] = 0.95
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 2 + 1     # ... until it is confident
    a[0], c[0] = eos, 1.0
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 1         # first response position
    t2, c2, a2 = _alp_case()
    a2[-1], c2[-1] = eos, 0.95
    assert o.predict_length(t2, c2, a2, ro, mask_id, eos, 0.9) == 20          # last position: nothing to cut


def test_length_prediction_decoded_positions():
    """A decoded position is judged by the token it holds, not by the attempt computed for it."""
    mask_id, eos, ro = 99, 7, 8
    t, c, a = _alp_case()
    t[ro + 4] = 11                                     # decoded, not [EOS]
    a[4], c[4] = eos, 0.99                             # the attempt at a decoded position is ignored
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == 20
    t[ro + 6] = eos                                    # a decoded [EOS] ends the response as it stands
    c[6] = 0.0
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 6 + 1
    t[3] = eos                                         # [EOS] inside the prompt is not part of the response
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 6 + 1
    a[1], c[1] = eos, 0.91                             # an earlier confident attempt still wins
    assert o.predict_length(t, c, a, ro, mask_id, eos, 0.9) == ro + 1 + 1


def test_length_prediction_against_a_vectorised_restatement_on_random_inputs():
    """Brute force over random inputs: the loop of the oracle against an independent array formulation."""
    rng = np.random.default_rng(5)
    mask_id, eos = 63, 5
    for trial in range(300):
        L = int(rng.integers(2, 60))
        ro = int(rng.integers(0, L))
        tokens = rng.integers(0, 8, L).astype(np.int32)
        tokens[ro:][rng.random(L - ro) < 0.6] = mask_id
        conf = rng.random(L - ro)
        am = rng.integers(0, 8, L - ro).astype(np.int32)
        thr = float(rng.choice([0.0, 0.3, 0.8, 1.0]))
        draft = np.where(tokens[ro:] == mask_id, am, tokens[ro:])
        sure = np.where(tokens[ro:] == mask_id, conf > thr, True)
        hits = np.flatnonzero((draft == eos) & sure)
        want = ro + int(hits[0]) + 1 if hits.size else L
        assert o.predict_length(tokens, conf, am, ro, mask_id, eos, thr) == want


# ------------------------------------------------------------------ accept-jump controller (Sec. 4.2.1)

M_ = 99          # MASK id of the hand-built cases


def _aj_inputs(block, cand_pos, cand_tok):
    """Four drafts of `block` plus blank step outputs (nothing unmasked, confidence 0.1, attempt 50)."""
    drafts = o.accept_jump_drafts(np.array(block, np.int32), np.array(cand_pos), np.array(cand_tok))
    b = drafts.shape[1]
    return drafts, np.full((4, b), 0.1), np.full((4, b), 50, np.int32), np.zeros((4, b), np.uint8)


def test_accept_jump_drafts_and_candidates_by_hand():
    block = [1, M_, M_, 4, M_, M_]
    d = o.accept_jump_drafts(np.array(block, np.int32), np.array([2, 5]), np.array([70, 80]))
    assert d.tolist() == [[1, M_, M_, 4, M_, M_], [1, M_, 70, 4, M_, M_], [1, M_, M_, 4, M_, 80], [1, M_, 70, 4, M_, 80]]
    d = o.accept_jump_drafts(np.array(block, np.int32), np.array([2, -1]), np.array([70, 0]))
    assert d[1].tolist() == d[3].tolist() == [1, M_, 70, 4, M_, M_] and d[2].tolist() == block
    conf = np.array([0.99, 0.3, 0.8, 0.99, 0.8, 0.5])
    am = np.array([10, 11, 12, 13, 14, 15], np.int32)
    pos, tok = o.speculative_candidates(np.array(block), conf, am, M_)
    assert pos.tolist() == [2, 4] and tok.tolist() == [12, 14]          # tie at 0.8: lower index first; decoded positions never
    pos, tok = o.speculative_candidates(np.array([1, 2, M_, 4]), conf[:4], am[:4], M_)
    assert pos.tolist() == [2, -1] and tok.tolist() == [12, 0]          # one MASK left
    pos, tok = o.speculative_candidates(np.array([1, 2, 3, 4]), conf[:4], am[:4], M_)
    assert pos.tolist() == [-1, -1]


def test_accept_jump_branches_by_hand():
    """Every branch of the rule, on inputs where the adopted draft is known by construction."""
    block, cp, ct = [1, M_, M_, 4, M_, M_], [2, 5], [70, 80]

    def run(setup):
        drafts, conf, am, um = _aj_inputs(block, cp, ct)
        setup(conf, am, um)
        return o.accept_jump(drafts, conf, am, um, np.array(cp), np.array(ct), M_)

    def accept(um, am, s, p, t):
        um[s, p], am[s, p] = 1, t

    # neither candidate is unmasked by block_0: block_0's own result (it unmasks position 1 here)
    ch, nb, *_ = run(lambda c, a, u: accept(u, a, 0, 1, 33))
    assert ch == 0 and nb.tolist() == [1, 33, M_, 4, M_, M_]
    # both verified in block_0: jump to block_3, whose step unmasks position 4
    def both(c, a, u):
        accept(u, a, 0, 2, 70); accept(u, a, 0, 5, 80); accept(u, a, 3, 4, 44); accept(u, a, 0, 1, 33)
    ch, nb, *_ = run(both)
    assert ch == 3 and nb.tolist() == [1, M_, 70, 4, 44, 80]            # block_0's extra position 1 is not carried over
    # only B verified, D fails in block_1: adopt block_1
    def only_b(c, a, u):
        accept(u, a, 0, 2, 70); accept(u, a, 1, 1, 21)
    ch, nb, *_ = run(only_b)
    assert ch == 1 and nb.tolist() == [1, 21, 70, 4, M_, M_]
    # only B verified in block_0, D verified in block_1: jump to block_3
    def b_then_d(c, a, u):
        accept(u, a, 0, 2, 70); accept(u, a, 1, 5, 80); accept(u, a, 3, 1, 23)
    ch, nb, *_ = run(b_then_d)
    assert ch == 3 and nb.tolist() == [1, 23, 70, 4, M_, 80]
    # only D verified in block_0, B fails in block_2 / succeeds in block_2
    ch, nb, *_ = run(lambda c, a, u: accept(u, a, 0, 5, 80))
    assert ch == 2 and nb.tolist() == [1, M_, M_, 4, M_, 80]
    def d_then_b(c, a, u):
        accept(u, a, 0, 5, 80); accept(u, a, 2, 2, 70)
    assert run(d_then_b)[0] == 3
    # a position unmasked with ANOTHER token than the speculated one does not verify the candidate
    ch, nb, *_ = run(lambda c, a, u: accept(u, a, 0, 2, 71))
    assert ch == 0 and nb.tolist() == [1, M_, 71, 4, M_, M_]
    # no candidates at all (first step of a block): block_0
    drafts, conf, am, um = _aj_inputs(block, [-1, -1], [0, 0])
    um[0, 1], am[0, 1] = 1, 9
    ch, nb, pos, tok, nd = o.accept_jump(drafts, conf, am, um, np.array([-1, -1]), np.array([0, 0]), M_)
    assert ch == 0 and nb.tolist() == [1, 9, M_, 4, M_, M_]


def _random_step_outputs(rng, S, b=None):
    """A block, k <= S // 2 ranked candidates among its MASK positions, the S blocks built from them and random
    step outputs in which candidates are often unmasked with the speculated token."""
    b = b or int(rng.integers(2, 20))
    n_cand = S // 2
    block = rng.integers(0, 8, b).astype(np.int32)
    block[rng.random(b) < 0.6] = M_
    masked = np.flatnonzero(block == M_)
    cp = np.full(n_cand, -1, np.int32)
    ct = rng.integers(0, 8, n_cand).astype(np.int32)
    k = min(n_cand, masked.size, int(rng.integers(0, n_cand + 1)))
    cp[:k] = rng.permutation(masked)[:k]
    drafts = o.speculative_drafts(block, cp, ct, S)
    conf = rng.random((S, b))
    am = rng.integers(0, 8, (S, b)).astype(np.int32)
    for c in range(n_cand):
        if cp[c] >= 0:
            am[:, cp[c]] = np.where(rng.random(S) < 0.75, ct[c], am[:, cp[c]])
    um = ((rng.random((S, b)) < 0.5) & (drafts == M_)).astype(np.uint8)
    return block, cp, ct, drafts, conf, am, um


def test_speculative_drafts_by_hand_and_equal_to_the_four_of_accept_jump():
    block = np.array([1, M_, M_, 4, M_, M_, M_], np.int32)
    d = o.speculative_drafts(block, np.array([2, 5, 1, 6]), np.array([70, 80, 60, 90]), 8)
    assert d.tolist() == [[1, M_, M_, 4, M_, M_, M_],                  # block_0
                          [1, M_, 70, 4, M_, M_, M_],                  # B
                          [1, M_, M_, 4, M_, 80, M_],                  # D
                          [1, M_, 70, 4, M_, 80, M_],                  # B + D
                          [1, 60, M_, 4, M_, M_, M_],                  # the third
                          [1, 60, 70, 4, M_, 80, M_],                  # top three
                          [1, M_, M_, 4, M_, M_, 90],                  # the fourth
                          [1, 60, 70, 4, M_, 80, 90]]                  # top four
    d = o.speculative_drafts(block, np.array([2, 5, -1, -1]), np.array([70, 80, 0, 0]), 8)
    assert d[4].tolist() == d[6].tolist() == block.tolist() and d[5].tolist() == d[7].tolist() == d[3].tolist()
    rng = np.random.default_rng(3)
    for _ in range(50):
        block, cp, ct, *_ = _random_step_outputs(rng, 4)
        assert np.array_equal(o.speculative_drafts(block, cp, ct, 4), o.accept_jump_drafts(block, cp, ct))
        assert np.array_equal(o.speculative_drafts(block, cp, ct, 8)[:4], o.accept_jump_drafts(block, cp, ct))


def test_speculative_jump_with_four_blocks_is_the_rule_of_accept_jump():
    """Sec. 4.2.1 fixes the rule for B and D: on four blocks the eight-block rule must give exactly that."""
    rng = np.random.default_rng(10)
    seen = set()
    for trial in range(1500):
        block, cp, ct, drafts, conf, am, um = _random_step_outputs(rng, 4)
        want = o.accept_jump(drafts, conf, am, um, cp, ct, M_)
        got = o.speculative_jump(drafts, conf, am, um, cp, ct, M_, 4)
        assert got[0] == want[0]
        for g, w_ in zip(got[1:], want[1:]):
            assert np.array_equal(g, w_)
        seen.add(want[0])
    assert seen == {0, 1, 2, 3}


def test_speculative_jump_eight_blocks_by_hand():
    block, cp, ct = [1, M_, M_, 4, M_, M_, M_, M_], [2, 5, 1, 6], [70, 80, 60, 90]

    def run(accepts):
        drafts = o.speculative_drafts(np.array(block, np.int32), np.array(cp), np.array(ct), 8)
        conf, am, um = np.full((8, 8), 0.1), np.full((8, 8), 50, np.int32), np.zeros((8, 8), np.uint8)
        conf[:, 7], conf[:, 4] = 0.3, 0.2                      # ranks the positions no draft touches
        for s, p, t in accepts:
            um[s, p], am[s, p] = 1, t
        return o.speculative_jump(drafts, conf, am, um, np.array(cp), np.array(ct), M_, 8)

    B_, D_, C_, E_ = (2, 70), (5, 80), (1, 60), (6, 90)         # (position, token) of the four candidates
    assert run([])[0] == 0
    assert run([(0, *C_)])[0] == 4                               # only the third verified: its own block
    assert run([(0, *E_)])[0] == 6
    assert run([(0, *C_), (0, *E_)])[0] == 4                     # two single-candidate blocks tie: the lower number
    assert run([(0, *B_), (0, *C_)])[0] == 1                     # {B, third} is no block: B's, nothing more there
    assert run([(0, *B_), (0, *D_), (0, *C_)])[0] == 5           # top three at once
    assert run([(0, *B_), (0, *D_), (0, *C_), (0, *E_)])[0] == 7
    assert run([(0, *B_), (0, *D_), (0, *E_)])[0] == 3           # {B, D, fourth} is no block: B + D
    assert run([(0, *B_), (1, *D_), (3, *C_), (5, *E_)])[0] == 7     # one candidate at a time, four jumps
    assert run([(0, *B_), (1, *D_), (3, *E_)])[0] == 3               # the chain stops where no block fits
    assert run([(0, *D_), (2, *B_), (2, *C_)])[0] == 5               # from D's block straight to the top three
    assert run([(0, *C_), (4, *B_), (4, *D_)])[0] == 5               # from the third's block too
    assert run([(0, 2, 71)])[0] == 0                                  # another token than the speculated one
    assert run([(1, *D_)])[0] == 0                                    # what a block that is never reached verifies is ignored
    ch, nb, pos, tok, nd = run([(0, *B_), (0, *D_), (3, 1, 33)])
    assert ch == 3 and nb.tolist() == [1, 33, 70, 4, M_, 80, M_, M_]
    assert pos.tolist() == [7, 4, 6, -1] and tok.tolist() == [50, 50, 50, 0]
    assert np.array_equal(nd, o.speculative_drafts(nb, pos, tok, 8))


def test_speculative_jump_invariants_on_random_inputs():
    """Brute force: the adopted block is the end of the only chain the rule allows, found by trying all paths."""
    rng = np.random.default_rng(11)
    seen = set()
    for trial in range(1500):
        block, cp, ct, drafts, conf, am, um = _random_step_outputs(rng, 8)
        ch, nb, pos, tok, nd = o.speculative_jump(drafts, conf, am, um, cp, ct, M_, 8)
        ok = lambda s, c: cp[c] >= 0 and drafts[s, cp[c]] == M_ and um[s, cp[c]] == 1 and am[s, cp[c]] == ct[c]
        sets = [frozenset(x) for x in o.SPEC_SETS]
        cur, hops = 0, 0
        while True:
            ver = sets[cur] | {c for c in range(4) if ok(cur, c)}
            reach = [s for s in range(8) if sets[cur] < sets[s] <= ver]
            if not reach:
                break
            size = max(len(sets[s]) for s in reach)
            cur = min(s for s in reach if len(sets[s]) == size)
            hops += 1
        assert ch == cur and hops <= 4
        seen.add(ch)
        # every candidate of the adopted block was verified in some block of the chain, so the new block holds it
        for c in o.SPEC_SETS[ch]:
            assert nb[cp[c]] == ct[c]
        assert np.array_equal(nb[um[ch] == 0], drafts[ch][um[ch] == 0]) and np.array_equal(nb[um[ch] == 1], am[ch][um[ch] == 1])
        still = np.flatnonzero(nb == M_)
        assert (pos >= 0).sum() == min(4, still.size) and len(set(pos[pos >= 0].tolist())) == (pos >= 0).sum()
        ranked = sorted(still, key=lambda i: (-conf[ch][i], i))[:4]
        assert pos[pos >= 0].tolist() == ranked and all(tok[j] == am[ch][pos[j]] for j in range(4) if pos[j] >= 0)
        assert np.array_equal(nd, o.speculative_drafts(nb, pos, tok, 8))
    assert seen == set(range(8))


def test_accept_jump_next_drafts_and_invariants_on_random_inputs():
    """Properties that any input must satisfy, and an independent restatement of the branch rule."""
    rng = np.random.default_rng(9)
    for trial in range(400):
        b = int(rng.integers(2, 20))
        block = rng.integers(0, 8, b).astype(np.int32)
        block[rng.random(b) < 0.6] = M_
        masked = np.flatnonzero(block == M_)
        cp = np.full(2, -1, np.int32)
        ct = rng.integers(0, 8, 2).astype(np.int32)
        k = min(2, masked.size, int(rng.integers(0, 3)))
        cp[:k] = rng.permutation(masked)[:k]
        drafts = o.accept_jump_drafts(block, cp, ct)
        conf = rng.random((4, b))
        am = rng.integers(0, 8, (4, b)).astype(np.int32)
        for c in range(2):                                   # make verification events common
            if cp[c] >= 0:
                am[:, cp[c]] = np.where(rng.random(4) < 0.7, ct[c], am[:, cp[c]])
        um = ((rng.random((4, b)) < 0.4) & (drafts == M_)).astype(np.uint8)
        ch, nb, pos, tok, nd = o.accept_jump(drafts, conf, am, um, cp, ct, M_)
        ok = lambda s, c: cp[c] >= 0 and drafts[s, cp[c]] == M_ and um[s, cp[c]] == 1 and am[s, cp[c]] == ct[c]
        want = {(True, True): 3, (False, False): 0}.get((ok(0, 0), ok(0, 1)))
        if want is None:
            want = (3 if ok(1, 1) else 1) if ok(0, 0) else (3 if ok(2, 0) else 2)
        assert ch == want
        src = drafts[ch]
        assert np.array_equal(nb[um[ch] == 0], src[um[ch] == 0]) and np.array_equal(nb[um[ch] == 1], am[ch][um[ch] == 1])
        assert np.array_equal(nd[0], nb)
        still = np.flatnonzero(nb == M_)
        assert all(p == -1 or nb[p] == M_ for p in pos) and (pos >= 0).sum() == min(2, still.size)
        if (pos >= 0).all():
            assert pos[0] != pos[1] and conf[ch][pos[0]] >= conf[ch][pos[1]]
            assert all(conf[ch][q] <= conf[ch][pos[1]] for q in still if q not in pos)
        for s, which in ((1, [0]), (2, [1]), (3, [0, 1])):
            diff = np.flatnonzero(nd[s] != nb)
            assert set(diff) <= {int(pos[c]) for c in which if pos[c] >= 0}


# ------------------------------------------------------------------ decoded-share stage (Sec. 4.2.2)

def _shared_case(seed=3, b=8, S=4, n_decoded=3):
    cfg = o.Config(n_layers=2, d_model=32, n_heads=2, head_dim=16, d_ff=48, vocab=40, mask_id=39)
    w = o.Weights(cfg, 77, 0.3)
    rng = np.random.default_rng(seed)
    L, off = 20, 6
    tokens = rng.integers(0, 38, L)
    tokens[off:] = cfg.mask_id
    dec = rng.permutation(b)[:n_decoded]
    tokens[off + dec] = rng.integers(0, 38, n_decoded)
    cache, _, _ = o.prefill(cfg, w, tokens)
    drafts = np.stack([tokens[off:off + b]] * S)
    masked = np.flatnonzero(drafts[0] == cfg.mask_id)
    for s in range(1, S):
        if masked.size:
            drafts[s, masked[(s - 1) % masked.size]] = int(rng.integers(0, 38))
    return cfg, w, cache, drafts, off


def test_shared_step_with_nothing_decoded_is_the_plain_step():
    """No decoded position: every speculative block is the whole block, nothing is borrowed (exact)."""
    cfg, w, cache, drafts, off = _shared_case(n_decoded=0)
    a = o.block_step(cfg, w, cache, drafts, off, 0.05)
    b_ = o.block_step_shared(cfg, w, cache, drafts, off, 0.05)
    for x, y in zip(a, b_):
        assert np.array_equal(x, y)


def test_shared_step_block0_and_copies_of_block0():
    """block_0 of the shared step is the plain step's block_0 (exact); a speculative block that holds
    block_0's own tokens reproduces block_0's outputs at the masked positions (by induction over the layers
    its rows see exactly the keys block_0's rows see), up to rounding order."""
    cfg, w, cache, drafts, off = _shared_case()
    drafts[2] = drafts[0]
    plain = o.block_step(cfg, w, cache, drafts[:1], off, 0.05)
    conf, am, um, z = o.block_step_shared(cfg, w, cache, drafts, off, 0.05, return_logits=True)
    assert np.array_equal(conf[0], plain[0][0]) and np.array_equal(am[0], plain[1][0]) and np.array_equal(um[0], plain[2][0])
    P = np.flatnonzero(drafts[0] == cfg.mask_id)
    assert np.allclose(z[2], z[0][P], rtol=0, atol=1e-12)
    assert np.allclose(conf[2, P], conf[0, P], rtol=1e-12) and np.array_equal(am[2, P], am[0, P])
    D = np.flatnonzero(drafts[0] != cfg.mask_id)
    assert np.all(conf[1:, D] == 0) and np.array_equal(am[1:, D], drafts[1:, D]) and not um[1:, D].any()


def test_shared_step_visibility():
    """Speculative blocks do not see each other; they do see block_0's decoded tokens through the borrowed K/V
    and do not see block_0's masked rows; decoded-position K/V really are block_0's (the result changes if
    they are recomputed inside the speculative block, which is what the plain step does)."""
    cfg, w, cache, drafts, off = _shared_case(S=4)
    base = o.block_step_shared(cfg, w, cache, drafts, off, 0.05, return_logits=True)[3]
    # another speculative block changes: block 1 unaffected
    d2 = drafts.copy()
    P = np.flatnonzero(drafts[0] == cfg.mask_id)
    d2[3, P[0]] = (d2[3, P[0]] + 1) % 38
    alt = o.block_step_shared(cfg, w, cache, d2, off, 0.05, return_logits=True)[3]
    assert np.array_equal(alt[1], base[1]) and np.array_equal(alt[2], base[2]) and not np.array_equal(alt[3], base[3])
    # the shared result is NOT the plain multi-draft step when a speculative token differs from block_0
    # (there the decoded positions' K/V would be recomputed with the speculative token in view) ...
    plain = o.block_step(cfg, w, cache, drafts, off, 0.05, return_logits=True)[3]
    assert np.abs(plain[1][P] - base[1]).max() > 1e-9
    # ... and equals a hand-assembled forward in which those K/V are taken from block_0 (one layer, by hand)
    cfg1 = o.Config(n_layers=1, d_model=32, n_heads=2, head_dim=16, d_ff=48, vocab=40, mask_id=39)
    w1 = o.Weights(cfg1, 77, 0.3)
    c1 = o.Cache(cache.k[:1], cache.v[:1])
    z1 = o.block_step_shared(cfg1, w1, c1, drafts, off, 0.05, return_logits=True)[3][1]
    D = np.flatnonzero(drafts[0] != cfg.mask_id)
    b = drafts.shape[1]
    pos = off + np.arange(b)
    def qkv(tok, pp):
        h = w1.embed_rows(tok)
        a = o.rmsnorm(h, w1.f64(o.T_G1, 0), cfg1.rms_eps)
        q = o.rope((a @ w1.f64(o.T_WQ, 0).T).reshape(-1, 2, 16), pp, cfg1.rope_base)
        k = o.rope((a @ w1.f64(o.T_WK, 0).T).reshape(-1, 2, 16), pp, cfg1.rope_base)
        return h, q, k, (a @ w1.f64(o.T_WV, 0).T).reshape(-1, 2, 16)
    _, _, k0, v0 = qkv(drafts[0], pos)
    h, q, k, v = qkv(drafts[1, P], pos[P])
    kk = np.concatenate([c1.k[0][:off], k0[D], k, c1.k[0][off + b:]])
    vv = np.concatenate([c1.v[0][:off], v0[D], v, c1.v[0][off + b:]])
    h = h + o.attention(q, kk, vv).reshape(-1, 32) @ w1.f64(o.T_WO, 0).T
    m = o.rmsnorm(h, w1.f64(o.T_G2, 0), cfg1.rms_eps)
    h = h + (o.silu(m @ w1.f64(o.T_WG, 0).T) * (m @ w1.f64(o.T_WU, 0).T)) @ w1.f64(o.T_WD, 0).T
    zz = o.rmsnorm(h, w1.f64(o.T_GF, 0), cfg1.rms_eps) @ w1.f64(o.T_LM, 0).T
    assert np.allclose(zz, z1, rtol=0, atol=1e-11)


def test_shared_step_fully_decoded_block():
    cfg, w, cache, drafts, off = _shared_case(n_decoded=8)
    conf, am, um = o.block_step_shared(cfg, w, cache, drafts[:1].repeat(3, 0), off, 0.05)
    assert not um.any() and np.all(conf[1:] == 0) and conf[0].min() > 0


# ------------------------------------------------------------------ the generation loop (Sec. 2.1 + 4.1 + 4.2)

def _gen_setup(seed=11, P=12, gain=6.0):
    rng = np.random.default_rng(seed)
    w = o.Weights(MICRO, seed, 0.25)
    w.set_values(o.T_GF, 0, np.full(MICRO.d_model, gain))
    return w, rng.integers(0, MICRO.vocab - 1, P).astype(np.int32)


def _n_masked(ev, P):
    return int((ev["tokens"][P:] == MICRO.mask_id).sum())


def test_generate_threshold_never_reached_decodes_one_position_per_forward():
    """tau above 1: only forced progress acts, so every forward (refresh or step) fills exactly one position,
    the most confident masked one of the current block, and R forwards fill R positions."""
    w, prompt = _gen_setup()
    P, R, b = len(prompt), 20, 8                                     # ragged last block of 4
    tokens, stats, events = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, tau=2.0))
    assert stats["n_refresh"] == 3 and stats["n_refresh"] + stats["n_step"] == R == len(events)
    assert stats["refresh_positions"] == 3 * (P + R) and stats["step_rows"] == 7 * 8 + 7 * 8 + 3 * 4
    assert not (tokens == MICRO.mask_id).any() and np.array_equal(tokens[:P], prompt)
    prev = np.concatenate([prompt, np.full(R, MICRO.mask_id, np.int32)])
    for n, ev in enumerate(events):
        diff = np.flatnonzero(ev["tokens"] != prev)
        assert diff.size == 1 and ev["block_off"] <= diff[0] < ev["block_off"] + ev["block_len"]
        assert prev[diff[0]] == MICRO.mask_id and ev["kind"] == ("refresh" if n in (0, 8, 16) else "step")
        prev = ev["tokens"]


def test_generate_threshold_always_reached_needs_refreshes_only():
    """tau below 0: the refresh's attempt fills its whole block, no step ever runs, and block k holds the greedy
    tokens of a full forward over the sequence as it stood when block k's cycle began."""
    w, prompt = _gen_setup(seed=12)
    P, R, b = len(prompt), 24, 8
    tokens, stats, events = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, tau=-1.0))
    assert stats["n_step"] == 0 and stats["n_refresh"] == 3 and [e["kind"] for e in events] == ["refresh"] * 3
    seq = np.concatenate([prompt, np.full(R, MICRO.mask_id, np.int32)])
    for k in range(3):
        _, _, am = o.prefill(MICRO, w, seq, resp_off=P)
        seq[P + k * b:P + (k + 1) * b] = am[k * b:(k + 1) * b]
        assert np.array_equal(events[k]["tokens"], seq)
    assert np.array_equal(tokens, seq)


def test_generate_steps_use_the_cache_of_the_cycles_refresh():
    """The first block cycle redone from the primitives: acceptance on the refresh's attempt, then steps against
    that same (ageing) cache, each on the block as the previous forward left it."""
    w, prompt = _gen_setup(seed=13)
    P, R, b, tau = len(prompt), 16, 8, 0.8
    _, _, events = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, tau=tau))
    seq = np.concatenate([prompt, np.full(R, MICRO.mask_id, np.int32)])
    cache, conf, am = o.prefill(MICRO, w, seq, resp_off=P)
    blk = seq[P:P + b].copy()
    take = conf[:b] > tau
    take[np.argmax(conf[:b])] = True
    blk[take] = am[:b][take]
    assert np.array_equal(events[0]["tokens"][P:P + b], blk) and (events[0]["tokens"][P + b:] == MICRO.mask_id).all()
    # the candidates a refresh hands to the first step: the two most confident positions it left masked
    left = sorted(np.flatnonzero(blk == MICRO.mask_id), key=lambda i: -conf[i])[:2]
    assert list(events[0]["cand_pos"][:len(left)]) == left and list(events[0]["cand_tok"][:len(left)]) == [am[i] for i in left]
    _, _, ev4 = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, n_drafts=4, tau=tau))
    assert np.array_equal(ev4[0]["tokens"], events[0]["tokens"]) and np.array_equal(ev4[0]["cand_pos"], events[0]["cand_pos"])
    d4 = np.stack([blk] * 4)
    d4[1, left[0]] = d4[3, left[0]] = am[left[0]]
    d4[2, left[1]] = d4[3, left[1]] = am[left[1]]
    c4, a4, u4 = o.block_step(MICRO, w, cache, d4, P, tau)
    s_ = ev4[1]["chosen"]
    assert s_ == 1, "the case is chosen so that the first step adopts a speculative block"
    assert np.array_equal(ev4[1]["tokens"][P:P + b], np.where(u4[s_] == 1, a4[s_], d4[s_]))
    n = 1
    while (blk == MICRO.mask_id).any():
        c, a, u = o.block_step(MICRO, w, cache, blk[None], P, tau)
        blk = np.where(u[0] == 1, a[0], blk)
        assert events[n]["kind"] == "step" and np.array_equal(events[n]["tokens"][P:P + b], blk)
        n += 1
    assert n > 1, "the case must exercise at least one step"
    assert events[n]["kind"] == "refresh" and events[n]["block_off"] == P + b


def test_generate_length_prediction_cuts_at_the_attempted_eos():
    """Sec. 4.1 inside the loop: the first refresh's attempt decides the first cut; the cut block is ragged; an
    [EOS] decoded inside a finished block ends generation at the next refresh."""
    w, prompt = _gen_setup(seed=14)
    P, R, b = len(prompt), 24, 8
    seq = np.concatenate([prompt, np.full(R, MICRO.mask_id, np.int32)])
    _, conf, am = o.prefill(MICRO, w, seq, resp_off=P)
    q = 8 + int(np.argmax(conf[8:20]))                                # a confident attempt in blocks 1-2
    eos, thr = int(am[q]), float(conf[q]) * 0.999
    first = min(i for i in range(R) if am[i] == eos and conf[i] > thr)
    tokens, stats, events = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, tau=0.6, eos_id=eos, truncate_thr=thr))
    assert events[0]["L"] == P + first + 1 and len(events[0]["tokens"]) == P + first + 1
    lens = [e["L"] for e in events]
    assert all(x >= y for x, y in zip(lens, lens[1:])) and stats["final_len"] == lens[-1] == len(tokens)
    assert not (tokens == MICRO.mask_id).any()
    # a refresh runs at the length the previous event left behind
    assert stats["refresh_positions"] == (P + R) + sum(events[i - 1]["L"] for i in range(1, len(events))
                                                       if events[i]["kind"] == "refresh")
    # never exceeded threshold: only a decoded [EOS] cuts.  Take the token block 0 really decodes first.
    full, _, ev_full = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, tau=0.6))
    eos2 = int(full[P + 3])
    j = int(np.flatnonzero(full[P:P + b] == eos2)[0])
    tokens2, stats2, ev2 = o.generate(MICRO, w, prompt, R, o.GenParams(block_len=b, tau=0.6, eos_id=eos2, truncate_thr=2.0))
    assert stats2["n_refresh"] == 2 and stats2["final_len"] == P + j + 1 and np.array_equal(tokens2, full[:P + j + 1])
    assert ev2[-1]["kind"] == "refresh" and ev2[-1]["block_len"] == 0


def test_generate_accept_jump_invariants_and_stage_switch():
    """Four drafts: every forward fills at least one position of the block, drafts other than block_0 do get
    adopted on peaked weights, a switch point beyond the block length never engages the decoded-share stage,
    and a switch point of 0 runs every step in it (rows: b + 3 * masked instead of 4 * b)."""
    seen = set()
    for seed in (21, 22, 23):
        w, prompt = _gen_setup(seed=seed, gain=8.0)
        P, R, b = len(prompt), 16, 8
        base = o.GenParams(block_len=b, n_drafts=4, tau=0.7)
        tokens, stats, events = o.generate(MICRO, w, prompt, R, base)
        assert not (tokens == MICRO.mask_id).any()
        prev = R
        for ev in events:
            assert _n_masked(ev, P) < prev
            prev = _n_masked(ev, P)
            seen.add(ev["chosen"])
        assert stats["n_step_shared"] == 0 and stats["step_rows"] == 4 * b * stats["n_step"]
        t2, s2, e2 = o.generate(MICRO, w, prompt, R, dataclasses_replace(base, share_from=b + 1))
        assert np.array_equal(t2, tokens) and s2 == stats
        t3, s3, e3 = o.generate(MICRO, w, prompt, R, dataclasses_replace(base, share_from=0))
        assert s3["n_step_shared"] == s3["n_step"] and not (t3 == MICRO.mask_id).any()
        rows, before = 0, None
        for ev in e3:
            if ev["kind"] == "shared":
                rows += b + 3 * before
            before = int((ev["tokens"][ev["block_off"]:ev["block_off"] + ev["block_len"]] == MICRO.mask_id).sum())
        assert rows == s3["step_rows"]
        _, _, e4 = o.generate(MICRO, w, prompt, R, dataclasses_replace(base, share_from=5))
        for prev_ev, ev in zip(e4, e4[1:]):
            if ev["kind"] != "refresh":
                blk = prev_ev["tokens"][ev["block_off"]:ev["block_off"] + ev["block_len"]]
                assert (ev["kind"] == "shared") == (int((blk != MICRO.mask_id).sum()) >= 5)
    assert seen - {0}, "no speculative draft was ever adopted: the case does not exercise the controller"


def test_generate_eight_blocks_in_the_decoded_share_stage():
    """n_drafts = 8: until the switch point the run is the four-draft accept-jump run, position for position; in
    the decoded-share stage a step forwards b + 7 * masked rows, and one such step is redone here from the
    primitives (eight blocks from the four ranked candidates, the shared-K/V forward, the jump rule)."""
    seen = set()
    for seed in (23, 34, 35):
        w, prompt = _gen_setup(seed=seed, gain=8.0)
        P, R, b = len(prompt), 16, 8
        four = o.GenParams(block_len=b, n_drafts=4, tau=0.85, share_from=b + 1)
        t4, s4, e4 = o.generate(MICRO, w, prompt, R, four)
        t8, s8, e8 = o.generate(MICRO, w, prompt, R, dataclasses_replace(four, n_drafts=8))
        assert np.array_equal(t4, t8) and s4 == s8 and len(e4) == len(e8)
        for a4, a8 in zip(e4, e8):
            assert a4["chosen"] == a8["chosen"] and np.array_equal(a4["tokens"], a8["tokens"])
            assert np.array_equal(a4["cand_pos"], a8["cand_pos"][:2]) and a8["cand_pos"].shape == (4,)
        p8 = o.GenParams(block_len=b, n_drafts=8, tau=0.85, share_from=2)
        tokens, stats, events = o.generate(MICRO, w, prompt, R, p8)
        assert not (tokens == MICRO.mask_id).any() and stats["n_step_shared"] > 0
        rows = 0
        redone = False
        for prev_ev, ev in zip(events, events[1:]):
            if ev["kind"] == "refresh":
                continue
            off, bb = ev["block_off"], ev["block_len"]
            blk = prev_ev["tokens"][off:off + bb]
            nm = int((blk == MICRO.mask_id).sum())
            assert (ev["kind"] == "shared") == (bb - nm >= 2)
            rows += bb + 7 * nm if ev["kind"] == "shared" else 4 * bb
            seen.add((ev["kind"], ev["chosen"]))
            if ev["kind"] == "shared" and not redone:
                # the cycle's cache: the refresh ran on the sequence as it stood when the block cycle began
                cyc = [x for x in events[:events.index(ev)] if x["kind"] == "refresh"][-1]
                before = events[events.index(cyc) - 1]["tokens"] if events.index(cyc) else \
                    np.concatenate([prompt, np.full(R, MICRO.mask_id, np.int32)])
                cache, _, _ = o.prefill(MICRO, w, before, resp_off=P)
                drafts = o.speculative_drafts(blk, prev_ev["cand_pos"], prev_ev["cand_tok"], 8)
                out = o.block_step_shared(MICRO, w, cache, drafts, off, 0.85)
                ch, nb, pos, tok, _ = o.speculative_jump(drafts, *out, prev_ev["cand_pos"], prev_ev["cand_tok"],
                                                         MICRO.mask_id, 8)
                assert ch == ev["chosen"] and np.array_equal(nb, ev["tokens"][off:off + bb])
                assert np.array_equal(pos, ev["cand_pos"]) and np.array_equal(tok, ev["cand_tok"])
                redone = True
        assert rows == stats["step_rows"] and redone
    assert {c for k, c in seen if k == "shared"} - {0, 1, 2, 3}, "none of the four extra blocks was ever adopted"
    # the row budget: eight blocks only where b + 7 * masked rows fit; a budget nothing exceeds changes nothing,
    # one that nothing fits gives the four-block run with the same switch point
    w, prompt = _gen_setup(seed=23, gain=8.0)
    p8 = o.GenParams(block_len=8, n_drafts=8, tau=0.85, share_from=2)
    ref8 = o.generate(MICRO, w, prompt, 16, p8)
    big = o.generate(MICRO, w, prompt, 16, dataclasses_replace(p8, row_budget=8 + 7 * 8))
    assert np.array_equal(ref8[0], big[0]) and ref8[1] == big[1]
    none = o.generate(MICRO, w, prompt, 16, dataclasses_replace(p8, row_budget=0))
    ref4 = o.generate(MICRO, w, prompt, 16, dataclasses_replace(p8, n_drafts=4))
    assert np.array_equal(none[0], ref4[0]) and none[1] == ref4[1]
    mid = o.generate(MICRO, w, prompt, 16, dataclasses_replace(p8, row_budget=8 + 7 * 3))
    rows, n8 = 0, 0
    for prev_ev, ev in zip(mid[2], mid[2][1:]):
        if ev["kind"] == "refresh":
            continue
        blk = prev_ev["tokens"][ev["block_off"]:ev["block_off"] + ev["block_len"]]
        nm = int((blk == MICRO.mask_id).sum())
        eight = ev["kind"] == "shared" and nm <= 3
        n8 += eight
        rows += (ev["block_len"] + (7 if eight else 3) * nm) if ev["kind"] == "shared" else 4 * ev["block_len"]
        assert ev["chosen"] < (8 if eight else 4)
    assert rows == mid[1]["step_rows"] and n8 > 0


def test_generate_stops_when_the_greedy_token_is_mask():
    """Untrained weights may attempt the MASK token itself at the forced position: the block's MASK count then
    stays as it was and the loop reports it instead of spinning (LM head row of MASK made dominant here)."""
    w, prompt = _gen_setup(seed=21, gain=8.0)
    lm = w.f64(o.T_LM).copy()
    lm[MICRO.mask_id] = 40.0 * lm.std()          # every hidden state with a positive mean now prefers MASK ...
    lm[:MICRO.mask_id] = 0.0                     # ... and nothing competes
    w.set_values(o.T_LM, 0, lm)
    w.set_values(o.T_EMBED, 0, np.abs(w.f64(o.T_EMBED)))
    for nd, sf in ((1, None), (4, None), (8, 0)):
        with pytest.raises(RuntimeError):
            o.generate(MICRO, w, prompt, 8, o.GenParams(block_len=4, n_drafts=nd, tau=0.5, share_from=sf))


def dataclasses_replace(p, **kw):
    import dataclasses
    return dataclasses.replace(p, **kw)
