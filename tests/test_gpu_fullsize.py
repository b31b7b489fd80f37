"""GPU parity at the full 8B shape (configs 1 and 2), in the launch configuration bench.py times.

The oracle needs about an hour of CPU for the 32-layer model, so its outputs are stored:
tests/golden/config12_oracle*.npz, written by tests/golden/make_8b_golden.py (which calls only
the oracle).  Stored per call: confidence / argmax / unmask of every row, the eight largest
logits of every row, 256 sampled vocabulary columns of every row, log-sum-exp, max |logit|, and
K/V of 48 sampled positions at three layers.  The 2-layer file exercises the full width
(d = 4096, F = 12288, V = 126464) through every kernel; the 32-layer file is the benchmarked model.
"""
import os

import numpy as np
import pytest

from paper_2511_21759_amd import binding as B
from paper_2511_21759_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LOGIT_TOL, KV_TOL, MARGIN, TAU_BAND = 2e-2, 1e-2, 1e-2, 1e-3
LITERAL = {"argmax_rows": 0, "unmask_positions": 0}     # rows on which the bar was asserted as stated


def check_unmask_literal(um, drafts, g, prefix, tau, mask_id, tag):
    """Acceptance flags against the stored oracle's wherever the bar as stated binds: MASK positions whose top-2
    probability margin exceeds 1e-2 and whose confidence is further than 1e-3 from tau; a position below tau is
    flagged only as the forced pick, compared where the most confident MASK position leads by more than 1e-2."""
    conf_o, ref = g[prefix + "_conf"], g[prefix + "_unmask"]
    top = g[prefix + "_top_logits"].astype(np.float64)
    margin = conf_o * (1.0 - np.exp(top[..., -2] - top[..., -1]))
    for s in range(drafts.shape[0]):
        masked = drafts[s] == mask_id
        if not masked.any():
            continue
        cm = np.sort(conf_o[s][masked])[::-1]
        forced_clear = cm.size < 2 or cm[0] - cm[1] > MARGIN
        for i in np.flatnonzero(masked):
            if not (margin[s][i] > MARGIN and abs(conf_o[s][i] - tau) > TAU_BAND):
                continue
            if not conf_o[s][i] > tau and not forced_clear and conf_o[s][i] >= cm[0] - MARGIN:
                continue
            assert um[s][i] == ref[s][i], "%s: unmask[%d][%d]" % (tag, s, i)
            LITERAL["unmask_positions"] += 1


def cuda_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()


def sampled_err(logits, g, prefix):
    """max |gpu - oracle| over the stored entries (sampled columns and top-8) of every row."""
    cols = g["step_logit_cols"]
    a = np.abs(logits[..., cols] - g[prefix + "_logits_sample"]).max()
    top = g[prefix + "_top_ids"].astype(np.int64)
    b = np.abs(np.take_along_axis(logits, top, -1) - g[prefix + "_top_logits"]).max()
    return float(max(a, b))


def check_rows(logits, conf, am, g, prefix, tag, same_gemm=True):
    e = sampled_err(logits, g, prefix)
    rel = e / float(g[prefix + "_logit_absmax"])
    assert rel <= LOGIT_TOL, "%s: logits rel err %.3g" % (tag, rel)
    band = 2.5 * e + 1e-5            # e is a sampled maximum: 25 % head-room on the exact 2e bound
    conf_o, am_o = g[prefix + "_conf"], g[prefix + "_argmax"]
    assert np.all(np.abs(np.log(conf) - np.log(conf_o)) <= band), "%s: confidence" % tag
    top = g[prefix + "_top_logits"].astype(np.float64)
    gap = top[..., -1] - top[..., -2]
    strict = gap > band
    assert np.array_equal(am[strict], am_o[strict]), "%s: argmax outside the error band" % tag
    # inside the band: any of the stored eight best tokens whose oracle logit is within the band of the largest
    ids = g[prefix + "_top_ids"]
    ok = ((ids == am[..., None]) & (top >= top[..., -1:] - band)).any(-1)
    assert np.all(ok[~strict]), "%s: argmax outside the error band" % tag
    # the bar as stated: no mismatch on any row whose two largest probabilities differ by more than 1e-2
    # (p1 = conf, p2 = conf * exp(z2 - z1), from the stored eight largest logits)
    margin = conf_o * (1.0 - np.exp(top[..., -2] - top[..., -1]))
    clear = margin > MARGIN
    bad = clear & (am != am_o)
    assert not bad.any(), "%s: argmax differs on %d of %d rows with top-2 probability margin > 1e-2" % (
        tag, int(bad.sum()), int(clear.sum()))
    LITERAL["argmax_rows"] += int(clear.sum())
    if same_gemm:
        # the fused statistics agree with the unfused logits when the same kernels produced both
        assert np.array_equal(am, logits.argmax(-1)), "%s: fused argmax vs stored logits" % tag
        lse = np.log(np.exp(logits - logits.max(-1, keepdims=True)).sum(-1))
        assert np.allclose(np.log(conf), -lse, atol=2e-4), "%s: fused confidence vs stored logits" % tag
    return e, rel, int(strict.sum()), strict.size


@pytest.mark.parametrize("fname", ["config12_oracle_2L.npz", "config12_oracle.npz"])
def test_configs_1_and_2_against_stored_oracle(fname):
    path = os.path.join(GOLDEN, fname)
    if not os.path.exists(path):
        pytest.skip("%s has not been generated (tests/golden/make_8b_golden.py)" % fname)
    g = np.load(path)
    nl = int(g["n_layers"])
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=nl)
    wl = W.config2()
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        L = wl.tokens.shape[1]
        cache = B.odb_cache_create(model, 1, L)
        tok = cuda_i32(wl.tokens)
        zp = B.odb_prefill_logits(model, cache, tok, wl.resp_off, shape["vocab"]).cpu().numpy()[0]
        conf_p, am_p = (t.cpu().numpy()[0] for t in B.odb_prefill(model, cache, tok, wl.resp_off))
        e, rel, ns, n = check_rows(zp, conf_p, am_p, g, "prefill", fname + " prefill")
        print("\n%s prefill: max sampled logit err %.4f (rel %.2e), %d/%d rows bit-exact-checked" % (fname, e, rel, ns, n))
        for i, layer in enumerate(g["kv_layers"]):
            for kv, ref, amax in ((0, g["k_sample"][i], g["k_absmax"][i]), (1, g["v_sample"][i], g["v_absmax"][i])):
                got = B.odb_cache_read(cache, int(layer), kv, 0, 0, L, 32, 128)[g["kv_pos"]]
                err = np.abs(got - ref).max() / amax
                assert err <= KV_TOL, "%s: cache layer %d kv %d: %.3g" % (fname, layer, kv, err)
        # config 2 (S = 4); its draft 0 is config 1
        d = cuda_i32(wl.drafts)
        z = B.odb_block_step_logits(model, cache, d, wl.block_off, shape["vocab"]).cpu().numpy()[0]
        conf, am, um = (t.cpu().numpy()[0] for t in B.odb_block_step(model, cache, d, wl.block_off, float(g["tau"])))
        B.odb_model_status(model)
        e, rel, ns, n = check_rows(z, conf, am, g, "step", fname + " step")
        assert np.array_equal(um, g["step_unmask"]), "unmask (tau = 0.9 is far from every confidence here)"
        d1 = cuda_i32(W.config1().drafts)
        c1, a1, u1 = (t.cpu().numpy()[0] for t in B.odb_block_step(model, cache, d1, wl.block_off, float(g["tau"])))
        # S = 1 and S = 4 run different GEMM kernels (other summation orders): same forced pick, confidences within binary16 noise
        assert np.array_equal(u1[0], um[0]) and np.allclose(c1[0], conf[0], rtol=5e-2)
        assert (a1[0] == am[0]).mean() >= 0.9
        print("%s step: max sampled logit err %.4f (rel %.2e), %d/%d rows bit-exact-checked" % (fname, e, rel, ns, n))
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


def test_batch4_long_block_against_stored_oracle():
    """Config 4's structure (batch 4, S = 8 drafts of a 64-token block: 2048 rows per step) at the full 8B
    width with two layers, sequences 0 and 3 of the batch against stored oracle outputs: batch indexing, the
    256 x 256 GEMM blocks with the fused norm, and the shared-K/V attention kernel at head_dim 128."""
    path = os.path.join(GOLDEN, "config4_small_oracle_2L.npz")
    if not os.path.exists(path):
        pytest.skip("config4_small_oracle_2L.npz has not been generated (tests/golden/make_8b_golden.py batch4)")
    g = np.load(path)
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=int(g["n_layers"]))
    wl = W.config4_small()
    assert wl.block_off == int(g["block_off"])
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        Bn, L = wl.tokens.shape
        cache = B.odb_cache_create(model, Bn, L)
        tok = cuda_i32(wl.tokens)
        zp = B.odb_prefill_logits(model, cache, tok, wl.resp_off, shape["vocab"]).cpu().numpy()
        conf_p, am_p = (t.cpu().numpy() for t in B.odb_prefill(model, cache, tok, wl.resp_off))
        d = cuda_i32(wl.drafts)
        z = B.odb_block_step_logits(model, cache, d, wl.block_off, shape["vocab"]).cpu().numpy()
        conf, am, um = (t.cpu().numpy() for t in B.odb_block_step(model, cache, d, wl.block_off, float(g["tau"])))
        B.odb_model_status(model)
        for i, bi in enumerate(g["seqs"]):
            view = {k: g[k][i] for k in g.files if g[k].ndim > 0 and g[k].shape[0] == len(g["seqs"]) and k != "seqs"}
            view["step_logit_cols"] = g["logit_cols"]
            e, rel, ns, n = check_rows(zp[bi], conf_p[bi], am_p[bi], view, "prefill", "batch4 prefill seq %d" % bi)
            e2, rel2, ns2, n2 = check_rows(z[bi], conf[bi], am[bi], view, "step", "batch4 step seq %d" % bi)
            assert np.array_equal(um[bi], view["step_unmask"]), "unmask of sequence %d" % bi
            print("\nseq %d: prefill logit err rel %.2e (%d/%d rows strict), step rel %.2e (%d/%d)" % (bi, rel, ns, n, rel2, ns2, n2))
            for layer in range(shape["n_layers"]):
                for kv, ref, amax in ((0, view["k_sample"][layer], view["k_absmax"][layer]),
                                      (1, view["v_sample"][layer], view["v_absmax"][layer])):
                    got = B.odb_cache_read(cache, layer, kv, int(bi), 0, L, 32, 128)[g["kv_pos"]]
                    err = np.abs(got - ref).max() / amax
                    assert err <= KV_TOL, "batch4: cache seq %d layer %d kv %d: %.3g" % (bi, layer, kv, err)
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


@pytest.mark.parametrize("resp", [512, 256, 128])
def test_config3_prefill_against_stored_oracle(resp):
    """Config 3's refreshes (512 prompt + 512 / 256 / 128 MASK positions: 1024, 768 and 640 rows, the lengths the
    adaptive length prediction shrinks the refresh to) at the full 8B width with two layers against stored oracle
    outputs: each length picks its own GEMM block shapes, and the K/V-sharing attention kernel runs over up to a
    thousand keys."""
    fname = "config3_r256_oracle_2L.npz" if resp == 256 else "config3_oracle_2L.npz"
    path = os.path.join(GOLDEN, fname)
    if not os.path.exists(path):
        pytest.skip("%s has not been generated (tests/golden/make_8b_golden.py prefill / prefill256)" % fname)
    g = np.load(path)
    tag = "r%d_" % resp
    view = {k[len(tag):]: g[k] for k in g.files if k.startswith(tag)}
    view["step_logit_cols"] = g["logit_cols"]
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=int(g["n_layers"]))
    tokens = W.config3(resp)
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        L = tokens.shape[1]
        cache = B.odb_cache_create(model, 1, L)
        tok = cuda_i32(tokens)
        z = B.odb_prefill_logits(model, cache, tok, 512, shape["vocab"]).cpu().numpy()[0]
        conf, am = (t.cpu().numpy()[0] for t in B.odb_prefill(model, cache, tok, 512))
        e, rel, ns, n = check_rows(z, conf, am, view, "prefill", "config3 prefill, %d response positions" % resp)
        print("\nconfig3 resp %d: logit err rel %.2e (%d/%d rows strict)" % (resp, rel, ns, n))
        for layer in range(shape["n_layers"]):
            for kv, ref, amax in ((0, view["k_sample"][layer], view["k_absmax"][layer]),
                                  (1, view["v_sample"][layer], view["v_absmax"][layer])):
                got = B.odb_cache_read(cache, layer, kv, 0, 0, L, 32, 128)[view["kv_pos"]]
                err = np.abs(got - ref).max() / amax
                assert err <= KV_TOL, "config3: cache layer %d kv %d: %.3g" % (layer, kv, err)
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


def test_decoded_share_step_against_stored_oracle():
    """The eight-block decoded-share step that bench.py times (config2_shared: a quarter of block_0 still MASK) at
    the full 8B width with two layers against stored oracle outputs, row by row."""
    path = os.path.join(GOLDEN, "config2_shared_oracle_2L.npz")
    if not os.path.exists(path):
        pytest.skip("config2_shared_oracle_2L.npz has not been generated (tests/golden/make_8b_golden.py shared)")
    g = np.load(path)
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=int(g["n_layers"]))
    wl = W.config2_shared()
    assert wl.block_off == int(g["block_off"])
    n_masked = int(g["n_masked"])
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        cache = B.odb_cache_create(model, 1, wl.tokens.shape[1])
        B.odb_prefill(model, cache, cuda_i32(wl.tokens), wl.resp_off)
        d = cuda_i32(wl.drafts)
        S, b = wl.drafts.shape[1:]
        z, rowout = B.odb_block_step_shared_logits(model, cache, d, wl.block_off, n_masked, shape["vocab"])
        z, rowout = z.cpu().numpy(), rowout.cpu().numpy()
        conf, am, um = (t.cpu().numpy()[0] for t in B.odb_block_step_shared(model, cache, d, wl.block_off, n_masked,
                                                                             float(g["tau"])))
        B.odb_model_status(model)
        computed = ~np.isnan(g["step_top_logits"][..., 0])                     # [S, b]
        assert sorted(rowout[rowout >= 0].tolist()) == np.flatnonzero(computed.reshape(-1)).tolist()
        # logits of the computed rows, gathered into [S, b, V] order through the row map
        e = 0.0
        zfull = {}
        for r, o_ in enumerate(rowout):
            if o_ < 0:
                continue
            s_, i_ = divmod(int(o_), b)
            zfull[(s_, i_)] = z[r]
            e = max(e, float(np.abs(z[r][g["logit_cols"]] - g["step_logits_sample"][s_, i_]).max()),
                    float(np.abs(z[r][g["step_top_ids"][s_, i_]] - g["step_top_logits"][s_, i_]).max()))
        rel = e / float(g["step_logit_absmax"])
        assert rel <= LOGIT_TOL, "decoded-share logits rel err %.3g" % rel
        band = 2.5 * e + 1e-5
        n_strict = 0
        for (s_, i_), zr in zfull.items():
            assert abs(np.log(conf[s_, i_]) - np.log(g["step_conf"][s_, i_])) <= band, (s_, i_)
            top = g["step_top_logits"][s_, i_].astype(np.float64)
            if top[-1] - top[-2] > band:
                assert am[s_, i_] == g["step_argmax"][s_, i_], (s_, i_)
                n_strict += 1
            else:
                ids = g["step_top_ids"][s_, i_]
                assert ((ids == am[s_, i_]) & (top >= top[-1] - band)).any(), (s_, i_)
        # positions that are not computed read as the call documents; random weights: only forced picks
        nc = ~computed
        assert np.all(conf[nc] == 0) and np.array_equal(am[nc], wl.drafts[0][nc]) and not um[nc].any()
        assert np.array_equal(um, g["step_unmask"]), "unmask (one forced pick per block, far from any tie)"
        print("\ndecoded-share step: %d rows, logit err rel %.2e, %d rows strict" % (len(zfull), rel, n_strict))
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


def test_decoded_share_step_properties_at_full_width():
    """The decoded-share step (ODB-dLLM Sec. 4.2.2) at the 8B width with two layers, head_dim 128, checked by the
    properties that pin its oracle: with nothing decoded it is the plain step; block_0 is the plain step's
    block_0; a speculative block that repeats block_0's tokens reproduces block_0 at the masked positions;
    speculative blocks do not see each other."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    wl = W.config2()
    mask_id = shape["mask_id"]
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        L = wl.tokens.shape[1]
        cache = B.odb_cache_create(model, 1, L)
        B.odb_prefill(model, cache, cuda_i32(wl.tokens), wl.resp_off)
        blk = wl.drafts[0, 0]
        masked = np.flatnonzero(blk == mask_id)
        assert 4 <= masked.size < 32
        rng = np.random.default_rng(17)
        drafts = np.stack([blk] * 8)[None].copy()                      # [1, 8, 32]
        for s in (1, 2, 3, 5, 6, 7):                                    # blocks 4 stays a copy of block_0
            drafts[0, s, masked[s % masked.size]] = int(rng.integers(0, 1000))
        d = cuda_i32(drafts)
        conf, am, um = (t.cpu().numpy()[0] for t in B.odb_block_step_shared(model, cache, d, wl.block_off, int(masked.size), wl.tau))
        B.odb_model_status(model)
        c0, a0, u0 = (t.cpu().numpy()[0, 0] for t in B.odb_block_step(model, cache, cuda_i32(drafts[:, :1]), wl.block_off, wl.tau))
        assert np.allclose(np.log(conf[0]), np.log(c0), atol=2e-2) and (am[0] == a0).mean() >= 0.9
        assert np.allclose(np.log(conf[4, masked]), np.log(conf[0, masked]), atol=2e-2)
        assert (am[4, masked] == am[0, masked]).mean() >= 0.8 and um[4].sum() == 1 and um[0].sum() == 1
        dec = np.flatnonzero(blk != mask_id)
        assert np.all(conf[1:][:, dec] == 0) and np.array_equal(am[1:][:, dec], drafts[0][1:][:, dec]) and not um[1:][:, dec].any()
        # another speculative block changes: the others are bit-identical (same rows, same kernels)
        d2 = drafts.copy()
        d2[0, 7, masked[0]] = 77
        conf2 = B.odb_block_step_shared(model, cache, cuda_i32(d2), wl.block_off, int(masked.size), wl.tau)[0].cpu().numpy()[0]
        assert np.array_equal(conf2[:7], conf[:7]) and not np.array_equal(conf2[7], conf[7])
        # nothing decoded: every block is computed in full, as in the plain step
        allm = np.full((1, 4, 32), mask_id, np.int32)
        allm[0, 1, 3], allm[0, 2, 9], allm[0, 3, 30] = 5, 6, 7
        tok2 = wl.tokens.copy()
        tok2[0, wl.block_off:wl.block_off + 32] = mask_id
        B.odb_prefill(model, cache, cuda_i32(tok2), wl.resp_off)
        cs, as_, us = (t.cpu().numpy()[0] for t in B.odb_block_step_shared(model, cache, cuda_i32(allm), wl.block_off, 32, wl.tau))
        cp, ap, up = (t.cpu().numpy()[0] for t in B.odb_block_step(model, cache, cuda_i32(allm), wl.block_off, wl.tau))
        assert np.allclose(np.log(cs[0]), np.log(cp[0]), atol=2e-2) and (as_[0] == ap[0]).mean() >= 0.9
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


def test_full_size_properties_without_an_oracle():
    """Properties that hold at any size (ODB-dLLM Sec. 2.1, Sec. 4.2), on the benchmarked 32-layer model:
    the generator matches sampled slices of the oracle's, a step on the unchanged block reproduces the
    refresh, drafts do not see each other, repeated calls are bit-identical."""
    from oracle import odb_oracle as o
    shape = W.MODEL_SHAPES["8b"]
    wl = W.config2()
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        d = shape["d_model"]
        for tid, layer, n in ((o.T_WO, 17, d * d), (o.T_WQ, 31, d * d), (o.T_WU, 3, d * shape["d_ff"])):
            got = B.odb_model_get_tensor(model, tid, layer, n)
            for start in (0, n // 3 + 5, n - 4096):
                ref = o.normal_bf16_bits(W.WEIGHT_SEED, tid, layer, start, 4096, W.WEIGHT_STD)
                gs = got[start:start + 4096]
                big = np.abs(B.bf16_bits_to_f32(ref)) >= 2.0 ** -16      # exact in the library's binary16 storage
                assert np.array_equal(gs[big], ref[big]), (tid, layer, start)
                assert np.all(np.abs(B.bf16_bits_to_f32(gs[~big]) - B.bf16_bits_to_f32(ref[~big])) <= 2.0 ** -24)
        L = wl.tokens.shape[1]
        cache = B.odb_cache_create(model, 1, L)
        tok = cuda_i32(wl.tokens)
        conf_p, am_p = B.odb_prefill(model, cache, tok, wl.resp_off)
        dr = cuda_i32(wl.drafts)
        conf, am, um = B.odb_block_step(model, cache, dr, wl.block_off, wl.tau)
        off = wl.block_off - wl.resp_off
        # draft 0 is the block as it stood at the refresh: cached step == full recompute up to bf16 noise
        assert torch.allclose(torch.log(conf[0, 0]), torch.log(conf_p[0, off:off + 32]), atol=0.15)
        assert (am[0, 0] == am_p[0, off:off + 32]).float().mean() > 0.8
        perm = [3, 1, 0, 2]
        c2, a2, u2 = B.odb_block_step(model, cache, dr[:, perm].contiguous(), wl.block_off, wl.tau)
        assert torch.equal(c2, conf[:, perm]) and torch.equal(a2, am[:, perm]) and torch.equal(u2, um[:, perm])
        c3, a3, u3 = B.odb_block_step(model, cache, dr, wl.block_off, wl.tau)
        assert torch.equal(c3, conf) and torch.equal(a3, am) and torch.equal(u3, um)
        assert um.sum().item() == 4 and (um.sum(-1) == 1).all()
        # two and three drafts run through other GEMM variants (64 rows: the 33..64-row kernels); drafts are
        # independent, so their results must agree with the four-draft call up to summation order
        for S in (2, 3):
            cS, aS, uS = B.odb_block_step(model, cache, dr[:, :S].contiguous(), wl.block_off, wl.tau)
            assert torch.allclose(torch.log(cS), torch.log(conf[:, :S]), atol=0.05), S
            assert (aS == am[:, :S]).float().mean() > 0.9 and (uS.sum(-1) == 1).all(), S
            cR, aR, uR = B.odb_block_step(model, cache, dr[:, :S].contiguous(), wl.block_off, wl.tau)
            assert torch.equal(cR, cS) and torch.equal(aR, aS) and torch.equal(uR, uS), S      # K-split projections: fixed order
        # five and six drafts (160 and 192 rows: two row blocks on the tile kernel, the LM head and, at 192 rows, the wide
        # projections on the 256-row kernel with part of a block empty)
        for pick in ([0, 1, 2, 3, 0], [0, 1, 2, 3, 0, 1]):
            cS, aS, uS = B.odb_block_step(model, cache, dr[:, pick].contiguous(), wl.block_off, wl.tau)
            assert torch.allclose(torch.log(cS), torch.log(conf[:, pick]), atol=0.05), len(pick)
            assert (aS == am[:, pick]).float().mean() > 0.9 and (uS.sum(-1) == 1).all(), len(pick)
            assert torch.equal(cS[:, 0], cS[:, 4]) and torch.equal(aS[:, 0], aS[:, 4]), len(pick)     # the same draft twice
        # one draft (32 rows): its down projection splits K over four workgroups and the last to arrive adds the
        # partial sums - in slice order, so repeated calls must agree bit for bit whoever arrives last
        c1, a1, u1 = B.odb_block_step(model, cache, dr[:, :1].contiguous(), wl.block_off, wl.tau)
        assert torch.allclose(torch.log(c1), torch.log(conf[:, :1]), atol=0.05) and (a1 == am[:, :1]).float().mean() > 0.9
        for _ in range(5):
            cr, ar, ur = B.odb_block_step(model, cache, dr[:, :1].contiguous(), wl.block_off, wl.tau)
            assert torch.equal(cr, c1) and torch.equal(ar, a1) and torch.equal(ur, u1)
        # a block of 16 (one row tile) against the same draft four times over (64 rows: other kernels throughout)
        d16 = dr[:, :1, :16].contiguous()
        c16, a16, u16 = B.odb_block_step(model, cache, d16, wl.block_off, wl.tau)
        c64, a64, u64 = B.odb_block_step(model, cache, d16.repeat(1, 4, 1).contiguous(), wl.block_off, wl.tau)
        assert torch.isfinite(c16).all() and (c16 > 0).all() and (c16 <= 1).all()
        assert torch.allclose(torch.log(c64), torch.log(c16).expand(-1, 4, -1), atol=0.05)
        assert (a64 == a16.expand(-1, 4, -1)).float().mean() > 0.9 and torch.equal(c64[:, 0], c64[:, 3])
        # seven copies (112 rows: seven of the eight row tiles of the 128-row kernels, the last one a repeat of the seventh)
        c112, a112, u112 = B.odb_block_step(model, cache, d16.repeat(1, 7, 1).contiguous(), wl.block_off, wl.tau)
        assert torch.allclose(torch.log(c112), torch.log(c16).expand(-1, 7, -1), atol=0.05)
        assert (a112 == a16.expand(-1, 7, -1)).float().mean() > 0.9 and torch.equal(c112[:, 0], c112[:, 6])
        assert torch.equal(u112[:, 0], u112[:, 6])
        B.odb_model_status(model)
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


def test_config4_at_its_real_lengths_against_stored_oracle():
    """Config 4 as bench.py times it (batch 4, 2048 prompt + 1024 response positions, block of 64, S = 8: 2048 step
    rows against 3008 cached keys per sequence) at the full 8B width with two layers.  Sequences and drafts are
    independent, so the stored oracle outputs of the refresh of sequences 0 and 3 (K/V at sampled positions) and
    of drafts 0 and 7 of sequence 0 and draft 3 of sequence 3 pin the whole call."""
    path = os.path.join(GOLDEN, "config4_oracle_2L.npz")
    if not os.path.exists(path):
        pytest.skip("config4_oracle_2L.npz has not been generated (tests/golden/make_8b_golden.py config4)")
    g = np.load(path)
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=int(g["n_layers"]))
    wl = W.config4()
    assert wl.block_off == int(g["block_off"])
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        Bn, L = wl.tokens.shape
        cache = B.odb_cache_create(model, Bn, L)
        B.odb_prefill(model, cache, cuda_i32(wl.tokens), L - 64)
        for bi in g["seqs"]:
            for layer in range(shape["n_layers"]):
                for kv, name in ((0, "k"), (1, "v")):
                    got = B.odb_cache_read(cache, layer, kv, int(bi), 0, L, 32, 128)[g["kv_pos"]]
                    err = np.abs(got - g["%s_sample_%d" % (name, bi)][layer]).max() / g["%s_absmax_%d" % (name, bi)][layer]
                    assert err <= KV_TOL, "config4: cache seq %d layer %d %s: %.3g" % (bi, layer, name, err)
        d = cuda_i32(wl.drafts)
        tau = float(g["tau"])
        z_all = B.odb_block_step_logits(model, cache, d, wl.block_off, shape["vocab"])
        conf, am, um = (t.cpu().numpy() for t in B.odb_block_step(model, cache, d, wl.block_off, tau))
        B.odb_model_status(model)
        for i, (bi, s_) in enumerate(g["picks"]):
            view = {k[len("p%d_" % i):]: g[k] for k in g.files if k.startswith("p%d_" % i)}
            view = {"step_" + k: v for k, v in view.items()}
            view["step_logit_cols"] = g["logit_cols"]
            z = z_all[bi, s_].cpu().numpy()
            e, rel, ns, n = check_rows(z, conf[bi, s_], am[bi, s_], view, "step", "config4 seq %d draft %d" % (bi, s_))
            assert np.array_equal(um[bi, s_], view["step_unmask"]), "unmask of sequence %d draft %d" % (bi, s_)
            print("\nconfig4 seq %d draft %d: logit err rel %.2e (%d/%d rows strict)" % (bi, s_, rel, ns, n))
        # the other drafts and sequences: finite, one forced pick each (random weights never reach tau)
        assert np.isfinite(conf).all() and (conf > 0).all() and (um.sum(-1) == (wl.drafts == shape["mask_id"]).any(-1)).all()
        del z_all
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


@pytest.mark.parametrize("gain", [8, 16])
def test_peaked_configs_1_and_2_assert_the_decision_bar_as_stated(gain):
    """Configs 1 and 2 at the full 8B width (two layers) with the final-norm gain at 8 / 16, where confidences
    straddle tau = 0.9 and most rows have a top-2 probability margin above 1e-2: argmax and unmask are asserted
    against the stored oracle on every such row, literally, in the refresh, the four-draft step and the one-draft
    step, and the counts of rows the bar bound on must not be zero."""
    path = os.path.join(GOLDEN, "config12_peaked_oracle_2L.npz")
    if not os.path.exists(path):
        pytest.skip("config12_peaked_oracle_2L.npz has not been generated (tests/golden/make_8b_golden.py peaked)")
    g0 = np.load(path)
    tag = "g%d_" % gain
    g = {k[len(tag):]: g0[k] for k in g0.files if k.startswith(tag)}
    g["step_logit_cols"] = g0["step_logit_cols"]
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=int(g0["n_layers"]))
    wl = W.config2()
    tau = float(g0["tau"])
    model = B.odb_model_create(shape)
    LITERAL.update(argmax_rows=0, unmask_positions=0)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        B.odb_model_set_tensor(model, B.T_GF, 0, np.full(shape["d_model"], {8: 0x4100, 16: 0x4180}[gain], np.uint16))
        cache = B.odb_cache_create(model, 1, wl.tokens.shape[1])
        tok = cuda_i32(wl.tokens)
        zp = B.odb_prefill_logits(model, cache, tok, wl.resp_off, shape["vocab"]).cpu().numpy()[0]
        conf_p, am_p = (t.cpu().numpy()[0] for t in B.odb_prefill(model, cache, tok, wl.resp_off))
        check_rows(zp, conf_p, am_p, g, "prefill", "peaked %d refresh" % gain)
        n_refresh = LITERAL["argmax_rows"]
        d = cuda_i32(wl.drafts)
        z = B.odb_block_step_logits(model, cache, d, wl.block_off, shape["vocab"]).cpu().numpy()[0]
        conf, am, um = (t.cpu().numpy()[0] for t in B.odb_block_step(model, cache, d, wl.block_off, tau))
        e, rel, ns, n = check_rows(z, conf, am, g, "step", "peaked %d step" % gain)
        check_unmask_literal(um, wl.drafts[0], g, "step", tau, shape["mask_id"], "peaked %d step" % gain)
        n_step = LITERAL["argmax_rows"] - n_refresh
        # config 1: draft 0 alone (32 rows: the few-row kernels)
        z1 = B.odb_block_step_logits(model, cache, d[:, :1].contiguous(), wl.block_off, shape["vocab"]).cpu().numpy()[0]
        c1, a1, u1 = (t.cpu().numpy()[0] for t in B.odb_block_step(model, cache, d[:, :1].contiguous(), wl.block_off, tau))
        g1 = {k: (v[:1] if k.startswith("step_") and getattr(v, "ndim", 0) >= 2 else v) for k, v in g.items()}
        check_rows(z1, c1, a1, g1, "step", "peaked %d one-draft step" % gain)
        check_unmask_literal(u1, wl.drafts[0][:1], g1, "step", tau, shape["mask_id"], "peaked %d one-draft step" % gain)
        B.odb_model_status(model)
        print("\npeaked gain %d: logit err rel %.2e; decision bar asserted as stated on %d refresh rows, %d + %d step rows, "
              "%d unmask positions; oracle step confidences %.3g .. %.3g" % (
                  gain, rel, n_refresh, n_step, LITERAL["argmax_rows"] - n_refresh - n_step, LITERAL["unmask_positions"],
                  g["step_conf"].min(), g["step_conf"].max()))
        assert n_refresh > 0 and n_step > 0 and LITERAL["unmask_positions"] > 0
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)
