"""GPU parity of the generation loop (odb_generate) against the oracle, in lock step.

A generation run is a chain of decisions, and one decision inside the numerical error band may
legitimately fall the other way and change everything after it.  So the run is not compared with
an independent oracle run as a whole.  Instead the library records the token sequence and the
candidates after every forward, and the test replays each forward with the oracle *from the
library's own state before it*.  Every decision of the oracle that is clear of the error band (a
position's greedy token and threshold test, the forced pick, the controller's choice of draft,
the cut, the ranking of the next candidates) must be the library's too, bit for bit; for the
others only the invariants are checked.  If every decision of every forward was clear, the run
must equal the oracle's own generate() from start to end.
"""
import numpy as np
import pytest

from oracle import odb_oracle as o
from paper_2511_21759_amd import binding as B
from paper_2511_21759_amd import workloads as W

from test_gpu_parity import Pair, cuda_i32, LOGIT_TOL, TAU_BAND

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def conf_bounds(conf, err):
    """Interval that the confidence of a row can reach when every logit moves by at most err and the greedy
    token stays: conf = 1 / (1 + sum_j exp(z_j - z_max)) and each difference moves by at most 2 err."""
    conf = np.asarray(conf, np.float64)
    s = (1.0 - conf) / conf
    return 1.0 / (1.0 + s * np.exp(2 * err)) - 1e-6, 1.0 / (1.0 + s * np.exp(-2 * err)) + 1e-6


def rows_clear(z, conf, tau, err):
    """Per row: the greedy token and the threshold decision survive a logit error of err."""
    if z.shape[0] == 0:
        return np.zeros(0, bool)
    part = np.partition(z, -2, axis=-1)
    lo, hi = conf_bounds(conf, err)
    return (part[:, -1] - part[:, -2] > 2 * err) & ((tau < lo) | (tau > hi)) & (np.abs(conf - tau) > TAU_BAND)


def ranking_clear(conf_masked, k, err):
    """The k most confident entries are separated from each other and from the rest by more than the band."""
    c = np.sort(np.asarray(conf_masked, np.float64))[::-1]
    lo, hi = conf_bounds(c, err)
    return all(lo[i] > hi[i + 1] for i in range(min(k, len(c) - 1)))


def draft_clear(tokens, z, conf, tau, mask_id, err):
    """Per position of one forwarded draft (tokens / z / conf over the same rows): True where the position is
    decoded already, or where what the forward decides there (greedy token, threshold, forced pick) is clear."""
    m = tokens == mask_id
    ok = np.ones(len(tokens), bool)
    ok[m] = rows_clear(z[m], conf[m], tau, err)
    lo, hi = conf_bounds(conf, err)
    if m.any() and not (lo[m] > tau).any() and not ranking_clear(conf[m], 1, err):
        ok &= ~(m & (hi >= lo[m].max()))                       # one of these is the forced pick, which one is open
    return ok


def replay(p, prompt, R, gp, events, snaps, err):
    """-> (forwards whose every decision was compared, positions compared bit-exactly, positions decided)."""
    cfg, w, mask = p.cfg, p.w, p.cfg.mask_id
    P, b, tau = len(prompt), gp["block_len"], gp["tau"]
    eos = gp.get("eos_id", -1)
    n_cand = 4 if gp["n_drafts"] == 8 else 2
    pre = np.concatenate([prompt, np.full(R, mask, np.int32)])
    L, cp, ct, cache = P + R, None, None, None
    n_clear = n_cmp = n_dec = 0
    for n, (e, post) in enumerate(zip(events, snaps)):
        off, bb, tag = e["block_off"], e["block_len"], "event %d (%s)" % (n, e["kind"])
        all_clear = True
        if e["kind"] == "refresh":
            cache, conf, am, z = o.prefill(cfg, w, pre[:L], P, return_logits=True)
            if eos >= 0:
                new_len = o.predict_length(pre[:L], conf, am, P, mask, eos, gp["truncate_thr"])
                m = pre[P:L] == mask
                top2 = np.argsort(z, axis=-1)[:, -2:]
                near = m & (top2 == eos).any(-1)                  # rows whose attempt is, or could flip to, [EOS]
                part = np.partition(z[near], -2, axis=-1)
                lo, hi = conf_bounds(conf[near], err)
                len_clear = not np.any(part[:, -1] - part[:, -2] <= 2 * err) and \
                    not np.any((lo <= gp["truncate_thr"]) & (gp["truncate_thr"] <= hi))
                if len_clear:
                    assert e["L"] == new_len, "%s: length %d, oracle %d" % (tag, e["L"], new_len)
                all_clear &= len_clear
            else:
                assert e["L"] == L, tag
            assert P < e["L"] <= L and np.array_equal(post[:off], pre[:off]), tag
            L = e["L"]
            cache = o.truncate_cache(cache, L)
            assert bb == max(0, min(b, L - off)), tag
            if bb == 0:
                assert n == len(events) - 1, "a cut into decoded territory ends generation"
                continue
            blk, c_b, a_b = pre[off:off + bb], conf[off - P:off - P + bb], am[off - P:off - P + bb]
            um = o.threshold_unmask(blk, c_b, tau, mask)
            new = np.where(um == 1, a_b, blk).astype(np.int32)
            pos, tok = o.speculative_candidates(new, c_b, a_b, mask, k=n_cand)
            ok = draft_clear(blk, z[off - P:off - P + bb], c_b, tau, mask, err)
            want_chosen, chosen_clear, c_ch = 0, True, c_b
        else:
            blk = pre[off:off + bb]
            m = blk == mask
            share = gp["n_drafts"] >= 4 and gp.get("share_from", -1) >= 0 and int((~m).sum()) >= gp["share_from"]
            assert e["kind"] == ("shared" if share else "step") and e["L"] == L and bb == min(b, L - off), tag
            # (eight blocks only in the decoded-share stage; the steps before it forward the first four)
            S_step = gp["n_drafts"] if share else 4
            if share and S_step == 8 and gp.get("row_budget", 0) > 0 and bb + 7 * int(m.sum()) > gp["row_budget"]:
                S_step = 4                                  # eight blocks would not fit the row budget
            drafts = blk[None] if gp["n_drafts"] == 1 else o.speculative_drafts(blk, cp, ct, S_step)
            if share:
                conf, am, um, zs = o.block_step_shared(cfg, w, cache, drafts, off, tau, return_logits=True)
                rows = [np.arange(bb)] + [np.flatnonzero(m)] * (len(drafts) - 1)
            else:
                conf, am, um, zs = o.block_step(cfg, w, cache, drafts, off, tau, return_logits=True)
                rows = [np.arange(bb)] * len(drafts)
            oks = []
            for s in range(len(drafts)):
                full = np.ones(bb, bool)
                full[rows[s]] = draft_clear(drafts[s][rows[s]], zs[s], conf[s][rows[s]], tau, mask, err)
                oks.append(full)
            if gp["n_drafts"] == 1:
                want_chosen, chosen_clear = 0, True
                new = np.where(um[0] == 1, am[0], blk).astype(np.int32)
                pos, tok = o.speculative_candidates(new, conf[0], am[0], mask)
            elif gp["n_drafts"] == 4:
                want_chosen, new, pos, tok, _ = o.accept_jump(drafts, conf, am, um, cp, ct, mask)
                # the controller looks at candidate B in block_0 and block_2, at candidate D in block_0 and block_1
                looks = [(0, cp[0]), (2, cp[0]), (0, cp[1]), (1, cp[1])]
                chosen_clear = all(oks[s][q] for s, q in looks if q >= 0)
            else:
                want_chosen, new, pos, tok, _ = o.speculative_jump(drafts, conf, am, um, cp, ct, mask, 8)
                # the walk may look at any candidate in any block that does not hold it already
                chosen_clear = all(oks[s][q] for s in range(len(drafts)) for q in cp[:len(drafts) // 2] if q >= 0)
            ok, c_ch = oks[want_chosen], conf[want_chosen]
        # invariants, whatever the margins
        got = post[off:off + bb]
        assert np.array_equal(post[:off], pre[:off]) and np.array_equal(post[off + bb:L], pre[off + bb:L]), tag
        assert np.array_equal(got[blk != mask], blk[blk != mask]), "%s: a decoded position changed" % tag
        assert e["n_masked"] == int((got == mask).sum()) < int((blk == mask).sum()), "%s: no progress" % tag
        assert len(e["cand_pos"]) == n_cand, tag
        for j in range(n_cand):
            q = e["cand_pos"][j]
            assert q == -1 or (0 <= q < bb and got[q] == mask), "%s: candidate on a decoded position" % tag
        real = [q for q in e["cand_pos"] if q >= 0]
        assert len(set(real)) == len(real) == min(n_cand, e["n_masked"]), tag
        # decisions, where they are clear of the error band
        n_dec += int((blk == mask).sum())
        if chosen_clear:
            assert e["chosen"] == want_chosen, "%s: adopted draft %d, oracle %d" % (tag, e["chosen"], want_chosen)
        if e["chosen"] == want_chosen:
            sel = ok & (blk == mask)
            assert np.array_equal(got[sel], new[sel]), "%s: block after the forward" % tag
            n_cmp += int(sel.sum())
            if ok.all() and ranking_clear(c_ch[new == mask], n_cand, err):
                assert np.array_equal(e["cand_pos"], pos) and np.array_equal(e["cand_tok"], tok), "%s: candidates" % tag
                n_clear += all_clear and chosen_clear
        pre, cp, ct = post.copy(), e["cand_pos"], e["cand_tok"]
    return n_clear, n_cmp, n_dec


def run_case(p, seed, P, R, gp, pick_eos=None):
    rng = np.random.default_rng(seed)
    cfg = p.cfg
    prompt = rng.integers(0, cfg.vocab - 1, P).astype(np.int32)
    start = np.concatenate([prompt, np.full(R, cfg.mask_id, np.int32)])
    # the error band: measured on the first refresh's logits, with a factor two of room for the later forwards
    cache = p.cache(1, P + R)
    _, conf0, am0, z0 = o.prefill(cfg, p.w, start, P, return_logits=True)
    zg = B.odb_prefill_logits(p.model, cache, cuda_i32(start[None]), P, cfg.vocab).cpu().numpy()[0]
    assert np.abs(zg - z0).max() <= LOGIT_TOL * np.abs(z0).max()
    err = 2 * float(np.abs(zg - z0).max())
    part0 = np.partition(z0, -2, axis=-1)
    print("\nerror band %.3g on logits of magnitude %.3g; median top-2 gap of the first attempt %.3g" % (
        err, np.abs(z0).max(), np.median(part0[:, -1] - part0[:, -2])))
    gp = dict(gp)
    if pick_eos:
        lo, hi = pick_eos
        q = lo + int(np.argmax(conf0[lo:hi]))
        gp["eos_id"], gp["truncate_thr"] = int(am0[q]), float(conf0[q]) * 0.9
    tokens = cuda_i32(start)
    tokens[P:] = 0                                       # the call writes the MASKs itself
    stats, events, snaps = B.odb_generate(p.model, cache, tokens, P, max_events=P + R + 8, event_tokens=True, **gp)
    snaps = snaps.cpu().numpy()
    final = tokens.cpu().numpy()[:stats["final_len"]]
    assert stats["n_events"] == len(events) == stats["n_refresh"] + stats["n_step"]
    assert not (final == cfg.mask_id).any() and np.array_equal(final[:P], prompt)
    assert np.array_equal(final, snaps[-1][:stats["final_len"]]) and B.odb_cache_length(cache) == stats["final_len"]
    kinds = [e["kind"] for e in events]
    assert stats["n_refresh"] == kinds.count("refresh") and stats["n_step_shared"] == kinds.count("shared")
    assert stats["refresh_positions"] == (P + R) + sum(events[i - 1]["L"] for i in range(1, len(events))
                                                       if kinds[i] == "refresh")
    n_clear, n_cmp, n_dec = replay(p, prompt, R, gp, events, snaps, err)
    og = o.GenParams(block_len=gp["block_len"], n_drafts=gp["n_drafts"], tau=gp["tau"],
                     eos_id=gp["eos_id"] if gp.get("eos_id", -1) >= 0 else None,
                     truncate_thr=gp.get("truncate_thr", 0.9),
                     share_from=gp["share_from"] if gp.get("share_from", -1) >= 0 else None,
                     row_budget=gp["row_budget"] if gp.get("row_budget", 0) > 0 else None)
    if n_clear == len(events):
        t_o, s_o, e_o = o.generate(cfg, p.w, prompt, R, og)
        assert np.array_equal(final, t_o), "every forward was clear of the error band, yet the runs differ"
        for k in ("n_refresh", "n_step", "n_step_shared", "refresh_positions", "step_rows", "final_len"):
            assert stats[k] == s_o[k], k
    return stats, events, (n_clear, n_cmp, n_dec)


# Weights for these runs: with the usual normal(0, 0.02) every MASK position of an undecoded response looks
# alike (confidences within 3 % of each other, far inside the error band) and the run would test nothing but
# ties.  Four times that scale makes attention position-dependent: the first attempt's confidences spread
# from 0.45 to 0.99 around the threshold and a dozen different tokens are attempted.
GEN_STD, GEN_GF = 0.08, 8.0

CASES = [
    # seed, P, R, params, eos window in the response (None: no length prediction)
    (1, 64, 96, dict(block_len=32, n_drafts=1, tau=0.9), None),
    (2, 64, 96, dict(block_len=32, n_drafts=4, tau=0.9), None),
    (3, 48, 128, dict(block_len=32, n_drafts=4, tau=0.9, share_from=16), (40, 100)),
    (4, 30, 50, dict(block_len=20, n_drafts=4, tau=0.8, share_from=0), None),
    (5, 40, 70, dict(block_len=48, n_drafts=1, tau=0.7), (20, 60)),
    (6, 32, 128, dict(block_len=64, n_drafts=4, tau=0.9, share_from=32), None),      # the largest block the shared step takes
    (7, 20, 130, dict(block_len=128, n_drafts=4, tau=0.85), None),                    # blocks longer than a wave, a two-position tail
    # eight blocks in the decoded-share stage (Sec. 4.2.2's four extra candidates), after four-draft steps / from the start
    (8, 48, 96, dict(block_len=32, n_drafts=8, tau=0.9, share_from=8), None),
    (9, 40, 80, dict(block_len=32, n_drafts=8, tau=0.85, share_from=0), (30, 70)),
    (10, 24, 128, dict(block_len=64, n_drafts=8, tau=0.9, share_from=24), None),
    (11, 40, 96, dict(block_len=32, n_drafts=8, tau=0.9, share_from=4, row_budget=128), None),       # eight blocks once they fit 128 rows
]


@pytest.mark.parametrize("seed,P,R,gp,pick_eos", CASES)
def test_generate_in_lock_step_with_the_oracle(seed, P, R, gp, pick_eos):
    p = Pair(W.MODEL_SHAPES["tiny"], std=GEN_STD, gf=GEN_GF)
    try:
        stats, events, (n_clear, n_cmp, n_dec) = run_case(p, seed, P, R, gp, pick_eos)
        chosen = sorted(set(e["chosen"] for e in events))
        print("\ngenerate %s: %d refreshes + %d steps (%d shared) for %d positions, final length %d, drafts adopted %s; "
              "%d of %d forwards compared in every decision, %d of %d position decisions compared bit-exactly" % (
                  gp, stats["n_refresh"], stats["n_step"], stats["n_step_shared"], R, stats["final_len"], chosen,
                  n_clear, len(events), n_cmp, n_dec))
        assert n_cmp >= 0.7 * n_dec, "too few decisions were clear of the error band to be compared bit-exactly"
        if pick_eos:
            assert stats["final_len"] < P + R, "the case is built so that the first refresh cuts the response"
    finally:
        p.close()


def test_generate_errors_and_truncate():
    p = Pair(W.MODEL_SHAPES["tiny"])
    try:
        cache = p.cache(1, 96)
        tok = torch.zeros(96, dtype=torch.int32, device="cuda")
        for kw in (dict(block_len=0), dict(block_len=300), dict(block_len=16, n_drafts=2), dict(block_len=16, n_drafts=8),
                   dict(block_len=128, n_drafts=8, share_from=4),
                   dict(block_len=128, n_drafts=4, share_from=4), dict(block_len=16, eos_id=p.cfg.mask_id),
                   dict(block_len=16, eos_id=p.cfg.vocab)):
            with pytest.raises(B.OdbError):
                B.odb_generate(p.model, cache, tok, 32, **kw)
        with pytest.raises(B.OdbError):
            B.odb_generate(p.model, cache, tok, 96, block_len=16)            # no response
        with pytest.raises(B.OdbError):
            B.odb_generate(p.model, p.cache(2, 96), tok, 32, block_len=16)   # batch 2
        with pytest.raises(B.OdbError):
            B.odb_generate(p.model, p.cache(1, 64), tok, 32, block_len=16)   # cache too short
        with pytest.raises(B.OdbError):
            B.odb_cache_truncate(cache, 1)                                   # nothing cached yet
        B.odb_prefill(p.model, cache, tok[None, :80].contiguous(), 40)
        B.odb_cache_truncate(cache, 50)
        assert B.odb_cache_length(cache) == 50
        for bad in (0, 51):
            with pytest.raises(B.OdbError):
                B.odb_cache_truncate(cache, bad)
    finally:
        p.close()


def test_truncated_cache_equals_the_oracle_on_the_kept_keys():
    """odb_cache_truncate followed by a step: the dropped positions are no longer keys (Sec. 4.1)."""
    p = Pair(W.MODEL_SHAPES["tiny"], gf=32.0)
    try:
        wl = W.decode_workload(p.shape, 64, 96, 32, 2, W.WEIGHT_SEED + 21)
        cache = p.cache(1, wl.tokens.shape[1])
        B.odb_prefill(p.model, cache, cuda_i32(wl.tokens), wl.resp_off)
        oc, *_ = o.prefill(p.cfg, p.w, wl.tokens[0], wl.resp_off)
        new_len = wl.block_off + 32 + 13                                    # ragged: not a multiple of the key tile
        B.odb_cache_truncate(cache, new_len)
        dg = cuda_i32(wl.drafts)
        z = B.odb_block_step_logits(p.model, cache, dg, wl.block_off, p.cfg.vocab).cpu().numpy()[0]
        _, _, _, z_o = o.block_step(p.cfg, p.w, o.truncate_cache(oc, new_len), wl.drafts[0], wl.block_off, 0.9,
                                    return_logits=True)
        _, _, _, z_full = o.block_step(p.cfg, p.w, oc, wl.drafts[0], wl.block_off, 0.9, return_logits=True)
        e_cut = np.abs(z - z_o).max() / np.abs(z_o).max()
        assert e_cut <= LOGIT_TOL and np.abs(z - z_full).max() > 10 * np.abs(z - z_o).max()
    finally:
        p.close()


@pytest.mark.parametrize("ND", [4, 8])
def test_generate_at_full_width_equals_the_composed_calls(ND):
    """8B width (d = 4096, F = 12288, V = 126464; 2 layers), where the oracle is too slow to replay a run: every
    forward of odb_generate must equal, bit for bit, what the separately tested entry points give on the state
    before it (odb_prefill / odb_block_step / odb_block_step_shared / odb_accept_jump or, with eight blocks,
    odb_speculative_jump, and the acceptance rule and candidate choice restated on the host from the library's
    own confidences)."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        B.odb_model_set_tensor(model, B.T_GF, 0, np.full(shape["d_model"], 0x4100, np.uint16))      # gain 8
        mask, P, R, b, tau, SHARE = shape["mask_id"], 100, 150, 32, 0.9, 16
        rng = np.random.default_rng(77)
        prompt = rng.integers(0, shape["vocab"] - 1, P).astype(np.int32)
        cache = B.odb_cache_create(model, 1, P + R)
        tokens = cuda_i32(np.concatenate([prompt, np.zeros(R, np.int32)]))
        # an [EOS] the first refresh attempts with confidence, two thirds into the response
        c0, a0 = B.odb_prefill(model, cache, cuda_i32(np.concatenate([prompt, np.full(R, mask, np.int32)])[None]), P)
        c0, a0 = c0.cpu().numpy()[0], a0.cpu().numpy()[0]
        late = [i for i in range(90, 130) if a0[i] not in a0[:90]]           # attempted nowhere earlier
        q = max(late, key=lambda i: c0[i])
        eos, thr = int(a0[q]), float(c0[q]) * 0.9
        stats, events, snaps = B.odb_generate(model, cache, tokens, P, block_len=b, n_drafts=ND, tau=tau, eos_id=eos,
                                              truncate_thr=thr, share_from=SHARE, max_events=400, event_tokens=True)
        snaps = snaps.cpu().numpy()
        assert stats["n_events"] == len(events) and stats["final_len"] < P + R
        final = tokens.cpu().numpy()[:stats["final_len"]]
        assert not (final == mask).any() and np.array_equal(final[:P], prompt)
        pre = np.concatenate([prompt, np.full(R, mask, np.int32)])
        L, cp, ct, kinds = P + R, None, None, set()
        for n, (e, post) in enumerate(zip(events, snaps)):
            off, bb, tag = e["block_off"], e["block_len"], "event %d (%s)" % (n, e["kind"])
            kinds.add(e["kind"])
            if e["kind"] == "refresh":
                seq = cuda_i32(pre[None, :L])
                conf_t, am_t = B.odb_prefill(model, cache, seq, P)
                new_len = int(B.odb_predict_length(model, seq, conf_t, am_t, P, eos, thr).cpu().numpy()[0])
                conf, am = conf_t.cpu().numpy()[0], am_t.cpu().numpy()[0]
                assert e["L"] == new_len, tag
                L = new_len
                B.odb_cache_truncate(cache, L)
                assert bb == max(0, min(b, L - off)), tag
                if bb == 0:
                    continue
                blk, c_b, a_b = pre[off:off + bb], conf[off - P:off - P + bb], am[off - P:off - P + bb]
                new = np.where(o.threshold_unmask(blk, c_b, np.float32(tau), mask) == 1, a_b, blk).astype(np.int32)
                pos, tok = o.speculative_candidates(new, c_b, a_b, mask, k=ND // 2)
                chosen = 0
            else:
                blk = pre[off:off + bb]
                share = int((blk != mask).sum()) >= SHARE
                assert e["kind"] == ("shared" if share else "step"), tag
                drafts = cuda_i32(o.speculative_drafts(blk, cp, ct, ND if share else 4)[None])
                if share:
                    out = B.odb_block_step_shared(model, cache, drafts, off, int((blk == mask).sum()), tau)
                else:
                    out = B.odb_block_step(model, cache, drafts, off, tau)
                if ND == 4:
                    ch, nd, npos, ntok = B.odb_accept_jump(model, drafts, *out, cuda_i32(cp[None]), cuda_i32(ct[None]))
                else:
                    ch, nd, npos, ntok = B.odb_speculative_jump(model, drafts, *out, cuda_i32(cp[None]), cuda_i32(ct[None]), 8)
                chosen, new = int(ch.cpu().numpy()[0]), nd.cpu().numpy()[0, 0]
                pos, tok = npos.cpu().numpy()[0], ntok.cpu().numpy()[0]
            assert e["chosen"] == chosen and np.array_equal(post[off:off + bb], new), tag
            assert np.array_equal(e["cand_pos"], pos) and np.array_equal(e["cand_tok"], tok), tag
            assert np.array_equal(post[:off], pre[:off]) and np.array_equal(post[off + bb:L], pre[off + bb:L]), tag
            pre, cp, ct = post.copy(), e["cand_pos"], e["cand_tok"]
        print("\nfull-width generate (%d blocks): %d refreshes + %d steps (%d shared), final length %d of %d, adopted %s" % (
            ND, stats["n_refresh"], stats["n_step"], stats["n_step_shared"], stats["final_len"], P + R,
            sorted(set(e["chosen"] for e in events))))
        assert kinds == {"refresh", "step", "shared"}, "the case must run all three kinds of forward (ran %s)" % kinds
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)
