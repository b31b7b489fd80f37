"""Writes tests/golden/config12_oracle.npz: the CPU oracle's outputs for the
8B-shaped decode workloads (config1: S=1, config2: S=4 drafts; same cache).

Calls only the oracle and the seeded workload generator; nothing here touches
the HIP library.  Takes the better part of an hour on 8 cores and ~25 GB of RAM
(the oracle widens every weight to float64 on use), which is why its outputs are
stored instead of being recomputed inside the GPU tests.

    python tests/golden/make_8b_golden.py [n_layers]   (n_layers defaults to 32)
    python tests/golden/make_8b_golden.py batch4       (config4_small_oracle_2L.npz: batch 4, S=8, b=64, 2 layers)
    python tests/golden/make_8b_golden.py prefill      (config3_oracle_2L.npz: the 1024- and 640-position refreshes, 2 layers)
    python tests/golden/make_8b_golden.py shared       (config2_shared_oracle_2L.npz: the eight-block decoded-share step, 2 layers)
    python tests/golden/make_8b_golden.py prefill256   (config3_r256_oracle_2L.npz: the 768-position refresh, 2 layers)
    python tests/golden/make_8b_golden.py config4      (config4_oracle_2L.npz: batch 4, L = 3072, S = 8, b = 64 at its real
                                                        lengths, 2 layers: sequence 0 drafts 0 and 7, sequence 3 draft 3)
    python tests/golden/make_8b_golden.py peaked       (config12_peaked_oracle_2L.npz: configs 1 / 2 with final-norm gain 8
                                                        and 16, so that confidences straddle tau and margins exceed 1e-2)
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import odb_oracle as o                       # noqa: E402
from paper_2511_21759_amd import workloads as W          # noqa: E402


def main():
    n_layers = int(sys.argv[1]) if len(sys.argv) > 1 else 32
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=n_layers)
    cfg = o.Config(**shape)
    w = o.Weights(cfg, W.WEIGHT_SEED, W.WEIGHT_STD, keep=True)
    wl = W.config2()
    assert np.array_equal(wl.tokens, W.config1().tokens) and np.array_equal(wl.drafts[0, :1], W.config1().drafts[0])
    t0 = time.time()
    cache, conf_p, am_p, z_p = o.prefill(cfg, w, wl.tokens[0], wl.resp_off, return_logits=True)
    print("prefill done %.0fs" % (time.time() - t0), flush=True)
    conf, am, um, z = o.block_step(cfg, w, cache, wl.drafts[0], wl.block_off, wl.tau, return_logits=True)
    print("step done %.0fs" % (time.time() - t0), flush=True)
    rng = np.random.default_rng(123)
    cols = np.sort(rng.choice(cfg.vocab, 256, replace=False))
    top = np.argsort(z, axis=-1)[..., -8:]
    top_p = np.argsort(z_p, axis=-1)[..., -8:]
    layers = sorted(set([0, n_layers // 2, n_layers - 1]))
    pos = np.sort(rng.choice(wl.tokens.shape[1], 48, replace=False))
    out = dict(
        n_layers=n_layers, tau=wl.tau, block_off=wl.block_off,
        step_conf=conf, step_argmax=am, step_unmask=um,
        step_logit_cols=cols, step_logits_sample=z[..., cols].astype(np.float32),
        step_top_ids=top.astype(np.int32), step_top_logits=np.take_along_axis(z, top, -1).astype(np.float32),
        step_logit_absmax=np.abs(z).max(), step_lse=np.log(np.exp(z - z.max(-1, keepdims=True)).sum(-1)) + z.max(-1),
        prefill_conf=conf_p, prefill_argmax=am_p,
        prefill_logits_sample=z_p[..., cols].astype(np.float32),
        prefill_top_ids=top_p.astype(np.int32),
        prefill_top_logits=np.take_along_axis(z_p, top_p, -1).astype(np.float32),
        prefill_logit_absmax=np.abs(z_p).max(),
        kv_layers=np.array(layers), kv_pos=pos,
        k_sample=cache.k[layers][:, pos].astype(np.float32), v_sample=cache.v[layers][:, pos].astype(np.float32),
        k_absmax=np.abs(cache.k[layers]).max(axis=(1, 2, 3)), v_absmax=np.abs(cache.v[layers]).max(axis=(1, 2, 3)),
    )
    name = "config12_oracle.npz" if n_layers == 32 else "config12_oracle_%dL.npz" % n_layers
    np.savez_compressed(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), **out)
    print("wrote", name, "%.0fs" % (time.time() - t0), flush=True)


def main_batch4():
    """Config 4's structure at the 8B width with 2 layers: sequences 0 and 3 of the batch of four."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    cfg = o.Config(**shape)
    w = o.Weights(cfg, W.WEIGHT_SEED, W.WEIGHT_STD, keep=True)
    wl = W.config4_small()
    rng = np.random.default_rng(321)
    cols = np.sort(rng.choice(cfg.vocab, 128, replace=False))
    pos = np.sort(rng.choice(wl.tokens.shape[1], 32, replace=False))
    seqs = [0, 3]
    out = dict(n_layers=2, tau=wl.tau, block_off=wl.block_off, seqs=np.array(seqs), logit_cols=cols, kv_pos=pos)
    t0 = time.time()
    acc = {k: [] for k in ("step_conf", "step_argmax", "step_unmask", "step_logits_sample", "step_top_ids",
                           "step_top_logits", "step_logit_absmax", "prefill_conf", "prefill_argmax",
                           "prefill_top_ids", "prefill_top_logits", "prefill_logits_sample", "prefill_logit_absmax",
                           "k_sample", "v_sample", "k_absmax", "v_absmax")}
    for bi in seqs:
        cache, conf_p, am_p, z_p = o.prefill(cfg, w, wl.tokens[bi], wl.resp_off, return_logits=True)
        conf, am, um, z = o.block_step(cfg, w, cache, wl.drafts[bi], wl.block_off, wl.tau, return_logits=True)
        print("sequence %d done %.0fs" % (bi, time.time() - t0), flush=True)
        top = np.argsort(z, axis=-1)[..., -8:]
        top_p = np.argsort(z_p, axis=-1)[..., -8:]
        acc["step_conf"].append(conf); acc["step_argmax"].append(am); acc["step_unmask"].append(um)
        acc["step_logits_sample"].append(z[..., cols].astype(np.float32))
        acc["step_top_ids"].append(top.astype(np.int32))
        acc["step_top_logits"].append(np.take_along_axis(z, top, -1).astype(np.float32))
        acc["step_logit_absmax"].append(np.abs(z).max())
        acc["prefill_conf"].append(conf_p); acc["prefill_argmax"].append(am_p)
        acc["prefill_top_ids"].append(top_p.astype(np.int32))
        acc["prefill_top_logits"].append(np.take_along_axis(z_p, top_p, -1).astype(np.float32))
        acc["prefill_logits_sample"].append(z_p[..., cols].astype(np.float32))
        acc["prefill_logit_absmax"].append(np.abs(z_p).max())
        acc["k_sample"].append(cache.k[:, pos].astype(np.float32)); acc["v_sample"].append(cache.v[:, pos].astype(np.float32))
        acc["k_absmax"].append(np.abs(cache.k).max(axis=(1, 2, 3))); acc["v_absmax"].append(np.abs(cache.v).max(axis=(1, 2, 3)))
    out.update({k: np.stack(v) for k, v in acc.items()})
    name = "config4_small_oracle_2L.npz"
    np.savez_compressed(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), **out)
    print("wrote", name, "%.0fs" % (time.time() - t0), flush=True)


def main_prefill(resps=(512, 128), name="config3_oracle_2L.npz", seed=654):
    """Config 3 (cache-refresh prefill, 512 prompt + 512 / 256 / 128 MASK positions) at the 8B width with 2 layers."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    cfg = o.Config(**shape)
    w = o.Weights(cfg, W.WEIGHT_SEED, W.WEIGHT_STD, keep=True)
    rng = np.random.default_rng(seed)
    cols = np.sort(rng.choice(cfg.vocab, 128, replace=False))
    out = dict(n_layers=2, logit_cols=cols, resp_lens=np.array(resps))
    t0 = time.time()
    for resp in resps:
        tokens = W.config3(resp)[0]
        pos = np.sort(rng.choice(tokens.shape[0], 32, replace=False))
        cache, conf, am, z = o.prefill(cfg, w, tokens, 512, return_logits=True)
        top = np.argsort(z, axis=-1)[..., -8:]
        tag = "r%d_" % resp
        out.update({tag + "kv_pos": pos, tag + "prefill_conf": conf, tag + "prefill_argmax": am,
                    tag + "prefill_logits_sample": z[..., cols].astype(np.float32),
                    tag + "prefill_top_ids": top.astype(np.int32),
                    tag + "prefill_top_logits": np.take_along_axis(z, top, -1).astype(np.float32),
                    tag + "prefill_logit_absmax": np.abs(z).max(),
                    tag + "k_sample": cache.k[:, pos].astype(np.float32), tag + "v_sample": cache.v[:, pos].astype(np.float32),
                    tag + "k_absmax": np.abs(cache.k).max(axis=(1, 2, 3)), tag + "v_absmax": np.abs(cache.v).max(axis=(1, 2, 3))})
        print("response %d done %.0fs" % (resp, time.time() - t0), flush=True)
    np.savez_compressed(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), **out)
    print("wrote", name, "%.0fs" % (time.time() - t0), flush=True)


def main_shared():
    """The decoded-share step of bench.py's config2_shared workload (eight blocks, a quarter of block_0 still MASK)
    at the 8B width with 2 layers.  Per computed row (block, position): confidence, argmax, unmask, the eight
    largest logits and 128 sampled columns; rows that are not computed keep NaN / -1."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    cfg = o.Config(**shape)
    w = o.Weights(cfg, W.WEIGHT_SEED, W.WEIGHT_STD, keep=True)
    wl = W.config2_shared()
    rng = np.random.default_rng(987)
    cols = np.sort(rng.choice(cfg.vocab, 128, replace=False))
    t0 = time.time()
    cache, _, _ = o.prefill(cfg, w, wl.tokens[0], wl.resp_off)
    drafts = wl.drafts[0]
    S, b = drafts.shape
    conf, am, um, zs = o.block_step_shared(cfg, w, cache, drafts, wl.block_off, wl.tau, return_logits=True)
    masked = np.flatnonzero(drafts[0] == cfg.mask_id)
    top_ids = np.full((S, b, 8), -1, np.int32)
    top_logits = np.full((S, b, 8), np.nan, np.float32)
    sample = np.full((S, b, 128), np.nan, np.float32)
    absmax = 0.0
    for s in range(S):
        rows = np.arange(b) if s == 0 else masked
        z = zs[s]
        if z.shape[0] == 0:
            continue
        top = np.argsort(z, axis=-1)[:, -8:]
        top_ids[s, rows] = top
        top_logits[s, rows] = np.take_along_axis(z, top, -1)
        sample[s, rows] = z[:, cols]
        absmax = max(absmax, float(np.abs(z).max()))
    name = "config2_shared_oracle_2L.npz"
    np.savez_compressed(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), n_layers=2, tau=wl.tau,
                        block_off=wl.block_off, logit_cols=cols, step_conf=conf, step_argmax=am, step_unmask=um,
                        step_top_ids=top_ids, step_top_logits=top_logits, step_logits_sample=sample,
                        step_logit_absmax=absmax, n_masked=masked.size)
    print("wrote", name, "%.0fs" % (time.time() - t0), flush=True)


def _row_record(z, cols):
    top = np.argsort(z, axis=-1)[..., -8:]
    return dict(logits_sample=z[..., cols].astype(np.float32), top_ids=top.astype(np.int32),
                top_logits=np.take_along_axis(z, top, -1).astype(np.float32), logit_absmax=np.abs(z).max())


def main_config4():
    """Config 4 at its real lengths (batch 4, 2048 prompt + 1024 response positions, block of 64, S = 8) at the 8B
    width with 2 layers.  Sequences and drafts are independent, so a subset pins the whole call: the refresh of
    sequences 0 and 3 (K/V at sampled positions), then drafts 0 and 7 of sequence 0 and draft 3 of sequence 3."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    cfg = o.Config(**shape)
    w = o.Weights(cfg, W.WEIGHT_SEED, W.WEIGHT_STD, keep=True)
    wl = W.config4()
    L = wl.tokens.shape[1]
    rng = np.random.default_rng(4321)
    cols = np.sort(rng.choice(cfg.vocab, 128, replace=False))
    pos = np.sort(rng.choice(L, 48, replace=False))
    picks = [(0, 0), (0, 7), (3, 3)]
    out = dict(n_layers=2, tau=wl.tau, block_off=wl.block_off, logit_cols=cols, kv_pos=pos, picks=np.array(picks),
               seqs=np.array([0, 3]))
    t0 = time.time()
    caches = {}
    for bi in (0, 3):
        # (only the cache is needed from the refresh: the LM head runs on the last position alone)
        caches[bi], _, _ = o.prefill(cfg, w, wl.tokens[bi], L - 1)
        out["k_sample_%d" % bi] = caches[bi].k[:, pos].astype(np.float32)
        out["v_sample_%d" % bi] = caches[bi].v[:, pos].astype(np.float32)
        out["k_absmax_%d" % bi] = np.abs(caches[bi].k).max(axis=(1, 2, 3))
        out["v_absmax_%d" % bi] = np.abs(caches[bi].v).max(axis=(1, 2, 3))
        print("refresh of sequence %d done %.0fs" % (bi, time.time() - t0), flush=True)
    for i, (bi, s) in enumerate(picks):
        conf, am, um, z = o.block_step(cfg, w, caches[bi], wl.drafts[bi, s:s + 1], wl.block_off, wl.tau, return_logits=True)
        rec = _row_record(z[0], cols)
        out.update({"p%d_conf" % i: conf[0], "p%d_argmax" % i: am[0], "p%d_unmask" % i: um[0]})
        out.update({"p%d_%s" % (i, k): v for k, v in rec.items()})
        print("sequence %d draft %d done %.0fs" % (bi, s, time.time() - t0), flush=True)
    name = "config4_oracle_2L.npz"
    np.savez_compressed(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), **out)
    print("wrote", name, "%.0fs" % (time.time() - t0), flush=True)


def main_peaked():
    """Configs 1 / 2 (same tokens and drafts) at the 8B width with 2 layers and the final-norm gain at 8 and 16: with
    normal(0, 0.02) weights every probability is about 1 / V, so neither tau = 0.9 nor the 1e-2 margin of the
    decision bar ever binds; the scaled gain (a power of two, exact in bf16) makes them bind."""
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    cfg = o.Config(**shape)
    w = o.Weights(cfg, W.WEIGHT_SEED, W.WEIGHT_STD, keep=True)
    wl = W.config2()
    rng = np.random.default_rng(246)
    cols = np.sort(rng.choice(cfg.vocab, 128, replace=False))
    out = dict(n_layers=2, tau=wl.tau, block_off=wl.block_off, step_logit_cols=cols, gains=np.array([8.0, 16.0]))
    t0 = time.time()
    for gf in (8.0, 16.0):
        w.set_values(o.T_GF, 0, np.full(cfg.d_model, gf, np.float32))
        cache, conf_p, am_p, z_p = o.prefill(cfg, w, wl.tokens[0], wl.resp_off, return_logits=True)
        conf, am, um, z = o.block_step(cfg, w, cache, wl.drafts[0], wl.block_off, wl.tau, return_logits=True)
        tag = "g%d_" % int(gf)
        out.update({tag + "step_conf": conf, tag + "step_argmax": am, tag + "step_unmask": um,
                    tag + "prefill_conf": conf_p, tag + "prefill_argmax": am_p})
        out.update({tag + "step_" + k: v for k, v in _row_record(z, cols).items()})
        out.update({tag + "prefill_" + k: v for k, v in _row_record(z_p, cols).items()})
        print("gain %g done %.0fs: step conf min %.3g median %.3g max %.3g" % (
            gf, time.time() - t0, conf.min(), np.median(conf), conf.max()), flush=True)
    name = "config12_peaked_oracle_2L.npz"
    np.savez_compressed(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), **out)
    print("wrote", name, "%.0fs" % (time.time() - t0), flush=True)


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "shared":
        main_shared()
    elif len(sys.argv) > 1 and sys.argv[1] == "prefill256":
        main_prefill((256,), "config3_r256_oracle_2L.npz", 655)
    elif len(sys.argv) > 1 and sys.argv[1] == "config4":
        main_config4()
    elif len(sys.argv) > 1 and sys.argv[1] == "peaked":
        main_peaked()
    elif len(sys.argv) > 1 and sys.argv[1] == "prefill":
        main_prefill()
    elif len(sys.argv) > 1 and sys.argv[1] == "batch4":
        main_batch4()
    else:
        main()
