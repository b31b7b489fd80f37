#!/usr/bin/env python3
"""Benchmark of the block-decode step and the cache-refresh prefill.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|config1|config2|config3|config4|...]

One "step" is one pass of the whole hot path over one batch of synthetic input:
odb_block_step on the 8B-shaped model against a prefilled cache (config1: S=1,
config2: S=4, config4: batch 4, S=8) or odb_prefill (config3, L=1024).  Inputs,
weights and the cache are resident in HBM before the timed region starts.

The default, `--workload all`, times config 2 (the paper's operating point: block_0
plus three speculative blocks, 128 rows per weight read) as the headline - `value`,
`ms_per_step`, `roofline` - with exactly K timed steps, and then configs 1, 3 and 4
the same way (at most 20 steps each); their records are in `config.also`.  The other
workloads (config2_jump, config2_shared, config3_chain, generate) are run one at a time.
Prints ONE JSON line.  Everything runs on one GPU; --gpus above 1 is refused.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0   # dense binary16 and bfloat16 MFMA share this peak

# rocprofv3 summaries of the same commands, tracked beside this script: the kernel-trace average of the dominant
# kernel and its HBM traffic per launch are read from there (they cannot be taken while this script times)
PROFILE_FILES = {"config1": "profiles/decode_step_config1_kernels.md", "config2": "profiles/decode_step_config2_kernels.md",
                 "config3": "profiles/prefill_config3_kernels.md", "config4": "profiles/decode_step_config4_kernels.md"}


def weight_bytes(shape):
    d, f, v, nl = shape["d_model"], shape["d_ff"], shape["vocab"], shape["n_layers"]
    per_layer = (3 * d * d + d * d + 2 * f * d + d * f) * 2
    return per_layer, per_layer * nl + v * d * 2


def kv_bytes_per_pos(shape):
    return shape["n_layers"] * 2 * shape["d_model"] * 2


def step_flops(shape, rows, keys_per_row):
    d, f, v, nl = shape["d_model"], shape["d_ff"], shape["vocab"], shape["n_layers"]
    gemm = 2 * rows * (nl * (4 * d * d + 3 * d * f) + v * d)
    attn = nl * 4 * rows * keys_per_row * d
    return gemm + attn


def profile_figures(name):
    """(average microseconds of the gate/up kernel in the tracked rocprofv3 kernel trace of this workload, its
    measured HBM bytes per launch from the tracked counter runs, the file) - None where the file has no such row."""
    rel = PROFILE_FILES.get(name)
    path = os.path.join(ROOT, rel) if rel else None
    if not path or not os.path.exists(path):
        return None, None, rel
    avg_us = traffic = None
    best_calls = best_disp = -1
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 6 or "EpiSwiGLU" not in cells[0]:
            continue
        try:
            nums = [float(c) for c in cells[1:]]
        except ValueError:
            continue
        # (the gate/up kernel of the timed steps is the row with the most launches; the set-up's refresh has its own)
        if len(cells) == 8 and nums[1] > best_calls:          # kernel | workgroups | calls | avg us | min | max | total ms | %
            best_calls, avg_us = nums[1], nums[2]
        elif len(cells) == 6 and nums[0] > best_disp:         # kernel | dispatches | fetch KiB | write KiB | read MB | write MB
            best_disp, traffic = nums[0], (nums[3] + nums[4]) * 1e6
    return avg_us, traffic, rel


def cpu_baseline_step(shape, wl, seed, std):
    """Times the oracle on a bounded sample of the step: ONE transformer layer (of
    n_layers) plus the LM head at full width on all rows of sequence 0, and scales
    the layer time by n_layers."""
    import numpy as np
    from oracle import odb_oracle as o
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    one = dict(shape, n_layers=1)
    cfg = o.Config(**one)
    w = o.Weights(cfg, seed, std)
    for tid in (o.T_WQ, o.T_WK, o.T_WV, o.T_WO, o.T_WG, o.T_WU, o.T_WD, o.T_LM):
        w.bits(tid, 0)                                   # generation is not part of the step
    S, b = wl.drafts.shape[1:]
    L = wl.tokens.shape[1]
    rng = np.random.default_rng(0)
    cache = o.Cache(rng.standard_normal((1, L, cfg.n_heads, cfg.head_dim)),
                    rng.standard_normal((1, L, cfg.n_heads, cfg.head_dim)))
    h = rng.standard_normal((S * b, cfg.d_model))
    t_lh, t_h, reps, t_start = [], [], 0, time.perf_counter()
    while reps < 3 or (time.perf_counter() - t_start < 12.0 and reps < 40):     # about 12 s of CPU work
        t0 = time.perf_counter()
        o.block_step(cfg, w, cache, wl.drafts[0], wl.block_off, wl.tau)
        t_lh.append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        o.confidence_argmax(o._head(cfg, w, h))
        t_h.append(time.perf_counter() - t0)
        reps += 1
    t_head = float(np.median(t_h))
    t_layer = max(float(np.median(t_lh)) - t_head, 1e-9)
    t_full = shape["n_layers"] * t_layer + t_head
    rows = wl.drafts.shape[0] * S * b
    return {"value": rows / (t_full * wl.drafts.shape[0]), "unit": "rows/s", "cores": int(cores), "kind": "oracle",
            "sample": "1 of %d layers + LM head at full width, all %d rows of sequence 0, float64, median of %d "
                      "repetitions (%.1f s of CPU work); layer time x%d (%.2fs layer, %.2fs head)" % (
                          shape["n_layers"], S * b, reps, time.perf_counter() - t_start, shape["n_layers"], t_layer,
                          t_head)}


def bench_generate(args, model, shape, B, W, np, torch):
    """Whole generations (ODB-dLLM Sec. 2.1 with Sec. 4.2 on): 256 prompt tokens, 256 response positions in
    blocks of 32, at the 8B shape.  Random weights never reach tau = 0.9, so the final norm gain is raised to
    8 (as in the parity tests' peaked variants): confidences then straddle the threshold.  Four decoders are
    timed on the same prompt: threshold only, accept-jump, accept-jump with the decoded-share stage from 20
    decoded positions on, and the same with eight blocks in that stage (Sec. 4.2.2's four extra candidates; from
    20 decoded positions on an eight-block step has at most 32 + 7 * 12 = 116 rows and stays within the kernels
    for up to 128 rows).
    No [EOS] is defined for synthetic weights, so length prediction stays off."""
    P, R, b = 256, 256, 32
    B.odb_model_set_tensor(model, B.T_GF, 0, np.full(shape["d_model"], 0x4100, np.uint16))     # bf16(8.0)
    rng = np.random.default_rng(W.WEIGHT_SEED + 31)
    prompt = torch.from_numpy(rng.integers(0, shape["vocab"] - 1, P).astype(np.int32)).cuda()
    cache = B.odb_cache_create(model, 1, P + R)
    modes = {"threshold": dict(n_drafts=1), "accept_jump": dict(n_drafts=4),
             "jump_share": dict(n_drafts=4, share_from=20), "jump_share8": dict(n_drafts=8, share_from=20, row_budget=128)}
    res = {}
    for mode, kw in modes.items():
        runs = []
        for it in range(args.warmup + args.steps):
            tokens = torch.zeros(P + R, dtype=torch.int32, device="cuda")
            tokens[:P] = prompt
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st, _, _ = B.odb_generate(model, cache, tokens, P, block_len=b, tau=0.9, **kw)
            torch.cuda.synchronize()
            st["wall_ms"] = (time.perf_counter() - t0) * 1e3
            if it >= args.warmup:
                runs.append(st)
        ms = float(np.mean([r["wall_ms"] for r in runs]))
        r0 = runs[0]
        res[mode] = {"ms_per_generation": ms, "positions_per_s": R / (ms * 1e-3), "n_refresh": r0["n_refresh"],
                     "n_step": r0["n_step"], "n_step_shared": r0["n_step_shared"],
                     "forwards": r0["n_refresh"] + r0["n_step"], "step_rows": r0["step_rows"],
                     "refresh_ms": float(np.mean([r["refresh_ms"] for r in runs])),
                     "step_ms": float(np.mean([r["step_ms"] for r in runs])),
                     "refresh_share_of_time": float(np.mean([r["refresh_ms"] / r["total_ms"] for r in runs]))}
    best = min((res["jump_share"], res["jump_share8"]), key=lambda r: r["ms_per_generation"])
    best_name = "jump_share" if best is res["jump_share"] else "jump_share8"
    out = {"metric": "generated positions/s, whole block-wise generation (8B shape, peaked synthetic weights)",
           "value": best["positions_per_s"], "unit": "positions/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": best["ms_per_generation"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": "generate: %d prompt + %d response positions, blocks of %d, tau 0.9, final norm gain 8; "
                                  "value is the faster accept-jump + decoded-share decoder (%s)" % (P, R, b, best_name),
                      "decoders": res},
           "roofline": None, "cpu_baseline": None}
    print(json.dumps(out))
    B.odb_cache_destroy(cache)
    B.odb_model_destroy(model)


class Setup:
    """One workload, ready to run: run() issues one step on torch's current stream."""

    def __init__(self, name, args, model, shape, B, W, np, torch):
        self.name, self.extra, self.wl, self.caches = name, {}, None, []
        per_layer_w, total_w = weight_bytes(shape)
        d = shape["d_model"]
        if name == "config3_chain":
            # Adaptive length prediction (ODB-dLLM Sec. 4.1) shortens the response from refresh to refresh.  With
            # random weights no [EOS] is ever confident, so the three lengths of config 3 are imposed and the
            # scan runs for its cost only ([EOS] id 2, threshold 0.9: the paper prints neither).
            toks = [torch.from_numpy(W.config3(r)).cuda() for r in (512, 256, 128)]
            self.caches = [B.odb_cache_create(model, 1, t.shape[1]) for t in toks]
            outs = [(torch.empty((1, t.shape[1] - 512), dtype=torch.float32, device="cuda"),
                     torch.empty((1, t.shape[1] - 512), dtype=torch.int32, device="cuda"),
                     torch.empty((1,), dtype=torch.int32, device="cuda")) for t in toks]

            def run():
                for t, c, (cf, am, nl) in zip(toks, self.caches, outs):
                    B.odb_prefill(model, c, t, 512, cf, am)
                    B.odb_predict_length(model, t, cf, am, 512, 2, 0.9, nl)
            self.run = run
            self.rows = sum(t.shape[1] for t in toks)
            self.rows_per_launch = self.rows / 3.0
            self.flops = sum(step_flops(shape, t.shape[1], t.shape[1]) - 2 * 512 * shape["vocab"] * d for t in toks)
            self.alg_bytes = 3 * total_w + self.rows * kv_bytes_per_pos(shape)
            self.label = "three cache refreshes of 1024, 768 and 640 positions, each with the length-prediction scan, 8B shape"
            self.unit, self.bound = "tokens/s", "mfma"
        elif name == "config3":
            tokens = torch.from_numpy(W.config3(args.resp)).cuda()
            Bn, L = tokens.shape
            cache = B.odb_cache_create(model, Bn, L)
            self.caches = [cache]
            conf = torch.empty((Bn, L - 512), dtype=torch.float32, device="cuda")
            am = torch.empty((Bn, L - 512), dtype=torch.int32, device="cuda")
            self.run = lambda: B.odb_prefill(model, cache, tokens, 512, conf, am)
            self.rows = self.rows_per_launch = Bn * L
            self.flops = step_flops(shape, self.rows, L) - 2 * Bn * 512 * shape["vocab"] * d   # LM head on response rows only
            self.alg_bytes = total_w + self.rows * kv_bytes_per_pos(shape)
            self.label = "cache-refresh prefill, 8B shape, 512 prompt + %d MASK, batch 1" % args.resp
            self.unit, self.bound = "tokens/s", "mfma"
        else:
            wl = {"config0": W.config0, "config1": W.config1, "config2": W.config2, "config2_jump": W.config2,
                  "config2_shared": W.config2_shared, "config4": W.config4}[name]()
            self.wl = wl
            Bn, L = wl.tokens.shape
            S, b = wl.drafts.shape[1:]
            cache = B.odb_cache_create(model, Bn, L)
            self.caches = [cache]
            tok = torch.from_numpy(wl.tokens).cuda()
            B.odb_prefill(model, cache, tok, wl.resp_off)
            drafts = torch.from_numpy(wl.drafts).cuda()
            conf = torch.empty((Bn, S, b), dtype=torch.float32, device="cuda")
            am = torch.empty((Bn, S, b), dtype=torch.int32, device="cuda")
            um = torch.empty((Bn, S, b), dtype=torch.uint8, device="cuda")
            self.run = lambda: B.odb_block_step(model, cache, drafts, wl.block_off, wl.tau, conf, am, um)
            if name == "config2_jump":
                # config 2's four drafts followed by the accept-jump controller (ODB-dLLM Sec. 4.2.1), which adopts a
                # draft and builds the next four on the device; the candidates are the two positions that drafts 1
                # and 2 of the workload unmask.  Timed with fixed inputs: one iteration of the loop.
                d0 = wl.drafts[0]
                cpos = [int(np.flatnonzero(d0[s] != d0[0])[0]) if (d0[s] != d0[0]).any() else -1 for s in (1, 2)]
                cand_pos = torch.tensor([cpos], dtype=torch.int32, device="cuda")
                cand_tok = torch.tensor([[int(d0[1][cpos[0]]) if cpos[0] >= 0 else 0,
                                          int(d0[2][cpos[1]]) if cpos[1] >= 0 else 0]], dtype=torch.int32, device="cuda")

                def run():
                    B.odb_block_step(model, cache, drafts, wl.block_off, wl.tau, conf, am, um)
                    B.odb_accept_jump(model, drafts, conf, am, um, cand_pos, cand_tok)
                self.run = run
            self.rows = Bn * S * b
            if name == "config2_shared":
                # decoded-share stage (ODB-dLLM Sec. 4.2.2): eight blocks, the speculative ones reduced to the still
                # masked positions; the plain eight-draft step on the same drafts is timed beside it
                n_masked = int((wl.drafts[:, 0] == shape["mask_id"]).sum(-1).max())
                plain = self.run
                for _ in range(3):
                    plain()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(10):
                    plain()
                torch.cuda.synchronize()
                self.extra = {"plain_8_draft_step_ms": (time.perf_counter() - t0) * 100.0, "n_masked": n_masked,
                              "rows_plain": self.rows}
                self.run = lambda: B.odb_block_step_shared(model, cache, drafts, wl.block_off, n_masked, wl.tau, conf, am, um)
                self.rows = Bn * (b + (S - 1) * n_masked)
            self.rows_per_launch = self.rows
            self.flops = step_flops(shape, self.rows, L)
            self.alg_bytes = total_w + Bn * (L - b) * kv_bytes_per_pos(shape)
            self.label = "block-decode step, %s shape, cache L=%d, block b=%d, S=%d drafts, batch %d" % (
                "tiny" if name == "config0" else "8B", L, b, S, Bn)
            self.unit = "rows/s"
            self.bound = "mfma" if name == "config4" else "hbm"     # config 4: 1600 flop per byte, far beyond the ridge
        torch.cuda.synchronize()
        self.B = B

    def close(self):
        for c in self.caches:
            self.B.odb_cache_destroy(c)


def measure(su, model, shape, steps, warmup, B, torch):
    """Times `steps` calls of su.run() after `warmup` untimed ones; then a second, instrumented pass over the same
    steps brackets every launch of the dominant kernel (the gate/up projection) with HIP events on the launch stream."""
    d, f = shape["d_model"], shape["d_ff"]
    for _ in range(warmup):
        su.run()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        su.run()
    ev1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ms_gpu = ev0.elapsed_time(ev1) / steps
    # An event pair also spans the dispatch latency after its start marker, which back-to-back launches hide and a
    # profiler's kernel trace does not count: the event-pair figure is a little pessimistic next to the rocprofv3
    # average of the same kernel, which is quoted beside it from the tracked profile.
    prof = B.odb_profile_kernel(model, su.run, steps)
    gu_bytes = 2 * f * d * 2 + su.rows_per_launch * d * 2 + su.rows_per_launch * f * 2
    gu_flops = 2 * su.rows_per_launch * 2 * f * d
    avg_s = prof["avg_ms"] * 1e-3
    trace_us, traffic, prof_file = profile_figures(su.name)
    if su.bound == "mfma":
        ach, peak, unit, alg = gu_flops / avg_s / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s", gu_flops
        step_frac = su.flops / (ms * 1e-3) / 1e12 / peak
    else:
        ach, peak, unit, alg = gu_bytes / avg_s / 1e9, HBM_PEAK_GBS, "GB/s", gu_bytes
        step_frac = su.alg_bytes / (ms * 1e-3) / 1e9 / peak
    roofline = {"bound": su.bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak, "traffic": traffic,
                "kernel": prof["kernel"], "launches": prof["launches"], "avg_us": prof["avg_ms"] * 1e3,
                "empty_pair_us": prof["avg_empty_pair_ms"] * 1e3, "algorithmic_per_launch": alg,
                # the same kernel in the tracked rocprofv3 kernel trace, and the fraction that duration gives
                "kernel_trace_avg_us": trace_us,
                "frac_kernel_trace": (alg / (trace_us * 1e-6) / (1e12 if su.bound == "mfma" else 1e9) / peak) if trace_us else None,
                "kernel_trace_source": prof_file,
                # the whole step against the same roof: all algorithmic bytes (or flops) of the step / step time
                "whole_step_frac": step_frac}
    return {"workload": "%s: %s" % (su.name, su.label), "rows_per_step": su.rows, "steps": steps, "warmup": warmup,
            "ms_per_step": ms, "ms_per_step_gpu_events": ms_gpu, "value": su.rows / (ms * 1e-3), "unit": su.unit,
            "steps_per_s": 1e3 / ms,
            "step_hbm": {"algorithmic_bytes": su.alg_bytes, "achieved_GBps": su.alg_bytes / (ms * 1e-3) / 1e9,
                         "frac_of_8TBps": su.alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "step_mfma": {"flops": su.flops, "achieved_TFLOPps": su.flops / (ms * 1e-3) / 1e12,
                          "frac_of_2.5PFLOPps": su.flops / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS},
            "roofline": roofline, **su.extra}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    choices=["all", "config0", "config1", "config2", "config2_jump", "config2_shared", "config3",
                             "config3_chain", "config4", "generate"])
    ap.add_argument("--resp", type=int, default=512, help="response length for config3 (512, 256 or 128)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region also run three 1 GiB device-to-device copies (a kernel of known "
                         "traffic, used to scale the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_21759_amd import binding as B
    from paper_2511_21759_amd import workloads as W

    if not os.path.exists(B.LIB_PATH):
        from paper_2511_21759_amd.build import build_library
        build_library()
    torch.cuda.set_device(0)
    name = args.workload
    shape = W.MODEL_SHAPES["tiny" if name == "config0" else "8b"]
    model = B.odb_model_create(shape)
    B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)

    if name == "generate":
        return bench_generate(args, model, shape, B, W, np, torch)

    head_name = "config2" if name == "all" else name
    su = Setup(head_name, args, model, shape, B, W, np, torch)
    head = measure(su, model, shape, args.steps, args.warmup, B, torch)
    wl = su.wl
    su.close()
    also = {}
    if name == "all":
        for other in ("config1", "config3", "config4"):
            so = Setup(other, args, model, shape, B, W, np, torch)
            also[other] = measure(so, model, shape, min(args.steps, 20), min(args.warmup, 3), B, torch)
            so.close()
    B.odb_model_status(model)       # no activation left the binary16 range in any of the timed calls

    cfg = {"workload": head["workload"], "rows_per_step": head["rows_per_step"], "steps_per_s": head["steps_per_s"]}
    cfg.update({k: v for k, v in head.items() if k in ("plain_8_draft_step_ms", "n_masked", "rows_plain")})
    if also:
        cfg["also"] = also
    out = {
        "metric": "block-decode tokens/s (8B shape, S drafts); achieved HBM GB/s vs peak"
                  if wl is not None else "cache-refresh prefill tokens/s; achieved bf16 TFLOP/s vs MFMA peak",
        "value": head["value"], "unit": head["unit"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "ms_per_step_gpu_events": head["ms_per_step_gpu_events"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": cfg, "step_hbm": head["step_hbm"], "step_mfma": head["step_mfma"], "roofline": head["roofline"],
    }
    if wl is not None and not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_step(shape, wl, W.WEIGHT_SEED, W.WEIGHT_STD)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))
    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    B.odb_model_destroy(model)


if __name__ == "__main__":
    main()
