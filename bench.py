#!/usr/bin/env python3
"""Benchmark of one Clover-2 speculative step (draft_tree -> verify_tree -> accept_and_compact)
on one MI355X.  Prints ONE JSON line.

  python bench.py --gpus 1 --steps K --warmup W [--config 3]

A "step" is one pass of the whole hot path over one batch of synthetic input (weights and KV
cache resident in HBM, prompt prefilled before the timed region).  The default workload is the
LLaMA3-8B-shaped batch-1 configuration (64-node tree over 1024 cached tokens); --config 4 and 5
run the ragged batch-8 and the long-context workloads.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
PREFILL_ROWS = 256           # prompt rows per pass of the prefill call (set-up; outside the timed region)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def layer_params(shape):
    H, d = shape.hidden, shape.head_dim
    nq, nkv, F = shape.n_q_heads, shape.n_kv_heads, shape.ffn
    return {"gemm_qkv": (nq + 2 * nkv) * d * H, "gemm_wo": H * nq * d, "gemm_gate_up": 2 * F * H, "gemm_down": H * F}


def verify_bytes(shape, B, N, L_sum):
    """Algorithmic HBM bytes of one verify_tree: every target weight once (2 bytes each), the
    cached K/V rows read once and the new K/V rows written once at 2 bytes per value (a bf16 cache:
    what the method needs; this library's caches hold a bf16 hi/lo pair, i.e. it moves 4, which is
    its own cost and does not count towards the achieved rate)."""
    weights = 2 * (shape.n_layers * sum(layer_params(shape).values()) + shape.vocab * shape.hidden)
    kv_row = 2 * shape.n_kv_heads * shape.head_dim * 2
    kv_read = shape.n_layers * kv_row * (L_sum + B * N)
    kv_write = shape.n_layers * kv_row * B * N
    return weights + kv_read + kv_write


def draft_bytes(shape, n_levels):
    H = shape.hidden
    w = 3 * H * H + shape.aug_layers * sum(layer_params(shape).values()) + H * H + \
        (n_levels - 1) * (3 * H * H + 2 * H * H) + n_levels * shape.vocab * H
    return 2 * w


def source_fingerprint():
    """sha256 over the kernel sources: a committed profile summary is used only while it was taken from THESE
    sources (it records the fingerprint it was measured with)."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2408_00264_amd", "csrc")
    for n in sorted(os.listdir(csrc)):
        if n.endswith((".hip", ".h")):
            h.update(n.encode())
            h.update(open(os.path.join(csrc, n), "rb").read())
    return h.hexdigest()[:16]


def profile_value(path, key, fingerprint):
    """`key: value` from a committed profile summary, or None when the file is missing, does not carry the key, or
    was measured with other kernel sources than the ones in this tree."""
    try:
        text = open(os.path.join(ROOT, "profiles", path)).read()
    except OSError:
        return None
    vals = {}
    for line in text.splitlines():
        if ":" in line:
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip()
    if vals.get("source_fingerprint") != fingerprint or key not in vals:
        return None
    try:
        return float(vals[key])
    except ValueError:
        return None


def cpu_baseline(shape, parent, rank, L, sample_layers, store, min_seconds):
    """The oracle, as it stands, timed on this host on a bounded sample of the same workload:
    `sample_layers` decoder layers of the verify pass (scaled to all layers), the LM head, the
    acceptance and one full draft_tree, for one sequence with L cached tokens."""
    from oracle import clover2_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    N = len(parent)
    dt = np.float32
    cfg = O.OracleConfig.from_shape(shape, L + 2 * N + 16, dt)
    cfg.n_layers = sample_layers
    W = O.Weights(store.get_f32, dt)
    rng = np.random.default_rng(0)
    seq = O.SeqState(cfg)
    seq.kv.k[:, :L] = rng.standard_normal(seq.kv.k[:, :L].shape, dtype=dt)
    seq.kv.v[:, :L] = rng.standard_normal(seq.kv.v[:, :L].shape, dtype=dt)
    seq.aug_kv.k[:, :L] = rng.standard_normal(seq.aug_kv.k[:, :L].shape, dtype=dt)
    seq.aug_kv.v[:, :L] = rng.standard_normal(seq.aug_kv.v[:, :L].shape, dtype=dt)
    seq.L = seq.aug_L = L
    tokens = rng.integers(0, shape.vocab, N)
    # touch every weight once so conversion to fp32 is outside the timing
    O.verify_tree(W, cfg, seq, tokens[:1], [-1])
    depth = O.tree_depths(parent)
    vis = O.ancestor_matrix(parent)
    t_layers = t_head = t_draft = 0.0
    reps = 0
    t_begin = time.perf_counter()
    while reps < 2 or time.perf_counter() - t_begin < min_seconds:
        t0 = time.perf_counter()
        x = W("embed")[tokens].astype(dt)
        for li in range(sample_layers):
            x = O.decoder_layer(W, f"layers.{li}.", cfg, x, seq.kv, li, L, L + depth, L + np.arange(N), vis)
        t1 = time.perf_counter()
        logits = O.rmsnorm(x, W("final_norm"), cfg.rms_eps) @ W("lm_head").T
        seq.L = L
        acc = O.accept_and_compact(cfg, seq, tokens, logits, x, parent)
        t2 = time.perf_counter()
        seq.L = seq.aug_L = L
        O.draft_tree(W, cfg, seq, acc["hid_acc"], acc["next_tok"], parent, rank)
        t3 = time.perf_counter()
        if reps:                      # the first repetition warms the draft weights and is not counted
            t_layers += t1 - t0; t_head += t2 - t1; t_draft += t3 - t2
        reps += 1
    n = reps - 1
    step_s = t_layers / n * shape.n_layers / sample_layers + t_head / n + t_draft / n
    return {"value": N / step_s, "unit": "tree-tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 sequence, L={L}, {N}-node tree, {n} timed repetitions ({t_layers + t_head + t_draft:.1f}s of "
                      f"CPU work): {sample_layers} of {shape.n_layers} verify layers ({t_layers / n:.2f}s each time, scaled "
                      f"to {shape.n_layers}), LM head + accept ({t_head / n:.2f}s), full draft_tree ({t_draft / n:.2f}s); "
                      f"fp32 NumPy", "est_step_ms": step_s * 1e3}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 4, 5])
    ap.add_argument("--layers", type=int, default=0, help="debug: override the number of target layers")
    ap.add_argument("--prompt", type=int, default=0, help="debug: override the prompt length")
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--library", default="", help="load another build of libclover.so (reported in the JSON line)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib", action="store_true",
                    help="also launch an elementwise kernel that reads 1 GiB and writes 1 GiB (three times), the "
                         "known-size reference for scaling hardware byte counters")
    ap.add_argument("--cpu-sample-layers", type=int, default=8)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time spent on the oracle baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
            "(the speculative step of one sequence batch lives on one device)")
        sys.exit(2)
    # The shipped library reads no environment variable; a tuning build does.  A number measured with a switch set
    # must not pass for the default path: refuse unless another library was named explicitly, and report the set.
    switches = sorted(k for k in os.environ if k.startswith("CLOVER_"))
    if switches and not args.library:
        log(f"bench.py: environment switches {switches} are set; unset them (the shipped library ignores them, a "
            "tuning build named with --library would not)")
        sys.exit(2)

    import torch
    from paper_2408_00264_amd import clover, synth
    if args.library:
        clover.load_library(os.path.abspath(args.library))

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    shape = synth.CONFIGS[args.config]
    if args.layers:
        shape = synth.scaled(shape, n_layers=args.layers)
    if args.prompt:
        shape = synth.scaled(shape, prompt_len=(args.prompt, args.prompt))
    B, N, D = shape.batch, shape.tree_nodes, shape.draft_depths
    parent, rank = synth.tree_for(shape)
    prompts = synth.make_prompts(shape)
    K, Wm = args.steps, args.warmup
    n_passes = 3 * K + Wm + 4
    max_seq = max(len(p) for p in prompts) + n_passes * (D + 1) + 2 * N + 64
    max_seq = (max_seq + 255) // 256 * 256

    t0 = time.time()
    store = synth.WeightStore(shape)
    keep = []
    if not args.no_cpu_baseline:
        sl = min(args.cpu_sample_layers, shape.n_layers)
        keep = [n for n in store.names() if not n.startswith("layers.") or int(n.split(".")[1]) < sl]
    dev_w = clover.upload_weights(store, keep_host=keep)
    log(f"[bench] weights generated and uploaded in {time.time() - t0:.1f}s")
    g = clover.Clover(shape, dev_w, parent, rank, B, max_seq, N, flags=args.flags, prefill_rows=PREFILL_ROWS)
    # set-up (outside the timed region): the prompts go through the library's prefill call, once to warm up and once
    # timed with an event pair around the prefill calls alone; its rate is reported beside the step's figures
    dev_prompts = [torch.from_numpy(np.ascontiguousarray(p, dtype=np.int32)).cuda() for p in prompts]
    for timed in (False, True):
        g.reset()
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pe[0].record()
        for b, t in enumerate(dev_prompts):
            g.prefill_prompt(b, t)
        pe[1].record()
        torch.cuda.synchronize()
    prefill_ms = pe[0].elapsed_time(pe[1])
    g.m.fill_(1)
    g.set_tree(parent, rank)
    g.draft_tree(B)
    torch.cuda.synchronize()
    lens0 = g.seq_len()
    n_prompt = sum(len(p) for p in prompts)
    log(f"[bench] prefill of {[len(p) for p in prompts]} tokens in {prefill_ms:.1f} ms "
        f"({n_prompt / prefill_ms * 1e3:.0f} tokens/s); lengths {lens0[:B].tolist()}")

    def run_steps(n, events=None):
        for i in range(n):
            if events is not None:
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                ev[0].record(); g.verify_tree(B); ev[1].record(); g.accept_and_compact(B); ev[2].record()
                g.draft_tree(B); ev[3].record()
                events.append(ev)
            else:
                g.verify_tree(B); g.accept_and_compact(B); g.draft_tree(B)

    if args.calib:
        ca = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        cb = torch.empty_like(ca)
        for _ in range(3):
            torch.add(ca, 1.0, out=cb)
        torch.cuda.synchronize()
        del ca, cb
    run_steps(Wm)
    torch.cuda.synchronize()
    g.seq_len()
    # ---- timed region: exactly K steps ----
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(K)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    lens1 = g.seq_len()
    # ---- second pass of K steps with one event pair per call (nothing recorded inside the calls) ----
    events = []
    torch.cuda.synchronize()
    run_steps(K, events)
    torch.cuda.synchronize()
    lens2 = g.seq_len()
    # ---- third pass with the library's HIP-event pairs around every kernel class, recorded on the library's own
    # stream (these add gaps between the kernels, so only the per-class sums of this pass are used) ----
    g.profile_enable(True)
    torch.cuda.synchronize()
    run_steps(K)
    torch.cuda.synchronize()
    prof = g.profile_collect()
    g.profile_enable(False)
    g.seq_len()
    ver = np.array([e[0].elapsed_time(e[1]) for e in events])
    acc = np.array([e[1].elapsed_time(e[2]) for e in events])
    dra = np.array([e[2].elapsed_time(e[3]) for e in events])
    L_sum = int(lens1[:B].sum())
    vbytes = verify_bytes(shape, B, N, L_sum)
    dbytes = draft_bytes(shape, D)
    kernels = {k: {"ms_per_step": v[0] / K, "launches_per_step": v[1] / K} for k, v in prof.items() if v[1]}
    ver_med = float(np.median(ver))

    # ---- per kernel class: bytes the class has to move per call and what it reached.  Up to 256 rows go through
    # one launch that streams the weights once (the <= 64-row, the 128-row panel and the 129..256-row tiled kernel);
    # the class timer brackets the whole call, so a class's rate is against ONE pass over its weights. ----
    rows = B * N
    passes = (rows + 255) // 256
    lp = layer_params(shape)
    classes = {}
    for name, params in list(lp.items()) + [("gemm_lm_head", shape.vocab * shape.hidden)]:
        if name in prof and prof[name][1]:
            ms = prof[name][0] / prof[name][1]
            classes[name] = {"weight_bytes": 2 * params, "avg_call_ms": ms, "weight_passes": passes,
                             "GBps": 2 * params / (ms * 1e-3) / 1e9, "frac": 2 * params / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # tree attention: K/V rows of the cached tokens and the tree nodes of one layer; the library's cache holds
    # 4 bytes per value (bf16 hi/lo pair), the method needs 2
    if "tree_attention" in prof and prof["tree_attention"][1]:
        ms = prof["tree_attention"][0] / prof["tree_attention"][1]
        kv_vals = 2 * shape.n_kv_heads * shape.head_dim * (L_sum + B * N)
        classes["tree_attention"] = {"kv_bytes_algorithmic": 2 * kv_vals, "kv_bytes_stored": 4 * kv_vals, "avg_call_ms": ms,
                                     "GBps_algorithmic": 2 * kv_vals / (ms * 1e-3) / 1e9,
                                     "GBps_stored": 4 * kv_vals / (ms * 1e-3) / 1e9,
                                     "frac": 2 * kv_vals / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                     "note": "attention kernel + the merge of its key splits"}

    # dominant kernel: the fused gate/up projection (largest weight stream of a layer); one launch = one pass over
    # both weight matrices for up to 256 rows.  Every product is issued twice (hi and lo activation planes), so the
    # launch sits under the HBM roof up to 2*P_mfma/(4*P_hbm) = 156 rows and under the bf16 MFMA roof above that;
    # the line reports the roof that binds the workload and keeps the other one beside it.
    dom_name = "gemm_gate_up (fused SwiGLU projection, one launch = one pass over both weight matrices)"
    dom_ms, dom_n = prof["gemm_gate_up"]
    dom_bytes = 2 * lp["gemm_gate_up"]
    dom_avg_ms = dom_ms / max(dom_n, 1) / passes
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9 if dom_n else 0.0
    rows_per_launch = (rows + passes - 1) // passes
    issued_tflops = 2 * 2 * rows_per_launch * lp["gemm_gate_up"] / (dom_avg_ms * 1e-3) / 1e12   # hi and lo planes
    fp = source_fingerprint()
    default_workload = not (args.layers or args.prompt or args.library or args.flags)
    traffic = profile_value(f"traffic_gemm_gate_up_config{args.config}.txt", "traffic_bytes_per_launch", fp) \
        if default_workload else None
    trace_us = profile_value(f"spec_step_config{args.config}_kernel_trace.txt", "gate_up_avg_us", fp) \
        if default_workload else None
    hbm_roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS}
    mfma_roof = {"bound": "mfma", "achieved": issued_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": issued_tflops / MFMA_BF16_PEAK_TFLOPS}
    mfma_bound = 4.0 * rows_per_launch / (MFMA_BF16_PEAK_TFLOPS * 1e12) > 2.0 / (HBM_PEAK_GBS * 1e9)
    main_roof, other_roof = (mfma_roof, hbm_roof) if mfma_bound else (hbm_roof, mfma_roof)
    out = {
        "metric": "verified tree-tokens/s over the whole speculative step (draft_tree + verify_tree + accept_and_compact)",
        "value": B * N / (ms_per_step * 1e-3), "unit": "tree-tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {shape.name}, batch {B}, {N}-node tree, "
                               f"cached lengths {lens1[:B].tolist()}, {shape.n_layers} layers",
                   "accepted_per_step": float((lens2[:B] - lens1[:B]).sum()) / (K * B),
                   "library": os.path.abspath(args.library) if args.library else "shipped",
                   "env_switches": switches},
        "calls_ms": {"verify_tree": {"median": ver_med, "p10": float(np.percentile(ver, 10)),
                                     "p90": float(np.percentile(ver, 90))},
                     "accept_and_compact": {"median": float(np.median(acc))},
                     "draft_tree": {"median": float(np.median(dra))}},
        "verify_hbm": {"algorithmic_bytes": vbytes, "GBps": vbytes / (ver_med * 1e-3) / 1e9,
                       "frac_of_peak": vbytes / (ver_med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "tree_tokens_per_s": B * N / (ver_med * 1e-3),
                       "weight_passes_per_gemm": passes},
        "draft_hbm": {"algorithmic_bytes": dbytes, "GBps": dbytes / (float(np.median(dra)) * 1e-3) / 1e9},
        "roofline": {"kernel": dom_name, **main_roof,
                     "traffic": int(traffic) if traffic else None, "other_roof": other_roof,
                     "bytes_per_launch": dom_bytes, "avg_launch_ms": dom_avg_ms,
                     "rows_per_launch": rows_per_launch,
                     "mfma_issued_TFLOPs": issued_tflops, "mfma_frac_of_bf16_peak": issued_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "kernel_trace_avg_launch_ms": trace_us * 1e-3 if trace_us else None,
                     "source_fingerprint": fp},
        "prefill": {"tokens": n_prompt, "ms": prefill_ms, "tokens_per_s": n_prompt / prefill_ms * 1e3,
                    "rows_per_pass": PREFILL_ROWS,
                    "note": "set-up through clover_prefill, one sequence after the other; not part of the timed step"},
        "kernel_classes": classes,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(shape, parent, rank, int(lens0[0]), min(args.cpu_sample_layers, shape.n_layers), store,
                                           args.cpu_seconds)
        log(f"[bench] cpu baseline in {time.time() - t0:.1f}s")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
