"""Benchmark of the Token Recycling decode step on one MI355X.

A "step" is one pass of the whole hot path: draft-tree gather, verification forward over the
80 tree nodes (tree attention, all projections, LM head), per-node top-k, greedy accept, matrix
update and KV compaction.  Workload: random-init 7B-shape Llama in bf16, batch 1, 80-node /
6-layer static tree, k = 8, seeded Zipf(1.1) prompt of 512 tokens with planted 8-gram repeats;
all inputs are resident in HBM before the timed region starts.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this build is
single-GPU by design.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--shape", default="7b")
    ap.add_argument("--prompt-len", type=int, default=0,
                    help="0: the prompt length of the shape's workload (7b 512, 13b 2048, 70b 4096)")
    ap.add_argument("--profile-steps", type=int, default=4)
    ap.add_argument("--cpu-steps", type=int, default=4, help="oracle steps timed for cpu_baseline (0 = skip)")
    ap.add_argument("--no-ar", action="store_true", help="skip the 1-node autoregressive comparison run")
    ap.add_argument("--no-hot", action="store_true", help="skip the hot-start rerun")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy a few times (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--sweep-nodes", default="",
                    help="comma-separated tree sizes: time the step for each (breadth-first prefixes of the 128-node "
                         "template) instead of the headline run, and print one JSON line with the table")
    ap.add_argument("--sweep-depth", default="",
                    help="comma-separated tree depths (layers including the root, 4..8): time the step for 80-node "
                         "templates of each depth instead of the headline run, cold and with the hot-start matrix "
                         "the cold run leaves, and print one JSON line with the table")
    ap.add_argument("--sweep-prefill", default="",
                    help="comma-separated prompt lengths: time prompt ingestion (tr_prefill) at each, print one JSON line")
    ap.add_argument("--sweep-attention", default="",
                    help="comma-separated prefix lengths: time the tree-attention op alone (attention kernel + split "
                         "merge, the shape's heads, 80-node tree, rotating cache layers) at each, instead of the "
                         "headline run, and print one JSON line with the table (no model is built)")
    return ap.parse_args()


def say(*a):
    """Progress line on stderr (stdout carries only the JSON line)."""
    print("[bench]", *a, file=sys.stderr, flush=True)


def timed_steps(eng, torch, n):
    torch.cuda.synchronize()
    l0 = int(eng.kv.d_len.item())
    t0 = time.perf_counter()
    for _ in range(n):
        eng.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, int(eng.kv.d_len.item()) - l0


def cpu_baseline(sh, w_gpu, tmpl, prompt, n_steps, synth):
    """The oracle as it stands, float32 batched mode, on the host cores: n_steps whole steps at the
    same shape after a KV prefix of synthetic N(0,1) values (the oracle's own prefill of 511 tokens
    would take minutes and is not part of a step)."""
    import numpy as np
    from oracle import tr_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    wn = synth.weights_to_numpy(w_gpu)
    cfg = O.Config(sh.n_layers, sh.d_model, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_ffn, sh.vocab,
                   sh.rms_eps, sh.rope_theta)
    tree = O.make_tree(tmpl.parent, tmpl.rank, 8)
    L = len(prompt) - 1
    kv = O.KVCache(cfg, L + n_steps * tree.n_layers + tree.n_nodes, np.float32)
    rng = np.random.default_rng(0)
    for l in range(cfg.n_layers):
        kv.k[l][:L] = rng.standard_normal((L, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32)
        kv.v[l][:L] = rng.standard_normal((L, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32)
    kv.len = L
    M = synth.init_matrix(sh.vocab, 8).astype(np.int64)
    root, emitted = int(prompt[-1]), 0
    t0 = time.perf_counter()
    for _ in range(n_steps):
        r = O.tr_step(cfg, wn, kv, M, tree, root, 8, dtype=np.float32)
        root = r.acc.bonus
        emitted += r.acc.n_accepted + 1
    dt = time.perf_counter() - t0
    return {"value": n_steps / dt, "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_steps} whole draft-verify-update steps, {sh.name} shape, float32 batched mode, "
                      f"KV prefix of {L} synthetic N(0,1) positions", "s_per_step": dt / n_steps,
            "tokens_per_s": emitted / dt}


def attention_microbench(sh, tmpl, torch, tr, L=1024, reps=5):
    """Tree attention alone (attention kernel + split merge) at the kernel-microbenchmark shape: 32 heads of
    128, L = 1024 committed positions, the 80-node tree, N(0,1) bf16 Q/K/V.  One launch per cache layer, so
    consecutive launches read different 18 MB K/V blocks (32 layers = 580 MB, beyond the Infinity Cache)."""
    n, H, hd = tmpl.n_nodes, sh.n_heads, sh.head_dim
    kv = tr.KVDesc(sh, L + n)
    kv.k.normal_()
    kv.v.normal_()
    kv.reset(L)
    ctx = tr.Context(64, 8, tmpl.parent, tmpl.rank, tmpl.n_layers)
    q = torch.randn(n, H, hd, device="cuda").to(torch.bfloat16)
    o = torch.zeros_like(q)
    ws = torch.empty(16 * 128 * H * (2 + hd) * 4 + 4096, dtype=torch.uint8, device="cuda")
    for layer in range(sh.n_layers):
        ctx.op_tree_attention(kv, layer, H, q, o, ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        for layer in range(sh.n_layers):
            ctx.op_tree_attention(kv, layer, H, q, o, ws)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * sh.n_layers)
    nbytes = (L + n) * sh.n_kv_heads * hd * 2 * 2 + 2 * n * H * hd * 2    # K, V, Q, O
    res = {"workload": f"H={H} Hkv={sh.n_kv_heads} hd={hd} L={L} N={n}, bf16, {sh.n_layers} rotating cache layers",
           "us_per_layer": us, "algorithmic_bytes_per_layer": nbytes, "achieved_GBs": nbytes / us * 1e-3,
           "frac_of_peak_hbm": nbytes / us * 1e-3 / PEAK_HBM_GBS, "traffic": None}
    # HBM bytes per layer from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, if a summary for this shape is recorded
    pmc = os.path.join(ROOT, "profiles", f"tree_attention_L{L}_pmc.txt")
    if H == 32 and sh.n_kv_heads == 32 and n == 80 and os.path.exists(pmc):
        for line in open(pmc):
            if line.startswith("traffic_bytes_per_layer:"):
                res["traffic"] = float(line.split(":")[1])
                res["traffic_source"] = os.path.relpath(pmc, ROOT)
    return res


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {a.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2408_08696_amd import synth, tr

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    tr.lib()
    torch.cuda.set_device(0)
    sh = synth.SHAPES[a.shape]
    if a.prompt_len <= 0:
        a.prompt_len = {"7b": 512, "13b": 2048, "70b": 4096}.get(a.shape, 512)
    tmpl = synth.tree80()
    K = 8
    if a.sweep_attention:
        rows = []
        for L in [int(v) for v in a.sweep_attention.split(",")]:
            r = attention_microbench(sh, tmpl, torch, tr, L=L, reps=3)
            r["prefix_len"] = L
            r["plan"] = dict(zip(("heads_per_workgroup", "key_splits"),
                                 tr.plan_attention(sh.n_heads, sh.n_kv_heads, tmpl.n_nodes, L + tmpl.n_nodes)))
            rows.append(r)
            say(f"L={L}: {r['us_per_layer']:.2f} us per layer")
        if a.calibrate_copy:
            # a copy of known size (256 MiB read + 256 MiB written) for calibrating rocprofv3 --pmc byte counters
            src, dst = (torch.ones(1 << 26, dtype=torch.float32, device="cuda") for _ in range(2))
            for _ in range(4):
                tr.op_stream(src, dst)
            torch.cuda.synchronize()
        print(json.dumps({"metric": "tree attention time vs prefix length", "unit": "us/layer", "n_gpus": 1,
                          "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"{sh.name}-shape heads (H={sh.n_heads}, Hkv={sh.n_kv_heads}, hd="
                                                 f"{sh.head_dim}), 80-node tree, N(0,1) Q/K/V, one launch per cache "
                                                 f"layer over {sh.n_layers} layers"},
                          "sweep": rows}))
        return
    # a model too large to hold twice (row-major + packed) is generated and packed one layer at a time;
    # the row-major originals are then gone, so the oracle baseline (which needs them) is skipped
    streaming_build = sh.weight_params() * 2 * 2 > 200e9
    if streaming_build:
        packed = synth.head_weights(sh, seed=0, device="cuda")
        packed["lm_head"] = tr.pack_weight(packed["lm_head"])
        packed["layers"] = []
        for l in range(sh.n_layers):
            lw = synth.layer_weights(sh, l, seed=0, device="cuda")
            packed["layers"].append(tr.pack_layer(sh, lw))
            del lw
            if l % 8 == 7:
                torch.cuda.synchronize()
                say(f"layer {l + 1}/{sh.n_layers} generated and packed")
        w = None
        model = tr.ModelDesc(sh, packed, pack=True, prepacked=True)
        del packed
    else:
        w = synth.make_weights(sh, seed=0, device="cuda")
        model = None
    prompt = synth.zipf_prompt(sh.vocab, a.prompt_len, seed=0, ngram=8).tolist()
    M0 = synth.init_matrix(sh.vocab, K)
    total_steps = a.warmup + a.steps + a.profile_steps
    cap = a.prompt_len + total_steps * tmpl.n_layers + tmpl.n_nodes + 64

    if a.sweep_prefill:
        # Prompt ingestion alone: len - 1 tokens through tr_prefill (the last prompt token is the first root),
        # average of --steps repetitions after one untimed call.
        if model is None:
            model = tr.ModelDesc(sh, w)
        del w
        lens = [int(v) for v in a.sweep_prefill.split(",")]
        e = tr.Engine(sh, None, tmpl, k=K, capacity=max(lens) + 256, keep_logits=False, model=model)
        rows = []
        for pl in lens:
            p = synth.zipf_prompt(sh.vocab, pl, seed=0, ngram=8).tolist()
            e.prefill(p)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(a.steps):
                e.prefill(p)
            torch.cuda.synchronize()
            dtp = (time.perf_counter() - t0) / a.steps
            rows.append({"prompt_tokens": pl - 1, "ms": dtp * 1e3, "tokens_per_s": (pl - 1) / dtp,
                         "weight_reads": -(-(pl - 1) // 512)})
            say(rows[-1])
        print(json.dumps({"metric": "prompt ingestion time", "unit": "ms", "n_gpus": 1, "steps": a.steps,
                          "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"{sh.name}-shape random-init Llama bf16, batch 1, Zipf prompts"},
                          "sweep": rows}))
        return

    if a.sweep_depth:
        # Step time and accepted length versus tree depth at a fixed 80 nodes (Section 5.1 / Figure 3b).  Step
        # time barely moves (the forward sees 80 rows whatever their arrangement); what a deeper tree changes is
        # how many drafts a step can accept, shown here cold and after a hot start (Section 3.1: the same prompt
        # again with the matrix the first run left behind).
        if model is None:
            model = tr.ModelDesc(sh, w)
        del w
        rows = []
        for dd in [int(v) for v in a.sweep_depth.split(",")]:
            t = synth.depth_template(dd)
            e = tr.Engine(sh, None, t, k=K, capacity=a.prompt_len + 2 * (a.warmup + a.steps) * t.n_layers + 256,
                          keep_logits=False, model=model)
            e.ctx.matrix_load(M0)
            e.prefill(prompt)
            timed_steps(e, torch, a.warmup)
            dts, tk = timed_steps(e, torch, a.steps)
            e.prefill(prompt)
            dth, tkh = timed_steps(e, torch, a.steps)
            rows.append({"n_layers": dd, "n_nodes": t.n_nodes, "layer_sizes": list(t.layer_sizes),
                         "ms_per_step": dts / a.steps * 1e3, "steps_per_s": a.steps / dts, "mat": tk / a.steps,
                         "tokens_per_s": tk / dts, "mat_hot_start": tkh / a.steps, "tokens_per_s_hot_start": tkh / dth})
            say(f"depth {dd}: {rows[-1]['ms_per_step']:.3f} ms/step, MAT {rows[-1]['mat']:.2f} cold, "
                f"{rows[-1]['mat_hot_start']:.2f} hot")
            del e
        print(json.dumps({"metric": "TR step time and accepted length vs tree depth at 80 nodes", "unit": "ms/step",
                          "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"{sh.name}-shape random-init Llama bf16, batch 1, prompt "
                                                 f"{a.prompt_len}, 80-node templates of 4..8 layers "
                                                 "(synth.depth_template)"},
                          "sweep": rows}))
        return

    if a.sweep_nodes:
        # Step time versus tree size (Section 5.1 / Figure 3a asks where verifying more nodes stops being
        # as cheap as one token): same model, prompt and KV length, one engine per tree size.
        if model is None:
            model = tr.ModelDesc(sh, w)
        del w
        rows = []
        for nn in [int(v) for v in a.sweep_nodes.split(",")]:
            t = synth.prefix_template(nn)
            e = tr.Engine(sh, None, t, k=K, capacity=a.prompt_len + (a.warmup + a.steps) * t.n_layers + 256,
                          keep_logits=False, model=model)
            e.ctx.matrix_load(M0)
            e.prefill(prompt)
            timed_steps(e, torch, a.warmup)
            dts, tk = timed_steps(e, torch, a.steps)
            rows.append({"n_nodes": nn, "n_layers": t.n_layers, "ms_per_step": dts / a.steps * 1e3,
                         "steps_per_s": a.steps / dts, "mat": tk / a.steps})
            del e
        base = rows[0]["ms_per_step"]
        for r in rows:
            r["cost_vs_first"] = r["ms_per_step"] / base
        print(json.dumps({"metric": "TR step time vs tree size", "unit": "ms/step", "n_gpus": 1, "steps": a.steps,
                          "warmup": a.warmup, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"{sh.name}-shape random-init Llama bf16, batch 1, prompt "
                                                 f"{a.prompt_len}, breadth-first prefixes of the 128-node template"},
                          "sweep": rows}))
        return

    if model is None:
        model = tr.ModelDesc(sh, w)
    eng = tr.Engine(sh, None, tmpl, k=K, capacity=cap, keep_logits=False, model=model)
    eng.ctx.matrix_load(M0)
    say("model ready; prefill")
    eng.prefill(prompt)                      # first call also pays one-time set-up; time the second
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.prefill(prompt)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    timed_steps(eng, torch, a.warmup)
    say("timing", a.steps, "steps")
    dt, toks = timed_steps(eng, torch, a.steps)
    say(f"{dt / a.steps * 1e3:.3f} ms/step")
    ms_step = dt / a.steps * 1e3
    steps_s = a.steps / dt
    mat = toks / a.steps

    # per-kernel-class durations from HIP events on the same stream, same launch configuration
    eng.ctx.profile_enable(True)
    timed_steps(eng, torch, a.profile_steps)
    prof = eng.ctx.profile_read()
    eng.ctx.profile_enable(False)
    breakdown = {k: {"launches_per_step": v[0] / a.profile_steps, "ms_per_step": v[1] / a.profile_steps}
                 for k, v in prof.items()}
    # dominant kernel: its own execution time from the start / stop events the library ties to each dispatch
    # (the figure rocprofv3 --kernel-trace reports for the same launches; profiles/ holds that summary)
    gu_launches, gu_ms = prof["gate_up_swiglu"]
    gu_bytes = 2 * sh.d_ffn * sh.d_model * 2                       # gate + up weights, bf16, read once
    gu_avg_s = gu_ms / gu_launches * 1e-3
    achieved = gu_bytes / gu_avg_s / 1e9
    roofline = {"kernel": "gate_up_swiglu (k_gemm_mfma, fused gate/up projection + SwiGLU)", "bound": "hbm",
                "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                "traffic": None, "avg_launch_us": gu_avg_s * 1e6, "algorithmic_bytes_per_launch": gu_bytes,
                "timing": "per-dispatch start/stop events (hipExtLaunchKernelGGL) over the profiled steps",
                "rocprof_summary": f"profiles/step_{sh.name}_tree80_kernel_stats.md"}
    # HBM bytes per launch of this kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, if a summary for this
    # workload has been recorded under profiles/ (bench.py cannot run the profiler on itself)
    pmc = os.path.join(ROOT, "profiles", f"gate_up_swiglu_{sh.name}_tree80_pmc.txt")
    if os.path.exists(pmc):
        for line in open(pmc):
            if line.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(line.split(":")[1])
                roofline["traffic_source"] = os.path.relpath(pmc, ROOT)
    wbytes = sh.weight_params() * 2
    step_roofline = {"weight_bytes": wbytes, "ms_at_peak_hbm": wbytes / (PEAK_HBM_GBS * 1e9) * 1e3,
                     "frac": wbytes / (PEAK_HBM_GBS * 1e9) * 1e3 / ms_step}

    out = {
        "metric": f"TR steps/s, {sh.name.upper()}-shape bf16, 1 GPU", "value": steps_s, "unit": "steps/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{sh.name}-shape random-init Llama bf16, batch 1, {tmpl.n_nodes}-node "
                               f"{tmpl.n_layers}-layer static tree, k=8, Zipf(1.1) prompt of {a.prompt_len} tokens "
                               "with planted 8-gram repeats, M init (i+j) mod V",
                   "n_layers": sh.n_layers, "d_model": sh.d_model, "vocab": sh.vocab},
        "tokens_per_s": steps_s * mat, "mat": mat,
        "prefill": {"prompt_tokens": len(prompt) - 1, "ms": prefill_s * 1e3,
                    "tokens_per_s": (len(prompt) - 1) / prefill_s, "how": "passes of up to 512 rows: wide projection kernel, attention per block of 128 rows"},
        "step_roofline": step_roofline, "roofline": roofline,
        "breakdown_ms_per_step": breakdown,
    }

    if not a.no_hot:
        # hot start (Section 3.1): same prompt again with the matrix the run above left behind
        eng.prefill(prompt)
        _, toks_hot = timed_steps(eng, torch, a.steps)
        out["mat_hot_start"] = toks_hot / a.steps
        out["tokens_per_s_hot_start"] = steps_s * toks_hot / a.steps
    del eng

    if not a.no_ar:
        say("autoregressive comparison")
        ar = tr.Engine(sh, None, synth.single(), k=K, capacity=a.prompt_len + a.warmup + a.steps + 64,
                       keep_logits=False, model=model)
        ar.ctx.matrix_load(M0)
        ar.prefill(prompt)
        timed_steps(ar, torch, a.warmup)
        dt_ar, toks_ar = timed_steps(ar, torch, a.steps)
        out["ar_tokens_per_s"] = toks_ar / dt_ar
        out["ar_ms_per_step"] = dt_ar / a.steps * 1e3
        out["speedup_vs_ar"] = out["tokens_per_s"] / out["ar_tokens_per_s"]
        out["step_cost_ratio_vs_ar"] = ms_step / out["ar_ms_per_step"]
        if "tokens_per_s_hot_start" in out:
            out["speedup_vs_ar_hot_start"] = out["tokens_per_s_hot_start"] / out["ar_tokens_per_s"]
        del ar

    # achievable streaming rate on this machine: the library's plain read kernel over 32 distinct 256 MiB
    # buffers (8 GiB, far beyond the 256 MB Infinity Cache), timed with events on the same stream
    bufs = [torch.ones(1 << 26, dtype=torch.float32, device="cuda") for _ in range(32)]
    for b_ in bufs[:4]:
        tr.op_stream(b_)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for b_ in bufs:
        tr.op_stream(b_)
    e1.record()
    torch.cuda.synchronize()
    stream_gbs = len(bufs) * bufs[0].numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    out["stream_read_ceiling_GBs"] = stream_gbs
    out["roofline"]["frac_of_stream_ceiling"] = achieved / stream_gbs
    out["step_roofline"]["frac_of_stream_ceiling"] = wbytes / (stream_gbs * 1e9) * 1e3 / ms_step
    if a.calibrate_copy:
        # a copy of known size (256 MiB read + 256 MiB written) for calibrating rocprofv3 --pmc byte counters
        for _ in range(4):
            tr.op_stream(bufs[0], bufs[1])
        torch.cuda.synchronize()
        out["calibrate_copy_bytes_each_way"] = bufs[0].numel() * 4
    del bufs

    say("attention microbenchmark, oracle baseline")
    out["tree_attention"] = attention_microbench(sh, tmpl, torch, tr)

    if a.cpu_steps > 0 and w is not None:
        out["cpu_baseline"] = cpu_baseline(sh, w, tmpl, prompt, a.cpu_steps, synth)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
