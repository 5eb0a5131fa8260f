#!/usr/bin/env python3
"""Benchmark of the lookahead-decoding hot path on one MI355X.

One "step" is one lookahead decoding step of a LLaMA-2-shaped model as the hot path sees
it: L back-to-back la_step_attention calls, one per layer and each on its own KV cache (so
the 256 MB Infinity Cache cannot hold what is streamed), followed by one la_verify call on
the step's verification logits.  Inputs are seeded synthetic tensors resident in HBM before
the timed region.  The reported value is microseconds per layer-step (step time / L).

Prints ONE JSON line.  `roofline`: algorithmic bytes (or flops) of one attention launch over its
measured time against the MI355X peak that bounds the shape (HBM 8 TB/s or bf16 MFMA 2.5 PFLOP/s)
and against what this machine reaches at best in the same run (`achievable`: a streaming read, a
register-resident MFMA loop), plus the HBM traffic recorded in profiles/.  `cpu_baseline`: the CPU
oracle timed on the host cores (all of them, and one).  The other objects time the remaining entry
points on their own.  --workload: llama2-7b (default), llama2-13b, llama2-70b-gqa, tiny, ragged,
llama2-7b-p256 (the 7B step on a 256-token prefix: the shape of the short-prefix kernel).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0

LAYERS = {"tiny": 8, "llama2-7b": 32, "llama2-13b": 40, "llama2-70b-gqa": 80, "llama2-7b-p256": 32}
RAGGED_W = (5, 10, 15, 20, 30)


def profile_traffic(workload):
    """HBM bytes per attention launch as the counters saw them, from the committed rocprofv3 summary
    of this workload (profiles/attention_<workload>.md: FETCH_SIZE + WRITE_SIZE per dispatch, each
    scaled by the same counter's reading for a plain copy).  A recorded value, not measured by this
    run: (bytes, "file @ commit it was taken at"), or (None, None) if there is no summary."""
    import re
    path = os.path.join(ROOT, "profiles", "attention_%s.md" % workload)
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", text, re.M)
    c = re.search(r"^traffic_taken_at\s*=\s*(\S+)", text, re.M)
    if not m:
        return None, None
    return int(m.group(1)), "profiles/attention_%s.md @ %s" % (workload, c.group(1) if c else "?")


def visible_pairs(W, N, G):
    n1 = N - 1
    return 1 + sum(2 + j for j in range(W)) + sum(2 + j + l for l in range(1, n1) for j in range(W)) \
        + G * sum(2 + k for k in range(n1))


def algorithmic_bytes(s):
    """HBM bytes one layer-step must move: K/V cache once, step K/V, q in, out (all bf16)."""
    T, H, KV, d, P = s.T, s.heads, s.kv_heads, s.head_dim, s.P
    return 2 * P * KV * d * 2 + 2 * T * KV * d * 2 + 2 * T * H * d * 2


def algorithmic_flops(s):
    return 4 * s.head_dim * s.heads * (s.T * s.P + visible_pairs(s.W, s.N, s.G))


def time_calls(torch, np, fn, calls, reps, use_graph):
    """Median microseconds per call of `fn`, `calls` of them back to back (as one HIP graph if
    use_graph), by events on the launch stream."""
    fn()
    torch.cuda.synchronize()
    run = fn
    if use_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(calls):
                fn()
        run = g.replay
    else:
        calls = 1
    run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ms = []
    replays = 4 if use_graph else 1   # (one replay alone also carries the start-up of a graph launch)
    for _ in range(reps):
        e0.record()
        for _ in range(replays):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1) / (calls * replays))
    return float(np.median(ms)) * 1e3


def measure_peaks(torch, np, binding):
    """What this machine reaches at best, in this run: a streaming read of 1 GiB (larger than the 256 MB
    Infinity Cache), a register-resident bf16 MFMA loop, and the clock the driver reports."""
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    buf.zero_()
    sink = torch.zeros(4, dtype=torch.int64, device="cuda")
    read_us = time_calls(torch, np, lambda: binding.la_probe_stream_read(buf, sink), 1, 10, False)
    del buf
    iters = 4096
    flops = []
    mfma_us = time_calls(torch, np, lambda: flops.append(binding.la_probe_mfma(iters, sink)), 1, 10, False)
    props = torch.cuda.get_device_properties(0)
    cycles, ticks = [int(v) for v in sink[:2].cpu()]
    return {"hbm_read_gbs": (1 << 30) / (read_us * 1e-6) / 1e9,
            "mfma_bf16_tflops": flops[-1] / (mfma_us * 1e-6) / 1e12,
            "clock_mhz_under_mfma_load": cycles / max(ticks, 1) * 100.0,   # shader cycles per 100 MHz tick
            "compute_units": props.multi_processor_count}


def roofline_object(abytes, aflops, us, peaks, kernel, traffic, traffic_source):
    t_hbm = abytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = aflops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if t_hbm >= t_mfma:
        roof = {"bound": "hbm", "achieved": abytes / (us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        best = peaks["hbm_read_gbs"]
    else:
        roof = {"bound": "mfma", "achieved": aflops / (us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s"}
        best = peaks["mfma_bf16_tflops"]
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = traffic
    roof["traffic_source"] = traffic_source     # a recorded profile value, not measured by this run
    roof["kernel"] = kernel
    roof["us_per_launch"] = us
    roof["algorithmic_bytes"] = abytes
    roof["algorithmic_flops"] = aflops
    roof["achievable"] = peaks
    roof["frac_of_achievable"] = roof["achieved"] / best
    return roof, max(t_hbm, t_mfma)


def run_ragged(args):
    """The ragged long-context sweep: eight sequences (GQA 32/8, prefixes drawn in 512 .. 16384),
    N = 5, G = W, W in {5, 10, 15, 20, 30}.  A step is ONE la_step_attention_batch launch over the
    eight sequences; `value` is its time at W = 15 (the paper's 7B setting).  For every W the line
    also has the eight single calls back to back and the roofline that bounds the launch."""
    import numpy as np
    import torch
    from paper_2402_02057_amd import binding, buildlib, workloads as wl
    from oracle import la_oracle as orc
    if not os.path.exists(buildlib.LIB):
        buildlib.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    use_graph = not args.no_graph
    peaks = measure_peaks(torch, np, binding)
    reps = max(10, min(args.steps, 50))
    sweep, host, value_us, value_roof, value_t = [], {}, None, None, None
    parity_err = 0.0
    widths = sorted(set(int(w) for w in args.ragged_w.split(",")) | {15})
    for W in widths:
        shapes = [wl.ragged_shape(seq, W) for seq in range(8)]
        s0 = shapes[0]
        descs = []
        for seq, s in enumerate(shapes):
            x = wl.attention_inputs(s, extra=seq)
            if W in (5, 30):
                host[(W, seq)] = x
            dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
            descs.append(dict(q=dev["q"], k_cache=dev["k_cache"], v_cache=dev["v_cache"], step_k=dev["step_k"],
                              step_v=dev["step_v"], out=torch.empty((s.T, s.heads, s.head_dim), dtype=torch.bfloat16,
                                                                    device="cuda"), P=s.P))

        def one_launch():
            binding.la_step_attention_batch(descs, W, s0.N, s0.G, s0.heads, s0.kv_heads, s0.head_dim)

        def eight_calls():
            for d_ in descs:
                binding.la_step_attention(d_["q"], d_["k_cache"], d_["v_cache"], d_["step_k"], d_["step_v"], d_["P"], W,
                                          s0.N, s0.G, s0.heads, s0.kv_heads, s0.head_dim, d_["out"])
        launch_us = time_calls(torch, np, one_launch, 4, reps, use_graph)
        calls_us = time_calls(torch, np, eight_calls, 2, reps, use_graph)
        abytes = sum(algorithmic_bytes(s) for s in shapes)
        aflops = sum(algorithmic_flops(s) for s in shapes)
        traffic, source = profile_traffic("ragged") if W == 15 else (None, None)
        roof, t_roof = roofline_object(abytes, aflops, launch_us, peaks, "step_attention_batch_kernel", traffic, source)
        sweep.append({"W": W, "rows": s0.T, "one_launch_us": launch_us, "eight_calls_us": calls_us,
                      "algorithmic_bytes": abytes, "algorithmic_flops": aflops, "bound": roof["bound"],
                      "roofline_us": t_roof * 1e6, "frac": roof["frac"], "frac_of_achievable": roof["frac_of_achievable"],
                      "frac_eight_calls": t_roof * 1e6 / calls_us})
        if W == 15:
            value_us, value_roof, value_t = launch_us, roof, t_roof
        if W in (5, 30):
            # parity of the launch that was timed: the two shortest sequences against the oracle
            one_launch()
            torch.cuda.synchronize()
            for seq in np.argsort([s.P for s in shapes])[:2]:
                s, x = shapes[seq], host[(W, int(seq))]
                want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], s.P, s.W, s.N,
                                          s.G, s.heads, s.kv_heads, s.head_dim)
                parity_err = max(parity_err, float(np.abs(descs[seq]["out"].float().cpu().numpy().astype(np.float64) - want).max()))
        del descs
    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle on the shortest sequence at W = 15, scaled by flops to the eight sequences
        shapes = [wl.ragged_shape(seq, 15) for seq in range(8)]
        seq = int(np.argmin([s.P for s in shapes]))
        s, x = shapes[seq], wl.attention_inputs(shapes[seq], extra=seq)
        t0 = time.perf_counter()
        n_done = 0
        while n_done < 3 and time.perf_counter() - t0 < 20.0:
            orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], s.P, s.W, s.N, s.G,
                               s.heads, s.kv_heads, s.head_dim)
            n_done += 1
        per = (time.perf_counter() - t0) / n_done
        scale = sum(algorithmic_flops(t) for t in shapes) / algorithmic_flops(s)
        cpu = {"value": per * scale * 1e6, "unit": "us/step", "cores": orc.threads(), "kind": "oracle",
               "sample": "the oracle's layer-step of the shortest sequence (P=%d, W=15), %d runs, scaled by "
                         "algorithmic flops (x%.1f) to the eight sequences" % (s.P, n_done, scale)}
    line = {
        "metric": "lookahead-step attention, us per step of the ragged sweep (8 sequences in one launch, W=15)",
        "value": value_us, "unit": "us/step", "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": value_us / 1e3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ragged sweep: 8 sequences H32/KV8/d128, P = %s, N=5, G=W; value at W=15" %
                               wl.ragged_prefix_lengths(), "graph": use_graph},
        "roofline": value_roof, "cpu_baseline": cpu, "sweep": sweep,
        "parity": {"attention_max_abs_err": parity_err},
    }
    print(json.dumps(line))
    if parity_err > 2e-2:
        print("bench.py: PARITY FAILURE", file=sys.stderr)
        sys.exit(1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama2-7b", choices=sorted(LAYERS) + ["ragged"])
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every call from Python instead of replaying the step as one HIP graph")
    ap.add_argument("--ragged-w", default=",".join(str(w) for w in RAGGED_W),
                    help="ragged workload: the window widths to run (W = 15 gives `value`)")
    ap.add_argument("--no-cache-hot", action="store_true",
                    help="skip the labelled cache-hot figure (profiles: keeps the kernel's statistics to the HBM-fed launches)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 64 MiB device copy a few times (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the hot path is one GPU's share; nothing here "
              "shards across GPUs); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.workload == "ragged":
        return run_ragged(args)

    import numpy as np
    import torch
    from paper_2402_02057_amd import binding, buildlib, workloads as wl

    if not os.path.exists(buildlib.LIB):
        buildlib.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    peaks = measure_peaks(torch, np, binding)
    s = wl.SHAPES[args.workload]
    L = args.layers or LAYERS[args.workload]
    T, H, KV, d, P = s.T, s.heads, s.kv_heads, s.head_dim, s.P

    # ---- inputs, resident in HBM: one independent draw per layer
    layers = []
    host0 = None
    for layer in range(L):
        x = wl.attention_inputs(s, extra=layer)
        if layer == 0:
            host0 = x
        layers.append({k: binding.bf16_tensor(v) for k, v in x.items()})
    outs = [torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    logits_h, cand_h, lens_h = wl.verify_inputs(s)
    logits = torch.from_numpy(logits_h).cuda()
    cand = torch.from_numpy(cand_h).cuda()
    alen = torch.empty((s.G,), dtype=torch.int32, device="cuda")
    acc = torch.empty((s.G, s.N - 1), dtype=torch.int32, device="cuda")
    # the whole end of a greedy step in one launch (timed on its own, not part of `value`)
    vs_h = wl.verify_step_inputs(s)
    vs = [torch.from_numpy(x).cuda() for x in vs_h[:4]]
    vs_out = [torch.empty((n,), dtype=torch.int32, device="cuda") for n in (s.N, 1, 1, s.W, s.G)]

    def verify_step():
        binding.la_verify_step(vs[0], vs[1], vs[2], vs[3], s.W, s.N, s.G, s.V, *vs_out)

    # sampling verification (Algorithm 4), also timed on its own
    sm_h = wl.verify_sample_inputs(s)
    sm = [torch.from_numpy(x).cuda() for x in sm_h]
    sm_out = [torch.empty((n,), dtype=torch.int32, device="cuda") for n in (s.N, 1)]

    def verify_sample():
        binding.la_verify_sample(sm[0], sm[1], sm[2], sm[3], sm[4], 1.0, s.N, s.G, s.V, *sm_out)

    def attention_layers():
        for x, o in zip(layers, outs):
            binding.la_step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"],
                                      P, s.W, s.N, s.G, H, KV, d, o)

    def step():
        attention_layers()
        binding.la_verify(logits, cand, s.G, s.N, s.V, alen, acc)

    step()
    torch.cuda.synchronize()
    run_step = step
    use_graph = not args.no_graph
    if use_graph:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            step()
        run_step = g.replay

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    us_per_layer = ms_per_step * 1e3 / L

    # ---- dominant kernel (attention) and the verify kernel, by HIP events on the launch stream
    reps = max(10, min(args.steps, 100))
    e = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    attn_ms, ver_ms, vs_ms, sm_ms = [], [], [], []
    if use_graph:
        # the L attention launches alone, and the verify launch alone, as graphs
        ga, gv = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(ga):
            attention_layers()
        with torch.cuda.graph(gv):
            for _ in range(32):
                binding.la_verify(logits, cand, s.G, s.N, s.V, alen, acc)
        verify_step()
        gs = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gs):
            for _ in range(32):
                verify_step()
        verify_sample()
        gm = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gm):
            for _ in range(32):
                verify_sample()
        run_attn, run_ver, run_vs, run_sm, ver_calls = ga.replay, gv.replay, gs.replay, gm.replay, 32
    else:
        run_attn = attention_layers
        run_ver = lambda: binding.la_verify(logits, cand, s.G, s.N, s.V, alen, acc)
        run_vs = verify_step
        run_sm = verify_sample
        ver_calls = 1
    # (several replays between the two events, as in the timed loop above: one replay alone also
    # carries the start-up of a graph launch, 0.3 us per kernel at 32 kernels per graph)
    attn_replays = 4 if use_graph else 1
    for _ in range(reps):
        e[0].record()
        for _ in range(attn_replays):
            run_attn()
        e[1].record()
        run_ver()
        e[2].record()
        run_vs()
        e[3].record()
        run_sm()
        e[4].record()
        torch.cuda.synchronize()
        attn_ms.append(e[0].elapsed_time(e[1]) / attn_replays)
        ver_ms.append(e[1].elapsed_time(e[2]) / ver_calls)
        vs_ms.append(e[2].elapsed_time(e[3]) / ver_calls)
        sm_ms.append(e[3].elapsed_time(e[4]) / ver_calls)
    attn_us = float(np.median(attn_ms)) * 1e3 / L       # per launch, launch gaps included
    verify_us = float(np.median(ver_ms)) * 1e3
    verify_step_us = float(np.median(vs_ms)) * 1e3
    verify_step_bytes = (1 + s.W + s.G * (s.N - 1)) * s.V * 4
    verify_sample_us = float(np.median(sm_ms)) * 1e3
    verify_sample_bytes = (2 + s.G * (s.N - 1)) * s.V * 4   # every row once, one row again for the draw
    # appending the accepted rows to an in-place cache (la_kv_commit), timed on its own: it follows
    # the best / n_out that verify_step left on the device
    cap = P + 64
    kc_cap = torch.zeros((KV, cap, d), dtype=torch.bfloat16, device="cuda")
    vc_cap = torch.zeros((KV, cap, d), dtype=torch.bfloat16, device="cuda")
    kc_cap[:, :P], vc_cap[:, :P] = layers[0]["k_cache"], layers[0]["v_cache"]

    def kv_commit():
        binding.la_kv_commit(kc_cap, vc_cap, layers[0]["step_k"], layers[0]["step_v"], P, s.W, s.N, s.G, KV, d,
                             vs_out[2], vs_out[1])
    kv_commit()
    run_kc, kc_calls = kv_commit, 1
    if use_graph:
        gk = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gk):
            for _ in range(32):
                kv_commit()
        run_kc, kc_calls = gk.replay, 32
    kc_ms = []
    for _ in range(reps):
        e[0].record()
        run_kc()
        e[1].record()
        torch.cuda.synchronize()
        kc_ms.append(e[0].elapsed_time(e[1]) / kc_calls)
    kv_commit_us = float(np.median(kc_ms)) * 1e3

    # rotary position embedding of the step's q and keys at the step's positions (la_step_rope), on
    # copies, timed on its own (its parity with the oracle is a GPU test: tests/test_gpu_rope.py)
    rope_q, rope_k = layers[0]["q"].clone(), layers[0]["step_k"].clone()
    rope_cos, rope_sin = [torch.from_numpy(x).cuda() for x in wl.rope_tables(P + s.W + s.N, d)]

    def rope():
        binding.la_step_rope(rope_q, rope_k, rope_cos, rope_sin, P, s.W, s.N, s.G, H, KV, d)
    rope()
    run_r, r_calls = rope, 1
    if use_graph:
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for _ in range(32):
                rope()
        run_r, r_calls = gr.replay, 32
    r_ms = []
    for _ in range(reps):
        e[0].record()
        run_r()
        e[1].record()
        torch.cuda.synchronize()
        r_ms.append(e[0].elapsed_time(e[1]) / r_calls)
    rope_us = float(np.median(r_ms)) * 1e3
    # the alternative: the keys alone in a pass of their own, the queries rotated inside the attention
    # kernel (la_step_attention_rope; its parity is tests/test_gpu_attention_rope.py).  Per layer a
    # model pays attention + rope either way: both sums are reported.
    rope_keys_us = time_calls(torch, np, lambda: binding.la_step_rope(None, rope_k, rope_cos, rope_sin, P, s.W, s.N,
                                                                      s.G, H, KV, d), 32, reps, use_graph)
    rot_it = iter(range(1 << 30))

    def attention_rope_layer():
        i = next(rot_it) % L
        x = layers[i]
        binding.la_step_attention_rope(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], rope_cos,
                                       rope_sin, P, s.W, s.N, s.G, H, KV, d, outs_rot[i])
    outs_rot = [torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    attention_rope_us = time_calls(torch, np, attention_rope_layer, L, reps, use_graph)
    # and with nothing rotated in memory: the attention kernel turns the step keys it stages as well,
    # the append turns the few key rows it copies (la_kv_commit_rope)
    rot2_it = iter(range(1 << 30))

    def attention_rope_all_layer():
        i = next(rot2_it) % L
        x = layers[i]
        binding.la_step_attention_rope(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], rope_cos,
                                       rope_sin, P, s.W, s.N, s.G, H, KV, d, outs_rot[i], rotate_keys=True)
    attention_rope_all_us = time_calls(torch, np, attention_rope_all_layer, L, reps, use_graph)
    kc_rot, vc_rot = kc_cap.clone(), vc_cap.clone()     # (caches of its own: kc_cap is compared with the oracle)
    kv_commit_rope_us = time_calls(torch, np, lambda: binding.la_kv_commit_rope(
        kc_rot, vc_rot, layers[0]["step_k"], layers[0]["step_v"], rope_cos, rope_sin, P, s.W, s.N, s.G, KV, d,
        vs_out[2], vs_out[1]), 32, reps, use_graph)

    # the ends of eight sequences' steps in ONE launch (la_verify_step_batch), timed on its own:
    # sequence 0 is the step above, the others are further seeded draws of the same shape
    vsb_h = [vs_h] + [wl.verify_step_inputs(s, extra) for extra in range(1, 8)]
    vsb = []
    for h in vsb_h:
        t4 = [torch.from_numpy(x).cuda() for x in h[:4]]
        vsb.append(dict(logits_cur=t4[0], logits_look=t4[1], logits_cand=t4[2], cand_tokens=t4[3],
                        out_tokens=torch.empty((s.N,), dtype=torch.int32, device="cuda"),
                        n_out=torch.empty((1,), dtype=torch.int32, device="cuda"),
                        best=torch.empty((1,), dtype=torch.int32, device="cuda"),
                        new_window=torch.empty((s.W,), dtype=torch.int32, device="cuda"),
                        accept_len=torch.empty((s.G,), dtype=torch.int32, device="cuda")))

    def verify_step_batch():
        binding.la_verify_step_batch(vsb, s.W, s.N, s.G, s.V)
    verify_step_batch()
    run_vb, vb_calls = verify_step_batch, 1
    if use_graph:
        gvb = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gvb):
            for _ in range(8):
                verify_step_batch()
        run_vb, vb_calls = gvb.replay, 8
    vb_ms = []
    for _ in range(reps):
        e[0].record()
        run_vb()
        e[1].record()
        torch.cuda.synchronize()
        vb_ms.append(e[0].elapsed_time(e[1]) / vb_calls)
    verify_step_batch_us = float(np.median(vb_ms)) * 1e3

    # the same append for every layer in ONE launch (la_kv_commit_batch): a step has as many appends
    # as layers, all following the same best / n_out.  Layer 0's cache holds the prefix, so that it
    # can be compared with the oracle's as a whole; the others only receive rows.
    commits = []
    for li, x in enumerate(layers):
        kc_l = torch.zeros((KV, cap, d), dtype=torch.bfloat16, device="cuda") if li == 0 else \
            torch.empty((KV, cap, d), dtype=torch.bfloat16, device="cuda")
        vc_l = torch.zeros_like(kc_l) if li == 0 else torch.empty_like(kc_l)
        if li == 0:
            kc_l[:, :P], vc_l[:, :P] = x["k_cache"], x["v_cache"]
        commits.append(dict(k_cache=kc_l, v_cache=vc_l, step_k=x["step_k"], step_v=x["step_v"], best=vs_out[2],
                            n_out=vs_out[1], P=P))

    def kv_commit_batch():
        binding.la_kv_commit_batch(commits, s.W, s.N, s.G, KV, d)
    kv_commit_batch()
    run_kb, kb_calls = kv_commit_batch, 1
    if use_graph:
        gkb = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gkb):
            for _ in range(8):
                kv_commit_batch()
        run_kb, kb_calls = gkb.replay, 8
    kb_ms = []
    for _ in range(reps):
        e[0].record()
        run_kb()
        e[1].record()
        torch.cuda.synchronize()
        kb_ms.append(e[0].elapsed_time(e[1]) / kb_calls)
    kv_commit_batch_us = float(np.median(kb_ms)) * 1e3

    # several independent steps in one launch (la_step_attention_batch), timed on its own: the first
    # eight layers' inputs stand for eight sequences.  Not part of `value` (one sequence per step).
    nb = min(8, L)
    descs = [dict(q=x["q"], k_cache=x["k_cache"], v_cache=x["v_cache"], step_k=x["step_k"], step_v=x["step_v"],
                  out=torch.empty_like(o), P=P) for x, o in zip(layers[:nb], outs[:nb])]

    def batch():
        binding.la_step_attention_batch(descs, s.W, s.N, s.G, H, KV, d)
    batch()
    run_b, b_calls = batch, 1
    if use_graph:
        gb = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gb):
            for _ in range(8):
                batch()
        run_b, b_calls = gb.replay, 8
    b_ms = []
    for _ in range(reps):
        e[0].record()
        run_b()
        e[1].record()
        torch.cuda.synchronize()
        b_ms.append(e[0].elapsed_time(e[1]) / b_calls)
    batch_us = float(np.median(b_ms)) * 1e3
    batch_equal = all(float((dsc["out"].float() - o.float()).abs().max()) <= 2e-2 for dsc, o in zip(descs, outs[:nb]))
    n_commit = int(vs_out[1].item())
    kv_commit_bytes = n_commit * KV * d * 2 * 2 * 2      # rows x (K, V) x (read, write)
    abytes = algorithmic_bytes(s)
    aflops = algorithmic_flops(s)
    traffic, traffic_source = profile_traffic(args.workload)
    kernel_name = "step_attention_rowtile_kernel" if binding.la_step_attention_kernel(P, s.W, s.N, s.G, H, KV, d) == 1 \
        else "step_attention_kernel"
    roof, t_roof = roofline_object(abytes, aflops, attn_us, peaks, kernel_name, traffic, traffic_source)
    t_hbm, t_mfma = abytes / (HBM_PEAK_GBS * 1e9), aflops / (MFMA_BF16_PEAK_TFLOPS * 1e12)

    # the same launch L times on ONE layer's buffers: the caches then come from the Infinity Cache
    # and the L2, not from HBM.  Labelled as such; never the headline.
    x0 = layers[0]

    def cache_hot():
        binding.la_step_attention(x0["q"], x0["k_cache"], x0["v_cache"], x0["step_k"], x0["step_v"], P, s.W, s.N, s.G,
                                  H, KV, d, outs[0])
    cache_hot_us = None if args.no_cache_hot else time_calls(torch, np, cache_hot, L, reps, use_graph)

    # the same layers over a KV cache of 8-bit floats (la_step_attention_fp8kv): the seeded draws
    # quantised per KV head, timed on their own.  Not part of `value`.
    f8_layers, f8_host0 = [], None
    for layer in range(L):
        x8 = wl.attention_inputs_fp8(s, extra=layer)
        if layer == 0:
            f8_host0 = x8
        dev8 = {k: torch.from_numpy(v).cuda() for k, v in x8.items() if k != "q"}
        dev8["q"] = layers[layer]["q"]
        f8_layers.append(dev8)
    f8_outs = [torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    f8_it = iter(range(1 << 30))

    def fp8_layer():
        i = next(f8_it) % L
        x8 = f8_layers[i]
        binding.la_step_attention_fp8kv(x8["q"], x8["k_cache"], x8["v_cache"], x8["step_k"], x8["step_v"],
                                        x8["k_scale"], x8["v_scale"], P, s.W, s.N, s.G, H, KV, d, f8_outs[i])
    for _ in range(L):
        fp8_layer()
    fp8_us = time_calls(torch, np, fp8_layer, L, reps, use_graph)
    fp8_bytes = 2 * P * KV * d + 2 * T * KV * d + 2 * T * H * d * 2

    if args.copy_calibration:
        # a copy kernel of known size: 64 MiB read + 64 MiB written per launch
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- validity: layer 0 and the verification against the CPU oracle
    from oracle import la_oracle as orc
    want = orc.step_attention(host0["q"], host0["k_cache"], host0["v_cache"], host0["step_k"],
                              host0["step_v"], P, s.W, s.N, s.G, H, KV, d)
    err = float(np.abs(outs[0].float().cpu().numpy().astype(np.float64) - want).max())
    want8 = orc.step_attention_fp8kv(f8_host0["q"], f8_host0["k_cache"], f8_host0["v_cache"], f8_host0["step_k"],
                                     f8_host0["step_v"], f8_host0["k_scale"], f8_host0["v_scale"], P, s.W, s.N, s.G,
                                     H, KV, d)
    err8 = float(np.abs(f8_outs[0].float().cpu().numpy().astype(np.float64) - want8).max())
    want_len, want_acc = orc.verify(logits_h, cand_h, s.G, s.N, s.V)
    exact = bool(np.array_equal(alen.cpu().numpy(), want_len) and np.array_equal(acc.cpu().numpy(), want_acc))
    w_out, w_best, w_window, w_len = orc.verify_step(*vs_h[:4], s.W, s.N, s.G, s.V)
    n = int(vs_out[1].item())
    exact_step = bool(vs_out[0].cpu().numpy()[:n].tolist() == w_out and int(vs_out[2].item()) == w_best and
                      np.array_equal(vs_out[3].cpu().numpy(), w_window) and
                      np.array_equal(vs_out[4].cpu().numpy(), w_len))

    exact_step_batch = True
    for h, x in zip(vsb_h[:3], vsb[:3]):      # (three of the eight: the oracle takes a while per sequence)
        b_out, b_best, b_window, b_len = orc.verify_step(*h[:4], s.W, s.N, s.G, s.V)
        nb_out = int(x["n_out"].item())
        exact_step_batch = exact_step_batch and bool(
            x["out_tokens"].cpu().numpy()[:nb_out].tolist() == b_out and int(x["best"].item()) == b_best and
            np.array_equal(x["new_window"].cpu().numpy(), b_window) and
            np.array_equal(x["accept_len"].cpu().numpy(), b_len))
    ok_h = np.zeros((KV, cap, d), np.uint16)
    ov_h = np.zeros((KV, cap, d), np.uint16)
    ok_h[:, :P], ov_h[:, :P] = host0["k_cache"], host0["v_cache"]
    orc.kv_commit(ok_h, ov_h, host0["step_k"], host0["step_v"], P, s.W, s.N, s.G, w_best, len(w_out))
    exact_commit = bool(np.array_equal(binding.bf16_bits(kc_cap), ok_h) and np.array_equal(binding.bf16_bits(vc_cap), ov_h))
    exact_commit_batch = bool(np.array_equal(binding.bf16_bits(commits[0]["k_cache"]), ok_h) and
                              np.array_equal(binding.bf16_bits(commits[0]["v_cache"]), ov_h))
    for c in commits[1:]:   # the other layers: the appended rows equal layer 0's choice of step rows
        rows = [0] + [1 + s.W * (s.N - 1) + w_best * (s.N - 1) + i for i in range(len(w_out) - 1)]
        src_k = c["step_k"][rows].transpose(0, 1)
        src_v = c["step_v"][rows].transpose(0, 1)
        exact_commit_batch = exact_commit_batch and bool(torch.equal(c["k_cache"][:, P:P + len(rows)], src_k)) \
            and bool(torch.equal(c["v_cache"][:, P:P + len(rows)], src_v))

    w_tokens = orc.verify_sample(*sm_h[:4], float(sm_h[4][0]), 1.0, s.N, s.G, s.V)
    n = int(sm_out[1].item())
    sample_equal = bool(sm_out[0].cpu().numpy()[:n].tolist() == w_tokens)
    sample_ok = sample_equal
    if not sample_equal:
        # fp32 against fp64: only a draw within rounding of what it is compared with may differ
        _, margin = orc.verify_sample_margin(*sm_h[:4], float(sm_h[4][0]), 1.0, s.N, s.G, s.V)
        sample_ok = margin < 2e-5

    cpu = None
    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host cores: repeated layer-steps of layer 0's inputs
        # plus one verification, until about 10 s of wall time have passed
        n_done, t_start = 0, time.perf_counter()
        while True:
            orc.step_attention(host0["q"], host0["k_cache"], host0["v_cache"], host0["step_k"],
                               host0["step_v"], P, s.W, s.N, s.G, H, KV, d)
            n_done += 1
            if time.perf_counter() - t_start > 10.0 or n_done >= 4 * L:
                break
        t_attn = time.perf_counter() - t_start
        t_start = time.perf_counter()
        orc.verify(logits_h, cand_h, s.G, s.N, s.V)
        t_ver = time.perf_counter() - t_start
        cpu = {"value": (t_attn / n_done + t_ver / L) * 1e6, "unit": "us/layer-step",
               "cores": orc.threads(), "kind": "oracle",
               "sample": "%d attention layer-steps of the %s shape (fp64, OpenMP over heads) + one "
                         "verification amortised over %d layers" % (n_done, s.name, L)}
        # and on one core (a few layer-steps)
        n_threads = orc.threads()
        orc.set_threads(1)
        n_one, t_start = 0, time.perf_counter()
        while n_one < 3 and time.perf_counter() - t_start < 8.0:
            orc.step_attention(host0["q"], host0["k_cache"], host0["v_cache"], host0["step_k"],
                               host0["step_v"], P, s.W, s.N, s.G, H, KV, d)
            n_one += 1
        cpu["one_core_value"] = ((time.perf_counter() - t_start) / n_one + t_ver / L) * 1e6
        cpu["one_core_sample"] = "%d attention layer-steps on one thread" % n_one
        orc.set_threads(n_threads)

    line = {
        "metric": "lookahead-step attention + verification, us per layer-step",
        "value": us_per_layer, "unit": "us/layer-step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: H%d/KV%d/d%d P=%d W=%d N=%d G=%d (T=%d), %d layers + verify "
                               "[%d,%d,%d] fp32" % (s.name, H, KV, d, P, s.W, s.N, s.G, T, L, s.G,
                                                     s.N - 1, s.V),
                   "layers": L, "graph": use_graph},
        "roofline": roof,
        "cpu_baseline": cpu,
        "verify_us": verify_us,
        "verify_step": {"us": verify_step_us, "algorithmic_bytes": verify_step_bytes,
                        "gbs": verify_step_bytes / (verify_step_us * 1e-6) / 1e9,
                        "frac_of_hbm_peak": verify_step_bytes / (verify_step_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "verify_sample": {"us": verify_sample_us, "algorithmic_bytes": verify_sample_bytes,
                          "gbs": verify_sample_bytes / (verify_sample_us * 1e-6) / 1e9,
                          "frac_of_hbm_peak": verify_sample_bytes / (verify_sample_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "verify_step_batch": {"sequences_per_launch": len(vsb), "us_per_launch": verify_step_batch_us,
                              "gbs": len(vsb) * verify_step_bytes / (verify_step_batch_us * 1e-6) / 1e9,
                              "frac_of_hbm_peak": len(vsb) * verify_step_bytes / (verify_step_batch_us * 1e-6) / 1e9
                              / HBM_PEAK_GBS},
        "rope": {"us": rope_us, "algorithmic_bytes": 2 * (T * H * d + T * KV * d) * 2,
                 "keys_only_us": rope_keys_us, "attention_with_q_rotation_us": attention_rope_us,
                 "per_layer_two_passes_us": attn_us + rope_us,
                 "per_layer_q_in_attention_us": attention_rope_us + rope_keys_us,
                 "attention_with_q_and_key_rotation_us": attention_rope_all_us,
                 "per_layer_all_in_attention_us": attention_rope_all_us,
                 "kv_commit_rope_us": kv_commit_rope_us},
        "kv_commit": {"us": kv_commit_us, "rows": n_commit, "algorithmic_bytes": kv_commit_bytes},
        "kv_commit_batch": {"layers_per_launch": L, "us_per_launch": kv_commit_batch_us,
                            "us_per_layer": kv_commit_batch_us / L},
        "batch": {"steps_per_launch": nb, "us_per_launch": batch_us, "us_per_step": batch_us / nb,
                  "frac_of_roofline": max(t_hbm, t_mfma) * nb / (batch_us * 1e-6)},
        "attention_tflops": aflops / (attn_us * 1e-6) / 1e12,
        "attention_gbs": abytes / (attn_us * 1e-6) / 1e9,
        "attention_fp8kv": {"us_per_launch": fp8_us, "algorithmic_bytes": fp8_bytes,
                            "gbs": fp8_bytes / (fp8_us * 1e-6) / 1e9,
                            "frac_of_roofline": max(fp8_bytes / (HBM_PEAK_GBS * 1e9), t_mfma) / (fp8_us * 1e-6),
                            "speedup_over_bf16_cache": attn_us / fp8_us,
                            "note": "keys and values as 8-bit floats with one scale per KV head; q and out bf16"},
        "attention_cache_hot": {"us_per_launch": cache_hot_us,
                                "note": "all launches on one layer's buffers (served by the caches, not HBM)"},
        "parity": {"attention_max_abs_err_layer0": err, "verify_bit_exact": exact,
                   "verify_step_bit_exact": exact_step, "verify_step_batch_bit_exact": exact_step_batch,
                   "verify_sample_equals_oracle": sample_equal,
                   "kv_commit_bit_exact": exact_commit, "kv_commit_batch_bit_exact": exact_commit_batch,
                   "batch_matches_single_calls": batch_equal, "attention_fp8kv_max_abs_err_layer0": err8},
    }
    print(json.dumps(line))
    if err > 2e-2 or err8 > 2e-2 or not exact or not exact_step or not exact_step_batch or not exact_commit or not exact_commit_batch \
            or not batch_equal or not sample_ok:
        print("bench.py: PARITY FAILURE", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
