#!/usr/bin/env python3
"""Benchmark of one EAGLE-3 speculative step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: feature fusion, draft-tree
expansion (depth D, top-K, N-node tree), tree-masked verification through every target layer plus the
LM head, and the acceptance walk (greedy and temperature 1).  Inputs (random-init LLaMA-shaped weights,
random KV caches) are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3] [--no-cpu-baseline] [--calibrate-copy]

--config c4 times the batched case instead (64 ragged sequences x 8-node trees: verification + acceptance, no
drafting) and prices its GEMMs against the MFMA peak.  --calibrate-copy appends three plain 256 MiB device copies
after the run, the reference that hardware-counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) are scaled by.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0       # MI355X dense bf16, published
COPY_BYTES = 256 << 20


def algorithmic_bytes(shape, n_new):
    """Bytes the method must move per step (weights once per forward, caches once per layer, logits out)."""
    b = 2 if shape.dtype == "bf16" else 4
    k, V, Vd, L, N, P, D = shape.hidden, shape.vocab, shape.draft_vocab, shape.n_layers, shape.n_nodes, shape.prefix_lo, shape.depth
    kv_row = 2 * shape.kv_dim * b
    layer_w = shape.layer_params() * b
    verify = L * (layer_w + (P + N) * kv_row) + V * k * b + N * V * 4 + 3 * N * k * 4
    draft_fwd = shape.draft_layer_params() * b + Vd * k * b + (P + n_new) * kv_row
    draft = 3 * k * k * b + D * draft_fwd
    accept = 2 * N * V * 4
    return {"verify": verify, "draft": draft, "accept": accept, "step": verify + draft + accept}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c3", choices=["c1", "c2", "c3", "c4", "c5", "chain", "ttt"])
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--n-new", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding): use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import eagle3_synth as S
    import paper_2503_01840_amd as E

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.config == "chain":
        print(json.dumps(bench_chain(args, S.get_shape("c4"), torch, S, E, dev)))
        return
    if args.config == "ttt":
        print(json.dumps(bench_ttt(args, torch, S, E, dev)))
        return
    shape = S.get_shape(args.config)
    if args.config == "c4":
        out = bench_batched(args, shape, torch, S, E, dev)
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_batched(shape)
        if args.calibrate_copy:
            calibrate_copy(torch, dev)
        print(json.dumps(out))
        return
    P, N, D, K, n_new = shape.prefix_lo, shape.n_nodes, shape.depth, shape.topk, args.n_new
    ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=64, max_depth=D, max_topk=K, max_new=max(8, n_new), device=dev)
    T = S.TensorIds
    tg = S.target_globals(shape, device=dev)
    target = {"layers": [S.layer_weights(shape, l, device=dev) for l in range(shape.n_layers)], **tg}
    draft = S.draft_weights(shape, device=dev)
    ctx.set_weights(target, draft)
    ks, vs = zip(*[S.kv_layer(shape, l, P + N, device=dev) for l in range(shape.n_layers)])
    plen = torch.tensor([P], dtype=torch.int32, device=dev)
    kv = E.KVCache(ks, vs, torch.tensor([0, P + N], dtype=torch.int32, device=dev), plen, P)
    d_slots = P + n_new + (D - 1) * K
    dk, dv = S.kv_layer(shape, 0, d_slots, device=dev, draft=True)
    dkv = E.KVCache([dk], [dv], torch.tensor([0, d_slots], dtype=torch.int32, device=dev), plen, P)
    taps = S.normal(S.SEED, T.TAPS, (3, n_new, shape.hidden), device=dev)
    tok_new = S.uniform_ints(S.SEED, T.TOK_NEW, (n_new,), 0, shape.vocab, device=dev)
    U = S.uniform01(S.SEED, T.UNIFORMS, (1, 2 * N), device=dev)
    logits = torch.empty(1, N, shape.vocab, dtype=torch.float32, device=dev)
    tapbuf = torch.empty(3, 1, N, shape.hidden, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]

    def step(record=False):
        if record: ev[0].record()
        g = E.eagle3_fuse_features(ctx, taps[0], taps[1], taps[2])
        if record: ev[1].record()
        tree = E.eagle3_draft_expand(ctx, g, tok_new, dkv, D, K, N)
        if record: ev[2].record()
        tt, pp = tree["tree_tok"][None], tree["parent"][None]
        E.eagle3_tree_verify(ctx, tt, pp, kv, logits=logits, taps=tapbuf)
        if record: ev[3].record()
        a0 = E.eagle3_accept(ctx, logits, tt, pp, 0.0)
        a1 = E.eagle3_accept(ctx, logits, tt, pp, 1.0, U)
        if record: ev[4].record()
        return a0, a1

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3

    # per-call split (events on the stream the kernels run on), outside the timed region
    parts = [0.0] * 4
    reps = min(args.steps, 10)
    for _ in range(reps):
        step(record=True)
        torch.cuda.synchronize()
        for i in range(4):
            parts[i] += ev[i].elapsed_time(ev[i + 1]) / reps

    # the same step with the caches flushed before it (a 512 MiB fill between steps evicts the 256 MB memory-side cache
    # and every L2), outside the timed region: back-to-back steps could otherwise find the first weights they read still
    # cached from the previous step's end
    flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    cold_ms = 0.0
    for i in range(reps):
        flush.fill_(i & 0xFF)
        ev[0].record()
        step()
        ev[4].record()
        torch.cuda.synchronize()
        cold_ms += ev[0].elapsed_time(ev[4]) / reps
    del flush

    # per-launch kernel durations of the weight-streaming GEMMs (HIP events attached to every dispatch on the stream
    # in use), by kernel: 64-weight-row workgroups (q/k/v, o, down), 128-weight-row ones (gate/up, LM head), draft GEMMs
    ctx.profile_begin()
    step()
    torch.cuda.synchronize()
    t64 = ctx.profile_read(1)
    t128 = ctx.profile_read(2)
    few = ctx.profile_read(0)
    ctx.profile_end()

    def kernel_line(name, what, tri):
        ms, n, by = tri
        if not n:
            return None
        return {"kernel": name, "projections": what, "launches_per_step": n, "avg_launch_us": ms / n * 1e3,
                "bytes_per_launch": by / n, "achieved": by / ms / 1e6, "unit": "GB/s", "frac": by / ms / 1e6 / HBM_PEAK_GBPS,
                "ms_per_step": ms}

    kernels = [k for k in (kernel_line("gemm_skinny_kernel<2>", "q/k/v, o, down at 60 activation rows", t64),
                           kernel_line("gemm_skinny128_kernel", "gate/up, LM head at 60 activation rows", t128),
                           kernel_line("gemm_skinny_kernel<1>", "every projection of the draft (<= 10 rows), feature fusion", few))
               if k]
    ab = algorithmic_bytes(shape, n_new)
    if not kernels:              # fp32 tiny configuration: exact-arithmetic kernels, everything sits in L2
        roofline = {"bound": "latency", "kernel": "fp32 exact-arithmetic path (tiny configuration)", "achieved": None,
                    "peak": None, "unit": "GB/s", "frac": None, "traffic": None,
                    "step_algorithmic_GB": ab["step"] / 1e9, "step_GBps": ab["step"] / ms_per_step / 1e6}
    else:
        dom = max(kernels, key=lambda k: k["ms_per_step"])          # the kernel with the largest share of the step
        traffic, traffic_src = stored_traffic(args.config, dom["kernel"])
        roofline = {
            "bound": "hbm", "kernel": dom["kernel"] + " (" + dom["projections"] + ")",
            "achieved": dom["achieved"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["frac"],
            "traffic": traffic, "traffic_source": traffic_src,
            "launches_per_step": dom["launches_per_step"], "avg_launch_us": dom["avg_launch_us"],
            "bytes_per_launch": dom["bytes_per_launch"], "kernels": kernels,
            "step_algorithmic_GB": ab["step"] / 1e9, "step_GBps": ab["step"] / ms_per_step / 1e6,
            "step_frac_of_hbm_peak": ab["step"] / ms_per_step / 1e6 / HBM_PEAK_GBPS,
        }

    out = {
        "metric": "tree tokens verified/s over the whole draft+verify step (%s-shape bs1)" % ("70B" if args.config == "c5" else "8B"),
        "value": N / ms_per_step * 1e3, "unit": "tree tokens verified/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "step_us": ms_per_step * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{args.config}: {shape.n_layers}-layer LLaMA-8B-shaped speculative step, batch 1, "
                               f"prefix {P}, tree N={N} depth={D} top-k={K}, n_new={n_new}, draft vocab {shape.draft_vocab}"
                   if args.config != "c5" else f"c5: 80-layer LLaMA-70B-shaped step, prefix {P}, N={N}, D={D}, K={K}",
                   "parallelism": "single GPU"},
        "call_us": {"fuse_features": parts[0] * 1e3, "draft_expand": parts[1] * 1e3, "tree_verify": parts[2] * 1e3,
                    "accept_greedy_plus_stochastic": parts[3] * 1e3},
        "verify_tree_tokens_per_s": N / parts[2] * 1e3,
        "ms_per_step_after_cache_flush": cold_ms,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, n_new)
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    print(json.dumps(out))


def calibrate_copy(torch, dev):
    """Three plain device-to-device copies of COPY_BYTES: what a counter run reads for them is the scale for
    the counters of every other dispatch."""
    a = torch.empty(COPY_BYTES // 4, dtype=torch.float32, device=dev).normal_()
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()


def stored_traffic(config, kernel):
    """HBM bytes per launch of `kernel` from the committed hardware-counter summary (rocprofv3 --pmc runs of this
    script are separate invocations, so the figure is a stored one): (bytes, "file @ commit it was measured at"), or
    (None, None) when no summary names this kernel."""
    path = os.path.join(ROOT, "profiles", f"{config}_gemm_pmc_traffic.txt")
    value = commit = None
    try:
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch[{kernel}]:"):
                value = float(line.split(":", 1)[1])
            elif line.startswith("measured_at_commit:"):
                commit = line.split(":", 1)[1].strip()
    except OSError:
        pass
    return (value, f"profiles/{os.path.basename(path)} @ {commit}") if value is not None else (None, None)


def bench_batched(args, shape, torch, S, E, dev):
    """c4: 64 ragged sequences, 8-node trees: one tree_verify + greedy and T=1 acceptance per step."""
    rb = S.ragged_batch(shape)
    B, N = shape.batch, shape.n_nodes
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=N, max_depth=shape.depth, max_topk=shape.topk, max_new=8, device=dev)
    tg = S.target_globals(shape, device=dev)
    ctx.set_weights({"layers": [S.layer_weights(shape, l, device=dev) for l in range(shape.n_layers)], **tg}, None)
    total = int(rb["kv_indptr"][-1])
    ks, vs = zip(*[S.kv_layer(shape, l, total, device=dev) for l in range(shape.n_layers)])
    kv = E.KVCache(ks, vs, torch.as_tensor(rb["kv_indptr"], device=dev), torch.as_tensor(rb["prefix_len"], device=dev),
                   int(rb["prefix_len"].max()))
    tt, pp = torch.as_tensor(rb["tree_tok"], device=dev), torch.as_tensor(rb["parent"], device=dev)
    logits = torch.empty(B, N, shape.vocab, device=dev)
    taps = torch.empty(3, B, N, shape.hidden, device=dev)
    U = S.uniform01(S.SEED, S.TensorIds.UNIFORMS, (B, 2 * N), device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def step(record=False):
        if record: ev[0].record()
        E.eagle3_tree_verify(ctx, tt, pp, kv, logits=logits, taps=taps)
        if record: ev[1].record()
        E.eagle3_accept(ctx, logits, tt, pp, 0.0)
        E.eagle3_accept(ctx, logits, tt, pp, 1.0, U)
        if record: ev[2].record()

    steps = min(args.steps, 10)
    for _ in range(min(args.warmup, 3)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    step(record=True)
    torch.cuda.synchronize()
    verify_ms, accept_ms = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2])
    ctx.profile_begin()
    step()
    torch.cuda.synchronize()
    g_ms, g_n, g_bytes = ctx.profile_read(3)
    ctx.profile_end()
    R = B * N
    flops = g_bytes * R                      # 2 N K bytes per launch -> 2 R N K FLOP
    kv_bytes = 2 * total * shape.kv_dim * 2 * shape.n_layers
    return {
        "metric": "tree tokens verified/s over verification + acceptance (8B-shape bs64)",
        "value": R / ms_per_step * 1e3, "unit": "tree tokens verified/s", "n_gpus": 1, "steps": steps,
        "warmup": min(args.warmup, 3), "ms_per_step": ms_per_step, "step_us": ms_per_step * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"c4: {shape.n_layers}-layer LLaMA-8B-shaped tree verification + acceptance, {B} sequences with "
                               f"{int(rb['prefix_len'].min())}..{int(rb['prefix_len'].max())}-token caches (ragged), {N}-node trees",
                   "parallelism": "single GPU"},
        "call_us": {"tree_verify": verify_ms * 1e3, "accept_greedy_plus_stochastic": accept_ms * 1e3},
        "roofline": {
            "bound": "mfma", "kernel": "gemm_wide_kernel (verification GEMMs, 512 activation rows)",
            "achieved": flops / g_ms / 1e9, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": flops / g_ms / 1e9 / MFMA_PEAK_TFLOPS, "traffic": None,
            "launches_per_step": g_n, "avg_launch_us": g_ms / g_n * 1e3, "flop_per_launch": flops / g_n,
            "gemm_ms_per_step": g_ms, "verify_flop_over_verify_time_frac": flops / verify_ms / 1e9 / MFMA_PEAK_TFLOPS,
            "kv_cache_GB_per_step": kv_bytes / 1e9, "weights_GB_per_step": g_bytes / 1e9,
        },
    }


def bench_chain(args, shape, torch, S, E, dev, length=3):
    """The serving regime of Sections 4.3 / 4.4 at the batch-64 shape: per step one batched chain draft (3 tokens per
    sequence, no tree), verification of the 64 four-node chains through the 32 target layers, acceptance, commit."""
    rb = S.ragged_batch(shape)
    B, N = shape.batch, length + 1
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=8, max_depth=4, max_topk=2, max_new=8, device=dev)
    tg = S.target_globals(shape, device=dev)
    ctx.set_weights({"layers": [S.layer_weights(shape, l, device=dev) for l in range(shape.n_layers)], **tg},
                    S.draft_weights(shape, device=dev))
    plen = rb["prefix_len"].astype("int64")
    import numpy as np
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(plen + 8)
    total = int(indptr[-1])
    ks, vs = zip(*[S.kv_layer(shape, l, total, device=dev) for l in range(shape.n_layers)])
    i32 = lambda a: torch.as_tensor(np.asarray(a), dtype=torch.int32, device=dev)
    plen0 = i32(plen)
    kv = E.KVCache(ks, vs, i32(indptr), plen0.clone(), int(plen.max()))
    dk, dv = S.kv_layer(shape, 0, total, device=dev, draft=True)
    dkv = E.KVCache([dk], [dv], i32(indptr), plen0.clone(), int(plen.max()))
    g = S.normal(S.SEED, S.TensorIds.G_NEW, (B, 1, shape.hidden), device=dev)
    tok = S.uniform_ints(S.SEED, S.TensorIds.TOK_NEW, (B, 1), 0, shape.vocab, device=dev)
    n_new = torch.ones(B, dtype=torch.int32, device=dev)
    parent = i32(np.tile(np.arange(-1, length), (B, 1)))
    logits = torch.empty(B, N, shape.vocab, device=dev)
    taps = torch.empty(3, B, N, shape.hidden, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]

    def step(record=False):
        if record: ev[0].record()
        chain_tok, _ = E.eagle3_draft_chain(ctx, g, tok, n_new, dkv, length)
        if record: ev[1].record()
        E.eagle3_tree_verify(ctx, chain_tok, parent, kv, logits=logits, taps=taps)
        if record: ev[2].record()
        al, path, bonus = E.eagle3_accept(ctx, logits, chain_tok, parent, 0.0)
        E.eagle3_commit(ctx, chain_tok, path, al, bonus, kv, taps, N, draft_kv=dkv, draft_rows=1)
        if record: ev[3].record()
        kv.prefix_len.copy_(plen0)                       # the same workload every step
        dkv.prefix_len.copy_(plen0)

    steps = min(args.steps, 10)
    for _ in range(min(args.warmup, 3)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    step(record=True)
    torch.cuda.synchronize()
    parts = [ev[i].elapsed_time(ev[i + 1]) for i in range(3)]
    return {
        "metric": "chain tokens verified/s over batched chain draft + verification + acceptance + commit (8B-shape bs64)",
        "value": B * N / ms_per_step * 1e3, "unit": "tree tokens verified/s", "n_gpus": 1, "steps": steps,
        "warmup": min(args.warmup, 3), "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"chain: {B} sequences, ragged caches of {int(plen.min())}..{int(plen.max())} tokens, chains of "
                               f"{length} draft tokens (no tree), {shape.n_layers}-layer LLaMA-8B-shaped target", "parallelism": "single GPU"},
        "call_us": {"draft_chain": parts[0] * 1e3, "tree_verify": parts[1] * 1e3, "accept_plus_commit": parts[2] * 1e3},
    }


def bench_ttt(args, torch, S, E, dev, T=2048, H=32, Hkv=8, d=128, s=2):
    """Training-time-test attention forward at an 8B-shaped training size: 2048 positions, third step."""
    q = S.normal(S.SEED, 1, (T, H, d), dtype=torch.bfloat16, device=dev)
    k = S.normal(S.SEED, 2, (s + 1, T, Hkv, d), dtype=torch.bfloat16, device=dev)
    v = S.normal(S.SEED, 3, (s + 1, T, Hkv, d), dtype=torch.bfloat16, device=dev)
    for _ in range(3):
        E.eagle3_ttt_attention(q, k, v)
    torch.cuda.synchronize()
    reps = 50
    t0 = time.perf_counter()
    for _ in range(reps):
        E.eagle3_ttt_attention(q, k, v)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    pairs = T * (T + 1) / 2 + s * T                      # visible (query, key) pairs per head
    flops = 4.0 * pairs * d * H                          # scores + values, what the method needs
    return {"metric": "training-time-test attention forward", "value": ms * 1e3, "unit": "us per call", "n_gpus": 1,
            "higher_is_better": False, "dtype": "bf16", "data": "synthetic", "ms_per_step": ms,
            "config": {"workload": f"ttt: T={T}, {H} heads / {Hkv} KV heads x {d}, simulated step {s}"},
            "roofline": {"bound": "mfma", "achieved": flops / ms / 1e9, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": flops / ms / 1e9 / MFMA_PEAK_TFLOPS, "traffic": None,
                         "note": "algorithmic FLOP of the visible pairs only; the kernel also spends MFMAs on the bf16 tail of exp(S) "
                                 "and on the masked half of the diagonal tiles"}}


def _threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count()


def cpu_baseline(shape, n_new, n_layers=8):
    """The oracle as it stands, timed on this machine's host cores on the SAME unit as `value` (one whole step: feature
    fusion, draft expansion, tree verification with the LM head, greedy and T=1 acceptance), over a bounded sample:
    everything in full except the target stack, of which `n_layers` layers are timed and scaled to all of them.
    Weights are generated beforehand (not timed)."""
    import numpy as np
    import torch
    import eagle3_synth as S
    from oracle import eagle3_oracle as O
    import pipeline as PL
    n_layers = min(n_layers, shape.n_layers)
    N, P, D, K = shape.n_nodes, shape.prefix_lo, shape.depth, shape.topk
    rnd = "bf16" if shape.dtype == "bf16" else "none"
    lazy = shape.vocab * shape.hidden > 5e8
    model = PL.OracleModel(shape, cache_layers=False, lazy_embed=lazy)
    if shape.dtype == "fp32":
        inp = PL.real_prefill_inputs(shape, model)
    else:
        inp = PL.synthetic_step_inputs(shape, n_new=n_new)
    dw = model.draft()
    taps = S.normal(S.SEED, S.TensorIds.TAPS, (3, n_new, shape.hidden))
    Ws = [O.weights_f64(S.layer_weights(shape, l)) for l in range(n_layers)]
    kvs = [tuple(O.as_f64(t) for t in PL.target_kv_cpu(shape, inp, l)) for l in range(n_layers)]
    dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    lm = O.as_f64(S.normal(S.SEED, S.TensorIds.LM_HEAD, (shape.vocab, shape.hidden), 0.02, 0.0, dt))
    fn = O.as_f64(S.normal(S.SEED, S.TensorIds.FINAL_NORM, (shape.hidden,), 0.02, 1.0, dt))
    U = S.uniform01(S.SEED, S.TensorIds.UNIFORMS, (2 * N,)).double().numpy()
    sub = shape.with_(n_layers=n_layers, taps=(0, 0, 0))
    t = {}
    t0 = time.perf_counter()
    O.fuse_features(dw["w_fc"], *[O.as_f64(taps[i]) for i in range(3)], rounding=rnd)
    t["fuse"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    tree = PL.oracle_draft(shape, model, inp, D, K, N)
    t["draft"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    x0 = model.embed()[np.asarray(tree["tree_tok"])]
    ver = O.tree_verify(sub, lambda l: Ws[l], {"lm_head": None}, tree["tree_tok"], tree["parent"], lambda l: kvs[l],
                        rounding=rnd, x0=x0)
    t["verify_layers_sample"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    rd = O._rounder(rnd)
    logits = rd(O.rmsnorm(ver["x_final"], fn, shape.rms_eps)) @ lm.T
    t["lm_head"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.accept_greedy(logits, tree["tree_tok"], tree["parent"])
    O.accept_stochastic(logits, tree["tree_tok"], tree["parent"], 1.0, U)
    t["accept"] = time.perf_counter() - t0
    step_s = t["fuse"] + t["draft"] + t["verify_layers_sample"] / n_layers * shape.n_layers + t["lm_head"] + t["accept"]
    return {"value": N / step_s, "unit": "tree tokens verified/s", "cores": _threads(), "kind": "oracle",
            "step_s_estimated": step_s, "timed_s": {k: round(v, 3) for k, v in t.items()},
            "sample": f"one whole step of the same workload through the fp64 NumPy oracle: fusion, draft expansion (depth {D}), "
                      f"LM head and both acceptance walks in full; {n_layers} of the {shape.n_layers} target layers timed and "
                      f"scaled to {shape.n_layers}"}


def cpu_baseline_batched(shape, n_seq=2, n_layers=2):
    """The oracle on the batched workload's unit (verification + acceptance of every sequence): `n_seq` sequences
    through `n_layers` target layers plus LM head and acceptance, scaled to the batch and to all layers."""
    import numpy as np
    import torch
    import eagle3_synth as S
    from oracle import eagle3_oracle as O
    rb = S.ragged_batch(shape)
    N = shape.n_nodes
    Ws = [O.weights_f64(S.layer_weights(shape, l)) for l in range(n_layers)]
    lm = O.as_f64(S.normal(S.SEED, S.TensorIds.LM_HEAD, (shape.vocab, shape.hidden), 0.02, 0.0, torch.bfloat16))
    fn = O.as_f64(S.normal(S.SEED, S.TensorIds.FINAL_NORM, (shape.hidden,), 0.02, 1.0, torch.bfloat16))
    import pipeline as PL
    emb = PL.LazyEmbedRows(shape)
    sub = shape.with_(n_layers=n_layers, taps=(0, 0, 0))
    rd = O._rounder("bf16")
    t_layers = t_rest = 0.0
    for b in range(n_seq):
        P, base = int(rb["prefix_len"][b]), int(rb["kv_indptr"][b])
        kvs = [tuple(O.as_f64(t) for t in S.kv_layer(shape, l, P, first_slot=base)) for l in range(n_layers)]
        U = S.uniform01(S.SEED + b, S.TensorIds.UNIFORMS, (2 * N,)).double().numpy()
        t0 = time.perf_counter()
        ver = O.tree_verify(sub, lambda l: Ws[l], {"lm_head": None}, rb["tree_tok"][b], rb["parent"][b],
                            lambda l: kvs[l], rounding="bf16", x0=emb[np.asarray(rb["tree_tok"][b])])
        t_layers += time.perf_counter() - t0
        t0 = time.perf_counter()
        logits = rd(O.rmsnorm(ver["x_final"], fn, shape.rms_eps)) @ lm.T
        O.accept_greedy(logits, rb["tree_tok"][b], rb["parent"][b])
        O.accept_stochastic(logits, rb["tree_tok"][b], rb["parent"][b], 1.0, U)
        t_rest += time.perf_counter() - t0
    step_s = (t_layers / n_layers * shape.n_layers + t_rest) / n_seq * shape.batch
    return {"value": shape.batch * N / step_s, "unit": "tree tokens verified/s", "cores": _threads(), "kind": "oracle",
            "step_s_estimated": step_s,
            "sample": f"{n_seq} of the {shape.batch} sequences through {n_layers} of the {shape.n_layers} target layers, LM head and "
                      f"both acceptance walks in full (fp64 NumPy oracle), scaled to the batch and to {shape.n_layers} layers"}


if __name__ == "__main__":
    main()
