#!/usr/bin/env python3
"""Bench of the verify path on one MI355X.

A step is one pass of the whole hot path on the benchmark's configs[2] (the workload the
metric is quoted on: LLaMA2-7B shape, bf16, batch 1, gamma = 8 new tokens against a
1024-token KV cache): psd_model_forward over the 8 rows, psd_spec_accept of the 8 draft
tokens against synthetic drafter logits, psd_kv_truncate to the accepted length (then the
cache length is put back to 1024 so every step sees the same shape).  Inputs are synthetic
and resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth


def weight_stream_bytes(shape):
    """Algorithmic bytes one forward pass must read for its projections: every weight matrix
    once, 2 bytes per bf16 weight (embedding rows and norm gains excluded: kilobytes)."""
    s = shape
    hd, kvd = s.n_q_heads * s.d_head, s.n_kv_heads * s.d_head
    per_layer = s.d_model * (hd + 2 * kvd) + hd * s.d_model + 3 * s.d_model * s.d_ffn
    return 2 * (s.n_layers * per_layer + s.vocab * s.d_model)


def stream_kernel_bytes(shape):
    """The share of weight_stream_bytes read by gemm_bf16_unit_kernel: the QKV, gate|up and lm_head
    projections (O runs on the column kernel, down on the unit kernel with the residual epilogue)."""
    s = shape
    hd, kvd = s.n_q_heads * s.d_head, s.n_kv_heads * s.d_head
    return 2 * (s.n_layers * (s.d_model * (hd + 2 * kvd) + 2 * s.d_model * s.d_ffn) + s.vocab * s.d_model)


def measured_traffic_bytes():
    """HBM bytes per launch of gemm_bf16_unit_kernel as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE (the committed summary under profiles/ records the commands); None if it is not there."""
    path = os.path.join(ROOT, "profiles", "bench_verify_step_llama2_7b_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_MB_PER_LAUNCH gemm_bf16_unit_kernel"):
                return float(line.split("=")[1]) * 1e6
    except OSError:
        pass
    return None


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix-core rate


def projection_bytes(shape):
    """bf16 weight bytes of the five projections of one layer / of the head."""
    s = shape
    hd, kvd = s.n_q_heads * s.d_head, s.n_kv_heads * s.d_head
    return {"QKV": 2 * s.d_model * (hd + 2 * kvd), "O": 2 * hd * s.d_model, "gate|up": 4 * s.d_model * s.d_ffn,
            "down": 2 * s.d_ffn * s.d_model, "lm_head": 2 * s.vocab * s.d_model}


def measure_ceilings(dev, quick=False, shape=None):
    """What the machine delivers on the two resources the kernels are bound by, from the library's two probe
    kernels: a plain streaming read of 2 GiB (more than the 256 MB Infinity Cache; best of several grid sizes)
    and a loop of nothing but 32x32x16 bf16 MFMAs on random operands.  Each figure is the best of the repeats."""
    import torch
    import paper_2510_26527_amd as psd
    n_bytes = 1 << 31
    src = torch.empty(n_bytes // 4, dtype=torch.int32, device=dev).random_(0, 1 << 30)
    sink = torch.zeros(1 << 20, dtype=torch.float32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    read = {}
    for blocks in ((2048,) if quick else (512, 1024, 2048, 4096, 8192)):
        best = 0.0
        for rep in range(3 if quick else 6):
            e0.record()
            psd.psd_probe_stream_read(src, sink, blocks)
            e1.record()
            torch.cuda.synchronize()
            if rep:
                best = max(best, n_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        read[blocks] = best
    # a plain read of exactly the bytes of each projection, back to back in a busy stream over rotating slices of
    # the 2 GiB buffer (nothing is served by a cache): what a step made of separate launches can at best take
    in_flow = None
    if shape is not None:
        in_flow = {}
        for name, nb in projection_bytes(shape).items():
            nb = nb // 16 * 16
            n_slices = max(2, n_bytes // nb)
            views = [src[i * (nb // 4):(i + 1) * (nb // 4)] for i in range(n_slices)]
            reps = max(1, 24 // n_slices + 1)
            for v in views:
                psd.psd_probe_stream_read(v, sink, 2048)
            e0.record()
            for _ in range(reps):
                for v in views:
                    psd.psd_probe_stream_read(v, sink, 2048)
            e1.record()
            torch.cuda.synchronize()
            in_flow[name] = {"MB": nb / 1e6, "us": e0.elapsed_time(e1) * 1e3 / (reps * n_slices)}
        per_layer = sum(in_flow[k]["us"] for k in ("QKV", "O", "gate|up", "down"))
        in_flow["weights_of_one_step_ms"] = (shape.n_layers * per_layer + in_flow["lm_head"]["us"]) * 1e-3
    del src
    seed = torch.empty(1024, dtype=torch.float32, device=dev).normal_(0, 1).to(torch.bfloat16)
    mfma = {}
    iters = 4000 if quick else 20000
    for blocks in ((512,) if quick else (256, 512, 1024)):
        best = 0.0
        for rep in range(3):
            e0.record()
            psd.psd_probe_mfma(seed, sink, blocks, iters)
            e1.record()
            torch.cuda.synchronize()
            flop = 2.0 * 32 * 32 * 16 * 4 * iters * 4 * blocks
            if rep:
                best = max(best, flop / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        mfma[blocks] = best
    return {"stream_read_GB/s": max(read.values()), "stream_read_by_blocks": read,
            "stream_read_frac_of_hbm_peak": max(read.values()) / HBM_PEAK_GBS,
            "mfma_bf16_TFLOP/s": max(mfma.values()), "mfma_by_blocks": mfma,
            "mfma_frac_of_published_peak": max(mfma.values()) / MFMA_BF16_PEAK_TFLOPS,
            "plain_read_of_each_projection_in_a_busy_stream": in_flow,
            "how": "psd_probe_stream_read over 2 GiB (non-temporal 16-byte loads, 8 in flight per lane); psd_probe_mfma "
                   "(32x32x16 bf16 on 4 accumulators per wavefront, random operands); best of the repeats"}


def ceilings_workload(args, dev):
    from paper_2510_26527_amd import synth
    c = measure_ceilings(dev, shape=synth.LLAMA2_7B)
    print(json.dumps({"metric": "measured ceilings of this MI355X", "unit": "GB/s and TFLOP/s", "n_gpus": 1,
                      "data": "synthetic", "config": {"workload": "library probe kernels: streaming read, MFMA-only loop"},
                      "published": {"hbm_GB/s": HBM_PEAK_GBS, "mfma_bf16_TFLOP/s": MFMA_BF16_PEAK_TFLOPS},
                      "ceilings": c}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--accept-iters", type=int, default=60)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run ten plain 1 GiB device-to-device copies (a kernel of known traffic, for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--workload", choices=["verify", "stress", "chain", "sweep", "ceilings", "tree"], default="verify",
                    help="verify (default): configs[2] verify step + configs[1] acceptance, the headline line; "
                         "stress: configs[4], 16 sequences x 16 rows of a Qwen2-7B-shaped model; "
                         "chain: configs[3], the full-size three-level chain with the agreement harness; "
                         "sweep: the projections of a LLaMA2-7B-shaped layer at 8 ... 4096 rows; "
                         "ceilings: the measured streaming-read and MFMA-only rates of this GPU")
    ap.add_argument("--sigma", type=float, default=0.25, help="noise of the agreement harness (--workload chain)")
    ap.add_argument("--tokens", type=int, default=512, help="tokens to generate (--workload chain)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (sequences of a batch are independent and "
              "would shard across GPUs without any exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2510_26527_amd as psd
    from paper_2510_26527_amd import runtime, synth
    if not os.path.exists(psd.LIB_PATH):
        from paper_2510_26527_amd import build
        build.build()
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs the GPU: no CPU fallback exists")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": "10 x copy of 1 GiB (reads 1 GiB, writes 1 GiB each)"}))
        return

    if args.workload == "stress":
        return stress_workload(args, dev)
    if args.workload == "chain":
        return chain_workload(args, dev)
    if args.workload == "sweep":
        return sweep_workload(args, dev)
    if args.workload == "ceilings":
        return ceilings_workload(args, dev)
    if args.workload == "tree":
        return tree_workload(args, dev)

    shape, gamma, ctx, max_len, temperature = synth.LLAMA2_7B, 8, 1024, 1088, 1.0
    w_cpu = synth.make_weights(shape, 3, torch.bfloat16)
    model = runtime.Model(shape, w_cpu, dev).pack()      # streaming copy of the weights for steps of <= 16 rows
    kv = runtime.KVCache(model, 1, max_len)
    ks, vs = synth.make_kv_fill(shape, 1, ctx, 4, torch.bfloat16)
    kv.load(ks, vs, ctx)
    tok_np = synth.make_tokens(shape.vocab, (1, gamma), 33)
    tokens = torch.from_numpy(tok_np).to(dev)
    p_buf = torch.empty((1, gamma, shape.vocab), dtype=torch.float32, device=dev)
    base = torch.full((1,), ctx, dtype=torch.int32, device=dev)
    acc = runtime.Acceptor(dev)
    uniforms = synth.make_uniforms((1, gamma + 1), 6, dev)

    # one forward outside the timed region fixes the synthetic drafter (q = p + N(0, 0.5^2))
    runtime.forward(model, kv, tokens, logits_out=p_buf)
    psd.psd_kv_truncate_to(kv.handle, ctx)
    q_logits, draft = synth.make_draft_from_target(p_buf, 0.5, 7)
    torch.cuda.synchronize()

    out = {}

    def step():
        runtime.forward(model, kv, tokens, logits_out=p_buf)
        n, tok, fl = acc(p_buf, q_logits, draft, uniforms, temperature)
        psd.psd_kv_truncate(kv.handle, base, n, 1, ctx + 1 + gamma)
        psd.psd_kv_truncate_to(kv.handle, ctx)          # back to the benchmark's cache length
        out["n"] = n

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    accepted = int(out["n"].item())

    # mean tokens committed per verify step (accepted + 1) over steps that differ only in their uniforms
    n_draws = 32
    kept = torch.zeros(n_draws, dtype=torch.int32, device=dev)
    for i in range(n_draws):
        u_i = synth.make_uniforms((1, gamma + 1), 1000 + i, dev)
        runtime.forward(model, kv, tokens, logits_out=p_buf)
        n_i, _, _ = acc(p_buf, q_logits, draft, u_i, temperature)
        kept[i:i + 1].copy_(n_i)
        psd.psd_kv_truncate_to(kv.handle, ctx)
    mean_committed = float(kept.float().mean().item()) + 1.0

    # the same step with the bonus row (n_new = gamma + 1: the x* row and the gamma draft tokens, as in the chain)
    tokens9 = torch.from_numpy(synth.make_tokens(shape.vocab, (1, gamma + 1), 34)).to(dev)
    p9 = torch.empty((1, gamma + 1, shape.vocab), dtype=torch.float32, device=dev)
    runtime.forward(model, kv, tokens9, logits_out=p9)
    psd.psd_kv_truncate_to(kv.handle, ctx)
    q9, draft9 = synth.make_draft_from_target(p9[:, :gamma], 0.5, 8)

    def step9():
        runtime.forward(model, kv, tokens9, logits_out=p9)
        n, tok, fl = acc(p9, q9, draft9, uniforms, temperature)
        psd.psd_kv_truncate(kv.handle, base, n, 1, ctx + 1 + gamma)
        psd.psd_kv_truncate_to(kv.handle, ctx)

    for _ in range(3):
        step9()
    torch.cuda.synchronize()
    t9 = time.perf_counter()
    for _ in range(min(args.steps, 30)):
        step9()
    torch.cuda.synchronize()
    ms9 = (time.perf_counter() - t9) * 1e3 / min(args.steps, 30)
    ceilings = measure_ceilings(dev, quick=True, shape=shape)

    # same steps again with every launch bracketed by HIP events on its stream
    launches_per_step = 40 * shape.n_layers + 64          # room in the event buffer: more than any path launches
    prof_steps = min(args.steps, 20)
    psd.psd_profile_enable(launches_per_step * prof_steps)
    for _ in range(prof_steps):
        step()
    prof = psd.psd_profile_collect()
    psd.psd_profile_enable(0)
    kernels = {k: {"launches_per_step": c / prof_steps, "avg_us": 1e3 * ms / c, "ms_per_step": ms / prof_steps}
               for k, (ms, c) in prof.items() if c}
    # dominant kernel: gemm_bf16_unit_kernel (QKV, gate|up and lm_head projections: 65 launches per step, 82 % of the
    # step's bytes); the O / down projections (column kernel) beside it
    sk_ms, sk_n = prof["gemm_skinny"]
    w_bytes = weight_stream_bytes(shape)
    stream_bytes = stream_kernel_bytes(shape)
    achieved = stream_bytes * prof_steps / (sk_ms * 1e-3) / 1e9
    roofline = {"kernel": "gemm_bf16_unit_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic_bytes(),
                "bytes_per_launch": stream_bytes * prof_steps / sk_n, "avg_launch_us": 1e3 * sk_ms / sk_n,
                "launches_per_step": sk_n / prof_steps,
                "measured_stream_read_GB/s": ceilings["stream_read_GB/s"],
                "frac_of_measured_stream_read": achieved / ceilings["stream_read_GB/s"]}
    gemm_ms = sk_ms
    others = (("gemm_column", "gemm_bf16_column_kernel (O) and gemm_bf16_unit_kernel<true> (down): the projections with the residual add",
               w_bytes - stream_bytes),)
    roofline["other_gemms"] = []
    for kind, label, nbytes in others:
        if kind in prof and prof[kind][1]:
            k_ms, k_n = prof[kind]
            gemm_ms += k_ms
            roofline["other_gemms"].append({"kernel": label, "achieved": nbytes * prof_steps / (k_ms * 1e-3) / 1e9,
                                            "unit": "GB/s", "bytes_per_launch": nbytes * prof_steps / k_n,
                                            "avg_launch_us": 1e3 * k_ms / k_n, "launches_per_step": k_n / prof_steps})
    roofline["all_weight_streaming_GB/s"] = w_bytes * prof_steps / (gemm_ms * 1e-3) / 1e9
    kv_bytes = 2 * shape.n_layers * shape.n_kv_heads * (ctx + gamma) * shape.d_head * 2
    step_floor_ms = (w_bytes + kv_bytes) / (HBM_PEAK_GBS * 1e9) * 1e3
    a_ms, a_n = prof["attn"]
    cmb_ms = prof["attn_combine"][0] if "attn_combine" in prof else 0.0
    attention = {"kernel": "attn_mfma_kernel (split over the KV length; builds q / k / v from the QKV partial sums)",
                 "bytes_per_layer": kv_bytes / shape.n_layers, "avg_launch_us": 1e3 * a_ms / a_n,
                 "GB/s": kv_bytes * prof_steps / (a_ms * 1e-3) / 1e9,
                 "GB/s_with_combine": kv_bytes * prof_steps / ((a_ms + cmb_ms) * 1e-3) / 1e9,
                 "frac_of_hbm_peak": kv_bytes * prof_steps / (a_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    # ---- the isolated acceptance workload (configs[1]): 64 x 8 x 32000 bf16, cold HBM
    sets = [synth.make_accept_inputs(64, 8, 32000, 100 + i, dtype=torch.bfloat16, device=dev) for i in range(6)]
    acc2 = runtime.Acceptor(dev)
    for s in sets:
        acc2(s["p"], s["q"], s["tokens"], s["uniforms"], 1.0)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(args.accept_iters):
        s = sets[i % len(sets)]
        acc2(s["p"], s["q"], s["tokens"], s["uniforms"], 1.0)
    e1.record(stream)
    torch.cuda.synchronize()
    call_us = e0.elapsed_time(e1) * 1e3 / args.accept_iters
    psd.psd_profile_enable(4 * args.accept_iters)
    for i in range(args.accept_iters):
        s = sets[i % len(sets)]
        acc2(s["p"], s["q"], s["tokens"], s["uniforms"], 1.0)
    aprof = psd.psd_profile_collect()
    psd.psd_profile_enable(0)
    a_bytes = 64 * 8 * 32000 * 2 * 2
    stats_us = 1e3 * aprof["accept_stats"][0] / aprof["accept_stats"][1]
    accept = {"workload": "configs[1]: 64 rows x gamma 8 x vocab 32000 bf16, 6 rotating input sets (393 MB)",
              "algorithmic_bytes": a_bytes, "call_us": call_us, "GB/s": a_bytes / call_us / 1e3,
              "frac_of_hbm_peak": a_bytes / call_us / 1e3 / HBM_PEAK_GBS,
              "stats_kernel_us": stats_us, "stats_kernel_GB/s": a_bytes / stats_us / 1e3,
              "draw_kernel_us": 1e3 * aprof["accept_draw"][0] / aprof["accept_draw"][1]}

    # ---- the oracle on the host cores, one whole step of the same workload
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import accept as oacc
        from oracle import forward as ofwd
        from threadpoolctl import threadpool_info
        cfg = ofwd.ModelConfig(**shape.asdict())
        okv = ofwd.KVCache(cfg, 1, max_len, np.float32)
        for l in range(shape.n_layers):
            okv.k[l][:, :, :ctx] = ks[l].float().numpy()
            okv.v[l][:, :, :ctx] = vs[l].float().numpy()
        okv.lens[:] = ctx
        c0 = time.perf_counter()
        ref = ofwd.forward(cfg, w_cpu, tok_np, okv)
        oacc.spec_accept(ref, q_logits.cpu().double().numpy(), draft.cpu().numpy(), uniforms.cpu().double().numpy(),
                         temperature)
        okv.truncate(ctx)
        c1 = time.perf_counter()
        threads = max([torch.get_num_threads()] + [p.get("num_threads", 1) for p in threadpool_info()])
        # the acceptance oracle alone on one configs[1] input set (single-threaded C, fp64)
        s0 = sets[0]
        a0 = time.perf_counter()
        oacc.spec_accept(s0["p"].float().cpu().numpy(), s0["q"].float().cpu().numpy(), s0["tokens"].cpu().numpy(),
                         s0["uniforms"].cpu().double().numpy(), 1.0)
        a1 = time.perf_counter()
        accept["cpu_oracle_ms"] = (a1 - a0) * 1e3
        accept["cpu_oracle_GB/s"] = a_bytes / (a1 - a0) / 1e9
        cpu_baseline = {"value": gamma / (c1 - c0), "unit": "tokens/s", "cores": threads, "kind": "oracle",
                        "sample": "one whole step of the same workload (32 layers + lm_head forward in numpy fp64, "
                                  "acceptance in C fp64, rollback), %.1f s" % (c1 - c0)}

    line = {
        "metric": "verify-step tokens/s (7B shape, γ=8, ctx 1k) + accept-kernel HBM GB/s",
        "value": gamma * 1e3 / ms_per_step, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "configs[2]: LLaMA2-7B-shaped random-init bf16, batch 1, gamma=8 new tokens on a "
                               "1024-token N(0,1) bf16 KV cache, forward + acceptance + KV rollback",
                   "gamma": gamma, "n_new": gamma, "kv_len": ctx, "batch": 1, "temperature": temperature},
        "accepted_this_step": accepted,
        "mean_tokens_committed_per_step": mean_committed,
        "expected_committed_tokens/s": mean_committed * 1e3 / ms_per_step,
        "with_bonus_row": {"n_new": gamma + 1, "ms_per_step": ms9, "verified_tokens/s": gamma * 1e3 / ms9},
        "step_floor_ms_at_hbm_peak": step_floor_ms,
        "step_floor_ms_at_measured_stream_read": (w_bytes + kv_bytes) / (ceilings["stream_read_GB/s"] * 1e9) * 1e3,
        "step_floor_ms_separate_launches": ceilings["plain_read_of_each_projection_in_a_busy_stream"]["weights_of_one_step_ms"],
        "ceilings": ceilings,
        "attention": attention,
        "roofline": roofline, "cpu_baseline": cpu_baseline, "accept_kernel": accept, "kernels": kernels,
    }
    print(json.dumps(line))


def tree_workload(args, dev):
    """A token-tree verify step at the headline shape: LLaMA2-7B-shaped model, 1024-token cache, one binary tree of
    depth 3 (root + 14 drafted nodes) per step: forward over the tree, acceptance down the tree, compaction of the
    accepted path.  The drafter is synthetic (q = p + N(0, 0.5^2), children drawn from q at their parent)."""
    import torch
    import paper_2510_26527_amd as psd
    from paper_2510_26527_amd import runtime, synth
    shape, ctx, max_len = synth.LLAMA2_7B, 1024, 1088
    parents = [-1] + [(i - 1) // 2 for i in range(1, 15)]
    n = len(parents)
    model = runtime.Model(shape, synth.make_weights(shape, 3, torch.bfloat16), dev).pack()
    kv = runtime.KVCache(model, 1, max_len)
    ks, vs = synth.make_kv_fill(shape, 1, ctx, 4, torch.bfloat16)
    kv.load(ks, vs, ctx)
    tokens = torch.from_numpy(synth.make_tokens(shape.vocab, (1, n), 33)).to(dev)
    p_buf = torch.empty((1, n, shape.vocab), dtype=torch.float32, device=dev)
    base = torch.full((1,), ctx, dtype=torch.int32, device=dev)
    runtime.forward_tree(model, kv, tokens, parents, logits_out=p_buf)
    psd.psd_kv_truncate_to(kv.handle, ctx)
    g = torch.Generator(device=dev).manual_seed(7)
    q_logits = p_buf + 0.5 * torch.randn(p_buf.shape, generator=g, device=dev)
    gum = -torch.log(-torch.log(torch.rand(p_buf.shape, generator=g, device=dev).clamp_min(1e-12)))
    for i in range(1, n):                                  # children: draws from the drafter's row at their parent
        tokens[0, i] = torch.argmax(q_logits[0, parents[i]] + gum[0, i]).to(torch.int32)
    runtime.forward_tree(model, kv, tokens, parents, logits_out=p_buf)      # the verifier's rows for those tokens
    psd.psd_kv_truncate_to(kv.handle, ctx)
    uniforms = synth.make_uniforms((1, n + 1), 6, dev)
    out = {}

    def step():
        runtime.forward_tree(model, kv, tokens, parents, logits_out=p_buf)
        ln, path, tok, fl = runtime.tree_accept(p_buf, q_logits, tokens, parents, uniforms, 1.0)
        psd.psd_kv_compact_tree(kv.handle, base, path, ln, n, n, ctx + n)
        psd.psd_kv_truncate_to(kv.handle, ctx)
        out["len"] = ln

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    prof_steps = min(args.steps, 20)
    psd.psd_profile_enable((40 * shape.n_layers + 64) * prof_steps)
    for _ in range(prof_steps):
        step()
    prof = psd.psd_profile_collect()
    psd.psd_profile_enable(0)
    kernels = {k: {"launches_per_step": c / prof_steps, "avg_us": 1e3 * t / c, "ms_per_step": t / prof_steps}
               for k, (t, c) in prof.items() if c}
    kept = []
    for i in range(32):                                    # committed tokens per step over steps that differ in their uniforms
        u_i = synth.make_uniforms((1, n + 1), 1000 + i, dev)
        ln, _, _, _ = runtime.tree_accept(p_buf, q_logits, tokens, parents, u_i, 1.0)
        kept.append(int(ln.item()) + 1)
    line = {
        "metric": "tree verify-step nodes/s (7B shape, binary tree of 15 nodes, ctx 1k)", "value": n * 1e3 / ms,
        "unit": "nodes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "LLaMA2-7B-shaped random-init bf16, batch 1, a 15-node binary token tree per step on a "
                               "1024-token cache: tree forward + tree acceptance + compaction", "n_nodes": n, "kv_len": ctx},
        "accepted_path_len_this_step": int(out["len"].item()),
        "mean_tokens_committed_per_step": sum(kept) / len(kept),
        "expected_committed_tokens/s": sum(kept) / len(kept) * 1e3 / ms,
        "kernels": kernels,
    }
    print(json.dumps(line))


def stress_workload(args, dev):
    """configs[4]: Qwen2-7B-shaped bf16 model, 16 independent sequences, 16 new rows each against 4096-token
    caches, per-sequence acceptance against a synthetic drafter (q = p + N(0, 0.5^2)), on-device rollback."""
    import torch
    import paper_2510_26527_amd as psd
    from paper_2510_26527_amd import runtime, synth
    shape, B, gamma, ctx, max_len = synth.QWEN2_7B, 16, 16, 4096, 4160
    w = synth.make_weights(shape, 5, torch.bfloat16, device=dev)
    model = runtime.Model(shape, w, dev)
    kv = runtime.KVCache(model, B, max_len)
    gen = torch.Generator(device=dev)
    gen.manual_seed(51)
    kv.k.normal_(generator=gen)
    kv.v.normal_(generator=gen)
    kv.load([kv.k[l, :, :, :ctx] for l in range(shape.n_layers)],
            [kv.v[l, :, :, :, :ctx].transpose(-1, -2) for l in range(shape.n_layers)], ctx)
    tokens = torch.from_numpy(synth.make_tokens(shape.vocab, (B, gamma), 55)).to(dev)
    p_buf = torch.empty((B, gamma, shape.vocab), dtype=torch.float32, device=dev)
    base = torch.full((B,), ctx, dtype=torch.int32, device=dev)
    acc = runtime.Acceptor(dev)
    uniforms = synth.make_uniforms((B, gamma + 1), 56, dev)
    runtime.forward(model, kv, tokens, logits_out=p_buf)
    psd.psd_kv_truncate_to(kv.handle, ctx)
    q_logits, draft = synth.make_draft_from_target(p_buf, 0.5, 57)
    out = {}

    def step():
        runtime.forward(model, kv, tokens, logits_out=p_buf)
        n, tok, fl = acc(p_buf, q_logits, draft, uniforms, 1.0)
        psd.psd_kv_truncate(kv.handle, base, n, 1, ctx + 1 + gamma)
        psd.psd_kv_truncate_to(kv.handle, ctx)          # back to the benchmark's cache length
        out["n"] = n

    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    prof_steps = 3
    psd.psd_profile_enable(3000 * prof_steps)
    for _ in range(prof_steps):
        step()
    prof = psd.psd_profile_collect()
    psd.psd_profile_enable(0)
    kernels = {k: {"launches_per_step": c / prof_steps, "avg_us": 1e3 * t / c, "ms_per_step": t / prof_steps}
               for k, (t, c) in prof.items() if c}
    # the oracle on the host cores: ONE of the 16 sequences (its 16 rows against its 4096-token cache), forward +
    # acceptance + rollback; the other fifteen would cost the same again each
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import accept as oacc
        from oracle import forward as ofwd
        from threadpoolctl import threadpool_info
        b0 = 0
        cfg = ofwd.ModelConfig(**shape.asdict())
        w_host = {k: v.cpu() for k, v in w.items()}
        okv = ofwd.KVCache(cfg, 1, max_len, np.float32)
        for l in range(shape.n_layers):
            okv.k[l][:, :, :ctx] = kv.k[l, b0:b0 + 1, :, :ctx].float().cpu().numpy()
            okv.v[l][:, :, :ctx] = kv.v[l, b0:b0 + 1, :, :, :ctx].transpose(-1, -2).float().cpu().numpy()
        okv.lens[:] = ctx
        tok_host = tokens[b0:b0 + 1].cpu().numpy()
        q_host, d_host = q_logits[b0:b0 + 1].cpu().double().numpy(), draft[b0:b0 + 1].cpu().numpy()
        u_host = uniforms[b0:b0 + 1].cpu().double().numpy()
        c0 = time.perf_counter()
        ref = ofwd.forward(cfg, w_host, tok_host, okv)
        oacc.spec_accept(ref, q_host, d_host, u_host, 1.0)
        okv.truncate(ctx)
        c1 = time.perf_counter()
        threads = max([torch.get_num_threads()] + [p.get("num_threads", 1) for p in threadpool_info()])
        cpu_baseline = {"value": gamma / (c1 - c0), "unit": "tokens/s", "cores": threads, "kind": "oracle",
                        "sample": "one of the 16 sequences (16 rows on a 4096-token cache: forward in numpy fp64, acceptance "
                                  "in C fp64, rollback), %.1f s; the whole step is 16 of these" % (c1 - c0)}
        del w_host, okv
    s = shape
    hd, kvd = s.n_q_heads * s.d_head, s.n_kv_heads * s.d_head
    flops = 2.0 * B * gamma * (s.n_layers * (s.d_model * (hd + 2 * kvd) + hd * s.d_model + 3 * s.d_model * s.d_ffn)
                               + s.vocab * s.d_model)
    g_ms = prof["gemm_tiled"][0] / prof_steps
    kv_bytes = 2.0 * s.n_layers * B * s.n_kv_heads * (ctx + gamma) * s.d_head * 2
    a_ms = prof["attn"][0] / prof_steps
    tf = flops / (g_ms * 1e-3) / 1e12
    line = {
        "metric": "stress verify-step tokens/s (Qwen2-7B shape, 16 sequences x gamma=16, ctx 4k)",
        "value": B * gamma * 1e3 / ms, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "configs[4]: Qwen2-7B-shaped random-init bf16, 16 sequences, gamma=16 new tokens each on "
                               "4096-token N(0,1) caches, forward + per-sequence acceptance + KV rollback",
                   "gamma": gamma, "n_new": gamma, "kv_len": ctx, "batch": B, "temperature": 1.0},
        "accepted_mean": float(out["n"].float().mean().item()),
        "roofline": {"kernel": "gemm_f16_tiled_kernel", "bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": tf / 2500.0, "traffic": None, "flop_per_step": flops, "ms_per_step": g_ms,
                     "note": "bf16 weights and fp16-rounded activations multiplied by 32x32x16 f16 MFMAs, fp32 accumulation; one MFMA pass"},
        "attention": {"kernel": "attn_mfma_wide_kernel", "bytes_per_step": kv_bytes, "ms_per_step": a_ms,
                      "GB/s": kv_bytes / (a_ms * 1e-3) / 1e9},
        "cpu_baseline": cpu_baseline, "kernels": kernels,
    }
    print(json.dumps(line))


def chain_workload(args, dev):
    """configs[3]: LLaMA3-8B-shaped target, 16-layer intermediate, one-layer draft sharing the target's embedding and
    lm_head; 256-token prompt, gamma_draft 6, gamma_intermediate 10, temperature 1, agreement harness at --sigma."""
    import torch
    import paper_2510_26527_amd as psd
    from paper_2510_26527_amd import chain as gchain
    from paper_2510_26527_amd import costmodel, runtime, shim, synth
    n_gen, n_prompt, max_len, gammas = args.tokens, 256, 256 + args.tokens + 128, [None, 10, 6]
    max_len = (max_len + 63) // 64 * 64
    tw = synth.make_weights(synth.LLAMA3_8B, 401, torch.bfloat16, device=dev)
    mw = synth.make_weights(synth.CHAIN_INTERMEDIATE, 402, torch.bfloat16, device=dev)
    dw = synth.make_weights(synth.CHAIN_DRAFT, 403, torch.bfloat16, device=dev,
                            share={"embed": tw["embed"], "lm_head": tw["lm_head"]})
    models = [runtime.Model(synth.LLAMA3_8B, tw, dev).pack(), runtime.Model(synth.CHAIN_INTERMEDIATE, mw, dev).pack(),
              runtime.Model(synth.CHAIN_DRAFT, dw, dev).pack()]
    levels = [gchain.Level(models[0], max_len, 11), gchain.Level(models[1], max_len, 11), gchain.Level(models[2], max_len, 7)]
    prompt = synth.make_tokens(synth.LLAMA3_8B.vocab, (n_prompt,), 77).tolist()
    tapes = [synth.make_tape(14, 0, 3 * n_gen, 16), synth.make_tape(14, 1, 6 * n_gen, 16),
             synth.make_tape(14, 2, 30 * n_gen, 1)[:, 0]]
    g = shim.AgreementShimChain(levels, gammas, tapes, args.sigma, noise_seed=5, temperature=1.0, max_len=max_len, timed=True)
    g.forward_log = []
    t0 = time.perf_counter()
    g.generate(prompt, n_gen)
    wall_ms = (time.perf_counter() - t0) * 1e3
    cpu_baseline = None if args.no_cpu_baseline else chain_cpu_baseline(g, levels, [tw, mw, dw], n_prompt, max_len)
    rep = costmodel.chain_report(n_gen, [lv.forwards for lv in levels], [lv.time_ms for lv in levels], g.accept_ms)
    # the target decoding alone, one token per forward, same kernels and cache length
    tgt = levels[0]
    at = n_prompt + n_gen // 2
    psd.psd_kv_truncate_to(tgt.kv.handle, at)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for it in range(40):
        if it == 8:
            e0.record()
        psd.psd_model_forward(tgt.model.handle, g.seq[at:at + 1], 1, tgt.kv.handle, tgt.rows[0:1], 1, tgt.ws)
        psd.psd_kv_truncate_to(tgt.kv.handle, at)
    e1.record()
    torch.cuda.synchronize()
    t_ar = e0.elapsed_time(e1) / 32
    chain_ms = rep["eq2_ms"] + rep["accept_ms"]
    line = {
        "metric": "three-level chain tokens/s (LLaMA3-8B-shaped target, harness sigma %.2f)" % args.sigma,
        "value": n_gen * 1e3 / chain_ms, "unit": "tokens/s", "n_gpus": 1, "steps": n_gen, "warmup": 0,
        "ms_per_step": chain_ms / n_gen, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "configs[3]: LLaMA3-8B-shaped target, 16-layer d=2048 intermediate, 1-layer draft, bf16 random "
                               "init, 256-token prompt, gamma_draft 6, gamma_intermediate 10, temperature 1",
                   "sigma": args.sigma, "tokens": n_gen},
        "value_counts": "GPU time of the three models' forwards and the acceptance calls (Eq. 2 + acceptance); the harness's "
                        "untimed target peeks and the host loop are excluded",
        "report": rep, "tokens_per_target_forward": n_gen / rep["F"][0],
        "target_only_ms_per_token": t_ar, "speedup_vs_target_only": t_ar * n_gen / chain_ms,
        "harness": {"peeks": g.peeks, "peek_ms": g.peek_ms, "wall_ms": wall_ms}, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(line))


def chain_cpu_baseline(g, levels, weights, n_prompt, max_len):
    """The oracle's forwards over the chain's first target cycle: every forward the three models made from the end
    of the prompt up to and including the target's first verification, replayed on the host cores from the same
    cache state (the prompt's K/V are copied from the GPU caches; the harness's untimed target peeks are left out,
    as they are from the GPU figure)."""
    import numpy as np
    import torch
    from oracle import forward as ofwd
    from threadpoolctl import threadpool_info
    shapes = [lv.model.shape for lv in levels]
    cfgs = [ofwd.ModelConfig(**sh.asdict()) for sh in shapes]
    w_host = [{k: v.cpu() for k, v in w.items()} for w in weights]
    okvs = []
    for lv, cfg, sh in zip(levels, cfgs, shapes):
        okv = ofwd.KVCache(cfg, 1, max_len, np.float32)
        for l in range(sh.n_layers):
            okv.k[l][:, :, :n_prompt - 1] = lv.kv.k[l, :, :, :n_prompt - 1].float().cpu().numpy()
            okv.v[l][:, :, :n_prompt - 1] = lv.kv.v[l, :, :, :, :n_prompt - 1].transpose(-1, -2).float().cpu().numpy()
        okv.lens[:] = n_prompt - 1
        okvs.append(okv)
    first = [k for k, ev in enumerate(g.forward_log) if ev[0] == 0 and ev[1] >= n_prompt - 1][0]
    cycle = [ev for ev in g.forward_log[:first + 1] if ev[1] >= n_prompt - 1]
    committed = len(cycle[-1][2]) - 1          # upper bound of what the cycle commits: its block + the extra token
    c0 = time.perf_counter()
    for i, start, toks in cycle:
        if int(okvs[i].lens[0]) > start:
            okvs[i].truncate(start)
        ofwd.forward(cfgs[i], w_host[i], np.asarray([toks], np.int32), okvs[i])
    c1 = time.perf_counter()
    threads = max([torch.get_num_threads()] + [p.get("num_threads", 1) for p in threadpool_info()])
    counts = [sum(1 for ev in cycle if ev[0] == i) for i in range(len(levels))]
    return {"value": committed / (c1 - c0), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "the forwards of the first target cycle (%d target, %d intermediate, %d draft forwards, at most %d "
                      "tokens committed) in numpy fp64, %.1f s; acceptance calls left out (milliseconds)"
                      % (counts[0], counts[1], counts[2], committed, c1 - c0)}


def sweep_workload(args, dev):
    """The four projections of LLaMA2-7B-shaped layers (plus a 32000-row lm_head) at M = 8 ... 4096 rows: one
    forward of a two-layer model per M on an empty cache; GEMM time from the per-launch timers.  Up to 16 rows
    the projections stream the weights (HBM-bound, GB/s); above, they run on the LDS-tiled MFMA kernel (TFLOP/s)."""
    import torch
    import paper_2510_26527_amd as psd
    from paper_2510_26527_amd import runtime, synth
    q = synth.LLAMA2_7B
    shape = synth.Shape(2, q.d_model, q.n_q_heads, q.n_kv_heads, q.d_head, q.d_ffn, q.vocab, q.rope_theta)
    w = synth.make_weights(shape, 3, torch.bfloat16, device=dev)
    model = runtime.Model(shape, w, dev).pack()
    s = shape
    hd, kvd = s.n_q_heads * s.d_head, s.n_kv_heads * s.d_head
    params = s.n_layers * (s.d_model * (hd + 2 * kvd) + hd * s.d_model + 3 * s.d_model * s.d_ffn) + s.vocab * s.d_model
    rows = []
    for M in (8, 16, 32, 64, 128, 256, 512, 1024, 4096):
        max_len = (M + 63) // 64 * 64
        kv = runtime.KVCache(model, 1, max_len)
        toks = torch.from_numpy(synth.make_tokens(s.vocab, (1, M), M)).to(dev)
        logits = torch.empty((1, M, s.vocab), dtype=torch.float32, device=dev)
        for _ in range(2):
            runtime.forward(model, kv, toks, logits_out=logits)
            psd.psd_kv_truncate_to(kv.handle, 0)
        reps = 5
        psd.psd_profile_enable(200 * reps)
        for _ in range(reps):
            runtime.forward(model, kv, toks, logits_out=logits)
            psd.psd_kv_truncate_to(kv.handle, 0)
        torch.cuda.synchronize()
        prof = psd.psd_profile_collect()
        psd.psd_profile_enable(0)
        g_ms = sum(prof[k][0] for k in ("gemm_skinny", "gemm_slot", "gemm_column", "gemm_tiled") if k in prof) / reps
        flops = 2.0 * M * params
        rows.append({"M": M, "gemm_ms": g_ms, "TFLOP/s": flops / (g_ms * 1e-3) / 1e12,
                     "frac_of_bf16_mfma_peak": flops / (g_ms * 1e-3) / 2.5e15,
                     "weight_GB/s": 2.0 * params / (g_ms * 1e-3) / 1e9,
                     "frac_of_hbm_peak": 2.0 * params / (g_ms * 1e-3) / 8e12,
                     "kernel": "weight streaming" if M <= 16 else "LDS-tiled MFMA"})
        kv.close()
        del logits
    print(json.dumps({"metric": "projection GEMMs of a LLaMA2-7B-shaped layer over M", "unit": "TFLOP/s and GB/s",
                      "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "two LLaMA2-7B-shaped layers + lm_head, one forward of M rows on an empty cache",
                                 "weights_GB": 2.0 * params / 1e9},
                      "note": "useful flops; up to 16 rows: bf16 weights streamed against hi + lo bf16 activations; above: one fp16 MFMA pass",
                      "sweep": rows}))


if __name__ == "__main__":
    main()
