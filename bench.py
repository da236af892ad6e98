#!/usr/bin/env python3
"""Benchmark of the FastCoT Jacobi decoding step on one MI355X.

A "step" is one pass of the whole hot path: window fetch, embedding, all decoder layers (fused
QKV + RoPE + cache write, window-causal attention, O-proj, gate/up + SwiGLU, down), final norm,
LM head with fused argmax, verification, accept/commit and window shift, for one batch.

Default workload: the Llama-2-7B-shaped bf16 model, batch 1, prompt 256, window 16, synthetic
random-init weights and uniform random token ids (seeded, see synthgen).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix cores, published
# HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a plain
# copy kernel of known size (profiles/hbm_traffic_7b_w16.md, hbm_traffic_13b_b8_w32.md); None where no counter
# run exists
MEASURED_TRAFFIC = {("7b", "gemm_gate_up"): 183.4e6, ("13b", "gemm_gate_up"): 400.1e6, ("70b", "gemm_gate_up"): 945.8e6}
WORKLOADS = {
    # name: (shape, batch, prompt, window, new tokens)
    "7b": ("7b", 1, 256, 16, 256),
    "70b": ("70b", 1, 512, 16, 128),
    "13b": ("13b", 8, 1024, 32, 256),
    "tiny": ("tiny", 1, 32, 8, 64),
}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def weight_bytes_per_step(s, esz):
    per_layer = {"gemm_qkv": s.d_model * (s.q_dim + 2 * s.kv_dim), "gemm_o": s.q_dim * s.d_model,
                 "gemm_gate_up": 2 * s.d_model * s.d_ffn, "gemm_down": s.d_ffn * s.d_model}
    out = {k: v * esz for k, v in per_layer.items()}
    out["lm_head"] = s.d_model * s.vocab * esz
    return out


def algorithmic_bytes(s, esz, B, W, n_committed):
    """Bytes the method itself must move per step: every streamed weight once, the committed K and
    V once (at the model's storage width), the window's K/V write, the embedding rows."""
    wb = weight_bytes_per_step(s, esz)
    weights = s.n_layers * (wb["gemm_qkv"] + wb["gemm_o"] + wb["gemm_gate_up"] + wb["gemm_down"]) + wb["lm_head"]
    kv_read = sum(s.n_layers * 2 * n * s.kv_dim * esz for n in n_committed)
    kv_write = s.n_layers * 2 * B * W * s.kv_dim * esz
    emb = B * W * s.d_model * 4
    return weights + kv_read + kv_write + emb


def cpu_baseline(shape, W, log_fn):
    """The oracle as it stands (fp32 build), timed on this host on a bounded sample."""
    import oracle
    import synthgen
    P, steps = 32, 3
    log_fn("cpu_baseline: building the oracle model (bf16-stored weights)")
    om = oracle.model_from_synth(shape, real="f32", bf16_storage=(shape.dtype == "bf16"))
    prompt = synthgen.prompts(1, P, shape.vocab)[0]
    buf = synthgen.buffer_init(1, steps * W + 2 * W, shape.vocab)[0]
    ss = om.session(P + (steps + 2) * W)
    ss.forward(prompt[:-1], 0, want_logits=False)
    n, g, newest, accepted = P - 1, 0, prompt[-1], 0
    t0 = time.time()
    for _ in range(steps):
        w = np.concatenate([[newest], buf[g:g + W - 1]]).astype(np.int32)
        _, o, _ = ss.forward(w, n, want_logits=False)
        K = oracle.verify(w, o)
        buf[g:g + W] = o
        newest = o[K]
        n += K + 1
        g += K + 1
        accepted += K + 1
    dt = time.time() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": accepted / dt, "unit": "accepted tokens/s", "ms_per_step": 1e3 * dt / steps, "cores": cores,
            "kind": "oracle",
            "sample": f"{steps} Jacobi steps of the fp32 oracle, batch 1, window {W}, context {P - 1}..{n}, same model shape"}


def time_launches(torch, fn, n):
    """Mean microseconds of n launches of fn(i) on torch's current stream (events around the batch)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(3):
        fn(i)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return 1e3 * e0.elapsed_time(e1) / n


def extras(torch, fc, synthgen, packed, log_fn, chain_bytes=None):
    """Secondary measurements: the device's plain streaming-read rate and the two kernels in isolation
    (window attention over a 2048-token cache; LM head + argmax), cache-cold by rotating buffer sets."""
    out = {}
    nbytes = min(packed.numel(), 8 << 30)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    us = time_launches(torch, lambda i: fc.stream_read(packed[:nbytes], sink), 5)
    out["stream_read_ceiling"] = {"bytes": int(nbytes), "us": round(us, 1), "GB/s": round(nbytes / us / 1e3, 0)}
    log_fn(f"plain streaming read of {nbytes / 1e9:.2f} GB: {us:.0f} us -> {nbytes / us / 1e3:.0f} GB/s")
    # the floor of a step made of separate launches: a chain of plain streaming reads with the byte counts of the
    # step's kernels (per layer QKV, the K/V the attention reads, O, gate/up, down; then the LM head), replayed
    # as one graph like the step itself
    if chain_bytes:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            fc.stream_read_chain(packed, chain_bytes, sink)          # warm (module load) outside the capture
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                total = fc.stream_read_chain(packed, chain_bytes, sink)
        us = time_launches(torch, lambda i: g.replay(), 10)
        out["stream_chain_floor"] = {"launches": len(chain_bytes), "bytes": int(total), "ms": round(us / 1e3, 4),
                                     "GB/s": round(total / us / 1e3, 0), "frac_of_8TBs": round(total / us / 1e3 / HBM_PEAK_GBS, 4)}
        log_fn(f"chain of {len(chain_bytes)} plain streaming launches with the step's byte counts ({total / 1e9:.2f} GB): "
               f"{us / 1e3:.3f} ms -> {total / us / 1e3:.0f} GB/s ({100 * total / us / 1e3 / HBM_PEAK_GBS:.1f}% of 8 TB/s)")
        del g
    # attention alone: 32 heads x 128, 2048 committed positions + 16 window rows, bf16 cache (one plane)
    n, W, H, Dh, S = 2048, 16, 32, 128, 2080
    sets = []
    for r in range(3):
        k = torch.from_numpy(synthgen.normal_bf16((n + W, H, Dh), 7, 2 * r, 1.0).view(np.int16)).cuda().view(torch.bfloat16)
        v = torch.from_numpy(synthgen.normal_bf16((n + W, H, Dh), 7, 2 * r + 1, 1.0).view(np.int16)).cuda().view(torch.bfloat16)
        sets.append(fc.kv_scatter(k, v, S))
    q = torch.from_numpy(synthgen.normal_f32((W, H, Dh), 7, 9, 1.0, False)).cuda()
    scratch = torch.zeros(fc.lib().fastcot_attn_scratch_bytes(W, H, Dh), dtype=torch.uint8, device="cuda")
    us = time_launches(torch, lambda i: fc.attn_window(q, *sets[i % 3], n, scratch), 120)
    kvb = 2 * (n + W) * H * Dh * 2
    out["attention_isolated"] = {"keys": n + W, "rows": W, "heads": H, "us": round(us, 2), "kv_bytes": kvb,
                                 "GB/s": round(kvb / us / 1e3, 0), "frac_of_8TBs": round(kvb / us / 1e3 / HBM_PEAK_GBS, 4)}
    log_fn(f"attention alone ({n + W} keys, {W} rows, {H} heads): {us:.1f} us, {kvb / us / 1e3:.0f} GB/s")
    del sets
    # LM head + argmax alone: 16 x 4096 activations, 4096 x 32000 weights, three weight copies in rotation
    M, d, V = 16, 4096, 32000
    wl = [fc.lmhead_pack(torch.from_numpy(synthgen.normal_bf16((d, V), 8, r, 0.02).view(np.int16)).cuda().view(torch.bfloat16))
          for r in range(3)]
    act = torch.from_numpy(synthgen.normal_f32((M, d), 8, 9, 1.0, False)).cuda()
    scr = torch.zeros(fc.lib().fastcot_lmhead_scratch_bytes(M, d, V), dtype=torch.uint8, device="cuda")
    us = time_launches(torch, lambda i: fc.lmhead_argmax(act, wl[i % 3], V, False, scr), 120)
    wb = d * V * 2
    out["lm_head_isolated"] = {"rows": M, "d": d, "vocab": V, "us": round(us, 2), "weight_bytes": wb,
                               "GB/s": round(wb / us / 1e3, 0), "frac_of_8TBs": round(wb / us / 1e3 / HBM_PEAK_GBS, 4)}
    log_fn(f"LM head + argmax alone ({M} x {d} x {V}): {us:.1f} us, {wb / us / 1e3:.0f} GB/s")
    return out


def step_only(torch, fc, synthgen, name, steps, warm, log_fn):
    """ms/step, fraction of the HBM roofline and per-kernel launch times of another workload (no generate run)."""
    shape_name, B, P, W, N = WORKLOADS[name]
    shape = synthgen.SHAPES[shape_name]
    max_seq = ((P + W * (steps + warm + 4) + 31) // 32) * 32
    cfg = fc.Config.from_shape(shape, B, max_seq, W)
    t0 = time.time()
    packed = fc.load_synth_weights(cfg, shape)
    ctx = fc.Context(cfg, packed)
    log_fn(f"secondary workload {name}: model resident after {time.time() - t0:.1f}s")
    ctx.prefill(synthgen.prompts(B, P, shape.vocab), [P] * B, synthgen.buffer_init(B, W * (steps + warm + 3), shape.vocab))
    for _ in range(warm):
        ctx.step(sync=False)
    ctx.stream.synchronize()
    n0 = ctx.state()["n"].copy()
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx.step(sync=False)
    ctx.stream.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / steps
    n1 = ctx.state()["n"]
    alg = algorithmic_bytes(shape, 2, B, W, (n0 + n1) / 2.0)
    rec = {"workload": f"llama2-{shape_name}-shaped, batch {B}, prompt {P}, window {W}", "steps": steps, "ms_per_step": round(ms, 4),
           "step_algorithmic_bytes": int(alg), "hbm_frac": round(alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    prof = ctx.profile_step(2)
    prof.pop("empty_kernel", None)
    rec["kernels_us"] = {k: round(v[0] * 1e3, 2) for k, v in prof.items()}
    if B * W > 32:
        # useful flops: 2 * rows * streamed parameters + attention; the GEMMs issue twice the useful MFMAs (bf16 hi + lo)
        ctxlen = float(np.mean((n0 + n1) / 2.0)) + W / 2.0
        flops = 2.0 * B * W * shape.n_params_streamed() + 4.0 * B * W * shape.q_dim * ctxlen * shape.n_layers
        tf = flops / (ms * 1e-3) / 1e12
        rec["useful_tflops"] = round(tf, 1)
        rec["mfma_frac_useful"] = round(tf / MFMA_BF16_PEAK_TFLOPS, 4)
        rec["mfma_frac_issued"] = round(2 * tf / MFMA_BF16_PEAK_TFLOPS, 4)
        wb = weight_bytes_per_step(shape, 2)
        gu_ms = prof.get("gemm_gate_up", (0.0, 0))[0]
        if gu_ms > 0:
            rec["gate_up_useful_tflops"] = round(2.0 * B * W * wb["gemm_gate_up"] / 2 / (gu_ms * 1e-3) / 1e12, 1)
    log_fn(f"secondary workload {name}: {ms:.3f} ms/step, {100 * rec['hbm_frac']:.1f}% of 8 TB/s" +
           (f", {rec['useful_tflops']:.0f} TFLOP/s useful ({100 * rec['mfma_frac_useful']:.1f}% of 2.5 PF)" if "useful_tflops" in rec else ""))
    ctx.close()
    del ctx, packed
    torch.cuda.empty_cache()
    return rec


def kv_format_study(args):
    """What a narrower K/V cache format would cost in logits: every step of a short run with the cached values
    rounded as the format would round them (FASTCOT_OPT_KV_EMULATE), against the same steps with the bf16 hi + lo
    pair the library stores (which the oracle tests hold to a few 1e-4).  Windows are replayed from the
    reference run, so all formats see identical inputs."""
    import torch
    import synthgen
    import paper_2311_08263_amd as fc
    modes = {"as computed": 0, "bf16": 1, "fp16": 2, "fp32 upper 24 bits": 3}
    rows = []
    for shape_name, P in (("7b", 256), ("13b", 1024), ("70b", 512)):
        shape = synthgen.SHAPES[shape_name]
        W, steps = 16, 3
        max_seq = ((P + 4 * W + 31) // 32) * 32
        cfg = fc.Config.from_shape(shape, 1, max_seq, W)
        log(f"kv format study: building {shape_name} weights")
        packed = fc.load_synth_weights(cfg, shape)
        prompts = synthgen.prompts(1, P, shape.vocab)
        buf = synthgen.buffer_init(1, 8 * W, shape.vocab)
        ref = None
        for kname, km in modes.items():
            for vname, vm in modes.items():
                if (km, vm) not in ((0, 0), (1, 1), (2, 2), (3, 3), (0, 1), (1, 0), (0, 2), (2, 0), (3, 2), (2, 3)):
                    continue
                ctx = fc.Context(cfg, packed)
                ctx.set_option(fc.binding.OPT_KV_EMULATE, km + 16 * vm)
                ctx.prefill(prompts, [P], buf)
                dbg = ctx.debug_logits(True)
                lgs = []
                for _ in range(steps):
                    ctx.step()
                    lgs.append(dbg[:W].clone())
                torch.cuda.synchronize()
                if ref is None:
                    ref = lgs
                # only steps whose inputs are the reference's count: compare while the windows agree (step 0 always does)
                err = float((lgs[0] - ref[0]).abs().max())
                rows.append({"shape": shape_name, "prompt": P, "K": kname, "V": vname, "bytes_per_value": {0: 4, 1: 2, 2: 2, 3: 3}[km] / 2 + {0: 4, 1: 2, 2: 2, 3: 3}[vm] / 2,
                             "max_abs_dlogit_step0": round(err, 6)})
                log(f"kv format {shape_name} prompt {P}: K {kname:20s} V {vname:20s} max |dlogit| {err:.2e}")
                ctx.close()
                del ctx
        # the same question for the GEMM inputs: activations as plain bf16 instead of the hi + lo pair, GEMM by GEMM
        for label, mask in (("QKV", 1), ("O", 2), ("gate/up", 4), ("down", 8), ("LM head", 16), ("O + down", 10), ("all", 31)):
            ctx = fc.Context(cfg, packed)
            ctx.set_option(fc.binding.OPT_ACT_EMULATE, mask)
            ctx.prefill(prompts, [P], buf)          # (the prompt pass of more than 32 rows keeps the pair)
            dbg = ctx.debug_logits(True)
            ctx.step()
            err = float((dbg[:W] - ref[0]).abs().max())
            rows.append({"shape": shape_name, "prompt": P, "plain_bf16_activations_into": label, "max_abs_dlogit_step0": round(err, 6)})
            log(f"activation format {shape_name}: plain bf16 into {label:10s} max |dlogit| {err:.2e}")
            ctx.close()
            del ctx
        del packed
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "max |dlogit| of the first step against the bf16 hi + lo pair cache, per emulated K/V storage format",
                      "n_gpus": 1, "data": "synthetic", "dtype": "bf16", "rows": rows}), flush=True)


def window_sweep(args):
    """Step time against window size and prompt length (the measurement of the paper's Fig. 2, Sec. 3.1:
    how large may the window grow before the step stops being free), batch 1, 7B and 13B shapes."""
    import torch
    import synthgen
    import paper_2311_08263_amd as fc
    rows = []
    for shape_name in ("7b", "13b"):
        shape = synthgen.SHAPES[shape_name]
        packed = None
        for P in (256, 1024, 4096):
            for W in (1, 2, 4, 8, 16, 32, 64, 128):
                steps, warm = 12, 3
                max_seq = ((P + W * (steps + warm + 3) + 31) // 32) * 32
                cfg = fc.Config.from_shape(shape, 1, max_seq, W)
                if packed is None:
                    log(f"window sweep: building {shape_name} weights")
                    packed = fc.load_synth_weights(cfg, shape)
                ctx = fc.Context(cfg, packed)
                ctx.prefill(synthgen.prompts(1, P, shape.vocab), [P], synthgen.buffer_init(1, W * (steps + warm + 2), shape.vocab))
                for _ in range(warm):
                    ctx.step(sync=False)
                ctx.stream.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    ctx.step(sync=False)
                ctx.stream.synchronize()
                ms = 1e3 * (time.perf_counter() - t0) / steps
                rows.append({"shape": shape_name, "prompt": P, "window": W, "ms_per_step": round(ms, 3)})
                log(f"window sweep {shape_name} prompt {P:5d} window {W:4d}: {ms:8.3f} ms/step")
                ctx.close()
                del ctx
        del packed
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "ms per Jacobi step against window size and prompt length (Fig. 2)", "unit": "ms",
                      "n_gpus": 1, "data": "synthetic", "dtype": "bf16", "rows": rows}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="7b", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-iters", type=int, default=3)
    ap.add_argument("--plain", action="store_true", help="time the plain kernels instead of the MFMA path")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the secondary measurements (streaming-read ceiling, isolated attention and LM head, perfect draft)")
    ap.add_argument("--plan", default="", help="launch-plan values for the timed context, as option=value pairs separated by commas "
                    "(FASTCOT_PLAN_* numbers of include/fastcot.h, e.g. 105=2 for two K slices per owner in the QKV GEMM)")
    ap.add_argument("--no-secondary-workloads", action="store_true",
                    help="skip the 13B batch-8 and 70B step measurements that follow the default workload")
    ap.add_argument("--window-sweep", action="store_true",
                    help="instead of the benchmark: ms/step for windows 1..128 x prompts 256..4096 on the 7B and 13B shapes")
    ap.add_argument("--kv-format-study", action="store_true",
                    help="instead of the benchmark: logit shift of narrower K/V cache formats (emulated) on the 7B, 13B and 70B shapes")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device-to-device copy of 512 MiB (the known-size kernel that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus above 1 is not supported "
                 "(sequences are independent, Eq. 2: a multi-GPU run would give each GPU its share of the batch and a copy of the weights)")

    if args.window_sweep:
        return window_sweep(args)
    if args.kv_format_study:
        return kv_format_study(args)

    import torch
    import synthgen
    import paper_2311_08263_amd as fc

    shape_name, B, P, W, N = WORKLOADS[args.workload]
    shape = synthgen.SHAPES[shape_name]
    esz = 4 if shape.dtype == "f32" else 2
    K, Wm = args.steps, args.warmup
    # room for the worst case of W accepted tokens per step
    max_seq = min(16000, ((P + W * (K + Wm + 2) + 2 * W + 31) // 32) * 32)
    max_seq = max(max_seq, ((P + N + 2 * W + 31) // 32) * 32)
    cfg = fc.Config.from_shape(shape, B, max_seq, W)
    t0 = time.time()
    log(f"workload {args.workload}: building synthetic weights ({shape.n_params_streamed() * esz / 1e9:.2f} GB streamed per step)")
    packed = fc.load_synth_weights(cfg, shape)
    ctx = fc.Context(cfg, packed)
    if args.plain:
        ctx.set_option(1, 1)
    for pair in filter(None, args.plan.split(",")):
        opt, val = pair.split("=")
        ctx.set_option(int(opt), int(val))
    log(f"model resident after {time.time() - t0:.1f}s; max_seq {max_seq}")
    prompts = synthgen.prompts(B, P, shape.vocab)
    lens = [P] * B
    buf_len = min(max_seq, W * (K + Wm + 2) + 2 * W)
    buf = synthgen.buffer_init(B, max(buf_len, N + 2 * W), shape.vocab)

    # ---- accepted tokens/s on the paper-shaped job: generate N tokens from the prompt
    ctx.prefill(prompts, lens, buf)
    ctx.generate(min(N, 4 * W))                        # warm (graph capture, caches)
    torch.cuda.synchronize()
    t0 = time.time()
    ctx.prefill(prompts, lens, buf)
    torch.cuda.synchronize()
    prefill_ms = 1e3 * (time.time() - t0)
    t0 = time.time()
    out = ctx.generate(N)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    gen_ms = ctx.step_times()
    gen_steps = int(out["steps"].max())
    tok_s = float(out["len"].sum()) / gen_s
    log(f"prefill {prefill_ms:.1f} ms; generate: {int(out['len'].sum())} tokens in {gen_steps} steps, {gen_s * 1e3:.1f} ms, "
        f"step median {np.median(gen_ms):.3f} p10 {np.percentile(gen_ms, 10):.3f} p90 {np.percentile(gen_ms, 90):.3f} ms")

    # ---- the other extreme of the accept path: a buffer that already holds the greedy continuation
    # (every draft verifies, W tokens per step); the model's own accepted stream is that continuation
    perfect = None
    if not args.no_extras:
        pbuf = buf.copy()
        pbuf[:, :N] = out["ids"][:, :N]
        ctx.prefill(prompts, lens, pbuf)
        torch.cuda.synchronize()
        t0 = time.time()
        pout = ctx.generate(N)
        torch.cuda.synchronize()
        ps = time.time() - t0
        perfect = {"tokens": int(pout["len"].sum()), "steps": int(pout["steps"].max()), "wall_ms": round(ps * 1e3, 2),
                   "tokens_per_s": round(float(pout["len"].sum()) / ps, 1),
                   "accepted_per_step": round(float(pout["len"].sum()) / max(int(pout["steps"].max()), 1) / B, 3),
                   "same_tokens": bool((pout["ids"][:, :N] == out["ids"][:, :N]).all())}
        log(f"perfect draft: {perfect['tokens']} tokens in {perfect['steps']} steps, {perfect['tokens_per_s']:.0f} tokens/s")

    # ---- exactly K timed steps after Wm warm-up steps (state continues, inputs resident)
    ctx.prefill(prompts, lens, buf)
    for _ in range(Wm):
        ctx.step(sync=False)
    ctx.stream.synchronize()
    torch.cuda.synchronize()
    n_before = ctx.state()["n"].copy()
    t0 = time.perf_counter()
    for _ in range(K):
        ctx.step(sync=False)
    ctx.stream.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = ctx.state()
    ms_per_step = 1e3 * dt / K
    accepted_timed = int((st["n"] - n_before).sum())
    n_mid = (n_before + st["n"]) / 2.0
    alg = algorithmic_bytes(shape, esz, B, W, n_mid)
    step_gbs = alg / (ms_per_step * 1e-3) / 1e9
    log(f"timed: {K} steps, {ms_per_step:.3f} ms/step, accepted {accepted_timed}, "
        f"algorithmic {alg / 1e9:.3f} GB/step -> {step_gbs:.0f} GB/s ({100 * step_gbs / HBM_PEAK_GBS:.1f}% of 8 TB/s)")

    if args.calibrate_copy:
        src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        log("calibration copy: 536870912 bytes read, 536870912 bytes written")

    # ---- per-kernel launch durations (HIP events on the context's stream), dominant kernel roofline
    prof = ctx.profile_step(args.profile_iters)
    wb = weight_bytes_per_step(shape, esz)
    table = []
    empty_ms = prof.pop("empty_kernel", (0.0, 0))[0]      # the event pair around a kernel that does nothing
    for kind, (ms, cnt) in prof.items():
        b = wb.get(kind)
        table.append((kind, ms, cnt, b))
        log(f"kernel {kind:14s} {cnt:4d}/step  {ms * 1e3:9.2f} us" + (f"  {b / (ms * 1e-3) / 1e9:7.0f} GB/s" if b else ""))
    log(f"event pair around an empty kernel: {empty_ms * 1e3:.2f} us (the floor of these event intervals; a profiler's begin-to-end "
        "durations of the long kernels are 2-3 us shorter than the figures above)")
    cands = [t for t in table if t[3]]
    dom = max(cands, key=lambda t: t[1] * t[2])
    achieved = dom[3] / (dom[1] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom[0], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get((args.workload, dom[0])),
                "bytes_per_launch": dom[3], "avg_launch_ms": round(dom[1], 5),
                "step_algorithmic_bytes": int(alg), "step_frac": round(step_gbs / HBM_PEAK_GBS, 4)}
    if B * W > 32 and not args.plain:
        # many rows: the GEMMs sit on the matrix-core side of the ridge (2 * rows flops per weight element
        # against 2 bytes).  Algorithmic flops = 2 * rows * K * N of the dominant GEMM; the kernel issues
        # twice that because activations enter as bf16 hi + lo.
        flops = 2.0 * B * W * dom[3] / esz
        tf = flops / (dom[1] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dom[0], "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": MEASURED_TRAFFIC.get((args.workload, dom[0])),
                    "flops_per_launch": flops, "issued_flops_per_launch": 2 * flops, "avg_launch_ms": round(dom[1], 5),
                    "step_algorithmic_bytes": int(alg), "step_hbm_frac": round(step_gbs / HBM_PEAK_GBS, 4)}

    # launch durations above are HIP-event intervals, which start when the previous event completes: they
    # contain the launch latency that a profiler's begin-to-end duration leaves out.  The same pair around an
    # empty kernel (same pass) is reported as the floor of such intervals.
    roofline["empty_kernel_event_ms"] = round(empty_ms, 5)
    # What the event pairs add per launch, from this run alone: the intervals of all launches of a step add up
    # to more than the graph-replayed step takes; the excess, spread over the launches, is the pairs' share.
    # `achieved` and `frac` stay on the raw intervals; the net figures are what a profiler's durations show.
    launches = sum(t[2] for t in table)
    if launches:
        over_ms = (sum(t[1] * t[2] for t in table) - ms_per_step) / launches
        net_ms = dom[1] - over_ms
        if over_ms > 0 and net_ms > 0:
            roofline["event_overhead_ms_per_launch"] = round(over_ms, 5)
            roofline["avg_launch_ms_net"] = round(net_ms, 5)
            roofline["frac_net"] = round(roofline["frac"] * dom[1] / net_ms, 4)
            log(f"event intervals exceed the replayed step by {over_ms * 1e3:.2f} us per launch; {dom[0]} net of that: "
                f"{net_ms * 1e3:.2f} us ({100 * roofline['frac_net']:.1f} % of peak)")
    extra = None
    if not args.no_extras and not args.plain and shape.dtype == "bf16":
        kv_pair = 2 * float(np.mean(n_mid)) * shape.kv_dim * 2 * 2        # K and V of the context, bf16 hi + lo planes
        per_layer = [wb["gemm_qkv"], kv_pair, wb["gemm_o"], wb["gemm_gate_up"], wb["gemm_down"]]
        chain = [int(b) for _ in range(shape.n_layers) for b in per_layer] + [wb["lm_head"]]
        extra = extras(torch, fc, synthgen, packed, log, chain if B * W <= 32 else None)
    # the other two configurations, steps only (the headline fields above stay this workload's)
    if not args.no_extras and not args.plain and args.workload == "7b" and not args.no_secondary_workloads:
        ctx.close()
        del ctx, packed
        torch.cuda.empty_cache()
        extra = extra or {}
        extra["step_13b_b8_w32"] = step_only(torch, fc, synthgen, "13b", 10, 3, log)
        extra["step_70b"] = step_only(torch, fc, synthgen, "70b", 10, 3, log)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, W, log)
        log(f"cpu_baseline: {cpu['ms_per_step']:.0f} ms/step on {cpu['cores']} threads")

    rec = {
        "metric": "ms per Jacobi step + accepted tokens/s, 7B-shaped bf16, window 16; % HBM roofline",
        "value": round(tok_s, 2), "unit": "accepted tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"llama2-{shape_name}-shaped random-init, batch {B}, prompt {P}, window {W}, "
                               f"{N} new tokens, greedy", "batch": B, "prompt": P, "window": W, "new_tokens": N,
                   "kernels": "plain" if args.plain else "mfma", **({"plan": args.plan} if args.plan else {})},
        "generate": {"tokens": int(out["len"].sum()), "steps": gen_steps, "wall_ms": round(gen_s * 1e3, 2),
                     "median_step_ms": round(float(np.median(gen_ms)), 4),
                     "p10_step_ms": round(float(np.percentile(gen_ms, 10)), 4),
                     "p90_step_ms": round(float(np.percentile(gen_ms, 90)), 4),
                     "prefill_ms": round(prefill_ms, 2),
                     "accepted_per_step": round(float(out["len"].sum()) / max(gen_steps, 1) / B, 3)},
        "hbm_roofline_pct_step": round(100 * step_gbs / HBM_PEAK_GBS, 2),
        "perfect_draft": perfect,
        "roofline": roofline,
        "secondary": extra,
        "cpu_baseline": cpu,
    }
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
