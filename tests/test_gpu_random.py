"""Seeded random configurations: the small fp32 model bit-exact against the oracle over random batches,
windows, per-sequence windows, stop conditions, compaction / graph settings and joining sequences; small bf16
models (grouped and plain heads, dimensions that are not powers of two) in follow mode over random batch x
window x prompt shapes, which walks through the launch choices of all three row regimes (up to 16 rows, up to
32, more).  The same generator ran several hundred cases of each kind during development; the counts here are
sized for seconds."""
import random

import numpy as np
import pytest

import oracle
import synthgen
from gpu_util import follow_steps, say

pytestmark = pytest.mark.gpu
TINY = synthgen.SHAPES["tiny"]
BF16_SHAPES = [synthgen.ModelShape(2, 768, 6, 3, 128, 768, 1504, init_std=0.05),
               synthgen.ModelShape(2, 512, 4, 1, 128, 1280, 2000, init_std=0.05),
               synthgen.ModelShape(3, 256, 2, 2, 128, 256, 1008, init_std=0.06)]


@pytest.mark.timeout(600)
def test_random_runs_fp32_bit_exact():
    import paper_2311_08263_amd as fc
    om = oracle.model_from_synth(TINY)
    rng = random.Random(20231108)
    packed = None
    for case in range(40):
        B, W, N, Pmax = rng.randint(1, 6), rng.randint(1, 12), rng.randint(8, 40), rng.randint(1, 24)
        lens = [rng.randint(1, Pmax) for _ in range(B)]
        lens[rng.randrange(B)] = Pmax
        seed = rng.randint(1, 10 ** 6)
        Lb = N + 12 * W                                   # room for the step-mode part below
        prompts = synthgen.prompts(B, Pmax, TINY.vocab, seed=seed)
        buf = synthgen.buffer_init(B, Lb, TINY.vocab, seed=seed + 1)
        for b in range(B):
            if rng.random() < 0.3:                        # a perfect draft
                buf[b, :] = om.greedy_ar(prompts[b, :lens[b]], Lb)
        wins = [rng.randint(1, W) for _ in range(B)] if rng.random() < 0.5 else None
        mode = rng.choice(["plain", "eos", "cap"])
        eos = int(om.greedy_ar(prompts[0, :lens[0]], N)[rng.randrange(N)]) if mode == "eos" else -1
        max_steps = rng.randint(1, 10) if mode == "cap" else 0
        compact, graph = rng.randint(0, 1), rng.randint(0, 1)
        desc = f"random fp32 case {case}: B{B} W{W} N{N} lens{lens} wins{wins} eos{eos} cap{max_steps} compact{compact} graph{graph} seed{seed}"
        say(desc)
        cfg = fc.Config.from_shape(TINY, B, Pmax + Lb + 2 * W + 16, W)
        if packed is None:
            packed = fc.load_synth_weights(cfg, TINY)
        ctx = fc.Context(cfg, packed)
        ctx.set_option(4, compact)
        ctx.set_option(2, graph)
        ctx.prefill(prompts, lens, buf)
        if wins:
            ctx.set_windows(wins)
        out = ctx.generate(N, max_steps=max_steps, eos_id=eos)
        for b in range(B):
            Wb = wins[b] if wins else W
            ref = om.jacobi_generate(prompts[b, :lens[b]], buf[b], Wb, N, max_steps=max_steps, eos=eos)
            L = len(ref["ids"])
            assert out["len"][b] == L and (out["ids"][b, :L] == ref["ids"]).all(), (desc, b)
            assert out["steps"][b] == ref["steps"], (desc, b)
            if not (eos >= 0 and L and ref["ids"][-1] == eos):
                assert (out["tail"][b][:Wb - 1] == ref["tail"]).all(), (desc, b)
        # step mode, with prompts that join
        ctx.prefill(prompts, lens, buf)
        if wins:
            ctx.set_windows(wins)
        occ = [dict(p=prompts[b, :lens[b]], buf=buf[b], W=(wins[b] if wins else W), ids=[], counts=[]) for b in range(B)]
        gone = []
        for s in range(rng.randint(3, 8)):
            if rng.random() < 0.4:
                slot, L2 = rng.randrange(B), rng.randint(1, Pmax)
                p2 = synthgen.prompts(1, L2, TINY.vocab, seed=seed + 10 + s)[0]
                b2 = synthgen.buffer_init(1, Lb, TINY.vocab, seed=seed + 20 + s)[0]
                ctx.join(slot, p2, b2)
                gone.append(occ[slot])
                occ[slot] = dict(p=p2, buf=b2, W=W, ids=[], counts=[])
            nacc, acc, _ = ctx.step()
            for b in range(B):
                occ[b]["ids"].extend(acc[b][:nacc[b]].tolist())
                occ[b]["counts"].append(int(nacc[b]))
        for q in gone + occ:
            if not q["counts"]:
                continue
            ref = om.jacobi_generate(q["p"], q["buf"], q["W"], Lb - 2 * q["W"], max_steps=len(q["counts"]))
            assert ref["steps"] == len(q["counts"]), desc
            assert q["counts"] == [k + 1 for k in ref["K"]], (desc, q["counts"])
            n = min(len(q["ids"]), len(ref["ids"]))
            assert q["ids"][:n] == ref["ids"].tolist()[:n], desc
        del ctx


@pytest.mark.timeout(600)
def test_random_shapes_bf16_follow_mode():
    import paper_2311_08263_amd as fc
    rng = random.Random(8263)
    models = {}
    worst = 0.0
    for case in range(36):
        si = case % len(BF16_SHAPES)
        shape = BF16_SHAPES[si]
        B = rng.randint(1, 5)
        W = rng.choice([1, 2, 3, 5, 8, 11, 16, 17, 24, 32, 33, 40, 64])
        P = rng.randint(2, 150)
        lens = [rng.randint(1, P) for _ in range(B)]
        lens[0] = P
        seed = rng.randint(1, 10 ** 6)
        S = ((P + 8 * W + 64 + 31) // 32) * 32
        cfg = fc.Config.from_shape(shape, B, S, W)
        if si not in models:
            models[si] = (fc.load_synth_weights(cfg, shape), oracle.model_from_synth(shape))
        packed, om = models[si]
        prompts = synthgen.prompts(B, P, shape.vocab, seed=seed)
        buf = synthgen.buffer_init(B, 8 * W + 16, shape.vocab, seed=seed + 1)
        wins = [rng.randint(1, W) for _ in range(B)] if rng.random() < 0.3 else None
        joins = None
        if rng.random() < 0.3:
            L2 = rng.randint(1, P)
            joins = {1: (rng.randrange(B), synthgen.prompts(1, L2, shape.vocab, seed=seed + 2)[0],
                         synthgen.buffer_init(1, 8 * W + 16, shape.vocab, seed=seed + 3)[0])}
            if wins:
                wins[joins[1][0]] = W                      # a newcomer runs the batch window
        say(f"random bf16 case {case}: shape{si} B{B} W{W} P{P} lens{lens} wins{wins} join{joins is not None} seed{seed}")
        ctx = fc.Context(cfg, packed)
        ctx.prefill(prompts, lens, buf)
        if wins:
            ctx.set_windows(wins if not joins else [w if b != joins[1][0] else W for b, w in enumerate(wins)])
        r = follow_steps(ctx, om, prompts, lens, 3, 2e-2, joins=joins, wins=wins)
        worst = max(worst, r["max_err"])
        del ctx
    print(f"random bf16 shapes: max |dlogit| {worst:.2e}")
    assert worst < 5e-3
