"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import os
import sys
import time

import numpy as np

import oracle
import synthgen


_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def say(msg: str) -> None:
    """Names the case before each GPU step, so a dying box still tells which one it was; the line also goes to a
    progress file (pytest holds stderr back until the test ends, and a long oracle pass would otherwise look
    like a hang from outside)."""
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)
    try:
        d = os.path.join(_ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "gpu_cases.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def margins(logits: np.ndarray) -> np.ndarray:
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def follow_steps(ctx, omodel, prompts, lens, n_steps, tol, margin=0.05, check_rows=None, joins=None, wins=None):
    """Follow mode: at every step the oracle is fed the GPU's own window at the GPU's own
    committed length and must reproduce its logits (within tol), its argmax wherever the
    oracle's top-1/top-2 margin exceeds `margin`, and -- from the GPU's argmax row -- exactly
    its verified count, accepted tokens, next committed length and next window slot 0.
    joins: {step: (slot, prompt, buffer)} -- before that step the prompt takes over the slot (and a
    fresh oracle session its place).  wins: per-sequence window sizes the context was told to use (the
    integer path then looks at the first wins[b] rows only).
    Returns dict(max_err, rows, low_margin_rows, K)."""
    B, W = ctx.B, ctx.cfg.window
    sessions = []
    for b in range(B):
        ss = omodel.session(ctx.cfg.max_seq)
        if lens[b] > 1:
            ss.forward(prompts[b, :lens[b] - 1], 0, want_logits=False)
        sessions.append(ss)
    dbg = ctx.debug_logits(True)
    st = ctx.state()
    max_err, rows, low, Ks = 0.0, 0, 0, []
    for step in range(n_steps):
        if joins and step in joins:
            slot, pr, bf = joins[step]
            ctx.join(slot, pr, bf)
            sessions[slot] = omodel.session(ctx.cfg.max_seq)
            if len(pr) > 1:
                sessions[slot].forward(np.asarray(pr[:-1]), 0, want_logits=False)
            st = ctx.state()
            assert st["n"][slot] == len(pr) - 1 and st["g"][slot] == 0 and st["window"][slot][0] == pr[-1]
            assert (st["window"][slot][1:] == np.asarray(bf)[:W - 1]).all()
        win, n0 = st["window"].copy(), st["n"].copy()
        say(f"follow step {step} n={n0.tolist()}")
        rs = ctx.step_rows()                # dense, or packed when the sequences have windows of their own
        nacc, acc, win_next = ctx.step()
        st = ctx.state()
        glog = dbg.cpu().numpy()
        for b in range(B):
            if nacc[b] == 0:
                continue
            olog, oam, _ = sessions[b].forward(win[b], int(n0[b]))
            Wr = int(rs[b + 1] - rs[b])     # rows the step computed for this sequence
            if wins is not None and Wr < W:
                assert Wr == wins[b]
            gl = glog[rs[b]:rs[b] + Wr]
            olog, oam = olog[:Wr], oam[:Wr]
            err = np.abs(gl - olog).max()
            max_err = max(max_err, float(err))
            assert err <= tol, f"step {step} seq {b}: |dlogit| {err} > {tol}"
            mg = margins(olog)
            o_gpu = st["o"][b][:Wr]
            clear = mg > margin
            assert (o_gpu[clear] == oam[clear]).all(), f"step {step} seq {b}: argmax differs on a clear-margin row"
            assert (o_gpu == gl.argmax(-1)).all(), "GPU argmax is not the argmax of the GPU's own logits"
            rows += Wr
            low += int((~clear).sum())
            # integer path, recomputed by the oracle from the GPU's own argmax row: no tolerance
            Wb = wins[b] if wins is not None else W
            K = oracle.verify(win[b][:Wb], o_gpu[:Wb])
            assert st["K"][b] == K and nacc[b] == K + 1
            assert (acc[b, :K + 1] == o_gpu[:K + 1]).all()
            assert st["n"][b] == n0[b] + K + 1
            assert win_next[b, 0] == o_gpu[K]
            Ks.append(K)
    ctx.debug_logits(False)
    return dict(max_err=max_err, rows=rows, low_margin_rows=low, K=Ks)


def follow_streamed(ctx, shape, prompts, lens, follow, n_steps, tol, margin=0.05, real="f64", label=""):
    """Follow mode at full depth for models whose weights the host does not hold: the GPU takes n_steps steps
    (its windows, committed lengths, logits and integer results recorded), then the oracle runs the prompt and
    those windows of the sequences in `follow` through the model one layer at a time (oracle.forward_streamed,
    weights regenerated per layer by synthgen) and must reproduce the GPU's logits within tol and its argmax
    wherever the oracle's margin exceeds `margin`.  The integer path is recomputed from the GPU's own argmax rows
    for every sequence of the batch, with no tolerance.  Returns dict(max_err, rows, low_margin_rows, K)."""
    B, W = ctx.B, ctx.cfg.window
    dbg = ctx.debug_logits(True)
    st = ctx.state()
    rec = []
    for step in range(n_steps):
        win, n0 = st["window"].copy(), st["n"].copy()
        say(f"{label} streamed follow: GPU step {step} n={n0.tolist()}")
        nacc, acc, win_next = ctx.step()
        st = ctx.state()
        glog = dbg.cpu().numpy()
        rec.append(dict(win=win, n0=n0, nacc=nacc.copy(), acc=acc.copy(), win_next=win_next.copy(), o=st["o"].copy(),
                        K=st["K"].copy(), n1=st["n"].copy(), glog={b: glog[b * W:(b + 1) * W].copy() for b in follow}))
    ctx.debug_logits(False)
    Ks = []
    for r in rec:                      # integer path of every sequence: Eq. 5 and the cache update, exact
        for b in range(B):
            if r["nacc"][b] == 0:
                continue
            o_gpu = r["o"][b]
            K = oracle.verify(r["win"][b], o_gpu)
            assert r["K"][b] == K and r["nacc"][b] == K + 1
            assert (r["acc"][b, :K + 1] == o_gpu[:K + 1]).all()
            assert r["n1"][b] == r["n0"][b] + K + 1
            assert r["win_next"][b, 0] == o_gpu[K]
            Ks.append(K)
    fields = dict(n_layers=shape.n_layers, d_model=shape.d_model, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                  head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab, rms_eps=shape.rms_eps,
                  rope_base=shape.rope_base)
    specs = list(synthgen.weight_tensors(shape))
    glob = {sp.name: synthgen.weight_array(shape, sp, as_bf16_bits=True) for sp in specs if sp.layer < 0}

    def layer_weights(l):
        return {sp.name: synthgen.weight_array(shape, sp, as_bf16_bits=True) for sp in specs if sp.layer == l}

    sequences, top = [], 0
    for b in follow:
        passes = []
        if lens[b] > 1:
            passes.append((prompts[b, :lens[b] - 1], 0, False))
        for r in rec:
            passes.append((r["win"][b], int(r["n0"][b]), True))
            top = max(top, int(r["n0"][b]) + W)
        sequences.append(passes)
    t0 = time.time()
    out = oracle.forward_streamed(fields, 1, glob, layer_weights, sequences, top, real=real,
                                  progress=lambda l: say(f"{label} streamed follow: oracle layer {l} done ({time.time() - t0:.0f}s)"))
    max_err, rows, low = 0.0, 0, 0
    for si, b in enumerate(follow):
        res = out[si][1:] if lens[b] > 1 else out[si]
        for step, (r, (olog, oam)) in enumerate(zip(rec, res)):
            if r["nacc"][b] == 0:
                continue
            gl = r["glog"][b]
            err = float(np.abs(gl - olog).max())
            max_err = max(max_err, err)
            assert err <= tol, f"step {step} seq {b}: |dlogit| {err} > {tol}"
            clear = margins(olog) > margin
            o_gpu = r["o"][b]
            assert (o_gpu[clear] == oam[clear]).all(), f"step {step} seq {b}: argmax differs on a clear-margin row"
            assert (o_gpu == gl.argmax(-1)).all(), "GPU argmax is not the argmax of the GPU's own logits"
            rows += W
            low += int((~clear).sum())
    return dict(max_err=max_err, rows=rows, low_margin_rows=low, K=Ks, oracle_s=time.time() - t0)
