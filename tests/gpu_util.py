"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import sys

import numpy as np

import oracle
import synthgen


def say(msg: str) -> None:
    """Names the case before each GPU step, so a dying box still tells which one it was."""
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


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
        nacc, acc, win_next = ctx.step()
        st = ctx.state()
        glog = dbg.cpu().numpy()
        for b in range(B):
            if nacc[b] == 0:
                continue
            olog, oam, _ = sessions[b].forward(win[b], int(n0[b]))
            gl = glog[b * W:(b + 1) * W]
            err = np.abs(gl - olog).max()
            max_err = max(max_err, float(err))
            assert err <= tol, f"step {step} seq {b}: |dlogit| {err} > {tol}"
            mg = margins(olog)
            o_gpu = st["o"][b]
            clear = mg > margin
            assert (o_gpu[clear] == oam[clear]).all(), f"step {step} seq {b}: argmax differs on a clear-margin row"
            assert (o_gpu == gl.argmax(-1)).all(), "GPU argmax is not the argmax of the GPU's own logits"
            rows += W
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
