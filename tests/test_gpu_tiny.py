"""GPU parity on the small fp32 configuration (2 layers, d 256, 4 heads x 64, FFN 688, vocab
1024; batch 1, prompt 32, window 8, 64 new tokens) and its edge cases.  Bars: token ids, step
counts and per-step verified counts bit-exact; |dlogit| <= 1e-4."""
import numpy as np
import pytest

import oracle
import synthgen
from gpu_util import follow_steps, margins, say

pytestmark = pytest.mark.gpu
TINY = synthgen.SHAPES["tiny"]
TOL = 1e-4


@pytest.fixture(scope="module")
def env():
    import paper_2311_08263_amd as fc
    om = oracle.model_from_synth(TINY)
    return fc, om


def make_ctx(fc, B, S, W):
    cfg = fc.Config.from_shape(TINY, B, S, W)
    packed = fc.load_synth_weights(cfg, TINY)
    return fc.Context(cfg, packed)


def test_generate_matches_oracle_free_run(env):
    fc, om = env
    P, W, N = 32, 8, 64
    prompt = synthgen.prompts(1, P, TINY.vocab)
    buf = synthgen.buffer_init(1, N + 2 * W, TINY.vocab)
    ref = om.jacobi_generate(prompt[0], buf[0], W, N)
    say("tiny generate B1 P32 W8 N64")
    ctx = make_ctx(fc, 1, P + N + 2 * W, W)
    ctx.prefill(prompt, [P], buf)
    out = ctx.generate(N)
    assert out["len"][0] == N
    assert (out["ids"][0] == ref["ids"]).all()
    assert out["steps"][0] == ref["steps"]
    assert (out["tail"][0] == ref["tail"]).all()
    assert (out["ids"][0] == om.greedy_ar(prompt[0], N)).all()


def test_generate_matches_stored_trajectory(env):
    """The same run against tests/golden/tiny_trajectory.json (written by the oracle alone)."""
    import json
    import os
    fc, _ = env
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_trajectory.json")) as f:
        g = json.load(f)
    P, W, N = g["config"]["prompt"], g["config"]["window"], g["config"]["new_tokens"]
    say("tiny generate against the stored trajectory")
    ctx = make_ctx(fc, 1, P + N + 2 * W, W)
    ctx.prefill(np.array([g["prompt"]], dtype=np.int32), [P], synthgen.buffer_init(1, N + 2 * W, TINY.vocab))
    Ks = []
    while True:
        nacc, acc, _ = ctx.step()
        Ks.append(int(nacc[0]) - 1)
        if sum(k + 1 for k in Ks) >= N:
            break
    assert Ks == g["K"]
    ctx.prefill(np.array([g["prompt"]], dtype=np.int32), [P], synthgen.buffer_init(1, N + 2 * W, TINY.vocab))
    out = ctx.generate(N)
    assert out["ids"][0].tolist() == g["ids"] and int(out["steps"][0]) == g["steps"] and out["tail"][0].tolist() == g["tail"]


def test_stepwise_logits_and_counts(env):
    fc, om = env
    P, W, N = 32, 8, 64
    prompt = synthgen.prompts(1, P, TINY.vocab)
    buf = synthgen.buffer_init(1, N + 2 * W, TINY.vocab)
    ref = om.jacobi_generate(prompt[0], buf[0], W, N)
    ctx = make_ctx(fc, 1, P + N + 2 * W, W)
    ctx.prefill(prompt, [P], buf)
    r = follow_steps(ctx, om, prompt, [P], ref["steps"], TOL, margin=4 * TOL)
    assert r["K"] == ref["K"].tolist()          # free-running trajectories coincide step by step
    assert r["max_err"] < TOL
    print("tiny max |dlogit|", r["max_err"])


@pytest.mark.parametrize("W", [1, 2, 5, 16])
def test_windows(env, W):
    fc, om = env
    P, N = 20, 40
    prompt = synthgen.prompts(1, P, TINY.vocab, seed=12)
    buf = synthgen.buffer_init(1, N + 2 * W, TINY.vocab, seed=3)
    ref = om.jacobi_generate(prompt[0], buf[0], W, N)
    say(f"tiny window W={W}")
    ctx = make_ctx(fc, 1, P + N + 2 * W, W)
    ctx.prefill(prompt, [P], buf)
    out = ctx.generate(N)
    assert (out["ids"][0] == ref["ids"]).all() and out["steps"][0] == ref["steps"]
    if W == 1:
        assert out["steps"][0] == N


def test_ragged_batch_eos_and_cap(env):
    """Sequences of different prompt lengths advance independently; EOS among the accepted tokens
    stops a sequence (approximate EOS does not); max_steps caps the iterations."""
    fc, om = env
    W, N, B = 4, 24, 3
    lens = [9, 1, 17]
    prompts = synthgen.prompts(B, 17, TINY.vocab, seed=5)
    buf = synthgen.buffer_init(B, N + 2 * W, TINY.vocab, seed=6)
    refs = [om.jacobi_generate(prompts[b, :lens[b]], buf[b], W, N) for b in range(B)]
    say("tiny ragged batch")
    ctx = make_ctx(fc, B, 17 + N + 2 * W, W)
    ctx.prefill(prompts, lens, buf)
    out = ctx.generate(N)
    for b in range(B):
        assert (out["ids"][b] == refs[b]["ids"]).all() and out["steps"][b] == refs[b]["steps"], b
        assert (out["tail"][b] == refs[b]["tail"]).all()
    # EOS: take a token of sequence 0's stream as EOS
    eos = int(refs[0]["ids"][7])
    refs = [om.jacobi_generate(prompts[b, :lens[b]], buf[b], W, N, eos=eos) for b in range(B)]
    ctx.prefill(prompts, lens, buf)
    out = ctx.generate(N, eos_id=eos)
    for b in range(B):
        L = len(refs[b]["ids"])
        assert out["len"][b] == L and (out["ids"][b, :L] == refs[b]["ids"]).all() and out["steps"][b] == refs[b]["steps"]
    # iteration cap
    refs = [om.jacobi_generate(prompts[b, :lens[b]], buf[b], W, N, max_steps=3) for b in range(B)]
    ctx.prefill(prompts, lens, buf)
    out = ctx.generate(N, max_steps=3)
    for b in range(B):
        L = len(refs[b]["ids"])
        assert out["steps"][b] == 3 and out["len"][b] == L and (out["ids"][b, :L] == refs[b]["ids"]).all()


def test_finished_sequences_leave_the_batch(env):
    """Sequences that finish early (a perfect draft needs N / W steps, a random buffer about N) trade slots with
    unfinished ones inside fastcot_generate, so later steps run fewer rows; outputs, step counts, tails and the
    state afterwards are those of the run without the trades and of the oracle, in the caller's order, and the
    answer phase still finds every sequence's cache."""
    fc, om = env
    W, N, B, P = 4, 32, 5, 11
    lens = [11, 7, 9, 11, 5]
    prompts = synthgen.prompts(B, P, TINY.vocab, seed=71)
    buf = synthgen.buffer_init(B, N + 2 * W, TINY.vocab, seed=72)
    for b in (0, 3):                                   # perfect drafts: these finish after N / W steps
        buf[b, :] = om.greedy_ar(prompts[b, :lens[b]], N + 2 * W)      # slot j of a window drafts generated token g + j - 1
    refs = [om.jacobi_generate(prompts[b, :lens[b]], buf[b], W, N) for b in range(B)]
    assert refs[0]["steps"] == N // W and refs[1]["steps"] > 2 * refs[0]["steps"]
    say("tiny batch with early finishers")
    ctx = make_ctx(fc, B, P + N + 4 * W + 16, W)
    res = {}
    trigger = np.array([3, 14, 15], dtype=np.int32)
    for compact in (1, 0):
        ctx.set_option(4, compact)
        ctx.prefill(prompts, lens, buf)
        out = ctx.generate(N)
        res[compact] = (out, ctx.state(), ctx.answer(trigger, 6))
    for b in range(B):
        assert (res[1][0]["ids"][b] == refs[b]["ids"]).all() and res[1][0]["steps"][b] == refs[b]["steps"], b
        assert (res[1][0]["tail"][b] == refs[b]["tail"]).all()
    for k in ("ids", "len", "steps", "tail"):
        assert (res[1][0][k] == res[0][0][k]).all(), k
    for k in ("n", "g", "done", "window"):
        assert (res[1][1][k] == res[0][1][k]).all(), k
    assert (res[1][2]["ids"] == res[0][2]["ids"]).all() and (res[1][2]["len"] == res[0][2]["len"]).all()


def test_graph_and_eager_agree_and_are_deterministic(env):
    fc, om = env
    P, W, N = 16, 8, 32
    prompt = synthgen.prompts(1, P, TINY.vocab, seed=8)
    buf = synthgen.buffer_init(1, N + 2 * W, TINY.vocab, seed=9)
    ctx = make_ctx(fc, 1, P + N + 2 * W, W)
    outs = []
    for graph in (1, 0, 1):
        ctx.set_option(2, graph)
        ctx.prefill(prompt, [P], buf)
        outs.append(ctx.generate(N))
    for o in outs[1:]:
        assert (o["ids"] == outs[0]["ids"]).all() and (o["steps"] == outs[0]["steps"]).all()


def test_capacity_and_state_errors(env):
    fc, om = env
    W = 4
    ctx = make_ctx(fc, 2, 64, W)
    prompt = synthgen.prompts(1, 8, TINY.vocab)
    buf = synthgen.buffer_init(1, 40, TINY.vocab)
    with pytest.raises(fc.FastcotError) as e:
        ctx.step()
    assert e.value.rc == -2
    with pytest.raises(fc.FastcotError) as e:
        ctx.prefill(synthgen.prompts(3, 8, TINY.vocab), [8, 8, 8], synthgen.buffer_init(3, 40, TINY.vocab))
    assert e.value.rc == -3
    with pytest.raises(fc.FastcotError) as e:
        ctx.prefill(synthgen.prompts(1, 60, TINY.vocab), [60], buf)
    assert e.value.rc == -3
    ctx.prefill(prompt, [8], buf)
    with pytest.raises(fc.FastcotError) as e:
        ctx.generate(60)        # buffer (40) shorter than 60 + 2W
    assert e.value.rc == -3
    out = ctx.generate(16)
    assert out["len"][0] == 16
    with pytest.raises(fc.FastcotError) as e:
        ctx.generate(16)
    assert e.value.rc == -2


@pytest.mark.parametrize("mode", ["cap", "eos", "budget"])
def test_answer_phase_matches_greedy_on_the_combined_context(env, mode):
    """Sec. 4.4 "Trigger Answer": prompt + exact tokens + glimpse (none after an EOS) + trigger, then greedy
    decoding; the oracle does the same with its greedy loop (Eq. 1) over the combined token list."""
    fc, om = env
    P, W, N, NA = 32, 8, 40, 12
    trigger = np.array([5, 77, 301], dtype=np.int32)
    prompt = synthgen.prompts(1, P, TINY.vocab, seed=31)
    buf = synthgen.buffer_init(1, N + 2 * W, TINY.vocab, seed=32)
    greedy = om.greedy_ar(prompt[0], N)
    eos = int(greedy[9]) if mode == "eos" else -1
    max_steps = 5 if mode == "cap" else 0
    ref = om.jacobi_generate(prompt[0], buf[0], W, N, max_steps=max_steps, eos=eos)
    say(f"tiny answer phase, stop by {mode}")
    ctx = make_ctx(fc, 1, P + N + 4 * W + NA + 8, W)
    ctx.prefill(prompt, [P], buf)
    out = ctx.generate(N, max_steps=max_steps, eos_id=eos)
    n_exact = int(out["len"][0])
    assert out["ids"][0][:n_exact].tolist() == ref["ids"].tolist()
    st = ctx.state()
    if mode == "eos":
        assert out["ids"][0][n_exact - 1] == eos
        combined = np.concatenate([prompt[0], out["ids"][0][:n_exact], trigger])
    else:
        # every exact token the run accepted (the last step may have accepted more than the budget), then
        # the glimpse
        g = int(st["g"][0])
        exact = om.greedy_ar(prompt[0], g)
        assert exact[:n_exact].tolist() == out["ids"][0][:n_exact].tolist() and exact[g - 1] == st["window"][0][0]
        combined = np.concatenate([prompt[0], exact, st["window"][0][1:], trigger])
    want = om.greedy_ar(combined.astype(np.int32), NA)
    ans = ctx.answer(trigger, NA)
    assert ans["len"][0] == NA and ans["ids"][0].tolist() == want.tolist()
    with pytest.raises(fc.FastcotError):
        ctx.step()                      # the windowed state is gone until the next prefill


def test_window_size_changes_between_steps(env):
    """Sec. 4.1: whatever the window, every step accepts at least the one exact token and the accepted stream
    is the greedy continuation (Eq. 1); the window may therefore change from step to step."""
    fc, om = env
    P, N, Wmax = 32, 48, 16
    prompt = synthgen.prompts(1, P, TINY.vocab, seed=61)
    buf = synthgen.buffer_init(1, N + 4 * Wmax, TINY.vocab, seed=62)
    greedy = om.greedy_ar(prompt[0], N + Wmax)
    say("tiny window schedule")
    ctx = make_ctx(fc, 1, P + N + 4 * Wmax, Wmax)
    ctx.prefill(prompt, [P], buf)
    got, schedule, i = [], [8, 8, 4, 16, 2, 1, 5, 16, 3], 0
    with pytest.raises(fc.FastcotError):
        ctx.set_window(Wmax + 1)                    # the plain path's passes are at most the configured window
    while len(got) < N:
        W = schedule[i % len(schedule)]
        i += 1
        ctx.set_window(W)
        nacc, acc, win = ctx.step()
        assert 1 <= nacc[0] <= W and win.shape == (1, W)
        got.extend(acc[0][:nacc[0]].tolist())
        assert win[0][0] == got[-1]
    assert got == greedy[:len(got)].tolist()


def test_sequences_join_a_running_batch(env):
    """Eq. 2 couples no two sequences: a prompt that takes over a slot between two steps produces, step by
    step, what it produces alone (accepted ids and verified counts of the oracle's run), and the sequences that
    stay are not disturbed -- whether the newcomer goes to slot 0 or trades places with it for its prefill."""
    fc, om = env
    W, B, N = 4, 3, 64
    L = N + 2 * W
    first = synthgen.prompts(B, 13, TINY.vocab, seed=81)
    lens = [13, 6, 10]
    late = synthgen.prompts(3, 19, TINY.vocab, seed=82)
    late_lens = [19, 1, 8]
    bufs = synthgen.buffer_init(B + 3, L, TINY.vocab, seed=83)
    bufs[4, :] = om.greedy_ar(late[1, :1], L)           # one newcomer with a perfect draft: W tokens per step
    say("tiny batch with joining sequences")
    ctx = make_ctx(fc, B, 19 + L + 16, W)
    ctx.prefill(first, lens, bufs[:B])
    occupant = [dict(prompt=first[b, :lens[b]], buf=bufs[b], ids=[], counts=[]) for b in range(B)]
    finished = []
    joins = {3: (1, 0), 5: (0, 1), 9: (2, 2)}            # before step s: (slot, which late prompt)
    with pytest.raises(fc.FastcotError):
        ctx.join(B, late[0, :19], bufs[3])
    for s in range(14):
        if s in joins:
            slot, k = joins[s]
            finished.append(occupant[slot])
            ctx.join(slot, late[k, :late_lens[k]], bufs[B + k])
            occupant[slot] = dict(prompt=late[k, :late_lens[k]], buf=bufs[B + k], ids=[], counts=[])
        nacc, acc, win = ctx.step()
        for b in range(B):
            occupant[b]["ids"].extend(acc[b][:nacc[b]].tolist())
            occupant[b]["counts"].append(int(nacc[b]))
            assert win[b][0] == occupant[b]["ids"][-1]
    for seq in finished + occupant:
        steps = len(seq["counts"])
        ref = om.jacobi_generate(seq["prompt"], seq["buf"], W, N, max_steps=steps)
        assert steps >= 2 and ref["steps"] == steps
        assert len(seq["ids"]) <= N and seq["ids"] == ref["ids"].tolist()
        assert seq["counts"] == [k + 1 for k in ref["K"]]
    assert max(occupant[0]["counts"]) == W                # the perfect draft was accepted whole
    ctx.prefill(first, lens, bufs[:B])
    ctx.generate(8)
    with pytest.raises(fc.FastcotError):                  # generate runs its batch to the end
        ctx.join(0, late[0, :19], bufs[3])


def test_per_sequence_window_sizes(env):
    """The window enters Eq. 4 / Eq. 5 per sequence: in a batch whose step computes W rows for everyone, a
    sequence told to use W_b of them produces the ids, step count and approximate tail of the oracle's run with
    window W_b, and its answer phase sees W_b - 1 glimpse tokens."""
    fc, om = env
    W, B, N, P, NA = 8, 4, 24, 12, 5
    wins = [8, 3, 1, 5]
    lens = [12, 9, 4, 12]
    prompts = synthgen.prompts(B, P, TINY.vocab, seed=101)
    buf = synthgen.buffer_init(B, N + 2 * W, TINY.vocab, seed=102)
    buf[3, :] = om.greedy_ar(prompts[3, :lens[3]], N + 2 * W)        # a perfect draft: W_b tokens per step
    refs = [om.jacobi_generate(prompts[b, :lens[b]], buf[b], wins[b], N) for b in range(B)]
    assert refs[2]["steps"] == N and refs[3]["steps"] == -(-N // wins[3])
    say("tiny per-sequence windows")
    ctx = make_ctx(fc, B, P + N + 4 * W + NA + 8, W)
    ctx.prefill(prompts, lens, buf)
    with pytest.raises(fc.FastcotError):
        ctx.set_windows([8, 9, 1, 1])
    ctx.set_windows(wins)
    out = ctx.generate(N)
    st = ctx.state()
    for b in range(B):
        assert out["len"][b] == N and (out["ids"][b] == refs[b]["ids"]).all(), b
        assert out["steps"][b] == refs[b]["steps"], b
        assert (out["tail"][b][:wins[b] - 1] == refs[b]["tail"]).all(), b
    trigger = np.array([9, 500], dtype=np.int32)
    ans = ctx.answer(trigger, NA)
    for b in range(B):
        g = int(st["g"][b])
        exact = om.greedy_ar(prompts[b, :lens[b]], g)
        combined = np.concatenate([prompts[b, :lens[b]], exact, st["window"][b][1:wins[b]], trigger]).astype(np.int32)
        assert ans["ids"][b].tolist() == om.greedy_ar(combined, NA).tolist(), b
    # step mode: counts per step, and a prefill puts every sequence back on the batch window
    ctx.prefill(prompts, lens, buf)
    ctx.set_windows(wins)
    for s in range(3):
        nacc, _, _ = ctx.step()
        assert [int(x) - 1 for x in nacc] == [int(refs[b]["K"][s]) for b in range(B)]
    ctx.prefill(prompts, lens, buf)
    full = [om.jacobi_generate(prompts[b, :lens[b]], buf[b], W, N) for b in range(B)]
    out = ctx.generate(N)
    for b in range(B):
        assert out["steps"][b] == full[b]["steps"] and (out["ids"][b] == full[b]["ids"]).all()
