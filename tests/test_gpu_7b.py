"""Full-size parity: the Llama-2-7B-shaped bf16 model (32 layers, d 4096, 32 heads x 128, FFN 11008,
vocab 32000), batch 1, prompt 256, window 16 -- the configuration the benchmark times, in the same
launch configuration (graph replay).  The oracle follows the GPU for a few steps (its prefill of
255 rows plus a step of 16 rows is about a minute of host time)."""
import time

import numpy as np
import pytest

import oracle
import synthgen
from gpu_util import follow_steps, say

pytestmark = pytest.mark.gpu
SHAPE = synthgen.SHAPES["7b"]


@pytest.fixture(scope="module")
def env():
    import paper_2311_08263_amd as fc
    t0 = time.time()
    cfg = fc.Config.from_shape(SHAPE, 1, 640, 16)
    kept = {}

    def gen():
        for spec in synthgen.weight_tensors(SHAPE):
            arr = synthgen.weight_array(SHAPE, spec, as_bf16_bits=True)
            if spec.layer < 0:
                kept[spec.name] = arr
            else:
                kept.setdefault(spec.name, []).append(arr)
            yield spec.name, spec.layer, arr
    say("7b: generating and packing weights")
    packed = fc.pack_weights(cfg, gen())
    fields = dict(n_layers=SHAPE.n_layers, d_model=SHAPE.d_model, n_heads=SHAPE.n_heads, n_kv_heads=SHAPE.n_kv_heads,
                  head_dim=SHAPE.head_dim, d_ffn=SHAPE.d_ffn, vocab=SHAPE.vocab, rms_eps=SHAPE.rms_eps,
                  rope_base=SHAPE.rope_base)
    om = oracle.Model(fields, kept, wdtype=1)
    say(f"7b: model ready in {time.time() - t0:.1f}s")
    return fc, cfg, packed, om


@pytest.mark.timeout(900)
def test_7b_follow_mode_full_size(env):
    """The oracle follows three full-size steps whose draft is the model's own continuation for the first 32
    tokens (taken from a run of the GPU alone) and random ids after that: two steps that verify and accept many
    tokens at once (Eq. 5 with K up to 15, the commit of 16 K/V rows, the shift by 16) and one that accepts a single
    token, all with logits, argmax and the integer path checked against the oracle."""
    fc, cfg, packed, om = env
    P, W, N = 256, 16, 256
    ctx = fc.Context(cfg, packed)
    prompts = synthgen.prompts(1, P, SHAPE.vocab)
    buf = synthgen.buffer_init(1, N + 2 * W, SHAPE.vocab)
    say("7b: the continuation (GPU alone, 32 tokens)")
    ctx.prefill(prompts, [P], buf)
    first = ctx.generate(2 * W)["ids"][0]
    draft = buf.copy()
    draft[0, :2 * W] = first
    say("7b: prefill with that draft")
    ctx.prefill(prompts, [P], draft)
    t0 = time.time()
    r = follow_steps(ctx, om, prompts, [P], 3, 2e-2)
    print(f"7b follow: max |dlogit| {r['max_err']:.3e} over {r['rows']} rows, {r['low_margin_rows']} low-margin, "
          f"K={r['K']}, oracle time {time.time() - t0:.1f}s")
    assert max(r["K"]) >= 8, "no step of the followed prefix verified a long draft"
    assert min(r["K"]) <= 2, "no step of the followed prefix rejected its draft early"
    st = ctx.state()
    assert st["n"][0] == P - 1 + st["g"][0]


@pytest.mark.timeout(600)
def test_7b_generate_invariants_and_plain_path_agreement(env):
    """Properties that hold at any size: every step accepts 1..W tokens, counts add up, a perfect
    draft (the stream itself as buffer) is accepted W at a time, and the plain kernels produce the
    same tokens up to the first token where the two paths' logits could differ by rounding."""
    fc, cfg, packed, om = env
    P, W, N = 256, 16, 64
    ctx = fc.Context(cfg, packed)
    prompts = synthgen.prompts(1, P, SHAPE.vocab)
    buf = synthgen.buffer_init(1, N + 2 * W, SHAPE.vocab)
    say("7b: generate 64")
    ctx.prefill(prompts, [P], buf)
    out = ctx.generate(N)
    assert out["len"][0] == N and (N + W - 1) // W <= out["steps"][0] <= N
    ms = ctx.step_times()
    print(f"7b: steps {out['steps'][0]}, median step {np.median(ms):.3f} ms")
    # perfect draft: feed the generated stream back as the buffer
    draft = np.concatenate([out["ids"][0], buf[0, :2 * W]])[None]
    ctx.prefill(prompts, [P], draft)
    out2 = ctx.generate(N)
    same = out2["ids"][0] == out["ids"][0]
    first_diff = int(np.argmin(same)) if not same.all() else N
    print(f"7b perfect draft: steps {out2['steps'][0]}, agreement up to token {first_diff}")
    assert first_diff >= W          # the first window at least is reproduced
    if same.all():
        assert out2["steps"][0] == (N + W - 1) // W
