"""GPU parity at the real layer shapes of the larger benchmark configurations, with the layer count
cut to 2 so that the oracle follows in seconds: Llama-2-70B-shaped (d 8192, 64 query heads / 8 KV
heads, FFN 28672: grouped-query attention) and Llama-2-13B-shaped (d 5120, 40 heads, FFN 13824),
the latter also at batch 8 x window 32 = 256 rows per step."""
import numpy as np
import pytest

import oracle
import synthgen
from gpu_util import follow_steps, say

pytestmark = pytest.mark.gpu

S70 = synthgen.small_variant(synthgen.SHAPES["70b"], n_layers=2)
S13 = synthgen.small_variant(synthgen.SHAPES["13b"], n_layers=2)
S7 = synthgen.small_variant(synthgen.SHAPES["7b"], n_layers=2)      # gate/up: 1376 n-tiles, shared half tiles


def build(fc, shape, B, S, W):
    cfg = fc.Config.from_shape(shape, B, S, W)
    kept = {}

    def gen():
        for spec in synthgen.weight_tensors(shape):
            arr = synthgen.weight_array(shape, spec, as_bf16_bits=True)
            if spec.layer < 0:
                kept[spec.name] = arr
            else:
                kept.setdefault(spec.name, []).append(arr)
            yield spec.name, spec.layer, arr
    packed = fc.pack_weights(cfg, gen())
    fields = dict(n_layers=shape.n_layers, d_model=shape.d_model, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                  head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab, rms_eps=shape.rms_eps,
                  rope_base=shape.rope_base)
    return fc.Context(cfg, packed), oracle.Model(fields, kept, wdtype=1)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,shape,B,W,P,steps", [("70b-shaped", S70, 1, 16, 41, 3), ("13b-shaped", S13, 1, 16, 37, 3),
                                                    ("13b-shaped batch 8 window 32", S13, 8, 32, 50, 2),
                                                    ("13b-shaped window 32", S13, 1, 32, 45, 2), ("70b-shaped window 24", S70, 1, 24, 41, 2),
                                                    ("7b-shaped", S7, 1, 16, 39, 3), ("7b-shaped window 32", S7, 1, 32, 39, 2)])
def test_layer_shapes_follow_mode(name, shape, B, W, P, steps):
    import paper_2311_08263_amd as fc
    say(f"{name}: B={B} W={W} P={P}")
    N = 64
    S = ((P + N + 2 * W + 31) // 32) * 32
    ctx, om = build(fc, shape, B, S, W)
    lens = [P - 2 * b for b in range(B)]
    prompts = synthgen.prompts(B, P, shape.vocab, seed=51)
    buf = synthgen.buffer_init(B, N + 2 * W, shape.vocab, seed=52)
    ctx.prefill(prompts, lens, buf)
    r = follow_steps(ctx, om, prompts, lens, steps, 2e-2)
    print(f"{name}: max |dlogit| {r['max_err']:.3e} over {r['rows']} rows ({r['low_margin_rows']} low-margin)")
    assert r["max_err"] < 5e-3
    ctx.close()


@pytest.mark.timeout(600)
def test_many_row_attention_grouped_heads():
    """The many-row attention kernel at the 70B layer shape (64 query heads on 8 K/V heads, workgroup ids strided by
    the K/V head count): a 300-token prompt goes through it in one chunk, then the oracle follows two steps."""
    import paper_2311_08263_amd as fc
    shape, B, W, P = S70, 1, 16, 300
    say(f"70b-shaped, many-row attention forced: P={P}")
    S = ((P + 64 + 2 * W + 31) // 32) * 32
    ctx, om = build(fc, shape, B, S, W)
    ctx.set_option(fc.binding.PLAN_ATTN_MANY_ROWS, 2)
    prompts = synthgen.prompts(B, P, shape.vocab, seed=61)
    buf = synthgen.buffer_init(B, 64 + 2 * W, shape.vocab, seed=62)
    ctx.prefill(prompts, [P], buf)
    r = follow_steps(ctx, om, prompts, [P], 2, 2e-2)
    print(f"70b-shaped many-row attention: max |dlogit| {r['max_err']:.3e} over {r['rows']} rows")
    assert r["max_err"] < 5e-3
    ctx.close()
