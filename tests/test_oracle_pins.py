"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the statement of the paper (section / equation) or the textbook fact it
checks.  The library pin uses the `transformers` Llama implementation in float64 as an
independent definition of the decoder forward and of greedy decoding.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
import synthgen

TINY = synthgen.SHAPES["tiny"]


def rand_gain_model(shape, seed=7, real="f64"):
    """Synthetic weights plus non-trivial RMSNorm gains (so a dropped gain is caught)."""
    rng = np.random.default_rng(seed)
    weights = {}
    for spec in synthgen.weight_tensors(shape):
        arr = synthgen.weight_array(shape, spec, synthgen.WEIGHT_SEED)
        # bigger weights than 0.02 so attention is far from uniform and mistakes show
        arr = (arr * 3.0).astype(np.float32)
        if spec.layer < 0:
            weights[spec.name] = arr
        else:
            weights.setdefault(spec.name, []).append(arr)
    weights["g1"] = [rng.uniform(0.5, 1.5, shape.d_model).astype(np.float32) for _ in range(shape.n_layers)]
    weights["g2"] = [rng.uniform(0.5, 1.5, shape.d_model).astype(np.float32) for _ in range(shape.n_layers)]
    weights["gf"] = rng.uniform(0.5, 1.5, shape.d_model).astype(np.float32)
    fields = dict(n_layers=shape.n_layers, d_model=shape.d_model, n_heads=shape.n_heads,
                  n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab,
                  rms_eps=shape.rms_eps, rope_base=shape.rope_base)
    return oracle.Model(fields, weights, real=real), weights


def hf_llama(shape, weights):
    import torch
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
                      rope_theta=shape.rope_base, max_position_embeddings=512, tie_word_embeddings=False,
                      attention_bias=False, mlp_bias=False, attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": weights["emb"], "lm_head.weight": weights["wlm"].T,
          "model.norm.weight": weights["gf"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj"}
    for l in range(shape.n_layers):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = weights[k][l].T     # library stores [out, in]
        sd[f"model.layers.{l}.input_layernorm.weight"] = weights["g1"][l]
        sd[f"model.layers.{l}.post_attention_layernorm.weight"] = weights["g2"][l]
    sd = {k: torch.tensor(np.ascontiguousarray(v), dtype=torch.float64) for k, v in sd.items()}
    missing = m.load_state_dict(sd, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k], missing
    return m


@pytest.mark.parametrize("n_kv", [4, 2, 1])
def test_forward_and_greedy_match_library_llama(n_kv):
    """Eq. (1) and the decoder forward: the oracle's cached, windowed forward equals the
    library's full-sequence causal forward in float64 (MHA and grouped-query variants), and
    the oracle's greedy loop equals the library's greedy generate."""
    import torch
    shape = synthgen.small_variant(TINY, n_kv_heads=n_kv, vocab=512)
    om, weights = rand_gain_model(shape)
    hf = hf_llama(shape, weights)
    toks = synthgen.tokens(40, 3, 9, shape.vocab)
    with torch.no_grad():
        ref = hf(torch.tensor(toks[None].astype(np.int64))).logits[0].numpy()
    ss = om.session(64)
    lg_a, _, _ = ss.forward(toks[:23], 0)          # "prefill" rows
    lg_b, am_b, _ = ss.forward(toks[23:31], 23)    # a window of 8 on top of the cache
    lg_c, _, _ = ss.forward(toks[31:40], 31)
    got = np.concatenate([lg_a, lg_b, lg_c])
    # the library evaluates the rotary angles in fp32 whatever the model dtype, hence 1e-5 and
    # not 1e-12; any structural mistake (sign, pairing, head mapping, gain) is O(0.1) or more
    assert np.abs(got - ref).max() < 1e-5
    assert (am_b == ref[23:31].argmax(-1)).all()
    # greedy decoding
    N = 24
    with torch.no_grad():
        gen = hf.generate(torch.tensor(toks[None, :12].astype(np.int64)), max_new_tokens=N, do_sample=False,
                          pad_token_id=0, eos_token_id=None)[0, 12:].numpy()
    assert (om.greedy_ar(toks[:12], N) == gen).all()


@pytest.fixture(scope="module")
def tiny_model():
    return oracle.model_from_synth(TINY)


@pytest.fixture(scope="module")
def tiny_greedy(tiny_model):
    p = synthgen.prompts(1, 32, TINY.vocab)[0]
    return p, tiny_model.greedy_ar(p, 64 + 16)


def test_window_one_is_greedy(tiny_model, tiny_greedy):
    """Sec. 3.1: a window with no extra tokens (the paper's size 0) is autoregressive decoding."""
    p, g = tiny_greedy
    r = tiny_model.jacobi_generate(p, synthgen.buffer_init(1, 64 + 2, TINY.vocab)[0], 1, 64)
    assert (r["ids"] == g[:64]).all() and r["steps"] == 64 and (r["K"] == 0).all()


@pytest.mark.parametrize("W", [2, 3, 8, 16])
@pytest.mark.parametrize("bseed", [2, 11])
def test_accepted_stream_is_greedy_for_any_window_and_buffer(tiny_model, tiny_greedy, W, bseed):
    """Sec. 4.1 / 4.2: the exact segment equals lossless (greedy) decoding whatever the buffer
    held; every iteration yields at least one exact token, at most W."""
    p, g = tiny_greedy
    N = 64
    r = tiny_model.jacobi_generate(p, synthgen.buffer_init(1, N + 2 * W, TINY.vocab, bseed)[0], W, N)
    assert (r["ids"] == g[:N]).all()
    assert ((r["K"] >= 0) & (r["K"] <= W - 1)).all()
    assert math.ceil(N / W) <= r["steps"] <= N
    # accepted counts add up: all but the last step stay below N
    acc = (r["K"] + 1).cumsum()
    assert acc[-1] >= N and (acc[:-1] < N).all()


def test_static_window_reaches_greedy_fixed_point(tiny_model, tiny_greedy):
    """Eq. (2): row j depends only on window slots before j, so iterating the same window
    position makes output t-1 exact after t iterations and stops changing within W iterations."""
    p, g = tiny_greedy
    W = 8
    ss = tiny_model.session(64)
    ss.forward(p[:-1], 0, want_logits=False)
    n = len(p) - 1
    w = np.concatenate([[p[-1]], synthgen.buffer_init(1, W - 1, TINY.vocab, 5)[0]]).astype(np.int32)
    for t in range(1, W + 1):
        _, o, _ = ss.forward(w, n, want_logits=False)
        assert (o[:t] == g[:t]).all(), t
        w = np.concatenate([[p[-1]], o[:-1]]).astype(np.int32)
    _, o2, _ = ss.forward(w, n, want_logits=False)
    assert (o2 == g[:W]).all() and (o2[:-1] == w[1:]).all()


def test_perfect_and_adversarial_drafts(tiny_model, tiny_greedy):
    """Eq. (5) closed forms: a buffer holding the greedy continuation verifies fully every
    iteration (steps = ceil(N/W)); a buffer of a token the model does not emit there verifies nothing."""
    p, g = tiny_greedy
    W, N = 8, 60
    r = tiny_model.jacobi_generate(p, g[:N + 2 * W], W, N)
    assert r["steps"] == math.ceil(N / W) and (r["K"] == W - 1).all() and (r["ids"] == g[:N]).all()
    bad = next(t for t in range(TINY.vocab) if t not in set(g.tolist()))
    r = tiny_model.jacobi_generate(p, np.full(N + 2 * W, bad, dtype=np.int32), W, N)
    assert r["K"][0] == 0 and (r["ids"] == g[:N]).all()


def test_zero_layer_model_trajectory_by_table_lookup():
    """Eq. (2), (5) and the cache update on a degenerate model: with no decoder layers each
    output is a fixed function T of its own input token, so the whole Jacobi trajectory (every
    window, every K, the buffer) follows from table lookups done here by hand."""
    shape = synthgen.small_variant(TINY, n_layers=0, vocab=64)
    m = oracle.model_from_synth(shape)
    emb = synthgen.weight_array(shape, next(s for s in synthgen.weight_tensors(shape) if s.name == "emb")).astype(np.float64)
    wlm = synthgen.weight_array(shape, next(s for s in synthgen.weight_tensors(shape) if s.name == "wlm")).astype(np.float64)
    nrm = emb / np.sqrt((emb ** 2).mean(-1, keepdims=True) + shape.rms_eps)
    T = (nrm @ wlm).argmax(-1)
    W, N = 4, 40
    prompt = synthgen.prompts(1, 5, shape.vocab)[0]
    buf0 = synthgen.buffer_init(1, N + 2 * W, shape.vocab)[0]
    # by hand
    buf, g, newest, ids, Ks = buf0.copy(), 0, prompt[-1], [], []
    while g < N:
        w = [newest] + [buf[g + j - 1] for j in range(1, W)]
        o = [T[t] for t in w]
        K = 0
        while K < W - 1 and o[K] == w[K + 1]:
            K += 1
        buf[g:g + W] = o
        ids += o[:K + 1]
        Ks.append(K)
        newest = o[K]
        g += K + 1
    r = m.jacobi_generate(prompt, buf0, W, N)
    assert r["K"].tolist() == Ks and r["steps"] == len(Ks)
    assert r["ids"].tolist() == [int(t) for t in ids[:N]]
    assert (r["buf"] == buf).all()
    assert r["tail"].tolist() == [int(t) for t in buf[g:g + W - 1]]


def test_verify_exhaustive_against_literal_definition():
    """Eq. (5): K is the largest k such that every approximate slot i <= k equals the fresh
    prediction for its position; checked for all windows over a 3-letter alphabet, W <= 4."""
    for W in (1, 2, 3, 4):
        for w in itertools.product(range(3), repeat=W):
            for o in itertools.product(range(3), repeat=W):
                lit = max(k for k in range(W) if all(o[i - 1] == w[i] for i in range(1, k + 1)))
                assert oracle.verify(w, o) == lit


def test_attention_window_matches_dense_masked_softmax():
    """Eq. (2) conditioning as a mask: window-causal attention equals dense softmax attention
    under an explicit (n+R) x R mask; later window slots and the cache tail do not leak."""
    rng = np.random.default_rng(0)
    n, R, H, Hkv, Dh = 37, 5, 4, 2, 16
    q = rng.normal(size=(R, H, Dh))
    k = rng.normal(size=(n + R, Hkv, Dh))
    v = rng.normal(size=(n + R, Hkv, Dh))
    out = oracle.attention_window(q, k, v, n)
    kk, vv = np.repeat(k, H // Hkv, axis=1), np.repeat(v, H // Hkv, axis=1)
    s = np.einsum("rhd,thd->hrt", q, kk) / math.sqrt(Dh)
    mask = np.arange(n + R)[None, :] <= (n + np.arange(R))[:, None]
    s = np.where(mask[None], s, -np.inf)
    pr = np.exp(s - s.max(-1, keepdims=True))
    pr /= pr.sum(-1, keepdims=True)
    ref = np.einsum("hrt,thd->rhd", pr, vv).reshape(R, H * Dh)
    assert np.abs(out - ref).max() < 1e-12
    # garbage in later slots must not change earlier rows
    k2, v2 = k.copy(), v.copy()
    k2[n + 3:], v2[n + 3:] = 1e3, -1e3
    out2 = oracle.attention_window(q, k2, v2, n)
    assert (out2[:3] == out[:3]).all()


def test_rope_rmsnorm_closed_forms():
    """Textbook facts: rotary embedding at position 0 is the identity and inner products
    depend only on the position difference; RMSNorm output has unit mean square."""
    rng = np.random.default_rng(1)
    q, k = rng.normal(size=64), rng.normal(size=64)
    assert (oracle.rope(q, 0, 1e4) == q).all()
    d0 = oracle.rope(q, 17, 1e4) @ oracle.rope(k, 5, 1e4)
    d1 = oracle.rope(q, 112, 1e4) @ oracle.rope(k, 100, 1e4)
    assert abs(d0 - d1) < 1e-10
    assert abs(np.linalg.norm(oracle.rope(q, 33, 1e4)) - np.linalg.norm(q)) < 1e-12
    # the pair (i, i + Dh/2) rotates by pos * base^(-2i/Dh)
    e = np.zeros(64); e[3] = 1.0
    r = oracle.rope(e, 7, 1e4)
    ang = 7 * 1e4 ** (-2 * 3 / 64)
    assert abs(r[3] - math.cos(ang)) < 1e-14 and abs(r[35] - math.sin(ang)) < 1e-14
    x = rng.normal(size=256) * 5
    assert abs((oracle.rmsnorm(x, None, 0.0) ** 2).mean() - 1) < 1e-12


def test_shift_consistency_bit_exact(tiny_model, tiny_greedy):
    """Eq. (2): the logits of a position given the same exact prefix are identical whether the
    position is row 0 of one forward or a later row of another."""
    p, g = tiny_greedy
    seq = np.concatenate([p, g[:8]]).astype(np.int32)
    a = tiny_model.session(64)
    la, _, _ = a.forward(seq, 0)
    b = tiny_model.session(64)
    b.forward(seq[:30], 0, want_logits=False)
    lb1, _, _ = b.forward(seq[30:35], 30)
    lb2, _, _ = b.forward(seq[35:40], 35)
    assert (la[30:35] == lb1).all() and (la[35:40] == lb2).all()


def test_stop_conditions(tiny_model, tiny_greedy):
    """Sec. 4.4: stop once EOS is among the verified tokens (approximate EOS is ignored), or at
    the iteration cap."""
    p, g = tiny_greedy
    N, W = 48, 8
    # an id whose first occurrence in the greedy stream is at a known index
    idx = 13
    eos = int(g[idx])
    first = int(np.where(g == eos)[0][0])
    r = tiny_model.jacobi_generate(p, np.full(N + 2 * W, eos, dtype=np.int32), W, N, eos=eos)
    assert r["ids"].tolist() == g[:first + 1].tolist()
    r = tiny_model.jacobi_generate(p, synthgen.buffer_init(1, N + 2 * W, TINY.vocab)[0], W, N, max_steps=3)
    assert r["steps"] == 3 and len(r["ids"]) == int((r["K"] + 1).sum()) and (r["ids"] == g[:len(r["ids"])]).all()


def test_fp32_build_agrees_with_fp64(tiny_greedy):
    p, g = tiny_greedy
    m32 = oracle.model_from_synth(TINY, real="f32")
    m64 = oracle.model_from_synth(TINY, real="f64")
    l32, _, _ = m32.session(64).forward(p, 0)
    l64, _, _ = m64.session(64).forward(p, 0)
    assert np.abs(l32 - l64).max() < 1e-5


def test_bf16_storage_is_exact():
    shape = synthgen.small_variant(TINY, dtype="bf16")
    a = oracle.model_from_synth(shape, bf16_storage=True)
    b = oracle.model_from_synth(shape, bf16_storage=False)
    t = synthgen.prompts(1, 12, shape.vocab)[0]
    la, _, _ = a.session(16).forward(t, 0)
    lb, _, _ = b.session(16).forward(t, 0)
    assert (la == lb).all()


def test_stored_tiny_trajectory_is_reproduced():
    """tests/golden/tiny_trajectory.json was written by tests/golden/make_golden.py from this oracle: the
    oracle, the input generators and the stored trajectory must still agree (regression pin, Sec. 4.1-4.4)."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "golden", "tiny_trajectory.json")) as f:
        stored = json.load(f)
    assert mod.trajectory() == stored
    # structure every trajectory has: each step accepts K+1 in 1..W, the counts add up to the output
    W, N = stored["config"]["window"], stored["config"]["new_tokens"]
    assert all(0 <= k <= W - 1 for k in stored["K"]) and len(stored["K"]) == stored["steps"]
    assert sum(k + 1 for k in stored["K"]) >= N > sum(k + 1 for k in stored["K"][:-1])


@pytest.mark.parametrize("real", ["f64", "f32"])
def test_layer_streamed_forward_is_the_forward_bit_for_bit(real):
    """oracle.forward_streamed (one layer's weights at a time: oracle_embed / oracle_layers / oracle_head over
    one-layer models) against Session.forward of the whole model, which the library pin above fixes: a prefill,
    then two windowed passes of which the second rewinds over positions the first wrote (the K/V a Jacobi step
    leaves past its accepted prefix), grouped K/V heads, random gains.  Equal to the last bit."""
    shape = synthgen.ModelShape(3, 128, 4, 2, 32, 352, 512, dtype="f32")
    model, weights = rand_gain_model(shape, seed=11, real=real)
    toks = synthgen.tokens(40, 9, 0x77, shape.vocab)
    passes = [(toks[:17], 0, False), (toks[17:25], 17, True), (toks[25:33], 20, True)]
    ss = model.session(48)
    want = []
    for t, p0, wl in passes:
        lg, am, _ = ss.forward(t, p0, want_logits=wl)
        want.append((lg, am))
    fields = dict(model.fields)
    got = oracle.forward_streamed(fields, 0, {k: weights[k] for k in ("emb", "wlm", "gf")},
                                  lambda l: {k: weights[k][l] for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")},
                                  [passes, passes[:2]], 48, real=real)
    for seq in got:
        assert seq[0] == (None, None)
        for (lg, am), (wlg, wam) in zip(seq[1:], want[1:]):
            assert (lg == wlg).all() and (am == wam).all()


def test_oracle_and_generators_under_address_and_ub_sanitizers(tmp_path):
    """Builds oracle/fastcot_oracle.c and synthgen/gen.c with -fsanitize=address,undefined into one host program
    that generates a tiny model and runs a short Jacobi trajectory and the layer-range calls; any out-of-bounds
    access, leak-free or not, or undefined operation aborts it."""
    import os
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    main = tmp_path / "san_main.c"
    main.write_text(r'''
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
typedef struct { int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab; float rms_eps, rope_base; int32_t wdtype; } oracle_shape;
void* oracle_model_new(const oracle_shape*); void oracle_model_free(void*); int oracle_model_set(void*, int, int, const void*);
void* oracle_session_new(const void*, int32_t); void oracle_session_free(void*);
int oracle_forward(void*, const int32_t*, int, int, double*, int32_t*, double*);
int oracle_embed(const void*, const int32_t*, int, double*); int oracle_layers(void*, int, int, int, int, double*);
int oracle_head(const void*, const double*, int, double*, int32_t*);
int oracle_jacobi_generate(const void*, const int32_t*, int32_t, int32_t*, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t*, int32_t*, int32_t*, int32_t*, int32_t, int32_t*);
int32_t oracle_greedy_ar(const void*, const int32_t*, int32_t, int32_t, int32_t, int32_t*);
double synth_sigma_sum(void);
void synth_tokens(int32_t*, size_t, uint64_t, uint64_t, int32_t);
void synth_normal_bf16(uint16_t*, size_t, uint64_t, uint64_t, float);
int main(void) {
    oracle_shape s = {2, 64, 4, 2, 16, 96, 128, 1e-5f, 1e4f, 1};
    const int d = 64, qd = 64, kvd = 32, F = 96, V = 128, L = 2;
    void* m = oracle_model_new(&s);
    float sc = (float)(0.05 / synth_sigma_sum());
    size_t sizes[10] = {(size_t)V * d, (size_t)d * V, 0, (size_t)d * qd, (size_t)d * kvd, (size_t)d * kvd, (size_t)qd * d, (size_t)d * F, (size_t)d * F, (size_t)F * d};
    uint16_t* keep[2 + 7 * 2]; int nk = 0;
    for (int t = 0; t < 2; ++t) { uint16_t* w = malloc(sizes[t] * 2); synth_normal_bf16(w, sizes[t], 5, 100 + t, sc); oracle_model_set(m, t, -1, w); keep[nk++] = w; }
    for (int l = 0; l < L; ++l) for (int t = 3; t < 10; ++t) { uint16_t* w = malloc(sizes[t] * 2); synth_normal_bf16(w, sizes[t], 5, l * 16 + t, sc); oracle_model_set(m, t, l, w); keep[nk++] = w; }
    int32_t prompt[9], buf[40], out[16], Ks[16], tail[4], greedy[16], olen = 0, osteps = 0;
    synth_tokens(prompt, 9, 1, 2, V); synth_tokens(buf, 40, 1, 3, V);
    if (oracle_jacobi_generate(m, prompt, 9, buf, 40, 5, 16, 0, -1, out, &olen, &osteps, Ks, 16, tail)) return 2;
    if (oracle_greedy_ar(m, prompt, 9, 16, -1, greedy) != 16 || olen != 16 || memcmp(out, greedy, 64)) return 3;
    /* layer-range calls against the whole forward */
    void* a = oracle_session_new(m, 16); void* b = oracle_session_new(m, 16);
    double la[9 * 128], lb[9 * 128], x[9 * 64]; int32_t am[9];
    if (oracle_forward(a, prompt, 9, 0, la, am, NULL)) return 4;
    if (oracle_embed(m, prompt, 9, x) || oracle_layers(b, 0, 1, 9, 0, x) || oracle_layers(b, 1, 2, 9, 0, x) || oracle_head(m, x, 9, lb, am)) return 5;
    if (memcmp(la, lb, sizeof(la))) return 6;
    oracle_session_free(a); oracle_session_free(b);
    for (int i = 0; i < nk; ++i) free(keep[i]);
    oracle_model_free(m);
    printf("sanitized run ok: %d tokens in %d steps\n", olen, osteps);
    return 0;
}
''')
    exe = tmp_path / "san_oracle"
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp",
                           "-o", str(exe), str(main), os.path.join(root, "oracle", "fastcot_oracle.c"),
                           os.path.join(root, "synthgen", "gen.c"), "-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1")
    r = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitized run ok" in r.stdout
