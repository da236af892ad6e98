"""ctypes wrapper of the CPU oracle (fastcot_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports this package.

Two builds of the same source: ``real = double`` (the parity reference) and
``real = float`` (the plain-fp32 variant, also the one timed as CPU baseline).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastcot_oracle.c")
_libs = {}

T = {"emb": 0, "wlm": 1, "gf": 2, "wq": 3, "wk": 4, "wv": 5, "wo": 6, "wg": 7, "wu": 8, "wd": 9, "g1": 10, "g2": 11}


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", ctypes.c_float), ("rope_base", ctypes.c_float), ("wdtype", ctypes.c_int32)]


def so_path(real: str) -> str:
    return os.path.join(_HERE, f"liboracle_{real}.so")


def build(force: bool = False) -> None:
    for real, ctype in (("f64", "double"), ("f32", "float")):
        so = so_path(real)
        if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(_SRC):
            subprocess.check_call(["gcc", "-O3", "-mavx2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                                   f"-DORACLE_REAL={ctype}", "-o", so, _SRC, "-lm"])


def lib(real: str = "f64"):
    if real not in _libs:
        build()
        L = ctypes.CDLL(so_path(real))
        vp, i32, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_double
        L.oracle_real_bytes.restype = ctypes.c_int
        L.oracle_model_new.restype = vp
        L.oracle_model_new.argtypes = [ctypes.POINTER(Shape)]
        L.oracle_model_free.argtypes = [vp]
        L.oracle_model_set.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp]
        L.oracle_session_new.restype = vp
        L.oracle_session_new.argtypes = [vp, i32]
        L.oracle_session_free.argtypes = [vp]
        L.oracle_session_len.argtypes = [vp]
        L.oracle_session_set_len.argtypes = [vp, i32]
        L.oracle_forward.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp, vp, vp]
        L.oracle_embed.argtypes = [vp, vp, ctypes.c_int, vp]
        L.oracle_layers.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
        L.oracle_head.argtypes = [vp, vp, ctypes.c_int, vp, vp]
        L.oracle_verify.argtypes = [vp, vp, i32]
        L.oracle_verify.restype = i32
        L.oracle_greedy_ar.argtypes = [vp, vp, i32, i32, i32, vp]
        L.oracle_greedy_ar.restype = i32
        L.oracle_jacobi_generate.argtypes = [vp, vp, i32, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
        L.oracle_attention_window.argtypes = [vp, vp, vp] + [ctypes.c_int] * 5 + [vp]
        L.oracle_attention_window.restype = None
        L.oracle_lmhead_argmax.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        L.oracle_lmhead_argmax.restype = None
        L.oracle_rmsnorm.argtypes = [vp, vp, ctypes.c_int, dbl, vp]
        L.oracle_rmsnorm.restype = None
        L.oracle_rope.argtypes = [vp, ctypes.c_int, ctypes.c_int, dbl]
        L.oracle_rope.restype = None
        _libs[real] = L
    return _libs[real]


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Model:
    """Weights in canonical layout: dict name -> array (global) or list of arrays (per layer).

    Linear weights are row-major [in, out]; 'emb' is [vocab, d].  Arrays are float32, or
    uint16 bf16 bit patterns when wdtype == 1.  Gains ('g1','g2' per layer, 'gf') default to 1.
    """

    def __init__(self, shape_fields: dict, weights: dict, wdtype: int = 0, real: str = "f64"):
        self.real = real
        self.L = lib(real)
        self.fields = dict(shape_fields)
        self.shape = Shape(wdtype=wdtype, **shape_fields)
        self.h = self.L.oracle_model_new(ctypes.byref(self.shape))
        self._keep = []
        want = np.uint16 if wdtype == 1 else np.float32
        for name, val in weights.items():
            per_layer = isinstance(val, (list, tuple))
            for l, arr in enumerate(val if per_layer else [val]):
                dt = np.float32 if name in ("gf", "g1", "g2") else want
                a = np.ascontiguousarray(arr, dtype=dt)
                self._keep.append(a)
                rc = self.L.oracle_model_set(self.h, T[name], l if per_layer else -1, a.ctypes.data)
                assert rc == 0, name

    def __del__(self):
        try:
            self.L.oracle_model_free(self.h)
        except Exception:
            pass

    def session(self, max_seq: int) -> "Session":
        return Session(self, max_seq)

    def greedy_ar(self, prompt, N: int, eos: int = -1) -> np.ndarray:
        prompt = _i32(prompt)
        out = np.zeros(N, dtype=np.int32)
        got = self.L.oracle_greedy_ar(self.h, prompt.ctypes.data, len(prompt), N, eos, out.ctypes.data)
        assert got >= 0, got
        return out[:got]

    def jacobi_generate(self, prompt, buf_init, W: int, N: int, max_steps: int = 0, eos: int = -1):
        """Returns dict(ids, steps, K, tail, buf)."""
        prompt = _i32(prompt)
        buf = _i32(buf_init).copy()
        out = np.zeros(max(N, 1), dtype=np.int32)
        olen, osteps = ctypes.c_int32(0), ctypes.c_int32(0)
        Ks = np.full(max(N, 1), -1, dtype=np.int32)
        tail = np.zeros(max(W - 1, 1), dtype=np.int32)
        rc = self.L.oracle_jacobi_generate(self.h, prompt.ctypes.data, len(prompt), buf.ctypes.data, len(buf), W, N,
                                           max_steps, eos, out.ctypes.data, ctypes.addressof(olen),
                                           ctypes.addressof(osteps), Ks.ctypes.data, len(Ks), tail.ctypes.data)
        assert rc == 0, rc
        return dict(ids=out[:olen.value], steps=osteps.value, K=Ks[:osteps.value], tail=tail[:W - 1], buf=buf)


class Session:
    def __init__(self, model: Model, max_seq: int):
        self.m = model
        self.L = model.L
        self.max_seq = max_seq
        self.h = self.L.oracle_session_new(model.h, max_seq)
        assert self.h, "oracle session allocation failed"

    def __del__(self):
        try:
            self.L.oracle_session_free(self.h)
        except Exception:
            pass

    @property
    def n(self) -> int:
        return self.L.oracle_session_len(self.h)

    @n.setter
    def n(self, v: int) -> None:
        assert self.L.oracle_session_set_len(self.h, v) == 0

    def forward(self, tokens, pos0: int, want_logits: bool = True, want_hidden: bool = False):
        """Rows at positions pos0.. ; returns (logits [R,V] float64 or None, argmax [R], hidden or None)."""
        tok = _i32(tokens)
        R = len(tok)
        V, d = self.m.fields["vocab"], self.m.fields["d_model"]
        logits = np.empty((R, V), dtype=np.float64) if want_logits else None
        hidden = np.empty((R, d), dtype=np.float64) if want_hidden else None
        amax = np.empty(R, dtype=np.int32)
        rc = self.L.oracle_forward(self.h, tok.ctypes.data, R, pos0,
                                   logits.ctypes.data if want_logits else None, amax.ctypes.data,
                                   hidden.ctypes.data if want_hidden else None)
        assert rc == 0, rc
        return logits, amax, hidden


def forward_streamed(shape_fields: dict, wdtype: int, global_weights: dict, layer_weights, sequences, max_seq: int,
                     real: str = "f64", progress=None):
    """The forward of Session.forward for models whose weights do not fit the host: one layer's weights at a time.

    global_weights: dict with 'emb', 'wlm' (and optionally 'gf').  layer_weights(l) -> dict name -> array for
    'wq','wk','wv','wo','wg','wu','wd' (optionally 'g1','g2') of layer l; it is called once per layer and the
    arrays are dropped afterwards.  sequences: list (one entry per sequence) of lists of passes
    (tokens, pos0, want_logits); the passes of a sequence run in order on one K/V cache, exactly as successive
    Session.forward calls would (a layer's K/V depends on no other layer's, so running all passes of a sequence
    through layer l before layer l+1 computes the same values).  Returns, per sequence and pass,
    (logits [R, V] float64 or None, argmax [R] or None).  Built from oracle_embed / oracle_layers /
    oracle_head, the bodies oracle_forward itself is made of."""
    L = lib(real)
    f0 = dict(shape_fields, n_layers=0)
    g = {k: v for k, v in global_weights.items() if k in ("emb", "wlm", "gf")}
    m0 = Model(f0, g, wdtype=wdtype, real=real)
    d, V = shape_fields["d_model"], shape_fields["vocab"]
    xs = []
    for passes in sequences:
        row = []
        for tok, pos0, _ in passes:
            tok = _i32(tok)
            x = np.empty((len(tok), d), dtype=np.float64)
            assert L.oracle_embed(m0.h, tok.ctypes.data, len(tok), x.ctypes.data) == 0
            row.append(x)
        xs.append(row)
    f1 = dict(shape_fields, n_layers=1)
    for l in range(shape_fields["n_layers"]):
        w = layer_weights(l)
        m1 = Model(f1, {k: [v] for k, v in w.items()}, wdtype=wdtype, real=real)
        for si, passes in enumerate(sequences):
            ss = m1.session(max_seq)
            for pi, (tok, pos0, _) in enumerate(passes):
                x = xs[si][pi]
                assert L.oracle_layers(ss.h, 0, 1, x.shape[0], int(pos0), x.ctypes.data) == 0
            del ss
        del m1, w
        if progress:
            progress(l)
    out = []
    for si, passes in enumerate(sequences):
        row = []
        for pi, (tok, pos0, want) in enumerate(passes):
            if not want:
                row.append((None, None))
                continue
            x = xs[si][pi]
            R = x.shape[0]
            logits = np.empty((R, V), dtype=np.float64)
            amax = np.empty(R, dtype=np.int32)
            assert L.oracle_head(m0.h, x.ctypes.data, R, logits.ctypes.data, amax.ctypes.data) == 0
            row.append((logits, amax))
        out.append(row)
    return out


def verify(w, o, real: str = "f64") -> int:
    w, o = _i32(w), _i32(o)
    return lib(real).oracle_verify(w.ctypes.data, o.ctypes.data, len(w))


def attention_window(q, k, v, n: int, real: str = "f64") -> np.ndarray:
    """q [R,H,Dh]; k, v [n+R,Hkv,Dh] -> out [R,H*Dh] (float64)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    R, H, Dh = q.shape
    Hkv = k.shape[1]
    assert k.shape[0] == n + R and v.shape == k.shape
    out = np.empty((R, H * Dh), dtype=np.float64)
    lib(real).oracle_attention_window(q.ctypes.data, k.ctypes.data, v.ctypes.data, n, R, H, Hkv, Dh, out.ctypes.data)
    return out


def lmhead_argmax(act, W, wdtype: int = 0, real: str = "f64", want_logits: bool = True):
    act = np.ascontiguousarray(act, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.uint16 if wdtype == 1 else np.float32)
    M, d = act.shape
    V = W.shape[1]
    logits = np.empty((M, V), dtype=np.float64) if want_logits else None
    amax = np.empty(M, dtype=np.int32)
    lib(real).oracle_lmhead_argmax(act.ctypes.data, W.ctypes.data, wdtype, M, d, V,
                                   logits.ctypes.data if want_logits else None, amax.ctypes.data)
    return logits, amax


def rmsnorm(x, g, eps: float, real: str = "f64") -> np.ndarray:
    dt = np.float64 if real == "f64" else np.float32
    x = np.ascontiguousarray(x, dtype=dt)
    out = np.empty_like(x)
    gp = None if g is None else np.ascontiguousarray(g, dtype=np.float32)
    lib(real).oracle_rmsnorm(x.ctypes.data, None if gp is None else gp.ctypes.data, len(x), eps, out.ctypes.data)
    return out


def rope(v, pos: int, base: float, real: str = "f64") -> np.ndarray:
    dt = np.float64 if real == "f64" else np.float32
    out = np.ascontiguousarray(v, dtype=dt).copy()
    lib(real).oracle_rope(out.ctypes.data, len(out), pos, base)
    return out


def model_from_synth(shape, seed=None, real: str = "f64", bf16_storage: bool = False) -> Model:
    """Oracle model over the synthetic weights of ``synthgen`` (the shared input recipe).

    ``shape`` is a synthgen.ModelShape.  With bf16_storage the weights are held as bf16 bit
    patterns (half the host memory of fp32; the values are identical).
    """
    import synthgen
    seed = synthgen.WEIGHT_SEED if seed is None else seed
    weights = {}
    for spec in synthgen.weight_tensors(shape):
        arr = synthgen.weight_array(shape, spec, seed, as_bf16_bits=bf16_storage)
        if spec.layer < 0:
            weights[spec.name] = arr
        else:
            weights.setdefault(spec.name, []).append(arr)
    fields = dict(n_layers=shape.n_layers, d_model=shape.d_model, n_heads=shape.n_heads,
                  n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab,
                  rms_eps=shape.rms_eps, rope_base=shape.rope_base)
    return Model(fields, weights, wdtype=1 if bf16_storage else 0, real=real)
