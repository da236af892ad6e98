"""ctypes binding of the C ABI in include/fastcot.h.

Argument marshalling only: every step of the decoding path runs in the library's
HIP kernels.  PyTorch is used to own device memory and the stream.  There is no CPU
fallback: without the built library, or without a GPU, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import build as _build

_lib = None
vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
N_KINDS = 16

T = {"emb": 0, "wlm": 1, "gf": 2, "wq": 3, "wk": 4, "wv": 5, "wo": 6, "wg": 7, "wu": 8, "wd": 9, "g1": 10, "g2": 11}
OPT_PLAIN_KERNELS, OPT_GRAPH, OPT_KV_PLANES, OPT_COMPACT, OPT_AUTOTUNE, OPT_DEBUG_STAGES, OPT_KV_EMULATE, OPT_ACT_EMULATE, OPT_PACKED_ROWS = 1, 2, 3, 4, 5, 6, 7, 8, 9
PLAN_NW, PLAN_KS, PLAN_SB, PLAN_ROT, PLAN_CO_SINGLE, PLAN_ATTN_SPLITS, PLAN_ATTN_BLOCKS, PLAN_ATTN_MANY_ROWS = 100, 105, 110, 115, 120, 121, 122, 123
_STATUS = {0: "OK", -1: "EINVAL", -2: "ESTATE", -3: "ECAPACITY", -4: "EHIP", -5: "ENOMEM"}


def status_name(rc: int) -> str:
    return _STATUS.get(rc, str(rc))


class FastcotError(RuntimeError):
    def __init__(self, rc: int, msg: str):
        super().__init__(f"{status_name(rc)}: {msg}")
        self.rc = rc


class Config(ctypes.Structure):
    _fields_ = [(n, i32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", f32), ("rope_base", f32)] + \
               [(n, i32) for n in ("dtype", "max_batch", "max_seq", "window")]

    @classmethod
    def from_shape(cls, s, max_batch: int, max_seq: int, window: int) -> "Config":
        return cls(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, s.rms_eps,
                   s.rope_base, 0 if s.dtype == "f32" else 1, max_batch, max_seq, window)


SYMBOLS = {
    "fastcot_weight_bytes": (sz, [ctypes.POINTER(Config)]),
    "fastcot_workspace_bytes": (sz, [ctypes.POINTER(Config)]),
    "fastcot_pack_tensor": (ctypes.c_int, [ctypes.POINTER(Config), i32, i32, vp, vp, vp]),
    "fastcot_init": (ctypes.c_int, [ctypes.POINTER(Config), vp, vp, sz, vp, ctypes.POINTER(vp)]),
    "fastcot_free": (None, [vp]),
    "fastcot_last_error": (ctypes.c_char_p, [vp]),
    "fastcot_prefill": (ctypes.c_int, [vp, i32, vp, i32, vp, vp, i32]),
    "fastcot_jacobi_step": (ctypes.c_int, [vp, vp, vp, vp]),
    "fastcot_generate": (ctypes.c_int, [vp, i32, i32, i32, vp, vp, vp, vp]),
    "fastcot_get_state": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp]),
    "fastcot_debug_logits": (ctypes.c_int, [vp, vp]),
    "fastcot_step_rows": (ctypes.c_int, [vp, vp]),
    "fastcot_set_option": (ctypes.c_int, [vp, i32, i32]),
    "fastcot_debug_read": (ctypes.c_int, [vp, i32, vp, sz]),
    "fastcot_step_times": (ctypes.c_int, [vp, vp, i32, vp]),
    "fastcot_profile_step": (ctypes.c_int, [vp, i32, vp, vp]),
    "fastcot_kernel_name": (ctypes.c_char_p, [i32]),
    "fastcot_attn_scratch_bytes": (sz, [i32, i32, i32]),
    "fastcot_set_window": (ctypes.c_int, [vp, i32]),
    "fastcot_join": (ctypes.c_int, [vp, i32, vp, i32, vp]),
    "fastcot_set_windows": (ctypes.c_int, [vp, vp]),
    "fastcot_answer": (ctypes.c_int, [vp, vp, i32, i32, i32, vp, vp]),
    "fastcot_stream_read": (ctypes.c_int, [vp, ctypes.c_size_t, vp, vp]),
    "fastcot_stream_read_chain": (ctypes.c_int, [vp, ctypes.c_size_t, vp, i32, vp, vp]),
    "fastcot_kv_scatter": (ctypes.c_int, [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp]),
    "fastcot_attn_window": (ctypes.c_int, [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]),
    "fastcot_attn_window_noalloc": (ctypes.c_int, [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]),
    "fastcot_lmhead_packed_bytes": (sz, [i32, i32]),
    "fastcot_lmhead_scratch_bytes": (sz, [i32, i32, i32]),
    "fastcot_lmhead_pack": (ctypes.c_int, [vp, i32, i32, vp, vp]),
    "fastcot_lmhead_argmax": (ctypes.c_int, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]),
    "fastcot_canonical_bytes": (sz, [ctypes.POINTER(Config)]),
    "fastcot_canonical_offset": (sz, [ctypes.POINTER(Config), i32, i32]),
    "fastcot_pack_weights": (ctypes.c_int, [ctypes.POINTER(Config), vp, vp, vp]),
}


def lib():
    """Loads libfastcot.so, building it first only if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.SO):
            _build.build()
        # PyTorch ships its own HIP runtime; load it first so that the library binds to the same
        # one (two runtimes in a process do not see each other's device state)
        import torch  # noqa: F401
        L = ctypes.CDLL(_build.SO)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(L, name)      # AttributeError = the library does not export the symbol
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


KERNEL_KINDS = None


def kernel_kinds():
    global KERNEL_KINDS
    if KERNEL_KINDS is None:
        KERNEL_KINDS = [lib().fastcot_kernel_name(k).decode() for k in range(N_KINDS)]
    return KERNEL_KINDS


def _check(rc: int, ctx=None) -> None:
    if rc != 0:
        raise FastcotError(rc, (lib().fastcot_last_error(ctx) or b"").decode())


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("the FastCoT library needs a GPU (no CPU fallback exists)")
    return torch


def _stream_ptr() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _i32arr(a):
    return np.ascontiguousarray(a, dtype=np.int32)


# ---------------------------------------------------------------------------- weights
def pack_weights(cfg: Config, tensors, gains=None):
    """tensors: iterable of (name, layer, host ndarray in canonical layout); returns the packed
    device buffer (torch uint8).  Each tensor is staged through one device buffer and rearranged
    by the library's pack kernel.  gains: optional dict name -> array / list of arrays."""
    torch = _torch()
    L = lib()
    nbytes = L.fastcot_weight_bytes(ctypes.byref(cfg))
    if nbytes == 0:
        raise FastcotError(-1, "invalid configuration")
    packed = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    st = _stream_ptr()
    for name, layer, arr in tensors:
        t = torch.from_numpy(np.ascontiguousarray(arr)).to("cuda", non_blocking=False)
        _check(L.fastcot_pack_tensor(ctypes.byref(cfg), T[name], layer, t.data_ptr(), packed.data_ptr(), st))
        torch.cuda.current_stream().synchronize()
        del t
    gains = gains or {}
    for name in ("gf", "g1", "g2"):
        layers = [-1] if name == "gf" else range(cfg.n_layers)
        for l in layers:
            g = gains.get(name)
            if g is not None and name != "gf":
                g = g[l]
            if g is None:
                _check(L.fastcot_pack_tensor(ctypes.byref(cfg), T[name], l, None, packed.data_ptr(), st))
            else:
                t = torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).to("cuda")
                _check(L.fastcot_pack_tensor(ctypes.byref(cfg), T[name], l, t.data_ptr(), packed.data_ptr(), st))
                torch.cuda.current_stream().synchronize()
    torch.cuda.current_stream().synchronize()
    return packed


def load_synth_weights(cfg: Config, shape, seed: Optional[int] = None):
    """Packed device weights of the synthetic random-init model (the shared input recipe)."""
    import synthgen
    seed = synthgen.WEIGHT_SEED if seed is None else seed

    def gen():
        for spec in synthgen.weight_tensors(shape):
            yield spec.name, spec.layer, synthgen.weight_array(shape, spec, seed, as_bf16_bits=(shape.dtype == "bf16"))
    return pack_weights(cfg, gen())


# ---------------------------------------------------------------------------- context
class Context:
    def __init__(self, cfg: Config, packed):
        torch = _torch()
        self.cfg = cfg
        self.packed = packed
        L = lib()
        wbytes = L.fastcot_workspace_bytes(ctypes.byref(cfg))
        if wbytes == 0:
            raise FastcotError(-1, "invalid configuration")
        self.workspace = torch.empty(wbytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()                     # packing ran on torch's current stream
        self.stream = torch.cuda.Stream()            # a capturable stream of its own, default priority
        self.h = vp()
        _check(L.fastcot_init(ctypes.byref(cfg), packed.data_ptr(), self.workspace.data_ptr(), wbytes,
                              self.stream.cuda_stream, ctypes.byref(self.h)))
        self.B = 0
        self._dbg = None

    def close(self):
        if getattr(self, "h", None):
            lib().fastcot_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, option: int, value: int) -> None:
        _check(lib().fastcot_set_option(self.h, option, value), self.h)

    def prefill(self, prompts, lens, buffer_init) -> None:
        prompts, lens, buffer_init = _i32arr(prompts), _i32arr(lens), _i32arr(buffer_init)
        B, max_P = prompts.shape
        assert buffer_init.shape[0] == B and lens.shape == (B,)
        _check(lib().fastcot_prefill(self.h, B, prompts.ctypes.data, max_P, lens.ctypes.data, buffer_init.ctypes.data,
                                     buffer_init.shape[1]), self.h)
        self.B = B

    def step(self, sync: bool = True):
        W = self.cfg.window
        if not sync:
            _check(lib().fastcot_jacobi_step(self.h, None, None, None), self.h)
            return None
        nacc = np.zeros(self.B, dtype=np.int32)
        acc = np.zeros((self.B, W), dtype=np.int32)
        win = np.zeros((self.B, W), dtype=np.int32)
        _check(lib().fastcot_jacobi_step(self.h, nacc.ctypes.data, acc.ctypes.data, win.ctypes.data), self.h)
        return nacc, acc, win

    def generate(self, max_new_tokens: int, max_steps: int = 0, eos_id: int = -1):
        W = self.cfg.window
        ids = np.zeros((self.B, max_new_tokens), dtype=np.int32)
        olen = np.zeros(self.B, dtype=np.int32)
        steps = np.zeros(self.B, dtype=np.int32)
        tail = np.zeros((self.B, max(W - 1, 1)), dtype=np.int32)
        _check(lib().fastcot_generate(self.h, max_new_tokens, max_steps, eos_id, ids.ctypes.data, olen.ctypes.data,
                                      steps.ctypes.data, tail.ctypes.data), self.h)
        return dict(ids=ids, len=olen, steps=steps, tail=tail[:, :W - 1])

    def set_window(self, window: int) -> None:
        """Window size of the following steps (between step() calls only)."""
        _check(lib().fastcot_set_window(self.h, window), self.h)
        self.cfg.window = window

    def set_windows(self, windows) -> None:
        """Per-sequence window sizes (each at most the batch window) from the next step on."""
        w = _i32arr(windows).reshape(-1)
        assert w.size == self.B
        _check(lib().fastcot_set_windows(self.h, w.ctypes.data), self.h)

    def join(self, slot: int, prompt, buffer_init) -> None:
        """A new prompt takes over one slot of the running batch (between step() calls only)."""
        prompt, buffer_init = _i32arr(prompt).reshape(-1), _i32arr(buffer_init).reshape(-1)
        _check(lib().fastcot_join(self.h, slot, prompt.ctypes.data, int(prompt.size), buffer_init.ctypes.data), self.h)

    def answer(self, trigger_ids, max_new_tokens: int, eos_id: int = -1):
        """Answer phase after generate(): glimpse + trigger enter the cache, then greedy decoding."""
        trig = _i32arr(trigger_ids).reshape(-1)
        ids = np.zeros((self.B, max_new_tokens), dtype=np.int32)
        olen = np.zeros(self.B, dtype=np.int32)
        _check(lib().fastcot_answer(self.h, trig.ctypes.data if trig.size else None, int(trig.size), max_new_tokens, eos_id,
                                    ids.ctypes.data, olen.ctypes.data), self.h)
        return dict(ids=ids, len=olen)

    def state(self):
        W = self.cfg.window
        n, g, done, K = (np.zeros(self.B, dtype=np.int32) for _ in range(4))
        win = np.zeros((self.B, W), dtype=np.int32)
        o = np.zeros((self.B, W), dtype=np.int32)
        _check(lib().fastcot_get_state(self.h, n.ctypes.data, g.ctypes.data, done.ctypes.data, win.ctypes.data,
                                       o.ctypes.data, K.ctypes.data), self.h)
        return dict(n=n, g=g, done=done, window=win, o=o, K=K)

    def step_rows(self) -> np.ndarray:
        """Row layout of the next step: rows of sequence b are out[b] .. out[b + 1] - 1 (out[B] = rows computed)."""
        out = np.zeros(self.B + 1, dtype=np.int32)
        _check(lib().fastcot_step_rows(self.h, out.ctypes.data), self.h)
        return out

    def debug_logits(self, on: bool = True):
        """Returns the device tensor [max_batch*W, vocab] the following steps fill (or None)."""
        torch = _torch()
        if on:
            self._dbg = torch.zeros(self.cfg.max_batch * self.cfg.window, self.cfg.vocab, dtype=torch.float32, device="cuda")
            _check(lib().fastcot_debug_logits(self.h, self._dbg.data_ptr()), self.h)
        else:
            _check(lib().fastcot_debug_logits(self.h, None), self.h)
            self._dbg = None
        return self._dbg

    def debug_read(self, what: int, rows: int, cols: int) -> np.ndarray:
        out = np.zeros((rows, cols), dtype=np.float32)
        _check(lib().fastcot_debug_read(self.h, what, out.ctypes.data, out.size), self.h)
        return out

    def step_times(self) -> np.ndarray:
        n = i32(0)
        _check(lib().fastcot_step_times(self.h, None, 0, ctypes.byref(n)), self.h)
        ms = np.zeros(max(n.value, 1), dtype=np.float32)
        _check(lib().fastcot_step_times(self.h, ms.ctypes.data, n.value, ctypes.byref(n)), self.h)
        return ms[:n.value]

    def profile_step(self, iters: int = 3):
        ms = np.zeros(N_KINDS, dtype=np.float32)
        cnt = np.zeros(N_KINDS, dtype=np.int32)
        _check(lib().fastcot_profile_step(self.h, iters, ms.ctypes.data, cnt.ctypes.data), self.h)
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(kernel_kinds()) if cnt[i]}


# ---------------------------------------------------------------------------- kernel isolation
def kv_scatter(k, v, max_seq: int):
    """k, v: device tensors [S, Hkv, Dh] (bf16 or fp32) -> (k_cache, vt_cache), each [Hkv, max_seq/32, 32*Dh] in the
    library's blocked fragment order; max_seq and Dh must be multiples of 32."""
    torch = _torch()
    S, Hkv, Dh = k.shape
    dt = 0 if k.dtype == torch.float32 else 1
    kc = torch.zeros(Hkv, max_seq // 32, 32 * Dh, dtype=k.dtype, device="cuda")
    if max_seq % 32:
        raise ValueError("max_seq must be a multiple of 32")
    vc = torch.zeros(Hkv, max_seq // 32, 32 * Dh, dtype=k.dtype, device="cuda")
    _check(lib().fastcot_kv_scatter(k.data_ptr(), v.data_ptr(), S, Hkv, Dh, max_seq, dt, kc.data_ptr(), vc.data_ptr(),
                                    _stream_ptr()))
    return kc, vc


def attn_window(q, kc, vc, n: int, scratch=None):
    """q: device fp32 [W,H,Dh]; kc/vc from kv_scatter; returns out fp32 [W, H*Dh]."""
    torch = _torch()
    W, H, Dh = q.shape
    Hkv, max_seq = kc.shape[0], kc.shape[1] * 32
    dt = 0 if kc.dtype == torch.float32 else 1
    if scratch is None:
        scratch = torch.zeros(lib().fastcot_attn_scratch_bytes(W, H, Dh), dtype=torch.uint8, device="cuda")
    out = torch.empty(W, H * Dh, dtype=torch.float32, device="cuda")
    _check(lib().fastcot_attn_window(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), n, W, H, Hkv, Dh, max_seq, dt,
                                     out.data_ptr(), scratch.data_ptr(), _stream_ptr()))
    return out


def attn_window_noalloc(q, kc, vc, n: int, out=None):
    """attn_window through the entry point that allocates nothing (scratch built into the library); `out` may be
    a preallocated fp32 [W, H*Dh] device tensor."""
    torch = _torch()
    W, H, Dh = q.shape
    Hkv, max_seq = kc.shape[0], kc.shape[1] * 32
    dt = 0 if kc.dtype == torch.float32 else 1
    if out is None:
        out = torch.empty(W, H * Dh, dtype=torch.float32, device="cuda")
    _check(lib().fastcot_attn_window_noalloc(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), n, W, H, Hkv, Dh, max_seq, dt,
                                             out.data_ptr(), _stream_ptr()))
    return out


def stream_read(buf, sink=None):
    """One plain streaming read over the device tensor `buf` on torch's current stream."""
    torch = _torch()
    if sink is None:
        sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    nbytes = (buf.numel() * buf.element_size()) // 16 * 16
    _check(lib().fastcot_stream_read(buf.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr()))
    return nbytes


def stream_read_chain(buf, launch_bytes, sink=None):
    """Back-to-back plain streaming reads of launch_bytes[i] bytes each over `buf` on torch's current stream."""
    torch = _torch()
    if sink is None:
        sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    lb = np.ascontiguousarray(launch_bytes, dtype=np.uint64)
    _check(lib().fastcot_stream_read_chain(buf.data_ptr(), buf.numel() * buf.element_size(), lb.ctypes.data, int(lb.size),
                                           sink.data_ptr(), _stream_ptr()))
    return int((lb // 1024 * 1024).sum())


def lmhead_pack(w_bf16):
    """w_bf16: device bf16 tensor [d, V] canonical -> packed device buffer."""
    torch = _torch()
    d, V = w_bf16.shape
    packed = torch.empty(lib().fastcot_lmhead_packed_bytes(d, V), dtype=torch.uint8, device="cuda")
    _check(lib().fastcot_lmhead_pack(w_bf16.data_ptr(), d, V, packed.data_ptr(), _stream_ptr()))
    return packed


def pack_weights_whole(cfg: Config, tensors, gains=None):
    """pack_weights through the one-call entry point: every tensor is first laid out in one canonical device
    buffer (so the model is on the device twice meanwhile), then fastcot_pack_weights rearranges them all."""
    torch = _torch()
    L = lib()
    nbytes, cbytes = L.fastcot_weight_bytes(ctypes.byref(cfg)), L.fastcot_canonical_bytes(ctypes.byref(cfg))
    if nbytes == 0 or cbytes == 0:
        raise FastcotError(-1, "invalid configuration")
    canon = torch.zeros(cbytes, dtype=torch.uint8, device="cuda")
    packed = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")

    def put(name, layer, arr):
        off = L.fastcot_canonical_offset(ctypes.byref(cfg), T[name], max(layer, 0))
        raw = torch.from_numpy(np.ascontiguousarray(arr).view(np.uint8).reshape(-1))
        canon[off:off + raw.numel()] = raw.to("cuda")
    for name, layer, arr in tensors:
        put(name, layer, arr)
    gains = gains or {}
    ones = np.ones(cfg.d_model, dtype=np.float32)
    for name in ("gf", "g1", "g2"):
        for l in ([-1] if name == "gf" else range(cfg.n_layers)):
            g = gains.get(name)
            if g is not None and name != "gf":
                g = g[l]
            put(name, l, np.asarray(ones if g is None else g, dtype=np.float32))
    _check(L.fastcot_pack_weights(ctypes.byref(cfg), canon.data_ptr(), packed.data_ptr(), _stream_ptr()))
    torch.cuda.current_stream().synchronize()
    return packed


def lmhead_argmax(act, packed, V: int, want_logits: bool = False, scratch=None, want_top2: bool = False):
    """act: device fp32 [M,d]; returns (ids int32 [M], top fp32 [M], logits or None) and, with want_top2, the
    runner-up logit of every row as a fourth entry."""
    torch = _torch()
    M, d = act.shape
    if scratch is None:
        scratch = torch.zeros(lib().fastcot_lmhead_scratch_bytes(M, d, V), dtype=torch.uint8, device="cuda")
    ids = torch.empty(M, dtype=torch.int32, device="cuda")
    top = torch.empty(M, dtype=torch.float32, device="cuda")
    logits = torch.empty(M, V, dtype=torch.float32, device="cuda") if want_logits else None
    top2 = torch.empty(M, dtype=torch.float32, device="cuda") if want_top2 else None
    _check(lib().fastcot_lmhead_argmax(act.data_ptr(), packed.data_ptr(), M, d, V, ids.data_ptr(), top.data_ptr(),
                                       top2.data_ptr() if want_top2 else None,
                                       logits.data_ptr() if want_logits else None, scratch.data_ptr(), _stream_ptr()))
    return (ids, top, logits, top2) if want_top2 else (ids, top, logits)
