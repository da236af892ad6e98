"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
sizes configurations, and rejects bad arguments before touching a GPU."""
import ctypes

import numpy as np
import os
import re

import synthgen
from paper_2311_08263_amd import binding


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(os.path.dirname(__file__), "..", "include", "fastcot.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fastcot_[a-z_0-9]+)\s*\(", hdr))
    assert declared, "no declarations found"
    L = ctypes.CDLL(binding._build.SO) if os.path.exists(binding._build.SO) else binding.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} is declared in fastcot.h but not exported"
    assert declared == set(binding.SYMBOLS), declared ^ set(binding.SYMBOLS)


def test_sizes_and_invalid_configs():
    L = binding.lib()
    s7 = synthgen.SHAPES["7b"]
    cfg = binding.Config.from_shape(s7, 1, 640, 16)
    wb = L.fastcot_weight_bytes(ctypes.byref(cfg))
    streamed = s7.n_params_streamed() * 2
    assert streamed < wb < streamed + s7.vocab * s7.d_model * 2 + (1 << 22)
    assert L.fastcot_workspace_bytes(ctypes.byref(cfg)) > 2 * 32 * 640 * 4096 * 2
    for field, bad in (("head_dim", 100), ("n_kv_heads", 5), ("dtype", 7), ("window", 0), ("max_seq", 10), ("vocab", 1001)):
        c = binding.Config.from_shape(s7, 1, 640, 16)
        setattr(c, field, bad)
        assert L.fastcot_weight_bytes(ctypes.byref(c)) == 0, field
        assert L.fastcot_workspace_bytes(ctypes.byref(c)) == 0, field


def test_null_arguments_are_rejected_without_a_gpu():
    L = binding.lib()
    assert L.fastcot_prefill(None, 1, None, 1, None, None, 1) == -1
    assert L.fastcot_jacobi_step(None, None, None, None) == -1
    assert L.fastcot_generate(None, 1, 0, -1, None, None, None, None) == -1
    assert L.fastcot_get_state(None, None, None, None, None, None, None) == -1
    one = np.ones(4, dtype=np.int32)
    assert L.fastcot_set_window(None, 4) == -1
    assert L.fastcot_set_windows(None, one.ctypes.data) == -1
    assert L.fastcot_step_rows(None, one.ctypes.data) == -1
    assert L.fastcot_join(None, 0, one.ctypes.data, 4, one.ctypes.data) == -1
    assert L.fastcot_answer(None, one.ctypes.data, 1, 4, -1, one.ctypes.data, one.ctypes.data) == -1
    assert b"NULL" in L.fastcot_last_error(None)
    cfg = binding.Config.from_shape(synthgen.SHAPES["tiny"], 1, 64, 4)
    out = ctypes.c_void_p()
    assert L.fastcot_init(ctypes.byref(cfg), None, None, 0, None, ctypes.byref(out)) == -1
    assert L.fastcot_pack_tensor(ctypes.byref(cfg), 99, 0, None, None, None) == -1
    assert L.fastcot_attn_window(None, None, None, 0, 1, 1, 1, 16, 16, 0, None, None, None) == -1
    assert L.fastcot_lmhead_argmax(None, None, 1, 32, 16, None, None, None, None, None, None) == -1
    assert L.fastcot_pack_weights(ctypes.byref(cfg), None, None, None) == -1
    assert L.fastcot_canonical_offset(ctypes.byref(cfg), 3, 99) == ctypes.c_size_t(-1).value
    assert L.fastcot_kernel_name(4) == b"attention"
