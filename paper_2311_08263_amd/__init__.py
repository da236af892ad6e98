"""MI355X-native FastCoT Jacobi decoding step (thin ctypes binding over libfastcot.so)."""
from .binding import (Config, Context, FastcotError, KERNEL_KINDS, attn_window, attn_window_noalloc, kv_scatter, lib, lmhead_argmax,  # noqa: F401
                      lmhead_pack, load_synth_weights, pack_weights, pack_weights_whole, status_name, stream_read, stream_read_chain)
