"""The attention entry point that allocates nothing (its scratch is an array built into the library) against the
ordinary entry point, which takes a caller-allocated scratch: two calls in a row, the second with a smaller
input, through the C ABI.  Both run the same kernel, so the outputs must be identical bit for bit; the first is
also held to the oracle."""
import numpy as np
import pytest

import oracle
import synthgen
from gpu_util import say

pytestmark = pytest.mark.gpu


def _case(fc, torch, n, W, H, Hkv, S, seed):
    Dh = 128
    q = synthgen.normal_f32((W, H, Dh), seed, 1, 1.0, False)
    kb = synthgen.normal_bf16((n + W, Hkv, Dh), seed, 2, 1.0)
    vb = synthgen.normal_bf16((n + W, Hkv, Dh), seed, 3, 1.0)
    kc, vc = fc.kv_scatter(torch.from_numpy(kb.view(np.int16)).cuda().view(torch.bfloat16),
                           torch.from_numpy(vb.view(np.int16)).cuda().view(torch.bfloat16), S)
    qd = torch.from_numpy(q).cuda()
    return q, kb, vb, qd, kc, vc


def test_attn_window_noalloc_matches_attn_window():
    import torch
    import paper_2311_08263_amd as fc
    S = 2080
    # every device buffer exists before the calls under test; the calls themselves allocate nothing
    big = _case(fc, torch, 2048, 16, 32, 32, S, 5)
    small = _case(fc, torch, 300, 7, 8, 2, S, 6)
    out_big = torch.empty(16, 32 * 128, dtype=torch.float32, device="cuda")
    out_small = torch.empty(7, 8 * 128, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    say("no-alloc attention: 2048 keys x 32 heads x 16 rows, then 300 keys x 8 heads (2 K/V heads) x 7 rows")
    allocs0 = torch.cuda.memory_stats()["allocation.all.allocated"]       # allocations made so far (never decreases)
    fc.attn_window_noalloc(big[3], big[4], big[5], 2048, out=out_big)
    fc.attn_window_noalloc(small[3], small[4], small[5], 300, out=out_small)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == allocs0
    ref_big = fc.attn_window(big[3], big[4], big[5], 2048)
    ref_small = fc.attn_window(small[3], small[4], small[5], 300)
    torch.cuda.synchronize()
    assert torch.equal(out_big, ref_big)
    assert torch.equal(out_small, ref_small)
    o = oracle.attention_window(big[0], synthgen.bf16_bits_to_f32(big[1]), synthgen.bf16_bits_to_f32(big[2]), 2048)
    assert np.abs(out_big.cpu().numpy() - o).max() < 1e-4
    o = oracle.attention_window(small[0], synthgen.bf16_bits_to_f32(small[1]), synthgen.bf16_bits_to_f32(small[2]), 300)
    assert np.abs(out_small.cpu().numpy() - o).max() < 1e-4


def test_attn_window_noalloc_rejects_sizes_beyond_its_array():
    import torch
    import paper_2311_08263_amd as fc
    q, kb, vb, qd, kc, vc = _case(fc, torch, 40, 4, 4, 4, 96, 7)
    L = fc.lib()
    out = torch.empty(32, 128 * 128, dtype=torch.float32, device="cuda")
    rc = L.fastcot_attn_window_noalloc(qd.data_ptr(), kc.data_ptr(), vc.data_ptr(), 40, 4, 128, 4, 128, 96, 1, out.data_ptr(), None)
    assert rc == -3 and b"64 heads" in L.fastcot_last_error(None)
    rc = L.fastcot_attn_window_noalloc(qd.data_ptr(), kc.data_ptr(), vc.data_ptr(), 40, 17, 4, 4, 128, 96, 1, out.data_ptr(), None)
    assert rc == -3
