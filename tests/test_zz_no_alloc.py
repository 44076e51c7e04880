"""The bf16 decode entry point that allocates nothing (its split partials live in a device array built into the
library) against the entry point that takes a caller workspace: same kernels, same split, so the two must agree bit
for bit.  Two calls in a row, the second on a smaller input, so that stale partials of the first call would show."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def b():
    from paper_2605_08317_amd import binding
    return binding


def _inputs(seq_lens, hq, hkv, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    n = sum(seq_lens) * hkv * 128
    K = torch.randn(n, generator=g).to(torch.bfloat16).cuda()
    V = torch.randn(n, generator=g).to(torch.bfloat16).cuda()
    q = torch.randn((len(seq_lens), hq, 128), generator=g).to(torch.bfloat16).cuda()
    return K, V, q


def _both(b, seq_lens, hq, hkv, seed):
    K, V, q = _inputs(seq_lens, hq, hkv, seed)
    ref_out, ref_lse = b.rdkv_decode_attn_bf16(K, V, seq_lens, hq, hkv, q)
    out = torch.full((len(seq_lens), hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((len(seq_lens), hq), float("nan"), dtype=torch.float32, device="cuda")
    b.rdkv_decode_attn_bf16_noalloc(K, V, seq_lens, hq, hkv, q, out, lse)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out), f"outputs differ for seq_lens={seq_lens}"
    assert torch.equal(lse, ref_lse), f"lse differs for seq_lens={seq_lens}"
    return out


def test_noalloc_bf16_decode_matches_the_workspace_entry_point(b):
    print("case: large then small, hq=32 hkv=8", flush=True)
    _both(b, [20000, 777, 4096], 32, 8, seed=1)      # many splits, ragged
    _both(b, [300], 32, 8, seed=2)                   # a smaller input right after: one split per head
    _both(b, [5000, 64], 16, 2, seed=3)              # another head grouping (g = 8) on the same array
    # the library's own bound is enforced before anything is launched
    assert b.lib.rdkv_decode_bf16_noalloc_max_bytes() == 8 << 20


def test_noalloc_rejects_a_batch_beyond_the_scratch_area(b):
    # one long sequence among 63 one-token ones: every (sequence, head) gets the long one's split count
    seq_lens = [1 << 20] + [1] * 63
    need = b.rdkv_decode_bf16_workspace_bytes(seq_lens, 64, 8)
    assert need > b.lib.rdkv_decode_bf16_noalloc_max_bytes()
    arr = (ctypes.c_int32 * len(seq_lens))(*seq_lens)
    one = ctypes.c_void_p(256)   # never dereferenced: the size check comes first
    st = b.lib.rdkv_decode_attn_bf16_noalloc(one, one, arr, len(seq_lens), 64, 8, 128, one, one, None, None)
    assert st == 3 and "scratch" in b.lib.rdkv_last_error().decode()
