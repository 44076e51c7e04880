"""The config's device-allocator hooks (a framework's caching allocator behind the library): the pass, the appended
zone and re-budgeting must give the same bytes and the same outputs as with the default allocator, and everything the
library took through the hooks must come back through them."""
import ctypes

import numpy as np
import pytest
import torch

from test_gpu_parity import B, _inputs

pytestmark = pytest.mark.gpu


def test_allocator_hooks_round_trip():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1500,))
    live = {}

    @b._ALLOC_FN
    def alloc(nbytes, user):
        p = torch.cuda.caching_allocator_alloc(nbytes)
        live[p] = nbytes
        return p

    @b._FREE_FN
    def free(ptr, user):
        assert ptr in live, "the library released memory it did not take through the hook"
        del live[ptr]
        torch.cuda.caching_allocator_delete(ptr)

    outs = []
    for kw in ({}, {"alloc": alloc, "free_": free}):
        cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs, **kw)
        cache = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
        arena = cache.export(b.RDKV_EXPORT_ARENA, np.uint8).copy()
        b.rdkv_cache_reserve_tail(cache, 96)
        rng = torch.Generator(device="cpu").manual_seed(5)
        kn = torch.randn((64, 1, wl.hkv, 128), generator=rng).to(torch.bfloat16).cuda()
        for i in range(64):
            b.rdkv_cache_append(cache, kn[i], kn[(i + 1) % 64])
        Q = torch.randn((1, wl.hq, 16, 128), generator=rng).to(torch.bfloat16).cuda()
        b.rdkv_cache_rebudget_tail(cache, b.Config([64], wl.hq, wl.hkv, budget_bits=[3.0], s_obs=16, **kw), Q)
        out, lse = b.rdkv_decode_attn(cache, dev["q"])
        torch.cuda.synchronize()
        outs.append((arena, out.cpu(), lse.cpu()))
        assert not kw or len(live) > 0          # the cache lives in hook memory
        cache.free()
        assert len(live) == 0                   # temporaries and the cache's buffers all came back
    assert np.array_equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])
