"""GPU parity of the appended-token zone (Zone C of Sec. 3.3, third term of Eq. 7): tokens appended after the
compression pass are attended to together with the compressed rows; outputs within 2e-3 of the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from test_gpu_parity import B, _np, _split, _check_decode, _inputs, _pack_both
from test_gpu_mixed import _pack_both_mixed, _random_maps

pytestmark = pytest.mark.gpu


def _new_tokens(rng, n, batch, hkv):
    k = torch.from_numpy(rng.standard_normal((n, batch, hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    v = torch.from_numpy(rng.standard_normal((n, batch, hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    return k, v


def _append_and_check(b, cache, ref, inp, dev, n_new, check_at, hkv, seed):
    rng = np.random.default_rng(seed)
    batch = len(inp["seq_lens"])
    kn, vn = _new_tokens(rng, n_new, batch, hkv)
    kd, vd = kn.cuda(), vn.cuda()
    b.rdkv_cache_reserve_tail(cache, n_new)
    for i in range(n_new):
        b.rdkv_cache_append(cache, kd[i], vd[i])
        O.append_tokens(ref, kn[i].float().numpy(), vn[i].float().numpy())
        if i + 1 in check_at:
            assert b.rdkv_cache_tail_len(cache) == i + 1
            print(f"[step] decode after {i + 1} appended tokens", flush=True)
            out, lse = b.rdkv_decode_attn(cache, dev["q"])
            torch.cuda.synchronize()
            ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
            _check_decode(out, lse, ref_out, ref_lse)
    with pytest.raises(RuntimeError):                       # the tail is full
        b.rdkv_cache_append(cache, kd[0], vd[0])
    with pytest.raises(RuntimeError):                       # reserved once
        b.rdkv_cache_reserve_tail(cache, 8)


@pytest.mark.parametrize("name,kw,n_new,check_at", [
    ("tiny", {"seq_lens": (900,)}, 5, (1, 5)),
    ("tiny", {"seq_lens": (700,)}, 300, (255, 256, 257, 300)),          # crosses a 256-token chunk of the tail
    ("batch70b", {"batch": 3, "len_range": (100, 700)}, 40, (1, 40)),     # ragged batch, 8 query heads per KV head
])
def test_append_tokenwise(name, kw, n_new, check_at):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    rng = np.random.default_rng(21)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.4, .25, .2, .1, .05])
            for T in inp["seq_lens"]]
    bits[0][0, :] = 0                                       # one head keeps nothing of the prompt: only the tail is left
    cache, ref = _pack_both(b, wl, inp, dev, bits)
    _append_and_check(b, cache, ref, inp, dev, n_new, check_at, wl.hkv, 22)
    cache.free()


def test_append_mixed():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1100,))
    bt, bc = _random_maps(np.random.default_rng(9), inp["seq_lens"], wl.hkv, [.4, .3, .2, .05, .05], [.1, .4, .3, .15, .05])
    cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    _append_and_check(b, cache, ref, inp, dev, 70, (1, 33, 70), wl.hkv, 23)
    cache.free()


def test_append_needs_a_reserved_tail():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(300,))
    bits = [np.full((wl.hkv, 300), 4, np.uint8)]
    cache, _ = _pack_both(b, wl, inp, dev, bits)
    k = torch.zeros((1, wl.hkv, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RuntimeError):
        b.rdkv_cache_append(cache, k, k)
    with pytest.raises(RuntimeError):
        b.rdkv_cache_reserve_tail(cache, 0)
    assert b.rdkv_cache_tail_len(cache) == 0
    cache.free()
