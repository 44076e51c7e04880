"""GPU parity of the per-token format (one scale and offset per token row, App. B; config group_size = 128): packed
bytes bit for bit against the oracle, decode within 2e-3, the fused pass, the paper's own arrangement (V per token, K
one scale per channel), re-budgeting, and the calibration utility with row-wide groups."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from test_gpu_parity import B, _np, _split, _check_decode, _inputs
from test_gpu_mixed import _random_maps, _assert_cache_equal_mixed

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw", [
    ("tiny", {"seq_lens": (1000,)}),
    ("layer8b", {"seq_lens": (3000,)}),
    ("batch70b", {"batch": 3, "len_range": (200, 1500)}),
])
def test_row_wide_pack_is_bit_exact_and_decodes(name, kw):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    rng = np.random.default_rng(51)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.3, .25, .2, .15, .1])
            for T in inp["seq_lens"]]
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, group_size=128)
    cache = b.rdkv_pack(cfg, dev["K"], dev["V"], torch.from_numpy(np.concatenate([x.reshape(-1) for x in bits])).cuda())
    Ks, Vs = _split(inp["K"], inp["seq_lens"], wl.hkv, wl.d), _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d)
    ref = O.build_cache_tokenwise(Ks, Vs, bits, group=128)
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_SEG_OFF, np.int64).reshape(-1, 4, 4), ref["seg_off"])
    arena = cache.export(b.RDKV_EXPORT_ARENA, np.uint8)
    assert np.array_equal(arena, ref["arena"]), "packed bytes differ"
    assert not np.array_equal(arena, O.build_cache_tokenwise(Ks, Vs, bits)["arena"])      # not the 32-channel format
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    cache.free()


def test_row_wide_fused_pass_and_rebudget():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(2500,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs, group_size=128)
    cache = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
    w_tok, _ = b.rdkv_weights(cfg, dev["K"], dev["Q_obs"])
    torch.cuda.synchronize()
    Ks, Vs = _split(inp["K"], inp["seq_lens"], wl.hkv, wl.d), _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d)
    ref = O.compress_tokenwise(Ks, Vs, [_np(inp["Q_obs"][0])], [np.float32(inp["budgets"][0])],
                               weights_override=[w_tok.cpu().numpy().reshape(wl.hkv, -1)], group=128)
    assert np.array_equal(cache.export(b.RDKV_EXPORT_ARENA, np.uint8), ref["arena"])
    # appended tokens, then compressed in the same format; a config of the other format is refused
    n_new = 96
    rng = np.random.default_rng(52)
    kn = torch.from_numpy(rng.standard_normal((n_new, 1, wl.hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    vn = torch.from_numpy(rng.standard_normal((n_new, 1, wl.hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    b.rdkv_cache_reserve_tail(cache, n_new)
    for i in range(n_new):
        b.rdkv_cache_append(cache, kn[i].cuda(), vn[i].cuda())
        O.append_tokens(ref, kn[i].float().numpy(), vn[i].float().numpy())
    Q = torch.from_numpy(rng.standard_normal((1, wl.hq, 32, 128)).astype(np.float32)).to(torch.bfloat16)
    with pytest.raises(b.RdkvError):
        b.rdkv_cache_rebudget_tail(cache, b.Config([n_new], wl.hq, wl.hkv, budget_bits=[3.0], s_obs=32), Q.cuda())
    cfg_t = b.Config([n_new], wl.hq, wl.hkv, budget_bits=[3.0], s_obs=32, group_size=128)
    b.rdkv_cache_rebudget_tail(cache, cfg_t, Q.cuda())
    K_tail = kn[:, 0].transpose(0, 1).contiguous().cuda().reshape(-1)
    w_t, _ = b.rdkv_weights(cfg_t, K_tail, Q.cuda())
    torch.cuda.synchronize()
    child = O.rebudget_tail(ref, [_np(Q[0])], [np.float32(3.0)], weights_override=[w_t.cpu().numpy().reshape(wl.hkv, -1)],
                            group=128)
    gen = b.rdkv_cache_generation(cache, 0, cfg_t)
    assert np.array_equal(gen.export(b.RDKV_EXPORT_ARENA, np.uint8), child["arena"])
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    cache.free()


@pytest.mark.parametrize("name,kw", [("tiny", {"seq_lens": (900,)}), ("batch70b", {"batch": 2, "len_range": (300, 900)})])
def test_the_papers_own_format_v_per_token_k_per_channel(name, kw):
    """App. B as printed: V rows with one scale per token, K channels with one scale over all retained tokens."""
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    bt, bc = _random_maps(np.random.default_rng(53), inp["seq_lens"], wl.hkv, [.3, .3, .2, .1, .1], [.1, .4, .3, .15, .05])
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, k_mode=b.RDKV_K_CHANNELWISE, k_scale_per_channel=1, group_size=128)
    cache = b.rdkv_pack(cfg, dev["K"], dev["V"], torch.from_numpy(np.concatenate([x.reshape(-1) for x in bt])).cuda(),
                        torch.from_numpy(np.concatenate([x.reshape(-1) for x in bc])).cuda())
    Ks, Vs = _split(inp["K"], inp["seq_lens"], wl.hkv, wl.d), _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d)
    ref = O.build_cache_mixed(Ks, Vs, bt, bc, k_per_channel_scale=True, group=128)
    _assert_cache_equal_mixed(b, cache, ref)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    cache.free()


def test_calibration_with_one_scale_per_token_row():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1500,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, group_size=128)
    ek, ev = b.rdkv_calibrate_eps(cfg, dev["K"], dev["V"])
    Ks, Vs = _split(inp["K"], inp["seq_lens"], wl.hkv, wl.d), _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d)
    rk, rv = O.calibrate_eps(Ks, Vs, group=128)
    np.testing.assert_allclose(ek, rk, rtol=1e-10)
    np.testing.assert_allclose(ev, rv, rtol=1e-10)
    ek32, ev32 = b.rdkv_calibrate_eps(b.Config(inp["seq_lens"], wl.hq, wl.hkv), dev["K"], dev["V"])
    assert np.all(ev > ev32)
    print(f"[calibration] V per token row eps(2,4,8) = {ev.mean(axis=0)}; groups of 32: {ev32.mean(axis=0)}", flush=True)
