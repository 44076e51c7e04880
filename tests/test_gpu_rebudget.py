"""GPU parity of streaming re-budgeting (the extension sketched in App. "Limitations and Future Work"): appended tokens
are compressed by the same pass and join the cache as a further generation.  The absorbed generation must equal the
oracle's bit for bit (bit map, kept positions, packed bytes) when both allocate from the library's own fp32 weights;
decode over prompt zones, generations and the new tail within 2e-3 of the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from test_gpu_parity import B, _np, _check_decode, _inputs, _pack_both, _assert_cache_equal
from test_gpu_mixed import _pack_both_mixed, _random_maps, _assert_cache_equal_mixed

pytestmark = pytest.mark.gpu


def _append(b, cache, ref, rng, n_new, batch, hkv):
    """n_new tokens per sequence into both caches; returns their rows as [batch][hkv][n_new][128] bf16 tensors."""
    kn = torch.from_numpy(rng.standard_normal((n_new, batch, hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    vn = torch.from_numpy(rng.standard_normal((n_new, batch, hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    kn[:, :, :, 5] *= 8.0                                        # a heavy key channel
    kd, vd = kn.cuda(), vn.cuda()
    for i in range(n_new):
        b.rdkv_cache_append(cache, kd[i], vd[i])
        O.append_tokens(ref, kn[i].float().numpy(), vn[i].float().numpy())
    return kn.permute(1, 2, 0, 3).contiguous(), vn.permute(1, 2, 0, 3).contiguous()


def _rebudget_both(b, cache, ref, wl, batch, k_rows, n_tail, budgets, s_obs, rng, **cfg_kw):
    """Runs the library's and the oracle's re-budgeting on the same tail; the oracle allocates from the weights the
    library computes for the same rows.  Returns the oracle's child."""
    Q_obs = torch.from_numpy(rng.standard_normal((batch, wl.hq, s_obs, 128)).astype(np.float32)).to(torch.bfloat16)
    cfg = b.Config([n_tail] * batch, wl.hq, wl.hkv, budget_bits=budgets, s_obs=s_obs, **cfg_kw)
    print(f"[step] rebudget tail of {n_tail} tokens, budgets {budgets}", flush=True)
    b.rdkv_cache_rebudget_tail(cache, cfg, Q_obs.cuda())
    assert b.rdkv_cache_tail_len(cache) == 0
    w_tok, _ = b.rdkv_weights(cfg, k_rows.reshape(-1).cuda(), Q_obs.cuda())
    torch.cuda.synchronize()
    w_list = [w.cpu().numpy() for w in w_tok.view(batch, wl.hkv, n_tail)]
    kw = {}
    if "tiers" in cfg_kw:
        kw = {"tiers": tuple(cfg_kw["tiers"]), "eps": tuple(cfg_kw["eps_v"])}
    child = O.rebudget_tail(ref, [_np(Q_obs[s]) for s in range(batch)], [np.float32(x) for x in budgets],
                            weights_override=w_list, **kw)
    return child, cfg


@pytest.mark.parametrize("name,kw,n_new,budgets", [
    ("tiny", {"seq_lens": (900,)}, 200, [3.0]),
    ("tiny", {"seq_lens": (500,)}, 64, [16.0]),                  # everything kept verbatim
    ("tiny", {"seq_lens": (400,)}, 64, [0.0]),                   # nothing kept: an empty generation
    ("batch70b", {"batch": 3, "len_range": (100, 700)}, 300, [0.5, 2.0, 6.0]),   # 8 query heads per KV head
])
def test_rebudget_matches_oracle(name, kw, n_new, budgets):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    batch = len(inp["seq_lens"])
    rng = np.random.default_rng(91)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.4, .25, .2, .1, .05])
            for T in inp["seq_lens"]]
    cache, ref = _pack_both(b, wl, inp, dev, bits)
    b.rdkv_cache_reserve_tail(cache, 320)
    k_rows, _ = _append(b, cache, ref, rng, n_new, batch, wl.hkv)
    st0 = cache.stats()
    child, cfg = _rebudget_both(b, cache, ref, wl, batch, k_rows, n_new, budgets, 32, rng)
    # the absorbed generation, bit for bit
    assert b.rdkv_cache_generations(cache) == 1
    gen = b.rdkv_cache_generation(cache, 0, cfg)
    np.testing.assert_array_equal(gen.export(b.RDKV_EXPORT_BITS_TOK, np.uint8),
                                  np.concatenate([x.reshape(-1) for x in child["bits"]]))
    _assert_cache_equal(b, gen, child)
    st1 = cache.stats()
    assert st1["stored_bytes"] == st0["stored_bytes"] + O.stored_bytes(child["counts"])
    assert st1["rows"] == [a + c for a, c in zip(st0["rows"], child["counts"].sum(axis=0).tolist())]
    for s in range(batch):
        for h in range(wl.hkv):
            assert int(child["bits"][s][h].astype(np.int64).sum()) <= int(np.floor(np.float64(np.float32(budgets[s])) * n_new))
    # decode right after, then with new tokens in the emptied tail
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    _append(b, cache, ref, rng, 7, batch, wl.hkv)
    assert b.rdkv_cache_tail_len(cache) == 7
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    cache.free()


def test_rebudget_twice_and_prompt_fully_evicted():
    """Two generations on a cache whose first KV head kept nothing of the prompt."""
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(700,))
    rng = np.random.default_rng(92)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.4, .25, .2, .1, .05])
            for T in inp["seq_lens"]]
    bits[0][0, :] = 0
    cache, ref = _pack_both(b, wl, inp, dev, bits)
    b.rdkv_cache_reserve_tail(cache, 128)
    for gen_i, (n_new, budget) in enumerate(((128, 4.0), (40, 1.0))):
        k_rows, _ = _append(b, cache, ref, rng, n_new, 1, wl.hkv)
        child, cfg = _rebudget_both(b, cache, ref, wl, 1, k_rows, n_new, [budget], 16, rng)
        assert b.rdkv_cache_generations(cache) == gen_i + 1
        _assert_cache_equal(b, b.rdkv_cache_generation(cache, gen_i, cfg), child)
        out, lse = b.rdkv_decode_attn(cache, dev["q"])
        torch.cuda.synchronize()
        _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    _append(b, cache, ref, rng, 3, 1, wl.hkv)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    cache.free()


def test_rebudget_argument_errors():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(300,))
    rng = np.random.default_rng(93)
    bits = [np.full((wl.hkv, 300), 4, np.uint8)]
    cache, ref = _pack_both(b, wl, inp, dev, bits)
    Q = torch.zeros((1, wl.hq, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RuntimeError):                                        # nothing appended (no tail at all)
        b.rdkv_cache_rebudget_tail(cache, b.Config([8], wl.hq, wl.hkv, budget_bits=[2.0], s_obs=8), Q)
    b.rdkv_cache_reserve_tail(cache, 64)
    _append(b, cache, ref, rng, 10, 1, wl.hkv)
    with pytest.raises(RuntimeError):                                        # wrong tail length
        b.rdkv_cache_rebudget_tail(cache, b.Config([9], wl.hq, wl.hkv, budget_bits=[2.0], s_obs=8), Q)
    with pytest.raises(RuntimeError):                                        # other head counts than the cache
        b.rdkv_cache_rebudget_tail(cache, b.Config([10], wl.hq * 2, wl.hkv, budget_bits=[2.0], s_obs=8), Q)
    with pytest.raises(RuntimeError):                                        # window longer than the tail
        b.rdkv_cache_rebudget_tail(cache, b.Config([10], wl.hq, wl.hkv, budget_bits=[2.0], s_obs=32), Q)
    with pytest.raises(RuntimeError):                                        # not the cache's own K format
        b.rdkv_cache_rebudget_tail(cache, b.Config([10], wl.hq, wl.hkv, budget_bits=[2.0], s_obs=8,
                                                   k_mode=b.RDKV_K_CHANNELWISE), Q)
    assert b.rdkv_cache_tail_len(cache) == 10 and b.rdkv_cache_generations(cache) == 0   # unchanged after errors
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    cache.free()


@pytest.mark.parametrize("name,kw,n_new,budgets,per_channel_scale", [
    ("tiny", {"seq_lens": (900,)}, 200, [3.0], False),
    ("tiny", {"seq_lens": (600,)}, 160, [1.5], True),            # one K scale per channel over the unit (App. B)
    ("batch70b", {"batch": 2, "len_range": (100, 700)}, 300, [1.0, 6.0], False),   # 8 query heads per KV head
])
def test_rebudget_mixed_matches_oracle(name, kw, n_new, budgets, per_channel_scale):
    """Channel-wise caches: the generation has its own channel bit map and K row layout per (sequence, KV head)."""
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    batch = len(inp["seq_lens"])
    rng = np.random.default_rng(94)
    bt, bc = _random_maps(rng, inp["seq_lens"], wl.hkv, [.3, .3, .2, .1, .1], [.1, .4, .3, .15, .05])
    cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc, per_channel_scale)
    b.rdkv_cache_reserve_tail(cache, 320)
    k_rows, _ = _append(b, cache, ref, rng, n_new, batch, wl.hkv)
    Q_obs = torch.from_numpy(rng.standard_normal((batch, wl.hq, 32, 128)).astype(np.float32)).to(torch.bfloat16)
    cfg = b.Config([n_new] * batch, wl.hq, wl.hkv, budget_bits=budgets, s_obs=32, k_mode=b.RDKV_K_CHANNELWISE,
                   k_scale_per_channel=int(per_channel_scale))
    print(f"[step] rebudget mixed tail of {n_new} tokens, budgets {budgets}", flush=True)
    b.rdkv_cache_rebudget_tail(cache, cfg, Q_obs.cuda())
    w_tok, w_ch = b.rdkv_weights(cfg, k_rows.reshape(-1).cuda(), Q_obs.cuda(), want_channel=True)
    torch.cuda.synchronize()
    wt = [w.cpu().numpy() for w in w_tok.view(batch, wl.hkv, n_new)]
    wc = [w.cpu().numpy() for w in w_ch.view(batch, wl.hkv, 128)]
    child = O.rebudget_tail(ref, [_np(Q_obs[s]) for s in range(batch)], [np.float32(x) for x in budgets],
                            weights_override=(wt, wc))
    gen = b.rdkv_cache_generation(cache, 0, cfg)
    np.testing.assert_array_equal(gen.export(b.RDKV_EXPORT_BITS_TOK, np.uint8),
                                  np.concatenate([x.reshape(-1) for x in child["bits"]]))
    _assert_cache_equal_mixed(b, gen, child)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    _append(b, cache, ref, rng, 5, batch, wl.hkv)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    _check_decode(out, lse, *O.decode(ref, _np(inp["q"])))
    cache.free()


def test_rebudget_at_full_size():
    """One layer of the 128K-token stack, in the launch configuration the benchmark times: compress, append 256
    tokens, re-budget them at 2 bits, append 9 more, decode.  The oracle redoes one sampled KV head end to end from the
    library's fp32 weights (prompt and tail): bit maps and the generation's bytes bit for bit, output within 2e-3."""
    from paper_2605_08317_amd import workloads as W
    b = B()
    wl = W.CONFIGS["stack128k"]
    T, n_new, h, g = wl.seq_lens[0], 256, 5, wl.hq // wl.hkv
    print("[case] full-size stack128k layer 3 with re-budgeting", flush=True)
    inp = W.make_inputs(wl, device="cuda", layer=3)
    cfg = b.Config([T], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs)
    cache = b.rdkv_compress(cfg, inp["K"], inp["V"], inp["Q_obs"])
    w_tok, _ = b.rdkv_weights(cfg, inp["K"], inp["Q_obs"])
    torch.cuda.synchronize()
    # the oracle's copy of head h: prompt zones from the library's weights
    Kh = inp["K"].view(wl.hkv, T, 128)[h].float().cpu().numpy()[None]
    Vh = inp["V"].view(wl.hkv, T, 128)[h].float().cpu().numpy()[None]
    bt = O.mckp_bisect(w_tok.view(wl.hkv, T)[h].cpu().numpy(), np.float32(inp["budgets"][0]))
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_BITS_TOK, np.uint8).reshape(wl.hkv, T)[h], bt)
    ref = O.build_cache_tokenwise([Kh], [Vh], [bt[None]])
    # 256 appended tokens
    rng = np.random.default_rng(95)
    kn = torch.from_numpy(rng.standard_normal((n_new + 9, 1, wl.hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    vn = torch.from_numpy(rng.standard_normal((n_new + 9, 1, wl.hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    kd, vd = kn.cuda(), vn.cuda()
    b.rdkv_cache_reserve_tail(cache, n_new)
    for i in range(n_new):
        b.rdkv_cache_append(cache, kd[i], vd[i])
        O.append_tokens(ref, kn[i, :, h:h + 1].float().numpy(), vn[i, :, h:h + 1].float().numpy())
    Q_obs = torch.from_numpy(rng.standard_normal((1, wl.hq, wl.s_obs, 128)).astype(np.float32)).to(torch.bfloat16)
    cfg_t = b.Config([n_new], wl.hq, wl.hkv, budget_bits=[2.0], s_obs=wl.s_obs)
    b.rdkv_cache_rebudget_tail(cache, cfg_t, Q_obs.cuda())
    k_rows = kn[:n_new, 0].permute(1, 0, 2).contiguous()                          # [hkv][n][128]
    w_tail, _ = b.rdkv_weights(cfg_t, k_rows.reshape(-1).cuda(), Q_obs.cuda())
    torch.cuda.synchronize()
    child = O.rebudget_tail(ref, [Q_obs[0, h * g:(h + 1) * g].float().numpy()], [np.float32(2.0)],
                            weights_override=[w_tail.view(wl.hkv, n_new)[h:h + 1].cpu().numpy()])
    gen = b.rdkv_cache_generation(cache, 0, cfg_t)
    np.testing.assert_array_equal(gen.export(b.RDKV_EXPORT_BITS_TOK, np.uint8).reshape(wl.hkv, n_new)[h], child["bits"][0][0])
    # the generation's segments of item h against the oracle's single-item child
    counts = gen.export(b.RDKV_EXPORT_COUNTS, np.int32).reshape(-1, 4)
    seg_off = gen.export(b.RDKV_EXPORT_SEG_OFF, np.int64).reshape(-1, 4, 4)
    arena = gen.export(b.RDKV_EXPORT_ARENA, np.uint8)
    np.testing.assert_array_equal(counts[h], child["counts"][0])
    for ti, bits in enumerate(O.PACK_ORDER):
        npad = (int(counts[h, ti]) + 63) // 64 * 64
        for si, nbytes in enumerate([npad * O.row_bytes(bits), npad * O.meta_bytes(bits)] * 2):
            got = arena[int(seg_off[h, ti, si]):int(seg_off[h, ti, si]) + nbytes]
            want = child["arena"][int(child["seg_off"][0, ti, si]):int(child["seg_off"][0, ti, si]) + nbytes]
            assert np.array_equal(got, want), f"generation bytes differ in tier {bits}, segment {si}"
    for i in range(n_new, n_new + 9):
        b.rdkv_cache_append(cache, kd[i], vd[i])
        O.append_tokens(ref, kn[i, :, h:h + 1].float().numpy(), vn[i, :, h:h + 1].float().numpy())
    out, lse = b.rdkv_decode_attn(cache, inp["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, inp["q"][:, h * g:(h + 1) * g].float().cpu().numpy())
    _check_decode(out[:, h * g:(h + 1) * g], lse[:, h * g:(h + 1) * g], ref_out, ref_lse)
    cache.free()
