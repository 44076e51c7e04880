"""GPU parity in mixed mode (V token-wise, K channel-wise on the retained tokens: Sec. 3.2 Stages 2-3):
bit maps, packed bytes and index tables bit for bit against the oracle given the same fp32 weights / bit maps;
decode within 2e-3 of the fp64 oracle (max|o - o_ref| / max|o_ref| per head)."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from paper_2605_08317_amd import workloads as W
from test_gpu_parity import B, _np, _split, _check_decode, _inputs

pytestmark = pytest.mark.gpu


def _random_maps(rng, seq_lens, hkv, p_tok, p_ch):
    tiers = np.array([0, 2, 4, 8, 16], np.uint8)
    bt = [rng.choice(tiers, size=(hkv, T), p=p_tok) for T in seq_lens]
    bc = [rng.choice(tiers, size=(hkv, 128), p=p_ch) for _ in seq_lens]
    return bt, bc


def _pack_both_mixed(b, wl, inp, dev, bt, bc, per_channel_scale=False):
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, k_mode=b.RDKV_K_CHANNELWISE,
                   k_scale_per_channel=int(per_channel_scale))
    bt_flat = torch.from_numpy(np.concatenate([x.reshape(-1) for x in bt])).cuda()
    bc_flat = torch.from_numpy(np.concatenate([x.reshape(-1) for x in bc])).cuda()
    cache = b.rdkv_pack(cfg, dev["K"], dev["V"], bt_flat, bc_flat)
    Ks = _split(inp["K"], inp["seq_lens"], wl.hkv, wl.d)
    Vs = _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d)
    ref = O.build_cache_mixed(Ks, Vs, bt, bc, k_per_channel_scale=per_channel_scale)
    return cache, ref


def _assert_cache_equal_mixed(b, cache, ref):
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_COUNTS, np.int32).reshape(-1, 4), ref["counts"])
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_TIER_IDX, np.int32), ref["tier_idx"])
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_SEG_OFF, np.int64).reshape(-1, 4, 4), ref["seg_off"])
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_BITS_CH, np.uint8).reshape(-1, 128), ref["bits_ch"])
    arena = cache.export(b.RDKV_EXPORT_ARENA, np.uint8)
    assert arena.shape == ref["arena"].shape
    if not np.array_equal(arena, ref["arena"]):
        bad = np.nonzero(arena != ref["arena"])[0]
        raise AssertionError(f"arena differs at {len(bad)} bytes, first at {bad[:8]}")
    assert cache.stats()["stored_bytes"] == O.stored_bytes_mixed(ref["counts"], ref["bits_ch"],
                                                                 k_per_channel_scale=ref["k_per_unit"])


CASES = [
    # workload, overrides, token tier probabilities (0,2,4,8,16), channel tier probabilities
    ("tiny", {"seq_lens": (700,)}, [.3, .3, .2, .1, .1], [.1, .4, .3, .15, .05]),
    ("tiny", {"seq_lens": (2100,)}, [.6, .2, .15, .05, .0], [.0, .6, .4, .0, .0]),        # no 8/16-bit channels
    ("tiny", {"seq_lens": (333,)}, [.0, .0, .0, .0, 1.], [.0, .0, .0, .0, 1.]),            # everything at 16 bits
    ("tiny", {"seq_lens": (500,)}, [.2, .2, .2, .2, .2], [1., .0, .0, .0, .0]),            # every channel evicted
    ("tiny", {"seq_lens": (900,), "hq": 2, "hkv": 2}, [.5, .2, .2, .1, .0], [.2, .2, .2, .2, .2]),
    ("batch70b", {"batch": 3, "len_range": (100, 1300)}, [.5, .2, .2, .05, .05], [.05, .45, .35, .1, .05]),
    # 8 query heads per KV head with short K rows (2- and 4-bit channels only) and with the longest ones (all 16-bit)
    ("batch70b", {"batch": 2, "len_range": (300, 900)}, [.3, .3, .2, .1, .1], [.2, .6, .2, .0, .0]),
    ("batch70b", {"batch": 2, "len_range": (200, 500)}, [.3, .3, .2, .1, .1], [.0, .0, .0, .1, .9]),
]


@pytest.mark.parametrize("name,kw,p_tok,p_ch", CASES)
def test_pack_mixed_is_bit_exact(name, kw, p_tok, p_ch):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    bt, bc = _random_maps(np.random.default_rng(7), inp["seq_lens"], wl.hkv, p_tok, p_ch)
    cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    _assert_cache_equal_mixed(b, cache, ref)
    cache.free()


@pytest.mark.parametrize("name,kw,p_tok,p_ch", CASES)
def test_decode_mixed(name, kw, p_tok, p_ch):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    bt, bc = _random_maps(np.random.default_rng(8), inp["seq_lens"], wl.hkv, p_tok, p_ch)
    bt[0][0, :] = 0                                    # one head with nothing retained: out = 0, lse = -inf
    cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    cache.free()


def test_all_16_bit_mixed_cache_is_the_uncompressed_cache():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1234,))
    bt = [np.full((wl.hkv, T), 16, np.uint8) for T in inp["seq_lens"]]
    bc = [np.full((wl.hkv, 128), 16, np.uint8) for _ in inp["seq_lens"]]
    cache, _ = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    d_out, d_lse = O.decode_dense(_split(inp["K"], inp["seq_lens"], wl.hkv, wl.d),
                                  _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d), _np(inp["q"]))
    _check_decode(out, lse, d_out, d_lse)
    cache.free()


@pytest.mark.parametrize("seq_lens,budgets", [
    ((5000,), (1.0,)),
    ((4096, 777, 9000), (0.4, 2.0, 4.0)),
    ((64, 2000), (0.0, 16.0)),
])
def test_allocate_mixed_is_bit_exact(seq_lens, budgets):
    b = B()
    hkv, hq = 2, 8
    rng = np.random.default_rng(5)
    w_tok = [(1.0 + rng.pareto(1.2, (hkv, T))).astype(np.float32) for T in seq_lens]
    w_ch = [np.exp(rng.normal(0, 1.0, (hkv, 128))).astype(np.float32) for _ in seq_lens]
    cfg = b.Config(seq_lens, hq, hkv, budget_bits=budgets, k_mode=b.RDKV_K_CHANNELWISE)
    print(f"[case] allocate mixed seq_lens={seq_lens} budgets={budgets}", flush=True)
    bits_tok, bits_ch = b.rdkv_allocate(cfg, torch.from_numpy(np.concatenate([w.reshape(-1) for w in w_tok])).cuda(),
                                        torch.from_numpy(np.concatenate([w.reshape(-1) for w in w_ch])).cuda())
    torch.cuda.synchronize()
    got_t, got_c = bits_tok.cpu().numpy(), bits_ch.cpu().numpy().reshape(-1, 128)
    off = 0
    for s, T in enumerate(seq_lens):
        for h in range(hkv):
            rt, rc = O.allocate_mixed(w_tok[s][h], w_ch[s][h], np.float32(budgets[s]))
            np.testing.assert_array_equal(got_t[off:off + T], rt)
            np.testing.assert_array_equal(got_c[s * hkv + h], rc)
            off += T


def test_mixed_workload_staged_pass_and_fused_compress():
    """The mixed-granularity benchmark configuration at a shorter context: supplied Pareto token weights, channel
    weights from the probe."""
    b = B()
    wl, inp, dev = _inputs("mixed", seq_lens=(6000,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs,
                   k_mode=b.RDKV_K_CHANNELWISE)
    _, w_ch = b.rdkv_weights(cfg, dev["K"], dev["Q_obs"], want_channel=True)
    bits_tok, bits_ch = b.rdkv_allocate(cfg, dev["w_tok"], w_ch)
    cache = b.rdkv_pack(cfg, dev["K"], dev["V"], bits_tok, bits_ch)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    Ks = _split(inp["K"], inp["seq_lens"], wl.hkv, wl.d)
    Vs = _split(inp["V"], inp["seq_lens"], wl.hkv, wl.d)
    wt = inp["w_tok"].numpy().reshape(wl.hkv, -1)
    wc = w_ch.cpu().numpy().reshape(wl.hkv, 128)
    np.testing.assert_allclose(wc, O.channel_weights(Ks[0], _np(inp["Q_obs"][0])), rtol=1e-5)
    bt = np.zeros((wl.hkv, inp["seq_lens"][0]), np.uint8)
    bc = np.zeros((wl.hkv, 128), np.uint8)
    for h in range(wl.hkv):
        bt[h], bc[h] = O.allocate_mixed(wt[h], wc[h], np.float32(inp["budgets"][0]))
    np.testing.assert_array_equal(bits_tok.cpu().numpy().reshape(wl.hkv, -1), bt)
    np.testing.assert_array_equal(bits_ch.cpu().numpy().reshape(wl.hkv, 128), bc)
    ref = O.build_cache_mixed(Ks, Vs, [bt], [bc])
    _assert_cache_equal_mixed(b, cache, ref)
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    st = cache.stats()
    hist = {t: int((bc == t).sum()) for t in (0, 2, 4, 8, 16)}
    print(f"[mixed] token rows(16,8,4,2)={st['rows']} evicted={st['evicted']} channel tiers={hist} "
          f"stored={st['stored_bytes']} dense={st['dense_bytes']}", flush=True)
    cache.free()
    # the fused pass computes its own token weights (Eq. 2) instead of the supplied ones; its maps must equal the
    # oracle's allocation from the library's own fp32 weights
    cache2 = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
    w_tok2, w_ch2 = b.rdkv_weights(cfg, dev["K"], dev["Q_obs"], want_channel=True)
    torch.cuda.synchronize()
    wt2 = w_tok2.cpu().numpy().reshape(wl.hkv, -1)
    wc2 = w_ch2.cpu().numpy().reshape(wl.hkv, 128)
    for h in range(wl.hkv):
        bt[h], bc[h] = O.allocate_mixed(wt2[h], wc2[h], np.float32(inp["budgets"][0]))
    np.testing.assert_array_equal(cache2.export(b.RDKV_EXPORT_BITS_TOK, np.uint8).reshape(wl.hkv, -1), bt)
    _assert_cache_equal_mixed(b, cache2, O.build_cache_mixed(Ks, Vs, [bt], [bc]))
    cache2.free()


@pytest.mark.parametrize("r_k", [0.4, 0.6])
def test_allocate_mixed_with_other_kv_splits(r_k):
    """B_K = r_K B_head (Sec. 3.2; Table 8 varies r_K): the V map takes 2 (1 - r_K) of the average budget, the K
    channels the rest spread over the retained tokens."""
    b = B()
    hkv, hq, T = 2, 8, 6000
    rng = np.random.default_rng(11)
    w_tok = (1.0 + rng.pareto(1.2, (hkv, T))).astype(np.float32)
    w_ch = np.exp(rng.normal(0, 1.0, (hkv, 128))).astype(np.float32)
    cfg = b.Config([T], hq, hkv, budget_bits=[1.5], k_mode=b.RDKV_K_CHANNELWISE, kv_split_rk=r_k)
    print(f"[case] allocate mixed r_K={r_k}", flush=True)
    bits_tok, bits_ch = b.rdkv_allocate(cfg, torch.from_numpy(w_tok.reshape(-1)).cuda(),
                                        torch.from_numpy(w_ch.reshape(-1)).cuda())
    torch.cuda.synchronize()
    got_t, got_c = bits_tok.cpu().numpy().reshape(hkv, T), bits_ch.cpu().numpy().reshape(hkv, 128)
    for h in range(hkv):
        rt, rc = O.allocate_mixed(w_tok[h], w_ch[h], np.float32(1.5), r_k=np.float32(r_k))
        np.testing.assert_array_equal(got_t[h], rt)
        np.testing.assert_array_equal(got_c[h], rc)
        n_kept = int((rt > 0).sum())
        total_bits = int(rt.astype(np.int64).sum()) * 128 + int(rc.astype(np.int64).sum()) * n_kept
        assert total_bits <= 1.5 * 2 * T * 128                    # whole-cache budget


# the paper's own K format (App. B): one scale and zero-point per channel over all retained tokens
@pytest.mark.parametrize("name,kw,p_tok,p_ch", [CASES[0], CASES[1], CASES[3], CASES[5], CASES[6]])
def test_per_channel_scale_pack_and_decode(name, kw, p_tok, p_ch):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    bt, bc = _random_maps(np.random.default_rng(12), inp["seq_lens"], wl.hkv, p_tok, p_ch)
    bt[0][0, :] = 0                                    # one head with nothing retained
    cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc, per_channel_scale=True)
    _assert_cache_equal_mixed(b, cache, ref)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    cache.free()


@pytest.mark.parametrize("counts", [(125, 1, 1, 1), (126, 2, 0, 0), (121, 3, 2, 2), (124, 0, 4, 0)])
@pytest.mark.parametrize("name,kw", [("tiny", {"seq_lens": (700,)}), ("batch70b", {"batch": 2, "len_range": (200, 500)})])
def test_k_rows_longer_than_64_words(name, kw, counts):
    """Channel maps whose sorted-channel row exceeds 64 words (the 16-bit segment nearly full and every other segment
    paying its padding: up to 68 words): Stage 3 of Alg. 1 produces them when the K average lies just under 16 bits."""
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    rng = np.random.default_rng(21)
    n16, n8, n4, n2 = counts
    bt, _ = _random_maps(rng, inp["seq_lens"], wl.hkv, [.2, .2, .2, .2, .2], [.2, .2, .2, .2, .2])
    bc = []
    for _ in inp["seq_lens"]:
        m = np.zeros((wl.hkv, 128), np.uint8)
        for h in range(wl.hkv):
            row = np.array([16] * n16 + [8] * n8 + [4] * n4 + [2] * n2 + [0] * (128 - sum(counts)), np.uint8)
            m[h] = rng.permutation(row)
        bc.append(m)
    print(f"[case] wide K rows {name} {kw} counts={counts}", flush=True)
    cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    _assert_cache_equal_mixed(b, cache, ref)
    out, lse = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, _np(inp["q"]))
    _check_decode(out, lse, ref_out, ref_lse)
    cache.free()
