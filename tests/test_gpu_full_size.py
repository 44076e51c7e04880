"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times (one
rdkv_compress and one rdkv_decode_attn call per layer / batch).  The oracle cannot redo a whole 128K-token layer in
seconds, so it recomputes sampled items (sequence, KV head) one by one from the library's own fp32 weights: their
bit maps, kept-position lists and packed bytes must match bit for bit, their decode outputs within 2e-3; the rest
is covered by properties that hold at any size (budget met, counts consistent with the bit map)."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from paper_2605_08317_amd import workloads as W
from test_gpu_parity import B, _rel_err, _elementwise_err, DECODE_TOL, WEIGHT_RTOL

pytestmark = pytest.mark.gpu


def _item_segments(arena, seg_off, item, sizes):
    """The four segments of every tier of one item, cut out of an arena."""
    out = []
    for ti in range(4):
        for si in range(4):
            o = int(seg_off[item, ti, si])
            out.append(arena[o:o + sizes[ti][si]])
    return out


def _seg_sizes_tokenwise(counts):
    sizes = []
    for ti, b in enumerate(O.PACK_ORDER):
        npad = (int(counts[ti]) + O.ROW_PAD_TOKENWISE - 1) // O.ROW_PAD_TOKENWISE * O.ROW_PAD_TOKENWISE
        sizes.append([npad * O.row_bytes(b), npad * O.meta_bytes(b), npad * O.row_bytes(b), npad * O.meta_bytes(b)])
    return sizes


def _seg_sizes_mixed(counts, bits_ch, per_channel_scale=False):
    sl = O.channel_slots(bits_ch)
    sizes = []
    for ti, b in enumerate(O.PACK_ORDER):
        nt = (int(counts[ti]) + 63) // 64
        k_meta = nt * O.k_meta_bytes_mixed(sl)
        if per_channel_scale:                      # one record per non-empty tier segment: half a tile's metadata
            k_meta = O.k_meta_bytes_mixed(sl) // 2 if nt else 0
        sizes.append([nt * O.k_tile_bytes_mixed(sl), k_meta,
                      nt * (16384 if b == 16 else 1024 * b), 0 if b == 16 else nt * 1024])
    return sizes


def _check_sampled_items(b, wl, inp, cache, out, lse, w_tok, samples, mixed=False, w_ch=None, per_channel_scale=False):
    hkv, d, g = wl.hkv, wl.d, wl.hq // wl.hkv
    seq_lens = inp["seq_lens"]
    counts = cache.export(b.RDKV_EXPORT_COUNTS, np.int32).reshape(-1, 4)
    seg_off = cache.export(b.RDKV_EXPORT_SEG_OFF, np.int64).reshape(-1, 4, 4)
    tier_idx = cache.export(b.RDKV_EXPORT_TIER_IDX, np.int32)
    bits_all = cache.export(b.RDKV_EXPORT_BITS_TOK, np.uint8)
    arena = cache.export(b.RDKV_EXPORT_ARENA, np.uint8)
    bits_ch_all = cache.export(b.RDKV_EXPORT_BITS_CH, np.uint8).reshape(-1, d) if mixed else None
    tok_off = np.concatenate([[0], np.cumsum([hkv * T for T in seq_lens])])
    idx_off = np.concatenate([[0], np.cumsum(counts.sum(axis=1))])
    # properties over every item: the bit map meets the budget and the tier counts are its histogram
    for s, T in enumerate(seq_lens):
        bt = bits_all[tok_off[s]:tok_off[s + 1]].reshape(hkv, T)
        v_avg = inp["budgets"][s] if not mixed else O.mixed_budgets(np.float32(inp["budgets"][s]), np.float32(0.5), T, None, d)[0]
        for h in range(hkv):
            assert int(bt[h].astype(np.int64).sum()) <= int(np.floor(np.float64(np.float32(v_avg)) * T))
            assert [int((bt[h] == t).sum()) for t in O.PACK_ORDER] == counts[s * hkv + h].tolist()
    K_views = W.split_sequences(inp["K"], seq_lens, hkv, d)
    V_views = W.split_sequences(inp["V"], seq_lens, hkv, d)
    w_views = W.split_sequences(w_tok, seq_lens, hkv, None)
    worst = 0.0
    for (s, h) in samples:
        item, T = s * hkv + h, seq_lens[s]
        print(f"[sample] sequence {s} KV head {h} T={T}", flush=True)
        Kh = K_views[s][h].float().cpu().numpy()[None]
        Vh = V_views[s][h].float().cpu().numpy()[None]
        wh = w_views[s][h].cpu().numpy()
        if mixed:
            bt, bc = O.allocate_mixed(wh, w_ch[item], np.float32(inp["budgets"][s]))
            np.testing.assert_array_equal(bits_ch_all[item], bc)
            ref = O.build_cache_mixed([Kh], [Vh], [bt[None]], [bc[None]], k_per_channel_scale=per_channel_scale)
            sizes = _seg_sizes_mixed(counts[item], bc, per_channel_scale)
        else:
            bt = O.mckp_bisect(wh, np.float32(inp["budgets"][s]))
            ref = O.build_cache_tokenwise([Kh], [Vh], [bt[None]])
            sizes = _seg_sizes_tokenwise(counts[item])
        np.testing.assert_array_equal(bits_all[tok_off[s] + h * T:tok_off[s] + (h + 1) * T], bt)
        np.testing.assert_array_equal(counts[item], ref["counts"][0])
        np.testing.assert_array_equal(tier_idx[idx_off[item]:idx_off[item + 1]], ref["tier_idx"])
        for got, want in zip(_item_segments(arena, seg_off, item, sizes), _item_segments(ref["arena"], ref["seg_off"], 0, sizes)):
            assert np.array_equal(got, want), "packed bytes of the sampled item differ"
        q = inp["q"][s:s + 1, h * g:(h + 1) * g].float().cpu().numpy()
        ro, rl = O.decode(ref, q)
        go = out[s, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)[None]
        gl = lse[s, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)[None]
        err = _rel_err(go, ro)
        worst = max(worst, err)
        print(f"[sample] decode error {err:.2e}; element-wise with floor {_elementwise_err(go, ro):.2e}", flush=True)
        assert err <= DECODE_TOL
        np.testing.assert_allclose(gl, rl, rtol=1e-4, atol=1e-4)
    print(f"[full size] worst sampled decode error {worst:.2e}", flush=True)


@pytest.mark.parametrize("name,layer,samples", [
    ("layer8b", 0, [(0, 0), (0, 5)]),
    ("stack128k", 0, [(0, 3)]),
    ("stack128k", 17, [(0, 6)]),
    ("batch70b", 0, [(0, 1), (7, 4), (15, 7)]),
])
def test_tokenwise_configs_at_full_size(name, layer, samples):
    b = B()
    wl = W.CONFIGS[name]
    print(f"[case] full-size {name} layer {layer}", flush=True)
    inp = W.make_inputs(wl, device="cuda", layer=layer)
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs)
    cache = b.rdkv_compress(cfg, inp["K"], inp["V"], inp["Q_obs"])
    w_tok, _ = b.rdkv_weights(cfg, inp["K"], inp["Q_obs"])
    out, lse = b.rdkv_decode_attn(cache, inp["q"])
    torch.cuda.synchronize()
    _check_sampled_items(b, wl, inp, cache, out, lse, w_tok, samples)
    cache.free()


@pytest.mark.parametrize("per_channel_scale", [False, True])
def test_mixed_config_at_full_size(per_channel_scale):
    b = B()
    wl = W.CONFIGS["mixed"]
    print(f"[case] full-size mixed, one K scale per channel: {per_channel_scale}", flush=True)
    inp = W.make_inputs(wl, device="cuda")
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs,
                   k_mode=b.RDKV_K_CHANNELWISE, k_scale_per_channel=int(per_channel_scale))
    _, w_ch = b.rdkv_weights(cfg, inp["K"], inp["Q_obs"], want_channel=True)
    bits_tok, bits_ch = b.rdkv_allocate(cfg, inp["w_tok"], w_ch)
    cache = b.rdkv_pack(cfg, inp["K"], inp["V"], bits_tok, bits_ch)
    out, lse = b.rdkv_decode_attn(cache, inp["q"])
    torch.cuda.synchronize()
    _check_sampled_items(b, wl, inp, cache, out, lse, inp["w_tok"], [(0, 2), (0, 7)], mixed=True,
                         w_ch=w_ch.cpu().numpy().reshape(-1, wl.d), per_channel_scale=per_channel_scale)
    st = cache.stats()
    print(f"[mixed full] token rows(16,8,4,2)={st['rows']} evicted={st['evicted']} stored={st['stored_bytes']} "
          f"dense={st['dense_bytes']}", flush=True)
    cache.free()


@pytest.mark.parametrize("layer,head", [(0, 3), (11, 6)])
def test_token_weights_of_a_128k_layer_against_the_oracle(layer, head):
    """Alg. 1 Stage 1 (Eq. 2) at the benchmark's full shape: T = 131072, S_w = 64, g = 4.  The library computes the
    whole layer; the oracle redoes one sampled KV head (its 256 window rows over all keys) in fp64, pooling included."""
    b = B()
    wl = W.CONFIGS["stack128k"]
    print(f"[case] full-size weights stack128k layer {layer} KV head {head}", flush=True)
    inp = W.make_inputs(wl, device="cuda", layer=layer)
    T, g = inp["seq_lens"][0], wl.hq // wl.hkv
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, s_obs=wl.s_obs)
    w_tok, w_ch = b.rdkv_weights(cfg, inp["K"], inp["Q_obs"], want_channel=True)
    torch.cuda.synchronize()
    got = w_tok.view(wl.hkv, T)[head].cpu().numpy().astype(np.float64)
    Kh = inp["K"].view(wl.hkv, T, wl.d)[head].float().cpu().numpy()[None]
    Qh = inp["Q_obs"][0, head * g:(head + 1) * g].float().cpu().numpy()
    ref = O.avg_pool(O.token_weights(Kh, Qh), 5)[0]
    err = np.abs(got - ref) / (np.abs(ref) + 1e-6 * ref.max())
    print(f"[weights full size] max rel err {err.max():.3e} at t={int(err.argmax())}, total mass {got.sum():.6f} "
          f"(oracle {ref.sum():.6f})", flush=True)
    assert err.max() <= WEIGHT_RTOL
    ref_c = O.channel_weights(Kh, Qh)[0]
    np.testing.assert_allclose(w_ch.view(wl.hkv, wl.d)[head].cpu().numpy(), ref_c, rtol=1e-5)


@pytest.mark.parametrize("hq", [32, 64])
def test_large_launch_whose_chunks_span_tiers(hq):
    """In a launch of hundreds of megabytes a workgroup's share of an item runs through several tiers (2-bit rows, then
    4-bit, then 8-bit, on one softmax state).  Four sequences of 64K tokens with random bit maps over all five widths;
    sampled items are recomputed by the oracle from the same maps (4 and 8 query heads per KV head)."""
    b = B()
    hkv, T, nseq, d = 8, 65536, 4, 128
    g = hq // hkv
    gen = torch.Generator(device="cuda").manual_seed(77)
    K = torch.randn((nseq, hkv, T, d), device="cuda", generator=gen).to(torch.bfloat16)
    V = torch.randn((nseq, hkv, T, d), device="cuda", generator=gen).to(torch.bfloat16)
    q = torch.randn((nseq, hq, d), device="cuda", generator=gen).to(torch.bfloat16)
    tiers = torch.tensor([0, 2, 4, 8, 16], dtype=torch.uint8, device="cuda")
    pick = torch.multinomial(torch.tensor([.25, .3, .2, .2, .05], device="cuda"), nseq * hkv * T, replacement=True, generator=gen)
    bits = tiers[pick]
    print(f"[case] chunks spanning tiers, g = {g}", flush=True)
    cfg = b.Config([T] * nseq, hq, hkv)
    cache = b.rdkv_pack(cfg, K.reshape(-1), V.reshape(-1), bits)
    st = cache.stats()
    print(f"[stats] stored {st['stored_bytes'] / 1e6:.0f} MB in {st['n_chunks']} chunks", flush=True)
    assert st["stored_bytes"] > 150e6 and st["n_chunks"] < 2200
    out, lse = b.rdkv_decode_attn(cache, q)
    torch.cuda.synchronize()
    bits_h = bits.view(nseq, hkv, T)
    samples = [(0, 0), (2, 5), (3, 7)]
    refs = [O.build_cache_tokenwise([K[s, h].float().cpu().numpy()[None]], [V[s, h].float().cpu().numpy()[None]],
                                    [bits_h[s, h].cpu().numpy()[None]]) for (s, h) in samples]

    def check(out, lse, what):
        worst = 0.0
        for (s, h), ref in zip(samples, refs):
            ro, rl = O.decode(ref, q[s:s + 1, h * g:(h + 1) * g].float().cpu().numpy())
            go = out[s, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)[None]
            gl = lse[s, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)[None]
            err = _rel_err(go, ro)
            worst = max(worst, err)
            assert err <= DECODE_TOL
            np.testing.assert_allclose(gl, rl, rtol=1e-4, atol=1e-4)
        print(f"[chunks spanning tiers] {what}: worst sampled decode error {worst:.2e}", flush=True)

    check(out, lse, "prompt")
    # a tail rebuilds the schedule: the chained pieces move to new places in the chunk table
    b.rdkv_cache_reserve_tail(cache, 64)
    kn = torch.randn((5, nseq, hkv, d), device="cuda", generator=gen).to(torch.bfloat16)
    vn = torch.randn((5, nseq, hkv, d), device="cuda", generator=gen).to(torch.bfloat16)
    for i in range(5):
        b.rdkv_cache_append(cache, kn[i], vn[i])
        for (s, h), ref in zip(samples, refs):
            O.append_tokens(ref, kn[i, s:s + 1, h:h + 1].float().cpu().numpy(), vn[i, s:s + 1, h:h + 1].float().cpu().numpy())
    out, lse = b.rdkv_decode_attn(cache, q)
    torch.cuda.synchronize()
    check(out, lse, "prompt + 5 appended tokens")
    cache.free()


def test_mixed_config_with_three_sequences():
    """Three 64K-token sequences of the mixed-granularity configuration (70 MB stored): the launch is no longer small,
    so the channel-wise kernel runs with four-wavefront workgroups and about two rounds of chunks."""
    b = B()
    wl = W.scaled(W.CONFIGS["mixed"], batch=3, seq_lens=(65536,) * 3, budgets=(1.0,))
    print("[case] full-size mixed, 3 sequences", flush=True)
    inp = W.make_inputs(wl, device="cuda")
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs, k_mode=b.RDKV_K_CHANNELWISE)
    _, w_ch = b.rdkv_weights(cfg, inp["K"], inp["Q_obs"], want_channel=True)
    bits_tok, bits_ch = b.rdkv_allocate(cfg, inp["w_tok"], w_ch)
    cache = b.rdkv_pack(cfg, inp["K"], inp["V"], bits_tok, bits_ch)
    out, lse = b.rdkv_decode_attn(cache, inp["q"])
    torch.cuda.synchronize()
    assert cache.stats()["stored_bytes"] > 48 << 20
    _check_sampled_items(b, wl, inp, cache, out, lse, inp["w_tok"], [(0, 1), (2, 6)], mixed=True,
                         w_ch=w_ch.cpu().numpy().reshape(-1, wl.d))
    cache.free()


def test_one_million_token_sequence():
    """The longest context tried: one sequence of 2^20 tokens (8 KV heads, 0.5 bit/elt).  The pass and the decode step
    on the whole sequence, the bf16 path beside it; the oracle redoes one KV head from the library's own weights."""
    b = B()
    T, hq, hkv, h = 1 << 20, 32, 8, 5
    g = hq // hkv
    gen = torch.Generator(device="cuda").manual_seed(5)
    K = torch.randn((hkv, T, 128), device="cuda", generator=gen).to(torch.bfloat16)
    V = torch.randn((hkv, T, 128), device="cuda", generator=gen).to(torch.bfloat16)
    Q = torch.randn((1, hq, 32, 128), device="cuda", generator=gen).to(torch.bfloat16)
    q = torch.randn((1, hq, 128), device="cuda", generator=gen).to(torch.bfloat16)
    print("[case] one sequence of 2^20 tokens", flush=True)
    cfg = b.Config([T], hq, hkv, budget_bits=[0.5])
    cache = b.rdkv_compress(cfg, K.reshape(-1), V.reshape(-1), Q)
    out, lse = b.rdkv_decode_attn(cache, q)
    w, _ = b.rdkv_weights(cfg, K.reshape(-1), Q)
    torch.cuda.synchronize()
    st = cache.stats()
    assert st["arena_bytes"] <= b.rdkv_cache_max_bytes(cfg) and st["rows"][3] + st["rows"][2] + st["rows"][1] + st["rows"][0] + st["evicted"] == hkv * T
    bt = O.mckp_bisect(w.view(hkv, T)[h].cpu().numpy(), np.float32(0.5))
    np.testing.assert_array_equal(cache.export(b.RDKV_EXPORT_BITS_TOK, np.uint8).reshape(hkv, T)[h], bt)
    Kh, Vh = K[h].float().cpu().numpy()[None], V[h].float().cpu().numpy()[None]
    qh = q[:, h * g:(h + 1) * g].float().cpu().numpy()
    ref = O.build_cache_tokenwise([Kh], [Vh], [bt[None]])
    ro, rl = O.decode(ref, qh)
    err = _rel_err(out[0, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)[None], ro)
    print(f"[2^20 tokens] decode error {err:.2e} over {int((bt > 0).sum())} retained tokens", flush=True)
    assert err <= DECODE_TOL
    np.testing.assert_allclose(lse[0, h * g:(h + 1) * g].cpu().numpy()[None], rl, rtol=1e-4, atol=1e-4)
    ws = torch.empty(b.rdkv_decode_bf16_workspace_bytes([T], hq, hkv), dtype=torch.uint8, device="cuda")
    o16, l16 = b.rdkv_decode_attn_bf16(K.reshape(-1), V.reshape(-1), [T], hq, hkv, q, workspace=ws)
    torch.cuda.synchronize()
    d_out, d_lse = O.decode_dense([Kh], [Vh], qh)
    assert _rel_err(o16[0, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)[None], d_out) <= DECODE_TOL
    np.testing.assert_allclose(l16[0, h * g:(h + 1) * g].cpu().numpy()[None], d_lse, rtol=1e-4, atol=1e-4)
    cache.free()
