"""GPU tests of the boundary's bookkeeping: the multiplier and step count of Alg. 2 reported per item, the a-priori
arena bound, bit maps with values that are no bit-width, exact ties in the per-unit step, and calls that return
without waiting for the stream."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from test_gpu_parity import B, _inputs, _np, _split

pytestmark = pytest.mark.gpu


def _bits_by_item(bits, seq_lens, hkv):
    out, off = [], 0
    for T in seq_lens:
        for h in range(hkv):
            out.append(bits[off:off + T])
            off += T
    return out


@pytest.mark.parametrize("seq_lens,budgets,eps", [
    ((5000, 700), (1.0, 3.0), O.EPS_V_LLAMA31_8B),
    ((9000,), (0.4,), O.EPS_BENNETT),
    ((64, 2000, 333), (0.0, 16.0, 7.5), O.EPS_BENNETT),          # the all-0 and all-16 shortcuts: no search
])
def test_lambda_and_iterations_match_the_oracle(seq_lens, budgets, eps):
    b = B()
    hkv, hq = 2, 8
    rng = np.random.default_rng(3)
    w = [np.exp(rng.normal(0, 2.0, (hkv, T))).astype(np.float32) for T in seq_lens]
    cfg = b.Config(seq_lens, hq, hkv, budget_bits=budgets, eps_v=eps)
    print(f"[case] lambda/iterations seq_lens={seq_lens} budgets={budgets}", flush=True)
    bits, _, lam, iters = b.rdkv_allocate_info(cfg, torch.from_numpy(np.concatenate([x.reshape(-1) for x in w])).cuda())
    torch.cuda.synchronize()
    bits, lam, iters = bits.cpu().numpy(), lam.cpu().numpy()[0], iters.cpu().numpy()[0]
    per_item = _bits_by_item(bits, seq_lens, hkv)
    for s, T in enumerate(seq_lens):
        for h in range(hkv):
            rb, info = O.mckp_bisect(w[s][h], np.float32(budgets[s]), O.TIERS, eps, return_info=True)
            i = s * hkv + h
            np.testing.assert_array_equal(per_item[i], rb)
            assert iters[i] == info["iters"]
            if info["lam"] is None:
                assert np.isnan(lam[i])
            else:
                assert lam[i] == info["lam"]                     # the same fp64 midpoints, bit for bit


def test_compress_keeps_lambda_and_iterations_with_the_cache():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(3000,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs)
    cache = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
    w_tok, _ = b.rdkv_weights(cfg, dev["K"], dev["Q_obs"])
    torch.cuda.synchronize()
    lam = cache.export(b.RDKV_EXPORT_LAMBDA, np.float64)
    iters = cache.export(b.RDKV_EXPORT_ITERATIONS, np.int32)
    w = w_tok.cpu().numpy().reshape(wl.hkv, -1)
    for h in range(wl.hkv):
        _, info = O.mckp_bisect(w[h], np.float32(inp["budgets"][0]), return_info=True)
        assert lam[h] == info["lam"] and iters[h] == info["iters"]
    st = cache.stats()
    assert st["alloc_info"] == 1 and st["iterations_max"] == iters.max()
    assert st["lambda_min"] == lam.min() and st["lambda_max"] == lam.max()
    # a cache packed from caller-supplied maps knows nothing about a search
    packed = b.rdkv_pack(cfg, dev["K"], dev["V"], torch.from_numpy(cache.export(b.RDKV_EXPORT_BITS_TOK, np.uint8)).cuda())
    st2 = packed.stats()
    assert st2["alloc_info"] == 0 and np.isnan(st2["lambda_min"]) and packed.export(b.RDKV_EXPORT_LAMBDA, np.float64).size == 0
    assert np.array_equal(packed.export(b.RDKV_EXPORT_ARENA, np.uint8), cache.export(b.RDKV_EXPORT_ARENA, np.uint8))
    packed.free()
    cache.free()


def test_mixed_mode_reports_both_searches():
    b = B()
    hkv, hq, T = 2, 8, 4000
    rng = np.random.default_rng(4)
    w_tok = (1.0 + rng.pareto(1.2, (hkv, T))).astype(np.float32)
    w_ch = np.exp(rng.normal(0, 1.0, (hkv, 128))).astype(np.float32)
    cfg = b.Config([T], hq, hkv, budget_bits=[1.5], k_mode=b.RDKV_K_CHANNELWISE)
    bt, bc, lam, iters = b.rdkv_allocate_info(cfg, torch.from_numpy(w_tok.reshape(-1)).cuda(),
                                              torch.from_numpy(w_ch.reshape(-1)).cuda())
    torch.cuda.synchronize()
    lam, iters = lam.cpu().numpy(), iters.cpu().numpy()
    for h in range(hkv):
        v_avg, _ = O.mixed_budgets(np.float32(1.5), np.float32(0.5), T, None, 128)
        rt, info_v = O.mckp_bisect(w_tok[h], np.float32(v_avg), O.TIERS, O.EPS_V_LLAMA31_8B, return_info=True)
        n_kept = int((rt > 0).sum())
        _, k_avg = O.mixed_budgets(np.float32(1.5), np.float32(0.5), T, n_kept, 128)
        rc, info_k = O.mckp_bisect(w_ch[h], np.float32(k_avg), O.TIERS, O.EPS_K_LLAMA31_8B, return_info=True)
        np.testing.assert_array_equal(bt.cpu().numpy().reshape(hkv, T)[h], rt)
        np.testing.assert_array_equal(bc.cpu().numpy().reshape(hkv, 128)[h], rc)
        assert (lam[0, h], iters[0, h]) == (info_v["lam"], info_v["iters"])
        assert (lam[1, h], iters[1, h]) == (info_k["lam"], info_k["iters"])


def test_exact_ties_take_the_lower_bit_width_on_the_gpu():
    """Weights sitting exactly on the thresholds lam * r_k the search visits (dyadic distortion table, so that every
    product is exact): the library must keep the lower bit-width, as the printed argmin of Alg. 2 does."""
    b = B()
    eps = (1.0, 0.5, 0.25, 0.125, 0.0)
    w = np.array([64.0] * 4 + [32.0] * 4 + [1.0] * 4, np.float32)
    for iters_cap, want in ((3, [2] * 4 + [0] * 8), (4, [4] * 4 + [2] * 4 + [0] * 4)):
        cfg = b.Config([12], 1, 1, budget_bits=[2.0], eps_v=eps, rel_tol=0.0, max_iters=iters_cap)
        bits, _, lam, it = b.rdkv_allocate_info(cfg, torch.from_numpy(w).cuda())
        torch.cuda.synchronize()
        rb, info = O.mckp_bisect(w, np.float32(2.0), O.TIERS, eps, rel_tol=np.float32(0.0), max_iters=iters_cap, return_info=True)
        assert bits.cpu().numpy().tolist() == want == rb.tolist()
        assert lam.cpu().numpy()[0, 0] == info["lam"] and it.cpu().numpy()[0, 0] == info["iters"]


@pytest.mark.parametrize("name,kw,mixed", [
    ("tiny", {}, False), ("layer8b", {"seq_lens": (6000,)}, False), ("stack128k", {"seq_lens": (8192,)}, False),
    ("batch70b", {"batch": 3, "len_range": (500, 2500)}, False), ("mixed", {"seq_lens": (6000,)}, True),
])
def test_arena_stays_below_the_a_priori_bound(name, kw, mixed):
    b = B()
    wl, inp, dev = _inputs(name, **kw)
    extra = {"k_mode": b.RDKV_K_CHANNELWISE} if mixed else {}
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs, **extra)
    bound = b.rdkv_cache_max_bytes(cfg)
    cache = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
    st = cache.stats()
    print(f"[bound] {name}: arena {st['arena_bytes']} <= bound {bound} ({st['arena_bytes'] / bound:.2f})", flush=True)
    assert 0 < st["arena_bytes"] <= bound
    tbound = b.rdkv_cache_max_table_bytes(cfg)
    print(f"[bound] {name}: tables {st['index_bytes']} <= bound {tbound} ({st['index_bytes'] / tbound:.2f})", flush=True)
    assert 0 < st["index_bytes"] <= tbound
    cache.free()
    # the largest budgets: every row at 16 bits
    cfg16 = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=[16.0] * len(inp["seq_lens"]), s_obs=wl.s_obs, **extra)
    cache = b.rdkv_compress(cfg16, dev["K"], dev["V"], dev["Q_obs"])
    assert cache.stats()["arena_bytes"] <= b.rdkv_cache_max_bytes(cfg16)
    cache.free()


def test_bit_maps_with_values_that_are_no_bit_width_are_rejected():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(500,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv)
    bits = torch.full((wl.hkv * 500,), 4, dtype=torch.uint8, device="cuda")
    bits[777] = 3
    with pytest.raises(b.RdkvError) as e:
        b.rdkv_pack(cfg, dev["K"], dev["V"], bits)
    assert e.value.status == 1 and "bits_tok" in str(e.value)
    bits[777] = 0
    b.rdkv_pack(cfg, dev["K"], dev["V"], bits).free()
    cfg_m = b.Config(inp["seq_lens"], wl.hq, wl.hkv, k_mode=b.RDKV_K_CHANNELWISE)
    bc = torch.full((wl.hkv * 128,), 2, dtype=torch.uint8, device="cuda")
    bc[5] = 6
    with pytest.raises(b.RdkvError) as e:
        b.rdkv_pack(cfg_m, dev["K"], dev["V"], bits, bc)
    assert e.value.status == 1 and "bits_ch" in str(e.value)


def test_weights_and_allocate_return_without_waiting():
    """The two staged calls enqueue their work and return: a long-running kernel ahead of them on the stream is still
    running when they come back (the event recorded right after them has not completed)."""
    b = B()
    wl, inp, dev = _inputs("layer8b", seq_lens=(20000,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs)
    w_tok, _ = b.rdkv_weights(cfg, dev["K"], dev["Q_obs"])          # warm-up: module load, staging ring
    b.rdkv_allocate(cfg, w_tok)
    torch.cuda.synchronize()
    blocker = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    ev = torch.cuda.Event()
    for _ in range(40):                                             # ~ tens of milliseconds of queued work
        blocker.add_(1.0)
    w_tok, _ = b.rdkv_weights(cfg, dev["K"], dev["Q_obs"])
    bits, _ = b.rdkv_allocate(cfg, w_tok)
    ev.record()
    returned_early = not ev.query()
    torch.cuda.synchronize()
    assert returned_early, "rdkv_weights / rdkv_allocate waited for the stream"
    ref = O.mckp_bisect(w_tok.cpu().numpy().reshape(wl.hkv, -1)[0], np.float32(inp["budgets"][0]))
    np.testing.assert_array_equal(bits.cpu().numpy().reshape(wl.hkv, -1)[0], ref)


@pytest.mark.parametrize("eps", [O.EPS_V_LLAMA31_8B, O.EPS_BENNETT])
def test_long_items_whose_weights_crowd_a_histogram_bucket(eps):
    """Items of 16K units and more run their streaming passes on many workgroups; the steps the weight histogram
    cannot decide are evaluated on a list of the still-undecided units.  Weights crowded into a narrow band defeat the
    histogram early: a list beyond its capacity (every step then reads every unit), a list that starts in device memory
    and shrinks into LDS as the bracket narrows, and an ordinary spread, side by side."""
    b = B()
    rng = np.random.default_rng(61)
    T = 50000
    w = np.empty((3, T), np.float32)
    w[0] = (1.0 + 1e-4 * rng.random(T)).astype(np.float32)                                   # all units in one bucket
    w[1] = np.concatenate([(3.0 + 3e-4 * rng.random(20000)), np.exp(rng.normal(0, 2, T - 20000))]).astype(np.float32)
    rng.shuffle(w[1])
    w[2] = np.exp(rng.normal(0, 2.0, T)).astype(np.float32)
    for budget in (0.7, 3.0):
        cfg = b.Config([T], 3, 3, budget_bits=[budget], eps_v=eps)
        print(f"[case] crowded weights budget={budget}", flush=True)
        bits, _, lam, iters = b.rdkv_allocate_info(cfg, torch.from_numpy(w.reshape(-1)).cuda())
        torch.cuda.synchronize()
        bits, lam, iters = bits.cpu().numpy().reshape(3, T), lam.cpu().numpy()[0], iters.cpu().numpy()[0]
        for h in range(3):
            rb, info = O.mckp_bisect(w[h], np.float32(budget), O.TIERS, eps, return_info=True)
            np.testing.assert_array_equal(bits[h], rb)
            assert iters[h] == info["iters"]
            assert (np.isnan(lam[h]) and info["lam"] is None) or lam[h] == info["lam"]


@pytest.mark.parametrize("batch", [1500, 3000])
def test_many_calls_in_a_row_reuse_the_staging_ring(batch):
    """The host tables of a call travel through a ring of pinned staging memory whose bytes are reused once the copy
    that read them has run.  Thousands of short sequences make the tables large (1500 sequences: 0.6 MB per call, the
    2 MB ring wraps after three calls; 3000 sequences: more than half the ring, the synchronous path) and the calls
    are queued without waiting in between; a sample of items of the last call is checked against the oracle."""
    b = B()
    hq, hkv, T, S_w = 8, 8, 40, 32
    rng = np.random.default_rng(71)
    K = torch.from_numpy(rng.standard_normal((batch, hkv, T, 128)).astype(np.float32)).to(torch.bfloat16).cuda()
    Q = torch.from_numpy(rng.standard_normal((batch, hq, S_w, 128)).astype(np.float32)).to(torch.bfloat16).cuda()
    budgets = [float(x) for x in rng.choice([0.5, 1.0, 2.0, 4.0], size=batch)]
    cfg = b.Config([T] * batch, hq, hkv, budget_bits=budgets, s_obs=S_w)
    print(f"[case] staging ring, {batch} sequences", flush=True)
    outs = []
    for _ in range(6):
        w, _ = b.rdkv_weights(cfg, K.reshape(-1), Q)
        bits, _ = b.rdkv_allocate(cfg, w)
        outs.append((w, bits))
    torch.cuda.synchronize()
    w, bits = outs[-1]
    for w2, bits2 in outs[:-1]:
        assert torch.equal(w, w2) and torch.equal(bits, bits2)
    w, bits = w.cpu().numpy().reshape(batch, hkv, T), bits.cpu().numpy().reshape(batch, hkv, T)
    Kc, Qc = K.float().cpu().numpy(), Q.float().cpu().numpy()
    for s in (0, 1, batch // 2, batch - 1):
        ref_w = O.avg_pool(O.token_weights(Kc[s], Qc[s]), 5)
        assert np.abs(w[s] - ref_w).max() <= 1e-5 * ref_w.max()
        for h in (0, hkv - 1):
            np.testing.assert_array_equal(bits[s, h], O.mckp_bisect(w[s, h], np.float32(budgets[s])))


def test_schedule_rebuilt_on_another_stream_than_the_one_that_packed():
    """The split workspace belongs to a stream: a cache packed on one stream, given a tail on a second and decoded on
    both must give the same (correct) result everywhere."""
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1500,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs)
    cache = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
    out0, lse0 = b.rdkv_decode_attn(cache, dev["q"])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        b.rdkv_cache_reserve_tail(cache, 64)                       # rebuilds the schedule, drops the workspaces
        out1, lse1 = b.rdkv_decode_attn(cache, dev["q"])
    side.synchronize()
    out2, lse2 = b.rdkv_decode_attn(cache, dev["q"])               # back on the first stream: a new workspace
    torch.cuda.synchronize()
    assert torch.equal(out0, out1) and torch.equal(out0, out2) and torch.equal(lse0, lse1) and torch.equal(lse0, lse2)
    cache.free()


def test_empty_and_degenerate_batches():
    """No sequences at all, sequences of zero length among others, a single token, and budgets of zero everywhere: every
    call returns, the outputs of items without retained tokens are 0 with lse = -inf, and appended tokens still count."""
    b = B()
    hq, hkv = 8, 2
    dev = "cuda"
    # no sequences
    cfg0 = b.Config([], hq, hkv, budget_bits=[])
    empty16 = torch.empty(0, dtype=torch.bfloat16, device=dev)
    cache = b.rdkv_pack(cfg0, empty16, empty16, torch.empty(0, dtype=torch.uint8, device=dev))
    st = cache.stats()
    assert st["n_items"] == 0 and st["stored_bytes"] == 0
    out, lse = b.rdkv_decode_attn(cache, torch.empty((0, hq, 128), dtype=torch.bfloat16, device=dev))
    assert out.numel() == 0
    cache.free()
    cache = b.rdkv_compress(cfg0, empty16, empty16, torch.empty((0, hq, 32, 128), dtype=torch.bfloat16, device=dev))
    cache.free()
    # sequences of length 0 and 1 beside an ordinary one (explicit maps: no probe needed)
    rng = np.random.default_rng(81)
    seq = [0, 1, 300]
    n_rows = sum(seq) * hkv
    K = torch.from_numpy(rng.standard_normal((n_rows, 128)).astype(np.float32)).to(torch.bfloat16).to(dev)
    V = torch.from_numpy(rng.standard_normal((n_rows, 128)).astype(np.float32)).to(torch.bfloat16).to(dev)
    q = torch.from_numpy(rng.standard_normal((3, hq, 128)).astype(np.float32)).to(torch.bfloat16).to(dev)
    bits = [np.zeros((hkv, 0), np.uint8), np.array([[4], [0]], np.uint8),
            rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(hkv, 300))]
    cfg = b.Config(seq, hq, hkv)
    cache = b.rdkv_pack(cfg, K.reshape(-1), V.reshape(-1), torch.from_numpy(np.concatenate([x.reshape(-1) for x in bits])).to(dev))
    out, lse = b.rdkv_decode_attn(cache, q)
    torch.cuda.synchronize()
    Kc, Vc = K.float().cpu().numpy(), V.float().cpu().numpy()
    Ks = [Kc[:0].reshape(hkv, 0, 128), Kc[:2].reshape(hkv, 1, 128), Kc[2:].reshape(hkv, 300, 128)]
    Vs = [Vc[:0].reshape(hkv, 0, 128), Vc[:2].reshape(hkv, 1, 128), Vc[2:].reshape(hkv, 300, 128)]
    ref = O.build_cache_tokenwise(Ks, Vs, bits)
    ref_out, ref_lse = O.decode(ref, q.float().cpu().numpy())
    from test_gpu_parity import _check_decode
    _check_decode(out, lse, ref_out, ref_lse)
    assert np.isneginf(lse.cpu().numpy()[0]).all() and not out[0].any()              # the empty sequence
    assert np.isneginf(lse.cpu().numpy()[1, hq // 2:]).all()                            # its second KV head evicted its token
    # appended tokens are attended to even where nothing of the prompt is left
    b.rdkv_cache_reserve_tail(cache, 4)
    kn = torch.from_numpy(rng.standard_normal((2, 3, hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    for i in range(2):
        b.rdkv_cache_append(cache, kn[i].to(dev), kn[1 - i].to(dev))
        O.append_tokens(ref, kn[i].float().numpy(), kn[1 - i].float().numpy())
    out, lse = b.rdkv_decode_attn(cache, q)
    torch.cuda.synchronize()
    ref_out, ref_lse = O.decode(ref, q.float().cpu().numpy())
    _check_decode(out, lse, ref_out, ref_lse)
    assert np.isfinite(lse.cpu().numpy()).all()
    cache.free()
    # a budget of zero: everything evicted by the pass itself
    seq = [64, 100]
    K = torch.from_numpy(rng.standard_normal((sum(seq) * hkv, 128)).astype(np.float32)).to(torch.bfloat16).to(dev)
    Q = torch.from_numpy(rng.standard_normal((2, hq, 32, 128)).astype(np.float32)).to(torch.bfloat16).to(dev)
    cache = b.rdkv_compress(b.Config(seq, hq, hkv, budget_bits=[0.0, 0.0]), K.reshape(-1), K.reshape(-1), Q)
    st = cache.stats()
    assert st["stored_bytes"] == 0 and st["evicted"] == sum(seq) * hkv
    out, lse = b.rdkv_decode_attn(cache, q[:2].contiguous())
    torch.cuda.synchronize()
    assert not out.any() and np.isneginf(lse.cpu().numpy()).all()
    cache.free()
