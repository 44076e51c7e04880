"""The decode entry points under HIP graph capture (the launch configuration bench.py times): a captured decode is
replayed several times with eager work and synchronisations in between, and every replay must reproduce the eager
result bit for bit (the kernels are deterministic: fixed summation orders, no atomics)."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from test_gpu_parity import B, _inputs, _pack_both, _check_decode, _np
from test_gpu_mixed import _pack_both_mixed, _random_maps

pytestmark = pytest.mark.gpu


def _replay_equals_eager(b, cache, q, other_cache=None):
    out_e, lse_e = b.rdkv_decode_attn(cache, q)
    torch.cuda.synchronize()
    out_g, lse_g = torch.empty_like(out_e), torch.empty_like(lse_e)
    b.rdkv_decode_attn(cache, q, out_g, lse_g)              # warm-up on the capture stream's allocator state
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        b.rdkv_decode_attn(cache, q, out_g, lse_g)
    for i in range(4):
        out_g.fill_(float("nan"))
        lse_g.fill_(float("nan"))
        if other_cache is not None:                           # eager work of the same library between the replays
            b.rdkv_decode_attn(other_cache, q)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), f"replay {i} differs from the eager result"
        assert torch.equal(lse_g, lse_e)


def test_graph_replay_tokenwise_with_16_bit_rows_and_a_tail():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(2500,))
    rng = np.random.default_rng(31)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.3, .25, .2, .15, .1])
            for T in inp["seq_lens"]]
    cache, _ = _pack_both(b, wl, inp, dev, bits)
    other, _ = _pack_both(b, wl, inp, dev, [np.full_like(bits[0], 4)])
    b.rdkv_cache_reserve_tail(cache, 64)
    kn = torch.randn((1, wl.hkv, 128), device="cuda").to(torch.bfloat16)
    for _ in range(5):
        b.rdkv_cache_append(cache, kn, kn)
    _replay_equals_eager(b, cache, dev["q"], other)
    cache.free()
    other.free()


def test_graph_replay_mixed():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1800,))
    bt, bc = _random_maps(np.random.default_rng(32), inp["seq_lens"], wl.hkv, [.3, .3, .2, .1, .1], [.1, .4, .3, .15, .05])
    cache, _ = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    _replay_equals_eager(b, cache, dev["q"])
    cache.free()


def test_graph_replay_bf16_path():
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(3000,))
    ws = torch.empty(b.rdkv_decode_bf16_workspace_bytes(inp["seq_lens"], wl.hq, wl.hkv), dtype=torch.uint8, device="cuda")
    out_e, lse_e = b.rdkv_decode_attn_bf16(dev["K"], dev["V"], inp["seq_lens"], wl.hq, wl.hkv, dev["q"], workspace=ws)
    torch.cuda.synchronize()
    out_g, lse_g = torch.empty_like(out_e), torch.empty_like(lse_e)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        b.rdkv_decode_attn_bf16(dev["K"], dev["V"], inp["seq_lens"], wl.hq, wl.hkv, dev["q"], out=out_g, lse=lse_g,
                                workspace=ws)
    for i in range(3):
        out_g.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e) and torch.equal(lse_g, lse_e), f"replay {i} differs"


def test_graph_recaptured_after_rebudget():
    """Re-budgeting replaces the decode schedule: a graph captured afterwards must replay the new schedule (prompt
    zones, the absorbed generation and the tokens appended since)."""
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1500,))
    rng = np.random.default_rng(33)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.4, .25, .2, .15, .0])
            for T in inp["seq_lens"]]
    cache, _ = _pack_both(b, wl, inp, dev, bits)
    other, _ = _pack_both(b, wl, inp, dev, [np.full_like(bits[0], 2)])
    b.rdkv_cache_reserve_tail(cache, 128)
    kn = torch.randn((100, 1, wl.hkv, 128), device="cuda").to(torch.bfloat16)
    for i in range(96):
        b.rdkv_cache_append(cache, kn[i], kn[99 - i])
    Q = torch.randn((1, wl.hq, 32, 128), device="cuda").to(torch.bfloat16)
    b.rdkv_cache_rebudget_tail(cache, b.Config([96], wl.hq, wl.hkv, budget_bits=[3.0], s_obs=32), Q)
    for i in range(96, 100):
        b.rdkv_cache_append(cache, kn[i], kn[99 - i])
    _replay_equals_eager(b, cache, dev["q"], other)
    cache.free()
    other.free()


@pytest.mark.parametrize("mixed", [False, True])
def test_one_graph_of_append_and_decode_replays_across_a_generation_loop(mixed):
    """The appended-token count lives in device memory: a graph that captured rdkv_cache_append followed by
    rdkv_decode_attn is replayed token after token, with new rows and a new query in the same buffers, and every
    replay must see all tokens appended so far (third term of Eq. 7)."""
    b = B()
    wl, inp, dev = _inputs("tiny", seq_lens=(1300,))
    rng = np.random.default_rng(41)
    if mixed:
        bt, bc = _random_maps(rng, inp["seq_lens"], wl.hkv, [.4, .3, .2, .05, .05], [.1, .4, .3, .15, .05])
        cache, ref = _pack_both_mixed(b, wl, inp, dev, bt, bc)
    else:
        bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(wl.hkv, T), p=[.4, .25, .2, .1, .05])
                for T in inp["seq_lens"]]
        cache, ref = _pack_both(b, wl, inp, dev, bits)
    n_new = 300                                                  # crosses a 256-token chunk of the tail
    b.rdkv_cache_reserve_tail(cache, n_new + 5)
    kn = torch.from_numpy(rng.standard_normal((n_new, 1, wl.hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    vn = torch.from_numpy(rng.standard_normal((n_new, 1, wl.hkv, 128)).astype(np.float32)).to(torch.bfloat16)
    qn = torch.from_numpy(rng.standard_normal((n_new, 1, wl.hq, 128)).astype(np.float32)).to(torch.bfloat16)
    kd, vd, qd = kn.cuda(), vn.cuda(), qn.cuda()
    kbuf, vbuf, qbuf = kd[0].clone(), vd[0].clone(), qd[0].clone()
    out_g = torch.empty((1, wl.hq, 128), dtype=torch.float32, device="cuda")
    lse_g = torch.empty((1, wl.hq), dtype=torch.float32, device="cuda")
    b.rdkv_cache_append(cache, kbuf, vbuf)                       # token 0 eagerly (also the warm-up)
    b.rdkv_decode_attn(cache, qbuf, out_g, lse_g)
    O.append_tokens(ref, kn[0].float().numpy(), vn[0].float().numpy())
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        b.rdkv_cache_append(cache, kbuf, vbuf)
        b.rdkv_decode_attn(cache, qbuf, out_g, lse_g)
    for i in range(1, n_new):
        kbuf.copy_(kd[i]); vbuf.copy_(vd[i]); qbuf.copy_(qd[i])
        g.replay()
        O.append_tokens(ref, kn[i].float().numpy(), vn[i].float().numpy())
        if i in (1, 2, 63, 64, 255, 256, n_new - 1):
            torch.cuda.synchronize()
            print(f"[step] replay after {i + 1} appended tokens", flush=True)
            ref_out, ref_lse = O.decode(ref, _np(qn[i]))
            _check_decode(out_g, lse_g, ref_out, ref_lse)
    torch.cuda.synchronize()
    assert b.rdkv_cache_tail_len_sync(cache) == n_new == b.rdkv_cache_tail_len(cache)
    cache.free()


def test_decode_steps_on_two_streams_may_overlap():
    """Every stream gets its own split workspace, so two streams can decode from one cache at once: many steps are
    queued on both streams before anything is awaited, and each stream's results must equal the serial ones."""
    b = B()
    wl, inp, dev = _inputs("layer8b", seq_lens=(20000,))
    cfg = b.Config(inp["seq_lens"], wl.hq, wl.hkv, budget_bits=inp["budgets"], s_obs=wl.s_obs)
    cache = b.rdkv_compress(cfg, dev["K"], dev["V"], dev["Q_obs"])
    rng = torch.Generator(device="cuda").manual_seed(5)
    qs = [torch.randn((1, wl.hq, 128), device="cuda", generator=rng).to(torch.bfloat16) for _ in range(2)]
    want = [b.rdkv_decode_attn(cache, q)[0].clone() for q in qs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [[torch.empty_like(want[0]) for _ in range(50)] for _ in range(2)]
    for k, st in enumerate(streams):                              # first use of each stream: its workspace is created
        with torch.cuda.stream(st):
            b.rdkv_decode_attn(cache, qs[k], outs[k][0])
    torch.cuda.synchronize()
    for i in range(50):
        for k, st in enumerate(streams):
            with torch.cuda.stream(st):
                b.rdkv_decode_attn(cache, qs[k], outs[k][i])
    torch.cuda.synchronize()
    for k in range(2):
        for i in range(50):
            assert torch.equal(outs[k][i], want[k]), f"stream {k} step {i} differs from the serial result"
    cache.free()
