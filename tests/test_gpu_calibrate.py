"""GPU parity of the distortion-table calibration (App. B "Calibration", App. "Calibrated Distortion Tables"): the library's per-slice eps(b),
b = 2, 4, 8, against the fp64 oracle on the same K and V.  Both sides take every rounding decision (codes, fp16 scale
and offset) in the same fp32 operations, and errors are summed in fp64 on both, so the only difference is the order of
the additions: relative tolerance 1e-10."""
import numpy as np
import pytest
import torch

from oracle import rdkv_oracle as O
from paper_2605_08317_amd import workloads as W
from test_gpu_parity import B

pytestmark = pytest.mark.gpu
TOL = 1e-10
MODES = {"tokenwise": {}, "channelwise": {"k_channelwise": True},
         "channelwise_whole": {"k_channelwise": True, "k_per_channel_scale": True}}


def _config(b, seq_lens, hq, hkv, mode):
    kw = {}
    if mode != "tokenwise":
        kw["k_mode"] = b.RDKV_K_CHANNELWISE
    if mode == "channelwise_whole":
        kw["k_scale_per_channel"] = 1
    return b.Config(seq_lens, hq, hkv, **kw)


def _data(seq_lens, hkv, seed, outliers=True):
    rng = np.random.default_rng(seed)
    Ks, Vs = [], []
    for T in seq_lens:
        k = rng.standard_normal((hkv, T, 128)).astype(np.float32)
        if outliers:
            k[:, :, rng.choice(128, 6, replace=False)] *= 10.0    # a few heavy K channels, as in the workloads
        v = (rng.standard_normal((hkv, T, 128)) * rng.uniform(0.2, 3.0, (hkv, T, 1))).astype(np.float32)
        Ks.append(torch.from_numpy(k).to(torch.bfloat16))
        Vs.append(torch.from_numpy(v).to(torch.bfloat16))
    return Ks, Vs


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("seq_lens,hkv", [((300,), 2), ((1, 33, 1000, 256, 31), 2), ((2049,), 1)])
def test_calibration_matches_oracle(mode, seq_lens, hkv):
    b = B()
    print(f"[case] calibrate {mode} seq_lens={seq_lens} hkv={hkv}", flush=True)
    Ks, Vs = _data(seq_lens, hkv, 31)
    Kd = torch.cat([k.reshape(-1) for k in Ks]).cuda()
    Vd = torch.cat([v.reshape(-1) for v in Vs]).cuda()
    ek, ev = b.rdkv_calibrate_eps(_config(b, list(seq_lens), 4 * hkv, hkv, mode), Kd, Vd)
    rk, rv = O.calibrate_eps([k.float().numpy() for k in Ks], [v.float().numpy() for v in Vs], **MODES[mode])
    assert ek.shape == rk.shape and ev.shape == rv.shape
    np.testing.assert_allclose(ek, rk, rtol=TOL, atol=0)
    np.testing.assert_allclose(ev, rv, rtol=TOL, atol=0)
    assert (ev > 0).all()                                   # (a one-token channel group is exact: eps_k may be 0)


def test_calibration_degenerate_and_grid_data():
    b = B()
    # all-zero and constant slices report exactly 0 in every format
    Z = torch.zeros(2 * 70 * 128, dtype=torch.bfloat16, device="cuda")
    C = torch.full((2 * 70 * 128,), 1.5, dtype=torch.bfloat16, device="cuda")
    for mode in MODES:
        for X in (Z, C):
            ek, ev = b.rdkv_calibrate_eps(_config(b, [70], 2, 2, mode), X, X)
            assert not ek.any() and not ev.any()
    # grid data (every inner element a quarter step off its code): the closed form of the oracle's pin
    rng = np.random.default_rng(5)
    s = 2.0 ** -7
    for bi, bits in enumerate((2, 4, 8)):
        Q = (1 << bits) - 1
        X = np.zeros((64, 4, 32), dtype=np.float32)
        for a in range(64):
            for g in range(4):
                inner = rng.choice(np.arange(1, min(Q, 64)), 30) + rng.choice([-0.25, 0.25], 30)
                X[a, g] = rng.permutation(np.concatenate([[0.0], s * inner, [s * Q]]))
        want = 64 * 4 * 30 * (s / 4) ** 2 / float((X.astype(np.float64) ** 2).sum())
        Xd = torch.from_numpy(X.reshape(-1)).to(torch.bfloat16).cuda()
        assert torch.equal(Xd.float().cpu(), torch.from_numpy(X.reshape(-1)))
        ek, ev = b.rdkv_calibrate_eps(_config(b, [64], 1, 1, "tokenwise"), Xd, Xd)
        assert ek[0, bi] == pytest.approx(want, rel=1e-12) and ev[0, bi] == pytest.approx(want, rel=1e-12)


def test_calibration_argument_errors():
    b = B()
    X = torch.zeros(128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RuntimeError):
        b.rdkv_calibrate_eps(b.Config([0], 1, 1), X, X)            # no token to calibrate on
    with pytest.raises(RuntimeError):
        b.rdkv_calibrate_eps(b.Config([1], 1, 1, head_dim=64), X, X)
    ek, ev = b.rdkv_calibrate_eps(b.Config([], 1, 1), X, X)        # empty batch: nothing to do
    assert ek.shape == (0, 3)


@pytest.mark.parametrize("mode,T", [("tokenwise", 131072), ("channelwise_whole", 131072), ("channelwise", 16384)])
def test_calibration_at_scale(mode, T):
    """One layer of the 128K-token workload (8 KV heads); the oracle recomputes one sampled head.  The 32-token
    channel groups take the oracle a Python loop per group, so that format is checked at 16K tokens."""
    b = B()
    wl = W.scaled(W.CONFIGS["stack128k"], seq_lens=(T,))
    print(f"[case] calibrate at scale {mode} T={T}", flush=True)
    inp = W.make_inputs(wl, device="cuda")
    ek, ev = b.rdkv_calibrate_eps(_config(b, [T], wl.hq, wl.hkv, mode), inp["K"], inp["V"])
    h = 5
    Kh = inp["K"].view(wl.hkv, T, 128)[h].float().cpu().numpy()[None]
    Vh = inp["V"].view(wl.hkv, T, 128)[h].float().cpu().numpy()[None]
    rk, rv = O.calibrate_eps([Kh], [Vh], **MODES[mode])
    np.testing.assert_allclose(ek[h], rk[0], rtol=TOL, atol=0)
    np.testing.assert_allclose(ev[h], rv[0], rtol=TOL, atol=0)
    print(f"[calibrate] eps_k mean {ek.mean(axis=0)} eps_v mean {ev.mean(axis=0)}", flush=True)
