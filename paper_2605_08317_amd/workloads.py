"""Seeded synthetic inputs shaped like the paper's long-context runs.

This module only draws random tensors; it holds none of the method's
arithmetic, so both the tests' CPU checker and the HIP library can be fed from
it.  The tensors stand in for prefill K/V caches and probe queries of
LLaMA-3.1-8B-shaped layers (Hq=32, Hkv=8, d=128): the real prompts, models and
calibration prefixes are not available and are not reconstructed.

All values are bf16.  K/V of a ragged batch are one flat tensor holding, per
sequence in batch order, a block [Hkv][T_s][d].
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int = 1
    hq: int = 8
    hkv: int = 2
    d: int = 128
    seq_lens: tuple = (4096,)          # fixed lengths; or use len_range
    len_range: Optional[tuple] = None  # (lo, hi): T_s ~ U{lo..hi} per sequence
    s_obs: int = 32
    outlier_channels: int = 0          # key channels per head scaled x10
    sink_frac: float = 0.0             # fraction of positions that are attention sinks
    sink_gain: float = 9.5
    budgets: tuple = (2.0,)            # avg bits/element per sequence, or choices if draw_budgets
    draw_budgets: bool = False
    pareto_weights: bool = False       # supply w_t ~ 1 + Pareto(1.2) instead of computing it
    k_channelwise: bool = False
    layers: int = 1
    seed_base: int = 0


CONFIGS = {
    # the five benchmark configurations; seed = 1000 * config number + layer
    "tiny": Workload("tiny", 1, 8, 2, 128, (4096,), None, 32, 4, 0.0, 9.5, (2.0,), seed_base=1000),
    "layer8b": Workload("layer8b", 1, 32, 8, 128, (32768,), None, 32, 3, 0.0, 9.5, (1.0,), seed_base=2000),
    "stack128k": Workload("stack128k", 1, 32, 8, 128, (131072,), None, 64, 0, 0.01, 9.5, (0.4,),
                          layers=32, seed_base=3000),
    "batch70b": Workload("batch70b", 16, 64, 8, 128, (), (8192, 32768), 32, 3, 0.0, 9.5,
                         (0.5, 1.0, 2.0, 4.0), draw_budgets=True, seed_base=4000),
    "mixed": Workload("mixed", 1, 32, 8, 128, (65536,), None, 32, 3, 0.0, 9.5, (1.0,),
                      pareto_weights=True, k_channelwise=True, seed_base=5000),
}


def scaled(wl: Workload, **kw) -> Workload:
    """The same recipe at other sizes (parity tests use shorter contexts)."""
    return replace(wl, **kw)


def _randn_bf16(shape, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)


def make_inputs(wl: Workload, device="cpu", layer: int = 0, want_v: bool = True):
    """Draw one layer's inputs.  Returns a dict:
      seq_lens  list[int]
      budgets   list[float]                       avg bits per element, per sequence
      K, V      bf16 flat [sum_s Hkv*T_s*d]       (V omitted when want_v is False)
      Q_obs     bf16 [batch, Hq, s_obs, d]        probe (observation-window) queries
      q         bf16 [batch, Hq, d]               the decode query
      w_tok     fp32 flat [sum_s Hkv*T_s] or None supplied token weights (Pareto)
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed_base + layer)
    cpu_gen = torch.Generator(device="cpu")
    cpu_gen.manual_seed(wl.seed_base + layer + 7919)

    if wl.len_range is not None:
        lo, hi = wl.len_range
        seq_lens = [int(x) for x in torch.randint(lo, hi + 1, (wl.batch,), generator=cpu_gen)]
    else:
        seq_lens = list(wl.seq_lens)
        assert len(seq_lens) == wl.batch
    if wl.draw_budgets:
        pick = torch.randint(0, len(wl.budgets), (wl.batch,), generator=cpu_gen)
        budgets = [float(wl.budgets[int(i)]) for i in pick]
    else:
        budgets = [float(wl.budgets[i % len(wl.budgets)]) for i in range(wl.batch)]

    d, hkv, hq = wl.d, wl.hkv, wl.hq
    g = hq // hkv
    Q_obs = _randn_bf16((wl.batch, hq, wl.s_obs, d), gen, dev)
    q = _randn_bf16((wl.batch, hq, d), gen, dev)
    Ks, Vs, Ws = [], [], []
    for s, T in enumerate(seq_lens):
        K = torch.randn((hkv, T, d), generator=gen, device=dev, dtype=torch.float32)
        if wl.outlier_channels:
            for h in range(hkv):
                ch = torch.randperm(d, generator=cpu_gen)[: wl.outlier_channels].to(dev)
                K[h, :, ch] *= 10.0
        if wl.sink_frac > 0.0:
            n_sink = max(1, int(round(wl.sink_frac * T)))
            for h in range(hkv):
                u = torch.randn((d,), generator=gen, device=dev, dtype=torch.float32)
                u = u / u.norm()
                pos = torch.randperm(T - 1, generator=cpu_gen)[: n_sink - 1] + 1
                pos = torch.cat([torch.zeros(1, dtype=pos.dtype), pos]).to(dev)
                K[h, pos] += wl.sink_gain * u
                Q_obs[s, h * g:(h + 1) * g] = (Q_obs[s, h * g:(h + 1) * g].float()
                                               + wl.sink_gain * u).to(torch.bfloat16)
                q[s, h * g:(h + 1) * g] = (q[s, h * g:(h + 1) * g].float()
                                           + wl.sink_gain * u).to(torch.bfloat16)
        Ks.append(K.to(torch.bfloat16).reshape(-1))
        del K
        if want_v:
            Vs.append(_randn_bf16((hkv * T * d,), gen, dev))
        if wl.pareto_weights:
            # 1 + Pareto(alpha = 1.2): (1 - U)^(-1/alpha) is Pareto with x_m = 1
            uu = torch.rand((hkv * T,), generator=gen, device=dev, dtype=torch.float32)
            Ws.append(1.0 + (1.0 - uu).clamp_min(1e-12).pow(-1.0 / 1.2))
    out = {
        "seq_lens": seq_lens,
        "budgets": budgets,
        "K": torch.cat(Ks),
        "Q_obs": Q_obs,
        "q": q,
        "w_tok": torch.cat(Ws) if Ws else None,
    }
    if want_v:
        out["V"] = torch.cat(Vs)
    return out


def split_sequences(flat, seq_lens, hkv, d):
    """Views [Hkv, T_s, d] (or [Hkv, T_s] when d is None) of a flat ragged tensor."""
    views, off = [], 0
    for T in seq_lens:
        n = hkv * T * (d if d else 1)
        shape = (hkv, T, d) if d else (hkv, T)
        views.append(flat[off:off + n].view(shape))
        off += n
    return views
