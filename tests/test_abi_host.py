"""Host-only checks of the C ABI: the shared library loads, exports every symbol
include/rdkv.h declares, and rejects bad arguments before anything is launched
(no compute call reaches a GPU here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_08317_amd", "librdkv.so")


@pytest.fixture(scope="module")
def b():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    from paper_2605_08317_amd import binding
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "rdkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(rdkv_[a-z0-9_]+)\s*\(", text))
    return sorted(n for n in names if not n.endswith("_fn"))


def test_library_exports_every_declared_symbol(b):
    declared = _declared_functions()
    assert len(declared) >= 14
    for name in declared:
        assert hasattr(b.lib, name), f"{name} is declared in rdkv.h but not exported"
    assert sorted(b.EXPORTED_SYMBOLS) == declared
    assert "gfx950" in b.rdkv_version()


def test_config_default_matches_paper_constants(b):
    cfg = b.Config([4096], 8, 2)
    c = cfg.c
    assert (c.s_obs, c.pool_kernel, c.causal, c.group_size, c.max_iters) == (32, 5, 1, 32, 64)
    assert list(c.tiers) == [0, 2, 4, 8, 16] and c.n_tiers == 5
    assert c.rel_tol == pytest.approx(1e-2) and c.kv_split_rk == 0.5
    # Table 9, LLaMA-3.1-8B row (tests/golden/table9_eps.txt)
    row = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "table9_eps.txt")) if l.startswith("LLaMA-3.1-8B")][0]
    assert [c.eps_k[i] for i in (1, 2, 3)] == pytest.approx([float(x) for x in row[1:4]], rel=1e-6)
    assert [c.eps_v[i] for i in (1, 2, 3)] == pytest.approx([float(x) for x in row[4:7]], rel=1e-6)
    assert c.eps_v[0] == 1.0 and c.eps_v[4] == 0.0 and c.eps_k[0] == 1.0 and c.eps_k[4] == 0.0


def _pack_status(b, cfg):
    h = ctypes.c_void_p(1234)
    st = b.lib.rdkv_pack(cfg.ref(), None, None, None, None, None, ctypes.byref(h))
    return st, h.value, b.lib.rdkv_last_error().decode()


def test_shape_errors_are_reported_before_any_launch(b):
    st, h, msg = _pack_status(b, b.Config([100], 8, 2, head_dim=64))
    assert st == 2 and h is None and "head_dim" in msg
    st, h, msg = _pack_status(b, b.Config([100], 7, 2))
    assert st == 2 and "multiple" in msg
    st, h, msg = _pack_status(b, b.Config([100], 32, 2))          # g = 16
    assert st == 2
    st, h, msg = _pack_status(b, b.Config([-5], 8, 2))
    assert st == 2 and "negative" in msg
    st, h, msg = _pack_status(b, b.Config([100], 8, 2, group_size=64))
    assert st == 2 and "group_size" in msg
    st, h, msg = _pack_status(b, b.Config([100], 8, 2))           # null K/V/bits with tokens to pack
    assert st == 1 and h is None
    assert b.lib.rdkv_pack(None, None, None, None, None, None, ctypes.byref(ctypes.c_void_p())) == 1


def test_allocate_and_compress_argument_checks(b):
    null = None
    cfg = b.Config([100], 8, 2)                                    # no budgets
    assert b.lib.rdkv_allocate(cfg.ref(), null, null, null, null, null) == 1
    cfg = b.Config([100], 8, 2, budget_bits=[-1.0])
    assert b.lib.rdkv_allocate(cfg.ref(), null, null, null, null, null) == 1
    cfg = b.Config([100], 8, 2, budget_bits=[1.0], tiers=[0, 4, 2])
    assert b.lib.rdkv_allocate(cfg.ref(), null, null, null, null, null) == 1
    cfg = b.Config([100], 8, 2, budget_bits=[1.0], tiers=[0, 3, 16])
    assert b.lib.rdkv_allocate(cfg.ref(), null, null, null, null, null) == 1
    cfg = b.Config([100], 8, 2, budget_bits=[1.0], max_iters=0)
    assert b.lib.rdkv_allocate(cfg.ref(), null, null, null, null, null) == 1
    cfg = b.Config([100], 8, 2, budget_bits=[1.0])                  # valid config, null buffers
    assert b.lib.rdkv_allocate(cfg.ref(), null, null, null, null, null) == 1
    h = ctypes.c_void_p()
    cfg = b.Config([20], 8, 2, budget_bits=[1.0])                   # shorter than the observation window
    assert b.lib.rdkv_compress(cfg.ref(), null, null, null, null, ctypes.byref(h)) == 2 and h.value is None
    cfg = b.Config([100], 8, 2, budget_bits=[1.0], pool_kernel=4)
    assert b.lib.rdkv_weights(cfg.ref(), null, null, null, null, null) == 1
    cfg = b.Config([100], 8, 2, budget_bits=[1.0], s_obs=65)
    assert b.lib.rdkv_weights(cfg.ref(), null, null, null, null, null) == 2


def test_decode_argument_checks_and_workspace_size(b):
    assert b.lib.rdkv_decode_attn(None, None, None, None, None) == 1
    seq = (ctypes.c_int32 * 1)(4096)
    assert b.lib.rdkv_decode_attn_bf16(None, None, seq, 1, 8, 2, 128, None, None, None, None, 0, None) == 1
    assert b.lib.rdkv_decode_attn_bf16(None, None, seq, 1, 8, 2, 64, None, None, None, None, 0, None) == 2
    assert b.rdkv_decode_bf16_workspace_bytes([4096], 8, 2) > 0
    assert b.rdkv_decode_bf16_workspace_bytes([4096], 8, 2, head_dim=64) == 0
    assert b.lib.rdkv_cache_export_bytes(None, 0) == 0
    assert b.lib.rdkv_cache_stats(None, None) == 1
    b.lib.rdkv_cache_free(None)                                     # a null handle is a no-op
    n, ms = ctypes.c_int64(), ctypes.c_double()
    assert b.lib.rdkv_kernel_timing_read(99, ctypes.byref(n), ctypes.byref(ms)) == 1
    assert b.lib.rdkv_kernel_timing_read(0, ctypes.byref(n), ctypes.byref(ms)) == 0 and n.value == 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in p.stderr


def test_calibration_and_rebudget_argument_checks(b):
    null = None
    cfg = b.Config([100], 8, 2)
    assert b.lib.rdkv_calibrate_eps(None, null, null, null, null, null) == 1           # no config
    assert b.lib.rdkv_calibrate_eps(cfg.ref(), null, null, null, null, null) == 1      # null K / V / outputs
    assert b.lib.rdkv_calibrate_eps(b.Config([100], 8, 2, head_dim=64).ref(), null, null, null, null, null) == 2
    assert b.lib.rdkv_calibrate_eps(b.Config([100], 8, 2, k_mode=7).ref(), null, null, null, null, null) == 1
    assert b.lib.rdkv_cache_rebudget_tail(None, cfg.ref(), null, null) == 1            # no cache
    assert b.lib.rdkv_cache_generations(None) == 0
    assert b.lib.rdkv_cache_generation(None, 0) is None
    assert b.lib.rdkv_cache_tail_len(None) == 0
    assert b.lib.rdkv_cache_reserve_tail(None, 16, null) == 1
    assert b.lib.rdkv_cache_append(None, null, null, null) == 1
    assert "null" in b.lib.rdkv_last_error().decode() or b.lib.rdkv_last_error().decode() != ""


def test_ctypes_structs_match_the_c_header(b, tmp_path):
    """The binding's ctypes mirror of rdkv_config / rdkv_stats against the header compiled as plain C."""
    import subprocess
    cfg_fields = [f[0] for f in b.rdkv_config._fields_]
    st_fields = [f[0] for f in b.rdkv_stats._fields_]
    src = tmp_path / "layout.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "rdkv.h"', 'int main(void) {',
             '  printf("%zu %zu\\n", sizeof(rdkv_config), sizeof(rdkv_stats));']
    lines += [f'  printf("%zu\\n", offsetof(rdkv_config, {f}));' for f in cfg_fields]
    lines += [f'  printf("%zu\\n", offsetof(rdkv_stats, {f}));' for f in st_fields]
    lines += ['  return 0;', '}']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(out[0]), int(out[1])] == [ctypes.sizeof(b.rdkv_config), ctypes.sizeof(b.rdkv_stats)]
    want = [getattr(b.rdkv_config, f).offset for f in cfg_fields] + [getattr(b.rdkv_stats, f).offset for f in st_fields]
    assert [int(x) for x in out[2:]] == want


def test_every_channel_bit_map_fits_the_widest_k_row_kernel(b):
    """A channel-wise K row is longest with 125 channels at 16 bits and one each at 8, 4 and 2 (every segment pays its
    padding): 64 + 1 + 1 + 1 words, evened to 68.  The decode kernel's widest instantiation must hold it; the
    library's own row-shape function is swept over every combination of tier counts."""
    import numpy as np
    widest = b.lib.rdkv_k_row_words_max()

    def words(n16, n8, n4, n2):
        m = np.zeros(128, np.uint8)
        m[:n16] = 16
        m[n16:n16 + n8] = 8
        m[n16 + n8:n16 + n8 + n4] = 4
        m[n16 + n8 + n4:n16 + n8 + n4 + n2] = 2
        return b.lib.rdkv_k_row_words(m.ctypes.data_as(ctypes.c_void_p))

    # hand-computed shapes: ceil4(n16)/2 + ceil(n8/4) + ceil(n4/8) + ceil(n2/16), evened
    assert words(128, 0, 0, 0) == 64
    assert words(125, 1, 1, 1) == 68
    assert words(126, 2, 0, 0) == 66
    assert words(0, 0, 0, 128) == 8
    assert words(0, 0, 0, 0) == 0
    assert words(1, 0, 0, 0) == 2
    assert words(0, 37, 0, 91) == 10 + 6
    worst = 0
    for n16 in range(0, 129):
        for n8 in range(0, 129 - n16, 1 if n16 > 100 else 7):
            for n4 in range(0, 129 - n16 - n8, 1 if n16 > 100 else 5):
                rest = 128 - n16 - n8 - n4
                for n2 in {rest, max(rest - 1, 0), min(rest, 1)}:
                    worst = max(worst, words(n16, n8, n4, n2))
    assert worst == 68 and worst <= widest
    bad = np.full(128, 3, np.uint8)
    assert b.lib.rdkv_k_row_words(bad.ctypes.data_as(ctypes.c_void_p)) == -1
    assert b.lib.rdkv_k_row_words(None) == -1


def test_cache_max_bytes_is_the_budget_bound(b):
    """kept tokens <= floor(avg * T) / 2 and 2 (16 b + 16) bytes per kept row (Sec. 3.2 budget bookkeeping): the bound
    is linear in the budget until every row sits at 16 bits, never below what the budget can buy, and 0 for a bad
    config."""
    T, hkv = 10000, 2
    pad = 63 * 2 * (256 + 144 + 80 + 48) + 16 * 256                 # padding rows of four tiers + segment alignment
    got = b.rdkv_cache_max_bytes(b.Config([T], 8, hkv, budget_bits=[1.0]))
    assert got == hkv * (32 * T + 32 * (T // 2) + pad) + 256          # 10000 bits: 5000 rows at 2 bits at most
    all16 = b.rdkv_cache_max_bytes(b.Config([T], 8, hkv, budget_bits=[16.0]))
    assert all16 == hkv * (512 * T + pad) + 256
    assert b.rdkv_cache_max_bytes(b.Config([T], 8, hkv, budget_bits=[40.0])) == all16
    assert b.rdkv_cache_max_bytes(b.Config([T], 8, hkv, budget_bits=[0.0])) == hkv * pad + 256
    # evict-only tier set {0, 16}: a kept row costs 16 bits, so at most B / 16 rows
    evict_only = b.rdkv_cache_max_bytes(b.Config([T], 8, hkv, budget_bits=[1.0], tiers=[0, 16], eps_v=[1.0, 0.0], eps_k=[1.0, 0.0]))
    assert evict_only == hkv * (32 * T + 32 * (T // 16) + pad) + 256
    two = b.rdkv_cache_max_bytes(b.Config([T, 300], 8, hkv, budget_bits=[1.0, 2.0]))
    assert two == got - 256 + hkv * (32 * 600 + 32 * 300 + pad) + 256
    assert b.rdkv_cache_max_bytes(b.Config([T], 8, hkv)) == 0         # no budgets
    assert b.lib.rdkv_cache_max_bytes(None) == 0
    mixed = b.rdkv_cache_max_bytes(b.Config([T], 8, hkv, budget_bits=[1.0], k_mode=b.RDKV_K_CHANNELWISE))
    assert 0 < mixed < all16
