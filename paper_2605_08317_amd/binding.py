"""Thin ctypes binding of librdkv (include/rdkv.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the
shared library.  PyTorch supplies device memory and streams.  There is no CPU
fallback: if the library is missing or fails to load, importing this module
raises.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librdkv.so")

RDKV_OK = 0
RDKV_K_TOKENWISE, RDKV_K_CHANNELWISE = 0, 1
(RDKV_EXPORT_COUNTS, RDKV_EXPORT_TIER_IDX, RDKV_EXPORT_SEG_OFF, RDKV_EXPORT_ARENA,
 RDKV_EXPORT_BITS_TOK, RDKV_EXPORT_BITS_CH, RDKV_EXPORT_LAMBDA, RDKV_EXPORT_ITERATIONS) = range(8)
STATUS_NAMES = {0: "RDKV_OK", 1: "RDKV_ERR_INVALID_ARG", 2: "RDKV_ERR_SHAPE", 3: "RDKV_ERR_UNSUPPORTED",
                4: "RDKV_ERR_ALLOC", 5: "RDKV_ERR_HIP", 6: "RDKV_ERR_INTERNAL"}

EXPORTED_SYMBOLS = [
    "rdkv_version", "rdkv_last_error", "rdkv_config_default", "rdkv_weights", "rdkv_allocate", "rdkv_allocate_info", "rdkv_pack", "rdkv_cache_max_bytes", "rdkv_cache_max_table_bytes",
    "rdkv_compress", "rdkv_decode_attn", "rdkv_decode_bf16_workspace_bytes", "rdkv_decode_attn_bf16",
    "rdkv_decode_bf16_noalloc_max_bytes", "rdkv_decode_attn_bf16_noalloc",
    "rdkv_cache_reserve_tail", "rdkv_cache_append", "rdkv_cache_tail_len", "rdkv_cache_tail_len_sync", "rdkv_calibrate_eps",
    "rdkv_cache_rebudget_tail", "rdkv_cache_generations", "rdkv_cache_generation",
    "rdkv_cache_stats", "rdkv_cache_export_bytes", "rdkv_cache_export", "rdkv_cache_free",
    "rdkv_kernel_timing_enable", "rdkv_kernel_timing_read", "rdkv_k_row_words", "rdkv_k_row_words_max",
]
(RDKV_TIME_DECODE_TIERED, RDKV_TIME_DECODE_BF16, RDKV_TIME_WEIGHTS, RDKV_TIME_ALLOCATE, RDKV_TIME_PACK,
 RDKV_TIME_CALIBRATE) = range(6)

_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class rdkv_config(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("seq_lens", ctypes.POINTER(ctypes.c_int32)),
        ("s_obs", ctypes.c_int32), ("pool_kernel", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("k_mode", ctypes.c_int32), ("group_size", ctypes.c_int32),
        ("budget_bits", ctypes.POINTER(ctypes.c_float)),
        ("kv_split_rk", ctypes.c_float), ("k_scale_per_channel", ctypes.c_int32),
        ("n_tiers", ctypes.c_int32), ("tiers", ctypes.c_int32 * 5),
        ("eps_v", ctypes.c_float * 5), ("eps_k", ctypes.c_float * 5),
        ("rel_tol", ctypes.c_float), ("max_iters", ctypes.c_int32),
        ("alloc", _ALLOC_FN), ("free_", _FREE_FN), ("alloc_user", ctypes.c_void_p),
    ]


class rdkv_stats(ctypes.Structure):
    _fields_ = [
        ("n_items", ctypes.c_int64), ("rows", ctypes.c_int64 * 4), ("evicted", ctypes.c_int64),
        ("stored_bytes", ctypes.c_int64), ("arena_bytes", ctypes.c_int64), ("index_bytes", ctypes.c_int64),
        ("n_chunks", ctypes.c_int64), ("dense_bytes", ctypes.c_int64),
        ("alloc_info", ctypes.c_int64), ("iterations_max", ctypes.c_int64),
        ("lambda_min", ctypes.c_double), ("lambda_max", ctypes.c_double),
    ]


class RdkvError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    cfgp = ctypes.POINTER(rdkv_config)
    lib.rdkv_version.restype = ctypes.c_char_p
    lib.rdkv_last_error.restype = ctypes.c_char_p
    lib.rdkv_config_default.argtypes = [cfgp]
    lib.rdkv_weights.argtypes = [cfgp, vp, vp, vp, vp, vp]
    lib.rdkv_allocate.argtypes = [cfgp, vp, vp, vp, vp, vp]
    lib.rdkv_allocate_info.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp]
    lib.rdkv_cache_max_bytes.argtypes = [cfgp]
    lib.rdkv_cache_max_bytes.restype = sz
    lib.rdkv_cache_max_table_bytes.argtypes = [cfgp]
    lib.rdkv_cache_max_table_bytes.restype = sz
    lib.rdkv_pack.argtypes = [cfgp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
    lib.rdkv_compress.argtypes = [cfgp, vp, vp, vp, vp, ctypes.POINTER(vp)]
    lib.rdkv_decode_attn.argtypes = [vp, vp, vp, vp, vp]
    lib.rdkv_decode_bf16_workspace_bytes.argtypes = [ctypes.POINTER(i32), i32, i32, i32, i32]
    lib.rdkv_decode_bf16_workspace_bytes.restype = sz
    lib.rdkv_decode_attn_bf16.argtypes = [vp, vp, ctypes.POINTER(i32), i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.rdkv_decode_bf16_noalloc_max_bytes.argtypes = []
    lib.rdkv_decode_bf16_noalloc_max_bytes.restype = sz
    lib.rdkv_decode_attn_bf16_noalloc.argtypes = [vp, vp, ctypes.POINTER(i32), i32, i32, i32, i32, vp, vp, vp, vp]
    lib.rdkv_cache_reserve_tail.argtypes = [vp, i32, vp]
    lib.rdkv_cache_append.argtypes = [vp, vp, vp, vp]
    lib.rdkv_cache_tail_len.argtypes = [vp]
    lib.rdkv_cache_tail_len.restype = i32
    lib.rdkv_cache_tail_len_sync.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.rdkv_calibrate_eps.argtypes = [cfgp, vp, vp, vp, vp, vp]
    lib.rdkv_cache_rebudget_tail.argtypes = [vp, cfgp, vp, vp]
    lib.rdkv_cache_generations.argtypes = [vp]
    lib.rdkv_cache_generations.restype = i32
    lib.rdkv_cache_generation.argtypes = [vp, i32]
    lib.rdkv_cache_generation.restype = vp
    lib.rdkv_cache_stats.argtypes = [vp, ctypes.POINTER(rdkv_stats)]
    lib.rdkv_cache_export_bytes.argtypes = [vp, i32]
    lib.rdkv_cache_export_bytes.restype = sz
    lib.rdkv_cache_export.argtypes = [vp, i32, vp, sz]
    lib.rdkv_cache_free.argtypes = [vp]
    lib.rdkv_cache_free.restype = None
    lib.rdkv_k_row_words.argtypes = [vp]
    lib.rdkv_k_row_words.restype = i32
    lib.rdkv_k_row_words_max.argtypes = []
    lib.rdkv_k_row_words_max.restype = i32
    lib.rdkv_kernel_timing_enable.argtypes = [i32]
    lib.rdkv_kernel_timing_read.argtypes = [i32, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)]
    return lib


lib = _load()


def _check(status):
    if status != RDKV_OK:
        raise RdkvError(status, lib.rdkv_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def rdkv_version():
    return lib.rdkv_version().decode()


class Config:
    """Owns an rdkv_config and the host arrays it points to."""

    def __init__(self, seq_lens, hq, hkv, head_dim=128, budget_bits=None, **overrides):
        self.c = rdkv_config()
        _check(lib.rdkv_config_default(ctypes.byref(self.c)))
        self._seq = (ctypes.c_int32 * len(seq_lens))(*[int(x) for x in seq_lens])
        self.c.batch, self.c.hq, self.c.hkv, self.c.head_dim = len(seq_lens), hq, hkv, head_dim
        self.c.seq_lens = ctypes.cast(self._seq, ctypes.POINTER(ctypes.c_int32))
        if budget_bits is not None:
            self._bud = (ctypes.c_float * len(seq_lens))(*[float(x) for x in budget_bits])
            self.c.budget_bits = ctypes.cast(self._bud, ctypes.POINTER(ctypes.c_float))
        for k, v in overrides.items():
            if k in ("tiers", "eps_v", "eps_k"):
                arr = getattr(self.c, k)
                for i, x in enumerate(v):
                    arr[i] = x
                if k == "tiers":
                    self.c.n_tiers = len(v)
            else:
                setattr(self.c, k, v)
        self.seq_lens = [int(x) for x in seq_lens]
        self.hq, self.hkv, self.d = hq, hkv, head_dim

    @property
    def total_tokens(self):
        return sum(self.seq_lens) * self.hkv

    def ref(self):
        return ctypes.byref(self.c)


class Cache:
    """Handle of a packed cache (library-owned device memory)."""

    def __init__(self, handle, cfg):
        self.h = handle
        self.cfg = cfg

    def stats(self):
        st = rdkv_stats()
        _check(lib.rdkv_cache_stats(self.h, ctypes.byref(st)))
        return {"n_items": st.n_items, "rows": list(st.rows), "evicted": st.evicted,
                "stored_bytes": st.stored_bytes, "arena_bytes": st.arena_bytes, "index_bytes": st.index_bytes,
                "n_chunks": st.n_chunks, "dense_bytes": st.dense_bytes, "alloc_info": st.alloc_info,
                "iterations_max": st.iterations_max, "lambda_min": st.lambda_min, "lambda_max": st.lambda_max}

    def export(self, what, dtype):
        n = lib.rdkv_cache_export_bytes(self.h, what)
        buf = np.zeros(n, dtype=np.uint8)
        if n:
            _check(lib.rdkv_cache_export(self.h, what, buf.ctypes.data_as(ctypes.c_void_p), n))
        return buf.view(dtype)

    def free(self):
        if self.h:
            lib.rdkv_cache_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def rdkv_weights(cfg, K, Q_obs, want_channel=False):
    w_tok = torch.empty(cfg.total_tokens, dtype=torch.float32, device=K.device)
    w_ch = torch.empty(len(cfg.seq_lens) * cfg.hkv * cfg.d, dtype=torch.float32, device=K.device) if want_channel else None
    _check(lib.rdkv_weights(cfg.ref(), _ptr(K), _ptr(Q_obs), _ptr(w_tok), _ptr(w_ch), _stream()))
    return w_tok, w_ch


def rdkv_allocate(cfg, w_tok, w_ch=None):
    bits_tok = torch.empty(cfg.total_tokens, dtype=torch.uint8, device=w_tok.device)
    bits_ch = None
    if cfg.c.k_mode == RDKV_K_CHANNELWISE:
        bits_ch = torch.empty(len(cfg.seq_lens) * cfg.hkv * cfg.d, dtype=torch.uint8, device=w_tok.device)
    _check(lib.rdkv_allocate(cfg.ref(), _ptr(w_tok), _ptr(w_ch), _ptr(bits_tok), _ptr(bits_ch), _stream()))
    return bits_tok, bits_ch


def rdkv_allocate_info(cfg, w_tok, w_ch=None):
    """(bits_tok, bits_ch, lambda, iterations): the last two as device tensors [maps, items]."""
    n = len(cfg.seq_lens) * cfg.hkv
    mixed = cfg.c.k_mode == RDKV_K_CHANNELWISE
    bits_tok = torch.empty(cfg.total_tokens, dtype=torch.uint8, device=w_tok.device)
    bits_ch = torch.empty(n * cfg.d, dtype=torch.uint8, device=w_tok.device) if mixed else None
    lam = torch.empty((2 if mixed else 1, n), dtype=torch.float64, device=w_tok.device)
    iters = torch.empty((2 if mixed else 1, n), dtype=torch.int32, device=w_tok.device)
    _check(lib.rdkv_allocate_info(cfg.ref(), _ptr(w_tok), _ptr(w_ch), _ptr(bits_tok), _ptr(bits_ch), _ptr(lam),
                                  _ptr(iters), _stream()))
    return bits_tok, bits_ch, lam, iters


def rdkv_cache_max_bytes(cfg):
    return int(lib.rdkv_cache_max_bytes(cfg.ref()))


def rdkv_cache_max_table_bytes(cfg):
    return int(lib.rdkv_cache_max_table_bytes(cfg.ref()))


def rdkv_pack(cfg, K, V, bits_tok, bits_ch=None):
    h = ctypes.c_void_p()
    _check(lib.rdkv_pack(cfg.ref(), _ptr(K), _ptr(V), _ptr(bits_tok), _ptr(bits_ch), _stream(), ctypes.byref(h)))
    return Cache(h, cfg)


def rdkv_compress(cfg, K, V, Q_obs):
    h = ctypes.c_void_p()
    _check(lib.rdkv_compress(cfg.ref(), _ptr(K), _ptr(V), _ptr(Q_obs), _stream(), ctypes.byref(h)))
    return Cache(h, cfg)


def rdkv_decode_attn(cache, q, out=None, lse=None):
    cfg = cache.cfg
    if out is None:
        out = torch.empty((len(cfg.seq_lens), cfg.hq, cfg.d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((len(cfg.seq_lens), cfg.hq), dtype=torch.float32, device=q.device)
    _check(lib.rdkv_decode_attn(cache.h, _ptr(q), _ptr(out), _ptr(lse), _stream()))
    return out, lse


def rdkv_cache_reserve_tail(cache, max_new_tokens):
    _check(lib.rdkv_cache_reserve_tail(cache.h, int(max_new_tokens), _stream()))


def rdkv_cache_append(cache, k_new, v_new):
    _check(lib.rdkv_cache_append(cache.h, _ptr(k_new), _ptr(v_new), _stream()))


def rdkv_cache_tail_len(cache):
    return int(lib.rdkv_cache_tail_len(cache.h))


def rdkv_cache_tail_len_sync(cache):
    n = ctypes.c_int32()
    _check(lib.rdkv_cache_tail_len_sync(cache.h, _stream(), ctypes.byref(n)))
    return n.value


@_ALLOC_FN
def _torch_alloc(nbytes, user):
    return torch.cuda.caching_allocator_alloc(nbytes)


@_FREE_FN
def _torch_free(ptr, user):
    torch.cuda.caching_allocator_delete(ptr)


def torch_allocator_hooks():
    """Config overrides that route the library's device allocations through PyTorch's caching allocator
    (`Config(..., **torch_allocator_hooks())`): hipMalloc / hipFree of the large scratch and arena buffers cost more
    than the kernels of a compression pass over one 128K-token layer."""
    return {"alloc": _torch_alloc, "free_": _torch_free}


class _Borrowed(Cache):
    """A generation of another cache: never freed from here."""

    def __init__(self, handle, cfg, owner):
        super().__init__(handle, cfg)
        self._owner = owner

    def free(self):
        self.h = None


def rdkv_cache_rebudget_tail(cache, cfg, Q_obs):
    _check(lib.rdkv_cache_rebudget_tail(cache.h, cfg.ref(), _ptr(Q_obs), _stream()))


def rdkv_cache_generations(cache):
    return int(lib.rdkv_cache_generations(cache.h))


def rdkv_cache_generation(cache, index, cfg):
    h = lib.rdkv_cache_generation(cache.h, int(index))
    if not h:
        raise IndexError(f"generation {index} does not exist")
    return _Borrowed(ctypes.c_void_p(h), cfg, cache)


def rdkv_calibrate_eps(cfg, K, V):
    """(eps_k, eps_v): float64 [items, 3] for b = 2, 4, 8."""
    n = len(cfg.seq_lens) * cfg.hkv
    eps_k = np.zeros((n, 3), dtype=np.float64)
    eps_v = np.zeros((n, 3), dtype=np.float64)
    _check(lib.rdkv_calibrate_eps(cfg.ref(), _ptr(K), _ptr(V), eps_k.ctypes.data_as(ctypes.c_void_p),
                                  eps_v.ctypes.data_as(ctypes.c_void_p), _stream()))
    return eps_k, eps_v


def rdkv_decode_bf16_workspace_bytes(seq_lens, hq, hkv, head_dim=128):
    arr = (ctypes.c_int32 * len(seq_lens))(*[int(x) for x in seq_lens])
    return lib.rdkv_decode_bf16_workspace_bytes(arr, len(seq_lens), hq, hkv, head_dim)


def rdkv_decode_attn_bf16(K, V, seq_lens, hq, hkv, q, head_dim=128, out=None, lse=None, workspace=None):
    arr = (ctypes.c_int32 * len(seq_lens))(*[int(x) for x in seq_lens])
    if workspace is None:
        n = lib.rdkv_decode_bf16_workspace_bytes(arr, len(seq_lens), hq, hkv, head_dim)
        workspace = torch.empty(max(n, 16), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty((len(seq_lens), hq, head_dim), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((len(seq_lens), hq), dtype=torch.float32, device=q.device)
    _check(lib.rdkv_decode_attn_bf16(_ptr(K), _ptr(V), arr, len(seq_lens), hq, hkv, head_dim, _ptr(q), _ptr(out),
                                     _ptr(lse), _ptr(workspace), workspace.numel(), _stream()))
    return out, lse


def rdkv_decode_attn_bf16_noalloc(K, V, seq_lens, hq, hkv, q, out, lse=None, head_dim=128):
    """The caller passes every buffer; nothing is allocated here or in the library."""
    arr = (ctypes.c_int32 * len(seq_lens))(*[int(x) for x in seq_lens])
    _check(lib.rdkv_decode_attn_bf16_noalloc(_ptr(K), _ptr(V), arr, len(seq_lens), hq, hkv, head_dim, _ptr(q),
                                             _ptr(out), _ptr(lse), _stream()))
    return out, lse


def rdkv_kernel_timing_enable(enable):
    _check(lib.rdkv_kernel_timing_enable(1 if enable else 0))


def rdkv_kernel_timing_read(kind):
    """(launches, total_ms) of the bracketed main kernel of one kind since the last read."""
    n, ms = ctypes.c_int64(), ctypes.c_double()
    _check(lib.rdkv_kernel_timing_read(kind, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value
