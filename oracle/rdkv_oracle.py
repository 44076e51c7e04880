"""CPU oracle for the RDKV hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow NumPy written from the paper (arxiv 2605.08317, "RDKV: Rate-Distortion
Bit Allocation for Joint Eviction and Quantization of the KV Cache").  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product (the HIP library and its Python binding) never does, and this file
imports nothing from the product.

Every function cites the passage it follows.  Floating point is fp64 except the
reference quantizer, which is fp32 in a fixed operation order so that its codes
can be compared bit for bit.

Conventions
-----------
* One "item" is one (sequence, KV head).  K, V of one sequence: float32 arrays
  [Hkv, T, d] whose values are exactly representable in bf16.
* Query head j belongs to KV head j // g, g = Hq // Hkv (Sec. 3, GQA).
* Tiers (bit-widths) B = {0, 2, 4, 8, 16} (Sec. 3); tier 16 keeps the input
  16-bit pattern, tier 0 stores nothing.

Parity pins for each function are in tests/test_oracle_pins.py; every
function here has at least one pin that is not a retyping of its own formula.
End-to-end accuracy on the paper's benchmarks is "parity unpinned" (the data
sets and models are not available).
"""
import functools
import math

import numpy as np

TIERS = (0, 2, 4, 8, 16)
PACK_ORDER = (16, 8, 4, 2)          # order of tier segments inside an item
GROUP = 32                          # quantization group size
ROW_PAD_TOKENWISE = 64              # tier segments are padded to whole 64-row tiles (both modes)
K_TOKEN_GROUP = 32                  # mixed mode: a K channel's group = 32 consecutive retained tokens of a segment
SEG_ALIGN = 256                     # byte alignment of every segment in the arena

# Table 9 (App. "Calibrated Distortion Tables"), LLaMA-3.1-8B row; eps(0) = 1 and eps(16) = 0 for every model.
EPS_V_LLAMA31_8B = (1.0, 0.313, 0.0140, 4.9e-5, 0.0)
EPS_K_LLAMA31_8B = (1.0, 0.149, 0.0062, 2.2e-5, 0.0)
# Bennett-style table: per-coordinate RMSE proportional to 2^-b (Eq. 5).
EPS_BENNETT = tuple(2.0 ** (-b) for b in TIERS)


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------
def _check_bf16_exact(x, name):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if np.any(x.view(np.uint32) & np.uint32(0xFFFF)):
        raise ValueError(f"{name}: values are not bf16-representable")
    return x


def bf16_bits(x):
    """uint16 bit patterns of a bf16-exact float32 array."""
    x = _check_bf16_exact(x, "bf16_bits")
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(bits):
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Stage 1: distortion weights
# --------------------------------------------------------------------------
def token_weights(K, Q_obs, causal=True):
    """Token weights w_t = sum over window queries and group heads of a_{tau,t}.

    Prop. 3.1 / Eq. 2 and Alg. 1 Stage 1: A = softmax(Q_window K^T / sqrt(d)),
    w_t^{(h)} = sum_{tau, g} a_{tau,g,t}.  The window holds the last S_w prefill
    positions; row i sits at absolute position T - S_w + i and (reading taken:
    weights come from the prefill forward pass, which is causal) attends only
    keys t <= that position.

    K: [Hkv, T, d]; Q_obs: [Hq, S_w, d].  Returns float64 [Hkv, T] (not pooled).
    """
    K = np.asarray(K, dtype=np.float64)
    Q_obs = np.asarray(Q_obs, dtype=np.float64)
    Hkv, T, d = K.shape
    Hq, Sw, d2 = Q_obs.shape
    assert d2 == d and Hq % Hkv == 0 and T >= Sw
    g = Hq // Hkv
    w = np.zeros((Hkv, T), dtype=np.float64)
    for h in range(Hkv):
        for j in range(g):
            Z = Q_obs[h * g + j] @ K[h].T / math.sqrt(d)          # [S_w, T]
            if causal:
                for i in range(Sw):
                    Z[i, T - Sw + i + 1:] = -np.inf
            Z = Z - Z.max(axis=1, keepdims=True)
            A = np.exp(Z)
            A = A / A.sum(axis=1, keepdims=True)
            w[h] += A.sum(axis=0)
    return w


def avg_pool(w, kernel=5):
    """AvgPool1d along t (Alg. 1 Stage 1, pooling kernel w = 5).

    Reading taken: stride 1, zero padding kernel//2 on both sides, divisor always
    `kernel` (padding counted), no renormalisation.
    """
    w = np.asarray(w, dtype=np.float64)
    if kernel <= 1:
        return w.copy()
    assert kernel % 2 == 1
    r = kernel // 2
    T = w.shape[-1]
    padded = np.zeros(w.shape[:-1] + (T + 2 * r,), dtype=np.float64)
    padded[..., r:r + T] = w
    out = np.zeros_like(w)
    for k in range(kernel):
        out += padded[..., k:k + T]
    return out / kernel


def channel_weights(K, Q_obs):
    """Channel weights w_c = ||Q[:,c]||_2 ||K[:,c]||_2 / sqrt(d)  (Prop. 3.2, Eq. 4).

    Q[:,c] stacks the window queries of all g query heads of the group (the only
    queries the probe provides); K[:,c] runs over all T keys of the uncompressed
    cache (Sec. 3.2 Stage 1).  Returns float64 [Hkv, d].
    """
    K = np.asarray(K, dtype=np.float64)
    Q_obs = np.asarray(Q_obs, dtype=np.float64)
    Hkv, T, d = K.shape
    Hq = Q_obs.shape[0]
    g = Hq // Hkv
    out = np.zeros((Hkv, d), dtype=np.float64)
    for h in range(Hkv):
        Qg = Q_obs[h * g:(h + 1) * g].reshape(-1, d)
        qn = np.sqrt((Qg * Qg).sum(axis=0))
        kn = np.sqrt((K[h] * K[h]).sum(axis=0))
        out[h] = qn * kn / math.sqrt(d)
    return out


# --------------------------------------------------------------------------
# Continuous reverse water-filling (Thm 3.3) -- check-only, never shipped
# --------------------------------------------------------------------------
def water_filling(c, B):
    """Minimise sum_u c_u 2^{-b_u} s.t. sum_u b_u <= B, b_u >= 0  (Eq. 5, Thm 3.3).

    c_u = w_u sigma_u > 0.  Returns (b, theta, lam): b_u = [log2(c_u/theta)]_+,
    theta = lam / ln 2 is the water level; the budget binds when B > 0.
    """
    c = np.asarray(c, dtype=np.float64)
    assert np.all(c > 0) and B >= 0
    order = np.argsort(-c, kind="stable")
    cs = c[order]
    logc = np.log2(cs)
    csum = np.cumsum(logc)
    U = len(c)
    theta = None
    for m in range(1, U + 1):
        log_theta = (csum[m - 1] - B) / m
        lower_ok = (m == U) or (logc[m] <= log_theta)
        if logc[m - 1] > log_theta - 1e-15 and lower_ok:
            theta = 2.0 ** log_theta
            break
    assert theta is not None
    b = np.maximum(0.0, np.log2(c / theta))
    return b, theta, theta * math.log(2.0)


# --------------------------------------------------------------------------
# Stage 2/3: discrete allocation (MCKP, Eq. 6) by Lagrangian bisection (Alg. 2)
# --------------------------------------------------------------------------
def hull_thresholds(tiers, eps):
    """Lower convex hull of the points (b_k, eps(b_k)) and its slope ratios.

    For a multiplier lam, argmin_b w eps(b) + lam b (Alg. 2, per-unit step) moves
    from hull vertex k-1 to k exactly when
        w (eps_{k-1} - eps_k) > lam (b_k - b_{k-1})  <=>  w > lam r_k,
    r_k = (b_k - b_{k-1}) / (eps_{k-1} - eps_k), increasing along the hull.
    Strict '>' means a tie takes the lower bit-width.  Tiers off the hull are
    never optimal.  Returns (hull_tiers, r) with hull_tiers[0] the lowest tier and
    r[k-1] the ratio of the edge into hull_tiers[k].
    """
    pts = sorted((int(b), float(np.float64(np.float32(e)))) for b, e in zip(tiers, eps))
    hull = []
    for p in pts:
        while len(hull) >= 2:
            (b0, e0), (b1, e1) = hull[-2], hull[-1]
            cross = (b1 - b0) * (p[1] - e0) - (e1 - e0) * (p[0] - b0)
            if cross <= 0.0:
                hull.pop()
            else:
                break
        hull.append(p)
    # keep the descending part only: an edge that does not lower eps is never taken
    keep = [hull[0]]
    for p in hull[1:]:
        if keep[-1][1] - p[1] > 0.0:
            keep.append(p)
        else:
            break
    hb = [p[0] for p in keep]
    r = [(keep[k][0] - keep[k - 1][0]) / (keep[k - 1][1] - keep[k][1]) for k in range(1, len(keep))]
    return hb, r


def classify(w, lam, hull_tiers, r):
    """Bit-width of each unit at multiplier lam: the highest hull tier k whose
    threshold lam * r_k is strictly exceeded by (double) w_u."""
    w64 = np.asarray(w, dtype=np.float32).astype(np.float64)
    idx = np.zeros(w64.shape, dtype=np.int64)
    for k, rk in enumerate(r):
        thr = np.float64(lam) * np.float64(rk)
        idx += (w64 > thr)
    return np.asarray(hull_tiers, dtype=np.uint8)[idx]


def argmin_bits(w, lam, tiers, eps):
    """Alg. 2 per-unit step in its printed form: argmin_b w_u eps(b) + lam b
    (lowest b on ties), fp64.  This is what `mckp_bisect` runs."""
    w64 = np.asarray(w, dtype=np.float32).astype(np.float64)
    tiers = np.asarray(tiers, dtype=np.float64)
    e = np.asarray([np.float64(np.float32(x)) for x in eps])
    order = np.argsort(tiers)
    cost = w64[:, None] * e[order][None, :] + lam * tiers[order][None, :]
    return tiers[order][np.argmin(cost, axis=1)].astype(np.uint8)


def budget_units(avg_bits, U):
    """Integer budget in summed bit-widths: floor(avg_bits * U), fp64."""
    return int(math.floor(float(np.float64(avg_bits)) * U))


def mckp_bisect(w, avg_bits, tiers=TIERS, eps=EPS_V_LLAMA31_8B, rel_tol=np.float32(1e-2),
                max_iters=64, return_info=False):
    """Lagrangian bisection knapsack solver (Alg. 2; constants of App. B:
    lam in [0, max w], relative tolerance 1e-2, at most 64 steps).

    Readings taken where the listing and Eq. 6 disagree: the returned allocation
    always satisfies sum b_u <= B (strict feasibility); the search stops at the
    first feasible iterate within the tolerance band below the budget, and
    otherwise returns the feasible iterate with the smallest multiplier seen.
    Integer comparisons on the summed bits avoid dividing by a zero budget.
    Every step evaluates the per-unit rule in its printed form, argmin_b w eps(b) +
    lam b with the lowest b on ties (`argmin_bits`); the convex hull only supplies
    the shortcuts (highest and lowest useful tier).  `classify` is the equivalent
    threshold form and is pinned against it separately.

    w: float32 [U].  avg_bits: float32 target average bits per unit.
    """
    w = np.ascontiguousarray(w, dtype=np.float32)
    U = w.shape[0]
    hull_tiers, r = hull_thresholds(tiers, eps)
    top, low = hull_tiers[-1], (hull_tiers[1] if len(hull_tiers) > 1 else 0)
    B_int = budget_units(np.float32(avg_bits), U)
    info = {"B_int": B_int, "iters": 0, "lam": None}
    if U == 0:
        bits = np.zeros(0, dtype=np.uint8)
    elif B_int >= top * U:
        bits = np.full(U, top, dtype=np.uint8)
    elif len(hull_tiers) == 1 or B_int < low:
        bits = np.full(U, hull_tiers[0], dtype=np.uint8)
    else:
        need = int(math.ceil((1.0 - float(np.float64(np.float32(rel_tol)))) * B_int))
        lo, hi = 0.0, float(np.float64(w.max()))
        best = None
        for it in range(max_iters):
            lam = (lo + hi) * 0.5
            cand = argmin_bits(w, lam, tiers, eps)        # the per-unit step as Alg. 2 prints it
            S = int(cand.astype(np.int64).sum())
            info["iters"] = it + 1
            if S <= B_int:
                best, hi = (cand, lam), lam
                if S >= need:
                    break
            else:
                lo = lam
        if best is None:
            bits = np.full(U, hull_tiers[0], dtype=np.uint8)
        else:
            bits, info["lam"] = best
    if return_info:
        return bits, info
    return bits


def mixed_budgets(avg_bits, r_k, T, n_kept, d):
    """Stage 2/3 budgets of Alg. 1 in average-bit form.

    B_head = 2 B_tok d 16 is split B_K = r_K B_head, B_V = (1 - r_K) B_head
    (r_K = 1/2 in the paper).  With avg_bits the average over all 2 T d cache
    scalars: V gets avg 2 (1 - r_K) avg_bits per token unit; K's budget is spread
    over kept tokens only, k_avg = 2 r_K avg_bits T / n_kept, capped at 16.
    """
    a = float(np.float64(np.float32(avg_bits)))
    rk = float(np.float64(np.float32(r_k)))
    v_avg = 2.0 * (1.0 - rk) * a
    if n_kept is None:
        return v_avg, None
    k_avg = 16.0 if n_kept == 0 else min(16.0, 2.0 * rk * a * T / n_kept)
    return v_avg, k_avg


# --------------------------------------------------------------------------
# Reference quantizer (App. B "K-cache dequantization fusion": k_hat = s (code - z))
# --------------------------------------------------------------------------
def quantize_groups(x, bits):
    """Asymmetric uniform quantizer on groups along the last axis.

    The paper fixes the form k_hat = s (code - z) with codes in [0, 2^b - 1] and
    leaves rounding and the scale format open.  Layout fixed by this build: fp32
    arithmetic in exactly this order, fp16 scale s and fp16 offset m = group
    minimum (z = -m/s), so x_hat = s*code + m:
        mn = min x + 0.0 (so that -0 becomes +0), mx = max x
        s  = fp16_rn((mx - mn) / Q),  Q = 2^b - 1        (IEEE fp32 divide)
        m  = fp16_rn(mn)
        code = clamp(rint((x - m) / s), 0, Q)  (ties to even);  all 0 if s == 0
    x: float32 [..., n] (n <= 32 for one group).  Returns (codes uint8, s fp16,
    m fp16) with s, m of shape x.shape[:-1].
    """
    assert bits in (2, 4, 8)
    x = np.ascontiguousarray(x, dtype=np.float32)
    Q = np.float32((1 << bits) - 1)
    mn = x.min(axis=-1) + np.float32(0.0)
    mx = x.max(axis=-1)
    with np.errstate(over="ignore"):
        s = ((mx - mn) / Q).astype(np.float32).astype(np.float16)
        m = mn.astype(np.float16)
    sf = s.astype(np.float32)[..., None]
    mf = m.astype(np.float32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        t = ((x - mf).astype(np.float32) / sf).astype(np.float32)
    t = np.rint(t)
    t = np.minimum(np.maximum(t, np.float32(0.0)), Q)
    t = np.where(sf == 0, np.float32(0.0), t)
    return t.astype(np.uint8), s, m


def quantize_rows(rows, bits, group=GROUP):
    """Quantizes token rows [n, d] with one scale and offset per `group` consecutive channels.

    group = 32: the groups of this build's default layout.  group = d: one scale and one offset per token row, the
    per-token format of the paper (App. B; Table 9 reports per-token errors for V).  The record of a row keeps its
    d / 32 metadata slots either way: with a row-wide group every slot repeats the row's scale and offset, so the
    physical layout and its readers are the same.  Returns (codes uint8 [n, d], scale fp16 [n, d / 32], offset fp16
    [n, d / 32])."""
    n, d = rows.shape
    assert group in (GROUP, d)
    c, s, m = quantize_groups(rows.reshape(n, d // group, group), bits)
    rep = group // GROUP
    return c.reshape(n, d), np.repeat(s, rep, axis=1), np.repeat(m, rep, axis=1)


def dequantize_groups(codes, s, m):
    """x_hat = s*code + m in fp64 (exact: code is an integer, s and m are fp16)."""
    return s.astype(np.float64)[..., None] * codes.astype(np.float64) + m.astype(np.float64)[..., None]


# --------------------------------------------------------------------------
# Stage 4: partition and packing (token-wise mode)
# --------------------------------------------------------------------------
def partition(bits):
    """Kept units grouped by tier (16, 8, 4, 2), ascending position inside a tier
    (Alg. 1 Stage 4: sort the kept tokens by bit-width into sub-segments)."""
    bits = np.asarray(bits, dtype=np.uint8)
    return {b: np.nonzero(bits == b)[0].astype(np.int32) for b in PACK_ORDER}


def pack_codes(codes, bits):
    """Little-endian bit packing of one row: element i sits at bit i*b of the row
    (App. B: 2-bit -> four elements per byte at offsets 0,2,4,6; 4-bit -> two per
    byte at offsets 0,4; 8-bit -> one per byte).  codes: uint8 [..., n]."""
    per = 8 // bits
    n = codes.shape[-1]
    assert n % per == 0
    c = codes.reshape(codes.shape[:-1] + (n // per, per)).astype(np.uint32)
    out = np.zeros(c.shape[:-1], dtype=np.uint32)
    for j in range(per):
        out |= c[..., j] << np.uint32(j * bits)
    return out.astype(np.uint8)


def unpack_codes(data, bits):
    per = 8 // bits
    mask = np.uint32((1 << bits) - 1)
    d32 = data.astype(np.uint32)
    parts = [(d32 >> np.uint32(j * bits)) & mask for j in range(per)]
    return np.stack(parts, axis=-1).reshape(data.shape[:-1] + (data.shape[-1] * per,)).astype(np.uint8)


def _round_up(x, a):
    return (x + a - 1) // a * a


def row_bytes(bits, d=128):
    return d * bits // 8


def meta_bytes(bits, d=128):
    return 0 if bits == 16 else (d // GROUP) * 4


def canonical_item(Kh, Vh, bits_tok, group=GROUP):
    """Canonical (layout-free) record of one item in token-wise mode: per tier the
    kept positions and, for K and V, per-element codes plus fp16 scale / offset
    bit patterns per group of 32 channels (group = d: one per token row, repeated in
    every slot); tier 16 keeps the input bf16 bits.
    In token-wise mode a token's K row and V row share its bit-width.
    Kh, Vh: float32 [T, d] bf16-exact."""
    Kh = _check_bf16_exact(Kh, "K")
    Vh = _check_bf16_exact(Vh, "V")
    T, d = Kh.shape
    assert d % GROUP == 0
    idx = partition(bits_tok)
    rec = {}
    for b in PACK_ORDER:
        pos = idx[b]
        ent = {"pos": pos}
        for name, X in (("k", Kh), ("v", Vh)):
            rows = X[pos]
            if b == 16:
                ent[name + "_codes"] = bf16_bits(rows).reshape(len(pos), d)
                ent[name + "_scale"] = np.zeros((len(pos), 0), dtype=np.uint16)
                ent[name + "_off"] = np.zeros((len(pos), 0), dtype=np.uint16)
            else:
                c, s, m = quantize_rows(rows, b, group)
                ent[name + "_codes"] = c
                ent[name + "_scale"] = np.ascontiguousarray(s).view(np.uint16)
                ent[name + "_off"] = np.ascontiguousarray(m).view(np.uint16)
        rec[b] = ent
    return rec


TILE64_ROWS = 64                    # tokens per tile of a quantized tier segment
TILE64_META_BYTES = 1024            # per tile and side: 16 bytes per token


@functools.lru_cache(maxsize=None)
def tile64_code_positions(bits, which):
    """Token-wise mode: where the code of (row r of a 64-row tile, channel c) lives inside
    the tile's data block of 64 * 16 * bits bytes.

    Layout fixed by this build (the paper's own layout, App. B, is row-major per token;
    any documented bijection serves Eq. 7).  One wavefront lane owns a run of 4*bits
    32-bit words; word W of lane L is stored at byte 1024*(W // 4) + 16*L + 4*(W % 4), so
    a wavefront reads 1 KiB per 16-byte load.  The run holds four *groups* of `bits` words;
    a group is unpacked in eight *steps* of four codes: with F = 16 / bits fields per 16-bit
    half, step s reads field f = s % F of both halves of the word pair p = s // F of the
    group, i.e. code k (0..3) of step s is at word 2p + k // 2, bit 16*(k % 2) + bits*f.
      K: lane = token r; group = c // 32 (the quantization group); step, code: c % 32 = 4 s + k
      V: lane = 32*(r // 32) + c % 32; group = c // 32; step, code: r % 32 = 4 s + k
    (K: a lane holds one token's row; V: a lane holds one channel for 32 tokens.)
    Returns (byte_offset [64,128] int64, bit_shift [64,128] int64)."""
    assert bits in (2, 4, 8) and which in ("k", "v")
    F = 16 // bits
    byte_off = np.zeros((TILE64_ROWS, 128), dtype=np.int64)
    shift = np.zeros((TILE64_ROWS, 128), dtype=np.int64)
    for r in range(TILE64_ROWS):
        for c in range(128):
            if which == "k":
                lane, grp, idx = r, c // 32, c % 32
            else:
                lane, grp, idx = 32 * (r // 32) + c % 32, c // 32, r % 32
            st, k = idx // 4, idx % 4
            W = grp * bits + 2 * (st // F) + k // 2
            bit = 8 * (1024 * (W // 4) + 16 * lane + 4 * (W % 4)) + 16 * (k % 2) + bits * (st % F)
            byte_off[r, c], shift[r, c] = bit // 8, bit % 8
    return byte_off, shift


@functools.lru_cache(maxsize=None)
def tile64_meta_positions(which):
    """fp16 element index (0..511) of the scale and of the offset of (row r, group)
    inside the tile's 1024-byte metadata block.
      K: row-major, 16 bytes per token: scales of the 4 groups, then their offsets
      V: per block of 4 tokens 64 bytes = 4 groups x 16 bytes: the group's scales of the 4 tokens,
         then its offsets of the 4 tokens"""
    sc = np.zeros((TILE64_ROWS, 4), dtype=np.int64)
    of = np.zeros((TILE64_ROWS, 4), dtype=np.int64)
    for r in range(TILE64_ROWS):
        for grp in range(4):
            if which == "k":
                sc[r, grp], of[r, grp] = 8 * r + grp, 8 * r + 4 + grp
            else:
                sc[r, grp] = 32 * (r // 4) + 8 * grp + r % 4
                of[r, grp] = 32 * (r // 4) + 8 * grp + 4 + r % 4
    return sc, of


def tile64_data_bytes(bits):
    return TILE64_ROWS * 128 * bits // 8


def pack_tiles64(codes, scale_bits, off_bits, bits, which):
    """Physical 64-row tiles of n rows (zero-padded to whole tiles).  codes uint8 [n,128];
    scale_bits, off_bits uint16 [n,4].  Returns (data uint8, meta uint8)."""
    n = codes.shape[0]
    R = TILE64_ROWS
    nt = (n + R - 1) // R
    cp = np.zeros((nt * R, 128), dtype=np.uint8)
    cp[:n] = codes
    sp = np.zeros((nt * R, 4), dtype=np.uint16)
    op = np.zeros((nt * R, 4), dtype=np.uint16)
    sp[:n], op[:n] = scale_bits, off_bits
    byte_off, shift = tile64_code_positions(bits, which)
    sc_idx, of_idx = tile64_meta_positions(which)
    data = np.zeros((nt, tile64_data_bytes(bits)), dtype=np.uint8)
    meta = np.zeros((nt, TILE64_META_BYTES // 2), dtype="<u2")
    cp = cp.reshape(nt, R, 128)
    for t in range(nt):
        contrib = (cp[t].astype(np.uint32) << shift.astype(np.uint32)).astype(np.uint8)
        np.bitwise_or.at(data[t], byte_off.reshape(-1), contrib.reshape(-1))
        meta[t, sc_idx.reshape(-1)] = sp[t * R:(t + 1) * R].reshape(-1)
        meta[t, of_idx.reshape(-1)] = op[t * R:(t + 1) * R].reshape(-1)
    return data.reshape(-1), meta.view(np.uint8).reshape(-1)


def unpack_tiles64(data, meta, n, bits, which):
    """Inverse of pack_tiles64 for the first n rows."""
    R = TILE64_ROWS
    nt = (n + R - 1) // R
    byte_off, shift = tile64_code_positions(bits, which)
    sc_idx, of_idx = tile64_meta_positions(which)
    data = np.asarray(data, dtype=np.uint8).reshape(nt, tile64_data_bytes(bits))
    meta = np.asarray(meta, dtype=np.uint8).view("<u2").reshape(nt, TILE64_META_BYTES // 2)
    mask = (1 << bits) - 1
    codes = ((data[:, byte_off] >> shift.astype(np.uint8)) & mask).astype(np.uint8)
    sc = meta[:, sc_idx].astype(np.uint16)
    of = meta[:, of_idx].astype(np.uint16)
    return codes.reshape(nt * R, 128)[:n], sc.reshape(nt * R, 4)[:n], of.reshape(nt * R, 4)[:n]


def physical_segments(rec, d=128):
    """Physical form of one item's canonical record.

    Per tier b with n rows, padded with zero rows to whole 64-row tiles:
      tier 16:      K data and V data are the bf16 rows, row-major; no metadata
      tiers 8,4,2:  K data = tiles of 64*16*b bytes (tile64_code_positions(b, 'k')),
                    K meta = tiles of 1024 bytes (tile64_meta_positions('k')), same for V
    Returns {b: (kd, km, vd, vm)} as flat uint8 arrays.
    """
    assert d == 128
    out = {}
    for b in PACK_ORDER:
        ent = rec[b]
        n = len(ent["pos"])
        npad = _round_up(n, ROW_PAD_TOKENWISE)
        segs = []
        for name in ("k", "v"):
            if b == 16:
                data = np.zeros((npad, 2 * d), dtype=np.uint8)
                data[:n] = ent[name + "_codes"].astype("<u2").view(np.uint8).reshape(n, 2 * d)
                segs += [data.reshape(-1), np.zeros(0, dtype=np.uint8)]
            else:
                data, meta = pack_tiles64(ent[name + "_codes"], ent[name + "_scale"], ent[name + "_off"], b, name)
                segs += [data, meta]
        out[b] = tuple(segs)
    return out


def build_cache_tokenwise(K_list, V_list, bits_list, group=GROUP):
    """Pack a ragged batch in token-wise mode.

    K_list[s], V_list[s]: float32 [Hkv, T_s, d]; bits_list[s]: uint8 [Hkv, T_s].
    Items are ordered sequence-major, head-minor.  The arena concatenates, per
    item and per tier in the order 16, 8, 4, 2, the four segments K data, K meta,
    V data, V meta, each starting on a 256-byte boundary (empty segments take no
    space).  Returns a dict with
      counts   int32 [items][4]         rows per tier (16, 8, 4, 2)
      tier_idx int32 [sum kept]         kept positions, item-major, tier order
      seg_off  int64 [items][4][4]      byte offset of each segment in the arena
      arena    uint8 [bytes]
      canon    list of canonical records (for tests)
    """
    items = []
    for Ks, Vs, bs in zip(K_list, V_list, bits_list):
        for h in range(Ks.shape[0]):
            items.append((Ks[h], Vs[h], bs[h]))
    d = K_list[0].shape[2]
    n_items = len(items)
    counts = np.zeros((n_items, 4), dtype=np.int32)
    seg_off = np.zeros((n_items, 4, 4), dtype=np.int64)
    chunks, tier_idx, canon = [], [], []
    cur = 0
    for i, (Kh, Vh, bh) in enumerate(items):
        rec = canonical_item(Kh, Vh, bh, group)
        canon.append(rec)
        phys = physical_segments(rec, d)
        for ti, b in enumerate(PACK_ORDER):
            counts[i, ti] = len(rec[b]["pos"])
            tier_idx.append(rec[b]["pos"])
            for si, seg in enumerate(phys[b]):
                cur = _round_up(cur, SEG_ALIGN)
                seg_off[i, ti, si] = cur
                flat = seg.reshape(-1)
                if flat.size:
                    chunks.append((cur, flat))
                    cur += flat.size
    total = _round_up(cur, SEG_ALIGN)
    arena = np.zeros(total, dtype=np.uint8)
    for off, flat in chunks:
        arena[off:off + flat.size] = flat
    return {
        "counts": counts,
        "tier_idx": np.concatenate(tier_idx).astype(np.int32) if tier_idx else np.zeros(0, np.int32),
        "seg_off": seg_off,
        "arena": arena,
        "canon": canon,
        "d": d,
        "hkv": K_list[0].shape[0],
        "seq_lens": [k.shape[1] for k in K_list],
    }


def stored_bytes(counts, d=128):
    """Bytes a decode step must read for the given per-tier row counts (unpadded):
    sum over tiers of n * 2 * (row bytes + metadata bytes)."""
    counts = np.asarray(counts, dtype=np.int64).reshape(-1, 4)
    per_row = np.array([2 * (row_bytes(b, d) + meta_bytes(b, d)) for b in PACK_ORDER], dtype=np.int64)
    return int((counts * per_row[None, :]).sum())


def unpack_item(cache, item):
    """Dequantised K_hat, V_hat (float64 [n_kept, d]) of one item, read back from the
    physical arena (not from the canonical record)."""
    d = cache["d"]
    arena, seg_off, counts = cache["arena"], cache["seg_off"], cache["counts"]
    ks, vs = [], []
    for ti, b in enumerate(PACK_ORDER):
        n = int(counts[item, ti])
        if n == 0:
            continue
        mats = []
        for which, name in ((0, "k"), (2, "v")):
            d_off = int(seg_off[item, ti, which])
            if b == 16:
                raw = arena[d_off:d_off + n * 2 * d].reshape(n, 2 * d)
                mats.append(bf16_from_bits(raw.view("<u2").astype(np.uint16)).astype(np.float64))
            else:
                nt = (n + TILE64_ROWS - 1) // TILE64_ROWS
                m_off = int(seg_off[item, ti, which + 1])
                codes, sc, of = unpack_tiles64(arena[d_off:d_off + nt * tile64_data_bytes(b)],
                                               arena[m_off:m_off + nt * TILE64_META_BYTES], n, b, name)
                s = sc.copy().view(np.float16)
                m = of.copy().view(np.float16)
                mats.append(dequantize_groups(codes.reshape(n, d // GROUP, GROUP), s, m).reshape(n, d))
        ks.append(mats[0])
        vs.append(mats[1])
    if not ks:
        return np.zeros((0, d)), np.zeros((0, d))
    return np.concatenate(ks), np.concatenate(vs)


# --------------------------------------------------------------------------
# Mixed mode (Sec. 3.2 Stages 2-3, the paper's own arrangement): V token-wise,
# K channel-wise on the retained tokens
# --------------------------------------------------------------------------
SLOT_PAD = {16: 4, 8: 4, 4: 8, 2: 16}   # channel slots of a K tier are padded to whole steps / whole 32-bit words


def channel_slots(bits_ch):
    """Sorted-channel order of one item's K rows (App. B: channels are sorted by
    bit-width into segments along the channel axis and the query is permuted to
    match).  Tiers in the order 16, 8, 4, 2, ascending channel index inside a tier.
    A retained token's K row is a run of 32-bit words: a 16-bit word holds 2 channels,
    an 8-bit word 4, a 4-bit word 8, a 2-bit word 16; every tier is padded to whole
    words (the 16-bit tier to whole word pairs = 4 channels) -- the paper pads its 2-
    and 4-bit segments to whole bytes the same way; padded channels carry zero codes
    and s = m = 0, so they contribute nothing.  Evicted channels (0 bits) get no slot.
    A *step* is 4 consecutive slots (one matrix-core operand in the decode kernel).
    Returns {'order': {b: channel indices}, 'npad': {b: padded slot count},
    'nw': {b: words per token}, 'slot_ch': one entry per slot, the channel it holds or
    -1 for padding, 'n_words', 'n_words_padded' (even), 'n_steps16', 'n_qsteps'}."""
    bits_ch = np.asarray(bits_ch, dtype=np.uint8)
    order, npad, nw, slot_ch = {}, {}, {}, []
    for b in PACK_ORDER:
        ch = np.nonzero(bits_ch == b)[0].astype(np.int64)
        order[b] = ch
        npad[b] = _round_up(len(ch), SLOT_PAD[b])
        nw[b] = npad[b] * b // 32
        slot_ch += list(ch) + [-1] * (npad[b] - len(ch))
    n_words = sum(nw.values())
    return {"order": order, "npad": npad, "nw": nw, "slot_ch": np.asarray(slot_ch, dtype=np.int64),
            "n_words": n_words, "n_words_padded": _round_up(n_words, 2),
            "n_steps16": npad[16] // 4, "n_qsteps": (npad[8] + npad[4] + npad[2]) // 4}


def k_tile_bytes_mixed(sl):
    """Bytes of one 64-token K tile: 64 tokens x an even number of 32-bit words."""
    return 256 * sl["n_words_padded"]


def k_meta_bytes_mixed(sl):
    """Per tile: for each of the two 32-token groups and each quantized step (4 slots),
    4 fp16 scales then 4 fp16 offsets."""
    return 32 * sl["n_qsteps"]


def quantize_channelwise(Krows, bits_ch, group_tokens=K_TOKEN_GROUP):
    """Channel-wise K quantization of retained rows.

    group_tokens = None: one scale and zero-point per channel over all the rows given --
    the paper's own format (App. B: s_c, z_c per channel; the rows are then all the
    retained tokens of a (sequence, KV head)).  group_tokens = 32 (this build's default
    layout): groups of 32 consecutive rows of a channel (half a tile of a tier segment;
    the last group may be short).  Same quantizer as elsewhere (fp16 scale, fp16 offset =
    group minimum, fp32 arithmetic in a fixed order).
    Krows: float32 [n, d] bf16-exact, in packed order.  Returns
      codes  uint16 [n, d]: integer codes (tiers 8/4/2), bf16 bit patterns (tier 16), 0 (tier 0)
      scale, off  uint16 [groups, d]: fp16 bit patterns (0 for tiers 16 and 0)."""
    Krows = _check_bf16_exact(Krows, "K")
    n, d = Krows.shape
    bits_ch = np.asarray(bits_ch, dtype=np.uint8)
    gt = max(n, 1) if group_tokens is None else group_tokens
    ng = (n + gt - 1) // gt
    codes = np.zeros((n, d), dtype=np.uint16)
    scale = np.zeros((ng, d), dtype=np.uint16)
    off = np.zeros((ng, d), dtype=np.uint16)
    for c in range(d):
        b = int(bits_ch[c])
        if b == 16:
            codes[:, c] = bf16_bits(Krows[:, c])
        elif b in (2, 4, 8):
            for t in range(ng):
                rows = slice(t * gt, min(n, (t + 1) * gt))
                cc, sc, mc = quantize_groups(Krows[rows, c][None, :], b)
                codes[rows, c] = cc[0]
                scale[t, c] = sc.view(np.uint16)[0]
                off[t, c] = mc.view(np.uint16)[0]
    return codes, scale, off


def dequantize_channelwise(codes, scale, off, bits_ch, group_tokens=K_TOKEN_GROUP):
    """K_hat float64 [n, d]: s*code + m for tiers 8/4/2, the bf16 value for tier 16,
    exactly zero for an evicted channel (Sec. 3.2: a 0-bit channel is removed).
    group_tokens = None: scale and off hold one row that serves every token."""
    n, d = codes.shape
    out = np.zeros((n, d), dtype=np.float64)
    for c in range(d):
        b = int(bits_ch[c])
        if b == 16:
            out[:, c] = bf16_from_bits(codes[:, c]).astype(np.float64)
        elif b in (2, 4, 8):
            t = np.zeros(n, dtype=np.int64) if group_tokens is None else np.arange(n) // group_tokens
            s = scale[:, c].copy().view(np.float16).astype(np.float64)[t]
            m = off[:, c].copy().view(np.float16).astype(np.float64)[t]
            out[:, c] = s * codes[:, c].astype(np.float64) + m
    return out


def _k_word_offset(W, r, nwp):
    """Byte offset, inside a K tile of nwp words per token, of word W of token r (0..63).
    Words go out in runs of four (a wavefront reads 1 KiB per 16-byte load, lane = token);
    if nwp is not a multiple of four the last two words form a run of their own."""
    full = 4 * (nwp // 4)
    if W < full:
        return 1024 * (W // 4) + 16 * r + 4 * (W % 4)
    return 256 * full + 8 * r + 4 * (W - full)


def _k_code_bit(b, j):
    """Bit position inside its 32-bit word of slot j of the word (a b-bit word holds
    32/b slots).  Slot j = 4k + e is element e of the word's step k; elements (0, 1)
    sit at one bit field of the low and high 16-bit half, elements (2, 3) at the next
    field: bit 16 (e % 2) + b (e // 2) + 2 b k.  A 16-bit word holds its two slots in
    its two halves."""
    if b == 16:
        return 16 * j
    k, e = j // 4, j % 4
    return 16 * (e % 2) + b * (e // 2) + 2 * b * k


def _k_slot_words(sl):
    """(tier b, slot index inside the tier, word index inside the row, slot inside the
    word) for every slot of the sorted-channel order."""
    out, word0 = [], 0
    for b in PACK_ORDER:
        per_word = 32 // b
        for s in range(sl["npad"][b]):
            out.append((b, s, word0 + s // per_word, s % per_word))
        word0 += sl["nw"][b]
    return out


def pack_k_tiles_mixed(codes, scale, off, bits_ch, per_unit=False):
    """Physical K tiles (64 tokens) of one tier segment in mixed mode.

    Tile data: token r of the tile owns n_words_padded 32-bit words (_k_word_offset);
    the words of the 16-bit channels come first, then the 8-, 4- and 2-bit words, slots
    in sorted-channel order inside a tier (_k_code_bit).
    Tile metadata: for token group G (rows 32G..32G+31 of the tile) and quantized step
    sq (4 consecutive slots of the 8/4/2-bit tiers): fp16 element 8 (G n_qsteps + sq) + e
    is the scale of the step's slot e, element + 4 its offset.
    per_unit (one scale per channel over all retained tokens, App. B): the metadata is a
    single record of that form for the whole segment (scale and off have one row).
    Rows beyond n in the last tile and padding slots are zero.
    Returns (data uint8, meta uint8)."""
    n, d = codes.shape
    sl = channel_slots(bits_ch)
    R = TILE64_ROWS
    nt = (n + R - 1) // R
    nwp, nqs = sl["n_words_padded"], sl["n_qsteps"]
    data = np.zeros((nt, 64 * nwp), dtype="<u4")
    meta = np.zeros((min(nt, 1), 8 * nqs) if per_unit else (nt, 16 * nqs), dtype="<u2")
    cp = np.zeros((nt * R, d), dtype=np.uint32)
    cp[:n] = codes
    cp = cp.reshape(nt, R, d)
    if not per_unit:
        ng = scale.shape[0]
        sg = np.zeros((2 * nt, d), dtype=np.uint16)
        og = np.zeros((2 * nt, d), dtype=np.uint16)
        sg[:ng], og[:ng] = scale, off
        sg, og = sg.reshape(nt, 2, d), og.reshape(nt, 2, d)
    rows = np.arange(R)
    qs = 0
    for (b, s, W, j), ch in zip(_k_slot_words(sl), sl["slot_ch"]):
        if b != 16:
            if ch >= 0 and per_unit:
                if nt > 0:
                    meta[0, 8 * (qs // 4) + qs % 4] = scale[0, ch]
                    meta[0, 8 * (qs // 4) + 4 + qs % 4] = off[0, ch]
            elif ch >= 0:
                for G in range(2):
                    meta[:, 8 * (G * nqs + qs // 4) + qs % 4] = sg[:, G, ch]
                    meta[:, 8 * (G * nqs + qs // 4) + 4 + qs % 4] = og[:, G, ch]
            qs += 1
        if ch < 0:
            continue
        widx = np.array([_k_word_offset(W, r, nwp) // 4 for r in rows])
        data[:, widx] |= cp[:, :, ch] << np.uint32(_k_code_bit(b, j))
    return data.view(np.uint8).reshape(-1), meta.view(np.uint8).reshape(-1)


def unpack_k_tiles_mixed(data, meta, n, bits_ch, d=128, per_unit=False):
    """Inverse of pack_k_tiles_mixed for the first n rows: (codes, scale, off)."""
    sl = channel_slots(bits_ch)
    R = TILE64_ROWS
    nt = (n + R - 1) // R
    ng = 1 if per_unit else (n + K_TOKEN_GROUP - 1) // K_TOKEN_GROUP
    nwp, nqs = sl["n_words_padded"], sl["n_qsteps"]
    data = np.asarray(data, dtype=np.uint8).view("<u4").reshape(nt, 64 * nwp)
    meta = np.asarray(meta, dtype=np.uint8).view("<u2").reshape((1, 8 * nqs) if per_unit else (nt, 16 * nqs))
    codes = np.zeros((nt, R, d), dtype=np.uint16)
    scale = np.zeros((max(2 * nt, 1), d), dtype=np.uint16)
    off = np.zeros((max(2 * nt, 1), d), dtype=np.uint16)
    rows = np.arange(R)
    qs = 0
    for (b, s, W, j), ch in zip(_k_slot_words(sl), sl["slot_ch"]):
        if b != 16:
            if ch >= 0 and per_unit:
                scale[0, ch] = meta[0, 8 * (qs // 4) + qs % 4]
                off[0, ch] = meta[0, 8 * (qs // 4) + 4 + qs % 4]
            elif ch >= 0:
                for G in range(2):
                    scale[G::2, ch] = meta[:, 8 * (G * nqs + qs // 4) + qs % 4]
                    off[G::2, ch] = meta[:, 8 * (G * nqs + qs // 4) + 4 + qs % 4]
            qs += 1
        if ch < 0:
            continue
        widx = np.array([_k_word_offset(W, r, nwp) // 4 for r in rows])
        codes[:, :, ch] = (data[:, widx] >> np.uint32(_k_code_bit(b, j))) & np.uint32((1 << b) - 1)
    return codes.reshape(nt * R, d)[:n], scale[:ng], off[:ng]


def _v16_position(r, c):
    """16-bit element index, inside a 16 KiB tile of 64 bf16 V rows, of (row r, channel c):
    lane 32 (r // 32) + c % 32 holds channel c for the 32 tokens of its tile half, eight
    tokens per 16-byte unit; unit u = 4 (c // 32) + (r % 32) // 8 sits at byte 1024 u + 16 lane."""
    lane, u = 32 * (r // 32) + c % 32, 4 * (c // 32) + (r % 32) // 8
    return (1024 * u + 16 * lane) // 2 + r % 8


def pack_v16_tiles(vbits):
    """Mixed mode keeps 16-bit V rows (Zone B of Sec. 3.3) in 64-token tiles with the
    lane assignment of the quantized V tiers (a lane holds one channel for 32 tokens).
    vbits: uint16 [n, 128].  Returns uint8 [tiles * 16384]."""
    n = vbits.shape[0]
    R = TILE64_ROWS
    nt = (n + R - 1) // R
    vp = np.zeros((nt * R, 128), dtype=np.uint16)
    vp[:n] = vbits
    vp = vp.reshape(nt, R, 128)
    out = np.zeros((nt, R * 128), dtype="<u2")
    for r in range(R):
        for c in range(128):
            out[:, _v16_position(r, c)] = vp[:, r, c]
    return out.view(np.uint8).reshape(-1)


def unpack_v16_tiles(data, n):
    R = TILE64_ROWS
    nt = (n + R - 1) // R
    w = np.asarray(data, dtype=np.uint8).view("<u2").reshape(nt, R * 128)
    out = np.zeros((nt, R, 128), dtype=np.uint16)
    for r in range(R):
        for c in range(128):
            out[:, r, c] = w[:, _v16_position(r, c)]
    return out.reshape(nt * R, 128)[:n]


def build_cache_mixed(K_list, V_list, bits_tok_list, bits_ch_list, k_per_channel_scale=False, group=GROUP):
    """Pack a ragged batch in mixed mode (Alg. 1 Stage 4 as printed: V rows sorted by
    b_t^V into sub-segments, K rows of the retained tokens with channels sorted by
    b_c^K).  bits_tok_list[s]: uint8 [Hkv, T_s] (V token map); bits_ch_list[s]: uint8
    [Hkv, d] (K channel map).  Arena: per item and per V tier (16, 8, 4, 2) the four
    segments K data, K meta, V data, V meta, each on a 256-byte boundary; the K
    segments hold the channel-wise tiles of that tier's tokens.
    k_per_channel_scale: the paper's own K format (App. B): one scale and zero-point per
    channel over all retained tokens of the item (instead of groups of 32 tokens); every
    non-empty tier segment then carries the same single metadata record.
    Same keys as build_cache_tokenwise plus 'bits_ch' [items, d], 'mixed' = True and
    'k_per_unit'."""
    items = []
    for Ks, Vs, bt, bc in zip(K_list, V_list, bits_tok_list, bits_ch_list):
        for h in range(Ks.shape[0]):
            items.append((Ks[h], Vs[h], bt[h], bc[h]))
    d = K_list[0].shape[2]
    n_items = len(items)
    counts = np.zeros((n_items, 4), dtype=np.int32)
    seg_off = np.zeros((n_items, 4, 4), dtype=np.int64)
    chunks, tier_idx, canon = [], [], []
    cur = 0
    for i, (Kh, Vh, bt, bc) in enumerate(items):
        Kh = _check_bf16_exact(Kh, "K")
        Vh = _check_bf16_exact(Vh, "V")
        idx = partition(bt)
        rec = {}
        if k_per_channel_scale:          # the unit is the channel over every retained token, whatever its V tier
            all_pos = np.concatenate([idx[b] for b in PACK_ORDER])
            kc_all, ks_all, ko_all = quantize_channelwise(Kh[all_pos], bc, None)
            row0 = 0
        for ti, b in enumerate(PACK_ORDER):
            pos = idx[b]
            n = len(pos)
            counts[i, ti] = n
            tier_idx.append(pos)
            if k_per_channel_scale:
                kc, ks, ko = kc_all[row0:row0 + n], ks_all, ko_all
                row0 += n
                kd, km = pack_k_tiles_mixed(kc, ks, ko, bc, per_unit=True)
            else:
                kc, ks, ko = quantize_channelwise(Kh[pos], bc)
                kd, km = pack_k_tiles_mixed(kc, ks, ko, bc)
            if b == 16:
                vcodes = bf16_bits(Vh[pos]).reshape(n, d)
                vd, vm = pack_v16_tiles(vcodes), np.zeros(0, dtype=np.uint8)
                rec[b] = {"pos": pos, "k_codes": kc, "k_scale": ks, "k_off": ko, "v_codes": vcodes}
            else:
                c, sc, m = quantize_rows(Vh[pos], b, group)       # group = d: one scale per V token row (App. B)
                sc, m = np.ascontiguousarray(sc), np.ascontiguousarray(m)
                vd, vm = pack_tiles64(c, sc.view(np.uint16), m.view(np.uint16), b, "v")
                rec[b] = {"pos": pos, "k_codes": kc, "k_scale": ks, "k_off": ko, "v_codes": c,
                          "v_scale": sc.view(np.uint16), "v_off": m.view(np.uint16)}
            for si, seg in enumerate((kd, km, vd, vm)):
                cur = _round_up(cur, SEG_ALIGN)
                seg_off[i, ti, si] = cur
                if seg.size:
                    chunks.append((cur, seg))
                    cur += seg.size
        canon.append(rec)
    arena = np.zeros(_round_up(cur, SEG_ALIGN), dtype=np.uint8)
    for o, flat in chunks:
        arena[o:o + flat.size] = flat
    return {
        "counts": counts,
        "tier_idx": np.concatenate(tier_idx).astype(np.int32) if tier_idx else np.zeros(0, np.int32),
        "seg_off": seg_off, "arena": arena, "canon": canon, "d": d, "hkv": K_list[0].shape[0],
        "seq_lens": [k.shape[1] for k in K_list], "mixed": True,
        "bits_ch": np.stack([it[3] for it in items]).astype(np.uint8),
        "k_per_unit": bool(k_per_channel_scale),
    }


def stored_bytes_mixed(counts, bits_ch, d=128, k_per_channel_scale=False):
    """Bytes a decode step must read in mixed mode (unpadded): per item and V tier with n
    rows, K codes n * sum_c b_c / 8, K metadata ceil(n / 32) * 4 per quantized channel (one fp16
    scale and offset per channel and group of 32 retained tokens; with one scale per channel
    the record is stored once per non-empty tier segment), and
    the V rows as in token-wise mode (n * (16 b + 16), or n * 256 at 16 bits)."""
    counts = np.asarray(counts, dtype=np.int64).reshape(-1, 4)
    total = 0
    for i in range(counts.shape[0]):
        bc = np.asarray(bits_ch[i], dtype=np.int64)
        kbits = int(bc.sum())
        nquant = int(((bc == 2) | (bc == 4) | (bc == 8)).sum())
        for ti, b in enumerate(PACK_ORDER):
            n = int(counts[i, ti])
            ngroups = (1 if n else 0) if k_per_channel_scale else (n + K_TOKEN_GROUP - 1) // K_TOKEN_GROUP
            total += n * kbits // 8 + ngroups * 4 * nquant
            total += n * (row_bytes(b, d) + meta_bytes(b, d))
    return total


def unpack_item_mixed(cache, item):
    """K_hat, V_hat (float64 [n_kept, d]) of one item of a mixed-mode cache, read back
    from the physical arena."""
    d = cache["d"]
    arena, seg_off, counts = cache["arena"], cache["seg_off"], cache["counts"]
    bc = cache["bits_ch"][item]
    sl = channel_slots(bc)
    tb, mb_ = k_tile_bytes_mixed(sl), k_meta_bytes_mixed(sl)
    ks, vs = [], []
    for ti, b in enumerate(PACK_ORDER):
        n = int(counts[item, ti])
        if n == 0:
            continue
        nt = (n + TILE64_ROWS - 1) // TILE64_ROWS
        o = [int(x) for x in seg_off[item, ti]]
        pu = cache.get("k_per_unit", False)
        kc, ksc, kof = unpack_k_tiles_mixed(arena[o[0]:o[0] + nt * tb], arena[o[1]:o[1] + (mb_ // 2 if pu else nt * mb_)],
                                            n, bc, d, per_unit=pu)
        ks.append(dequantize_channelwise(kc, ksc, kof, bc, None if pu else K_TOKEN_GROUP))
        if b == 16:
            vbits = unpack_v16_tiles(arena[o[2]:o[2] + nt * 16384], n)
            vs.append(bf16_from_bits(vbits).astype(np.float64))
        else:
            codes, sc, of = unpack_tiles64(arena[o[2]:o[2] + nt * tile64_data_bytes(b)],
                                           arena[o[3]:o[3] + nt * TILE64_META_BYTES], n, b, "v")
            vs.append(dequantize_groups(codes.reshape(n, d // GROUP, GROUP), sc.copy().view(np.float16),
                                        of.copy().view(np.float16)).reshape(n, d))
    if not ks:
        return np.zeros((0, d)), np.zeros((0, d))
    return np.concatenate(ks), np.concatenate(vs)


def allocate_mixed(w_tok, w_ch, avg_bits, r_k=np.float32(0.5), tiers=TIERS, eps_v=EPS_V_LLAMA31_8B,
                   eps_k=EPS_K_LLAMA31_8B, rel_tol=np.float32(1e-2), max_iters=64):
    """Stages 2 and 3 of Alg. 1 for one item: the V token map from the token weights
    with average 2 (1 - r_K) avg_bits, then the K channel map from the channel weights
    with the K budget spread over the retained tokens only.  w_tok: float32 [T];
    w_ch: float32 [d].  Returns (bits_tok uint8 [T], bits_ch uint8 [d])."""
    T, d = len(w_tok), len(w_ch)
    v_avg, _ = mixed_budgets(avg_bits, r_k, T, None, d)
    bits_tok = mckp_bisect(w_tok, np.float32(v_avg), tiers, eps_v, rel_tol, max_iters)
    n_kept = int((bits_tok > 0).sum())
    _, k_avg = mixed_budgets(avg_bits, r_k, T, n_kept, d)
    if n_kept == 0:
        return bits_tok, np.zeros(d, dtype=np.uint8)
    bits_ch = mckp_bisect(w_ch, np.float32(k_avg), tiers, eps_k, rel_tol, max_iters)
    return bits_tok, bits_ch


# --------------------------------------------------------------------------
# Decode (Sec. 3.3, Eq. 7): dense attention on the compressed cache (K_hat, V_hat)
# --------------------------------------------------------------------------
def attention_rows(q, Kh, Vh):
    """softmax(q K^T / sqrt(d)) V for each row of q over the given rows; fp64.
    q: [g, d]; Kh, Vh: [n, d].  Returns (out [g, d], lse [g]); n == 0 gives
    out = 0, lse = -inf."""
    q = np.asarray(q, dtype=np.float64)
    g, d = q.shape
    if Kh.shape[0] == 0:
        return np.zeros((g, d)), np.full(g, -np.inf)
    z = q @ Kh.T / math.sqrt(d)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    l = e.sum(axis=1, keepdims=True)
    return (e / l) @ Vh, (zmax + np.log(l))[:, 0]


def append_tokens(cache, k_new, v_new):
    """Zone C of Sec. 3.3 (third term of Eq. 7): tokens generated after the compression
    pass are kept uncompressed and attended to like any other row.  The paper keeps them
    in FP16; here the bf16 input values are kept verbatim (as for the 16-bit tier).
    k_new, v_new: float32 [batch, Hkv, d], bf16-exact: one new token per sequence.
    The rows are appended to cache['tail'][item] = (K rows, V rows)."""
    k_new = _check_bf16_exact(k_new, "k_new")
    v_new = _check_bf16_exact(v_new, "v_new")
    hkv, d = cache["hkv"], cache["d"]
    batch = len(cache["seq_lens"])
    assert k_new.shape == (batch, hkv, d) and v_new.shape == (batch, hkv, d)
    tail = cache.setdefault("tail", [(np.zeros((0, d)), np.zeros((0, d))) for _ in range(batch * hkv)])
    for s in range(batch):
        for h in range(hkv):
            tk, tv = tail[s * hkv + h]
            tail[s * hkv + h] = (np.concatenate([tk, k_new[s, h][None].astype(np.float64)]),
                                 np.concatenate([tv, v_new[s, h][None].astype(np.float64)]))


def decode(cache, q):
    """One decode step over a packed cache (token-wise or mixed).  q: [batch, Hq, d]
    (bf16 exact).  Every retained token enters with its dequantised K row and V row;
    evicted tokens (tier 0) are absent and evicted K channels are zero; appended tokens
    (append_tokens) enter with their bf16 rows (Eq. 7), appended tokens that were
    compressed later (rebudget_tail) with their dequantised rows.
    Returns out float64 [batch, Hq, d], lse float64 [batch, Hq]."""
    q = np.asarray(q, dtype=np.float64)
    batch, Hq, d = q.shape
    hkv = cache["hkv"]
    g = Hq // hkv
    out = np.zeros((batch, Hq, d))
    lse = np.zeros((batch, Hq))
    for s in range(batch):
        for h in range(hkv):
            item = s * hkv + h
            Kh, Vh = unpack_item_mixed(cache, item) if cache.get("mixed") else unpack_item(cache, item)
            for child in cache.get("absorbed", []):
                Kc, Vc = unpack_item_mixed(child, item) if child.get("mixed") else unpack_item(child, item)
                Kh, Vh = np.concatenate([Kh, Kc]), np.concatenate([Vh, Vc])
            if "tail" in cache:
                Kh, Vh = np.concatenate([Kh, cache["tail"][item][0]]), np.concatenate([Vh, cache["tail"][item][1]])
            o, l = attention_rows(q[s, h * g:(h + 1) * g], Kh, Vh)
            out[s, h * g:(h + 1) * g] = o
            lse[s, h * g:(h + 1) * g] = l
    return out, lse


def decode_dense(K_list, V_list, q):
    """Uncompressed decode: softmax(q K^T / sqrt(d)) V over all T tokens (Sec. 3)."""
    q = np.asarray(q, dtype=np.float64)
    batch, Hq, d = q.shape
    out = np.zeros((batch, Hq, d))
    lse = np.zeros((batch, Hq))
    for s in range(batch):
        Ks = np.asarray(K_list[s], dtype=np.float64)
        Vs = np.asarray(V_list[s], dtype=np.float64)
        hkv = Ks.shape[0]
        g = Hq // hkv
        for h in range(hkv):
            o, l = attention_rows(q[s, h * g:(h + 1) * g], Ks[h], Vs[h])
            out[s, h * g:(h + 1) * g] = o
            lse[s, h * g:(h + 1) * g] = l
    return out, lse


# --------------------------------------------------------------------------
# Streaming re-budgeting (App. "Limitations and Future Work": the extension to the decode phase)
# --------------------------------------------------------------------------
def rebudget_tail(cache, Qobs_list, budgets, tiers=TIERS, eps=EPS_V_LLAMA31_8B, pool_kernel=5, causal=True,
                  rel_tol=np.float32(1e-2), max_iters=64, weights_override=None, eps_k=EPS_K_LLAMA31_8B,
                  r_k=np.float32(0.5), group=GROUP):
    """The paper sketches the extension in one sentence: attention weights are gathered over a
    buffer of recent decode tokens and the same knapsack allocation is applied to compress
    them.  Reading taken here: the buffer is the whole appended-token zone; its n tokens are
    treated as a sequence of their own and go through Alg. 1 unchanged, in the mode of the
    cache (token-wise, or V token-wise and K channel-wise on the kept tokens) -- the probe
    queries are the decode queries of the last S_w appended tokens, window row i at tail
    position n - S_w + i, softmax over the tail's keys only -- with a budget of their own.
    The compressed rows join the cache as one more generation (cache['absorbed']); the tail is
    empty afterwards and can take new tokens.
    Qobs_list[s]: [Hq, S_w, d]; budgets[s]: average bits per element of the tail of sequence s.
    weights_override: token-wise caches: list of float32 [Hkv, n] token weights; mixed caches:
    (list of [Hkv, n] token weights, list of [Hkv, d] channel weights).
    Returns the child cache (also appended to cache['absorbed'])."""
    hkv, d = cache["hkv"], cache["d"]
    batch = len(cache["seq_lens"])
    tail = cache["tail"]
    n = tail[0][0].shape[0]
    assert n > 0 and all(t[0].shape[0] == n for t in tail)
    K_list = [np.stack([tail[s * hkv + h][0] for h in range(hkv)]).astype(np.float32) for s in range(batch)]
    V_list = [np.stack([tail[s * hkv + h][1] for h in range(hkv)]).astype(np.float32) for s in range(batch)]
    if cache.get("mixed"):
        bt_list, bc_list = [], []
        for s in range(batch):
            if weights_override is not None:
                w_tok = np.asarray(weights_override[0][s], dtype=np.float32)
                w_ch = np.asarray(weights_override[1][s], dtype=np.float32)
            else:
                w_tok = avg_pool(token_weights(K_list[s], Qobs_list[s], causal), pool_kernel).astype(np.float32)
                w_ch = channel_weights(K_list[s], Qobs_list[s]).astype(np.float32)
            bt = np.zeros((hkv, n), dtype=np.uint8)
            bc = np.zeros((hkv, d), dtype=np.uint8)
            for h in range(hkv):
                bt[h], bc[h] = allocate_mixed(w_tok[h], w_ch[h], budgets[s], r_k, tiers, eps, eps_k, rel_tol, max_iters)
            bt_list.append(bt)
            bc_list.append(bc)
        child = build_cache_mixed(K_list, V_list, bt_list, bc_list, k_per_channel_scale=cache["k_per_unit"],
                                  group=group)
        child["bits"] = bt_list
    else:
        child = compress_tokenwise(K_list, V_list, Qobs_list, budgets, tiers, eps, pool_kernel, causal, rel_tol,
                                   max_iters, weights_override, group)
    cache.setdefault("absorbed", []).append(child)
    cache["tail"] = [(np.zeros((0, d)), np.zeros((0, d))) for _ in range(batch * hkv)]
    return child


# --------------------------------------------------------------------------
# Distortion-table calibration (App. B "Calibration"; App. "Calibrated Distortion Tables", Table 9)
# --------------------------------------------------------------------------
CALIB_BITS = (2, 4, 8)


def _nmse(x, x_hat):
    """Normalized squared error of one (sequence, KV head) slice: sum (x - x_hat)^2 / sum x^2
    in fp64; a slice that is all zero reports 0."""
    x = np.asarray(x, dtype=np.float64)
    den = float((x * x).sum())
    if den == 0.0:
        return 0.0
    e = x - np.asarray(x_hat, dtype=np.float64)
    return float((e * e).sum()) / den


def calibrate_eps(K_list, V_list, k_channelwise=False, k_per_channel_scale=False, group=GROUP):
    """eps(b) of this build's quantizer on supplied K and V, b in (2, 4, 8): the normalized
    distortion the knapsack of Eq. 6 consumes (App. "Calibrated Distortion Tables": per-token NMSE for V, per-channel NMSE
    for K; eps(0) = 1 and eps(16) = 0 hold by definition and are not computed).  The paper
    estimates the table once per (layer, head) slice and averages; the slice values are
    returned here and averaging is left to the caller.

    Every token is retained (calibration sees the uncompressed prefix).  V: every token row in
    groups of `group` channels (32, or d = one scale per token row: the "per-token" of Table 9).  K: as V when k_channelwise is false (K rows share the token map);
    else per channel in groups of 32 consecutive tokens starting at token 0 (the last group may
    be short), or one scale per channel over all tokens with k_per_channel_scale (App. B).
    Returns (eps_k, eps_v): float64 [items, 3], item = s * Hkv + h."""
    rows_k, rows_v = [], []
    for Ks, Vs in zip(K_list, V_list):
        Ks = _check_bf16_exact(Ks, "K")
        Vs = _check_bf16_exact(Vs, "V")
        hkv, T, d = Ks.shape
        for h in range(hkv):
            ek, ev = [], []
            for b in CALIB_BITS:
                cv, sv, mv = quantize_groups(Vs[h].reshape(T, d // group, group), b)
                ev.append(_nmse(Vs[h], dequantize_groups(cv, sv, mv).reshape(T, d)))
                if not k_channelwise:
                    ck, sk, mk = quantize_groups(Ks[h].reshape(T, d // group, group), b)
                    ek.append(_nmse(Ks[h], dequantize_groups(ck, sk, mk).reshape(T, d)))
                else:
                    gt = None if k_per_channel_scale else K_TOKEN_GROUP
                    bc = np.full(d, b, dtype=np.uint8)
                    ck, sk, mk = quantize_channelwise(Ks[h], bc, group_tokens=gt)
                    ek.append(_nmse(Ks[h], dequantize_channelwise(ck, sk, mk, bc, group_tokens=gt)))
            rows_k.append(ek)
            rows_v.append(ev)
    return (np.asarray(rows_k, dtype=np.float64).reshape(-1, 3),
            np.asarray(rows_v, dtype=np.float64).reshape(-1, 3))


# --------------------------------------------------------------------------
# Whole compression pass, token-wise mode (Alg. 1 with K sharing the token map)
# --------------------------------------------------------------------------
def compress_tokenwise(K_list, V_list, Qobs_list, budgets, tiers=TIERS, eps=EPS_V_LLAMA31_8B,
                       pool_kernel=5, causal=True, rel_tol=np.float32(1e-2), max_iters=64,
                       weights_override=None, group=GROUP):
    """Weights -> pooling -> per-item bisection -> pack.  `weights_override`, if
    given, is a list of float32 [Hkv, T_s] arrays used instead of the computed
    weights (the bit-exact comparisons feed both sides identical fp32 weights)."""
    bits_list, w_list = [], []
    for s, (Ks, Qs) in enumerate(zip(K_list, Qobs_list)):
        if weights_override is not None:
            w = np.asarray(weights_override[s], dtype=np.float32)
        else:
            w = avg_pool(token_weights(Ks, Qs, causal), pool_kernel).astype(np.float32)
        w_list.append(w)
        bits = np.stack([mckp_bisect(w[h], budgets[s], tiers, eps, rel_tol, max_iters)
                         for h in range(w.shape[0])])
        bits_list.append(bits)
    cache = build_cache_tokenwise(K_list, V_list, bits_list, group)
    cache["bits"] = bits_list
    cache["weights"] = w_list
    return cache
