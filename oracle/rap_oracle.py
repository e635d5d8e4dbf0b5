"""Float64 CPU oracle for the RAP decode hot path.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition of what the decode-time path of RAP
(RoPE-Aligned Pruning) computes.  It exists to check the HIP library; it shares
no code with it, imports nothing from it, and must only be imported by the
tests, the smoke entry and the CPU-baseline leg of the benchmark.

Everything is NumPy float64.  bf16 storage is handled as raw uint16 bit
patterns; the two converters below are written from the IEEE-754 layout
(1 sign, 8 exponent, 7 fraction bits = the top half of a binary32).

Passages of the paper each function follows:

  inv_freq, rope_full      Sec. "Motivation: RoPE Incompatibility", Eq. (rope):
                           pair (j, j') rotated by R(t, theta_j),
                           theta_j = theta_base^(-2j/D), half-apart pairing
                           (x, x + D/2).
  rope_full_adjacent,      the other pairing named under Eq. (rope): neighbouring dims
  select_pairs_adjacent    (2x-1, 2x) in the paper's 1-based count, (2x, 2x+1) from 0; the
                           selection E_k for that pairing in the compact order.
  rope_compact             Sec. "RAP", index-aware rotation on the compressed
                           matrices (original indices of the retained pairs);
                           App. "Method", Eq. (selection-rope-intertwine),
                           block R_{t,S}.
  append_ref               Sec. "Background" (each new K_t, V_t is written into
                           a cache) + Sec. "Step 3: RAP Construction"
                           (the cache holds K_latent = RoPE(X W~_k), width 2m).
  attn_ref                 Eq. (attn) with the GQA remark under it;
                           Eq. (latent-score).
  rope_queries_ref         Eq. (latent-score), query side: RoPE(X W~_q) with the kept pairs of
                           the query head's KV head.
  attn_full_masked_ref     App. "Method", Eq. (masked-logit-equivalence): the
                           full-width right-hand side with removed pairs zeroed.
  mx4_*, append_mx4_ref,   the 4-bit (microscaling FP4) form of the cache: Sec. "Introduction" and
  attn_mx4_ref             "Related Work" (KV quantisation composes with RAP); format and scale rule
                           from the OCP Microscaling Formats specification.
  merge_partials_ref       log-sum-exp combination of row-partitioned softmax
                           partials (algebraic identity of Eq. (attn); the paper
                           itself has no split kernel).
  kept_pairs, kv_bytes_*   App. "Cost model" (Cache = rho * 2SD) and the
                           rounding of a budget to whole pairs; Tab. (effsweep),
                           Tab. (serving).

Parity pins (tests/test_oracle_*.py): rho=1 reduction to textbook RoPE attention,
zero-mask identity, intertwining identity, relative-position invariance, closed
forms, brute force with scalar math, and the paper's printed cost-table values.
Every function here has at least one such pin; nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# bf16 <-> float64, from the bit layout
# --------------------------------------------------------------------------


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as float64.

    A bf16 is the upper 16 bits of an IEEE binary32, so widening is a shift.
    """
    b = np.asarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("bf16 bit patterns must be uint16")
    with np.errstate(invalid="ignore"):      # signalling-NaN patterns are fine to widen
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    """Round float64 to bf16, nearest-even, in ONE rounding (no float32 detour).

    bf16 has 8 significant bits, exponent range of binary32 (normal minimum
    2^-126, subnormal quantum 2^-133, largest finite (2 - 2^-7) * 2^127).
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, dtype=np.uint16)
    sign = np.signbit(x)
    a = np.abs(x)

    nan = np.isnan(x)
    inf = np.isinf(x)
    fin = ~(nan | inf)

    af = np.where(fin, a, 0.0)
    m, e = np.frexp(af)                     # af = m * 2^e, m in [0.5, 1)
    # quantum of the target binade: 8 significant bits -> 2^(e-8); never finer
    # than the subnormal quantum 2^-133.
    qexp = np.maximum(e - 8, -133)
    scaled = np.ldexp(af, -qexp)            # exact (power-of-two scaling)
    n = np.rint(scaled)                     # ties to even
    val = np.ldexp(n, qexp)                 # the rounded magnitude, exact in f64

    # encode val (exactly representable in bf16, or overflowed past max finite)
    m2, e2 = np.frexp(val)                  # val = m2 * 2^e2
    biased = e2 - 1 + 127                   # exponent field if normal
    normal = (val > 0) & (biased >= 1)
    frac_n = np.rint(np.ldexp(m2, 8)).astype(np.int64) - 128      # 7 fraction bits
    with np.errstate(invalid="ignore", over="ignore"):            # lanes not taken by the selects below
        sub_n = np.rint(np.ldexp(np.minimum(val, 1.0), 133)).astype(np.int64)   # subnormal count
    mag = np.where(normal, (biased.astype(np.int64) << 7) | frac_n, sub_n)
    mag = np.where(biased >= 255, 0x7F80, mag)                     # overflow -> inf
    mag = np.where(val == 0, 0, mag)

    mag = np.where(inf, 0x7F80, mag)
    mag = np.where(nan, 0x7FC0, mag)
    out = (mag.astype(np.uint16) | (sign.astype(np.uint16) << np.uint16(15))).astype(np.uint16)
    out = np.where(nan, np.uint16(0x7FC0), out).astype(np.uint16)
    return out


# --------------------------------------------------------------------------
# RoPE
# --------------------------------------------------------------------------


def inv_freq(theta_base: float, d_head: int) -> np.ndarray:
    """theta_j = theta_base^(-2j/D), j = 0 .. D/2-1 (0-based pair index)."""
    j = np.arange(d_head // 2, dtype=np.float64)
    return np.float64(theta_base) ** (-2.0 * j / np.float64(d_head))


def rope_full(x: np.ndarray, t, theta_base: float) -> np.ndarray:
    """Full-width rotation of x[..., D] at position(s) t (broadcast over ...).

    Pair j couples dims (j, j + D/2); the 2x2 block is
    [[cos, -sin], [sin, cos]] with angle t * theta_j.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    phi = np.asarray(t, dtype=np.float64)[..., None] * inv_freq(theta_base, d)
    c, s = np.cos(phi), np.sin(phi)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def rope_compact(x: np.ndarray, t, keep: np.ndarray, theta_base: float, d_head: int) -> np.ndarray:
    """Index-aware rotation of a compact row x[..., 2P].

    Compact order: element c (< P) is original dim keep[c], element c + P is
    original dim keep[c] + D/2.  Pair c rotates at the ORIGINAL frequency index
    keep[c], not at c.
    """
    x = np.asarray(x, dtype=np.float64)
    keep = np.asarray(keep)
    p = keep.shape[-1]
    if x.shape[-1] != 2 * p:
        raise ValueError("row width must be 2 * number of kept pairs")
    f = inv_freq(theta_base, d_head)[keep]                      # [..., P]
    phi = np.asarray(t, dtype=np.float64)[..., None] * f
    c, s = np.cos(phi), np.sin(phi)
    a, b = x[..., :p], x[..., p:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def rope_compact_freq(x: np.ndarray, t, pair_freq: np.ndarray) -> np.ndarray:
    """Rotation of a compact row [..., 2P] whose pair c turns by pair_freq[c] radians per position:
    the form Eq. (rope) takes under the RoPE variants of Sec. "Practical Considerations" (a scaled
    frequency table gathered at the kept pairs) and under the hybrid rule (frequency 0 = a kept
    channel pair that is not rotated).  Same block [[cos, -sin], [sin, cos]] on (c, c + P)."""
    x = np.asarray(x, dtype=np.float64)
    pair_freq = np.asarray(pair_freq, dtype=np.float64)
    p = pair_freq.shape[-1]
    if x.shape[-1] != 2 * p:
        raise ValueError("compact row must have 2P elements")
    phi = np.asarray(t, dtype=np.float64)[..., None] * pair_freq
    c, s_ = np.cos(phi), np.sin(phi)
    a, b = x[..., :p], x[..., p:]
    return np.concatenate([a * c - b * s_, a * s_ + b * c], axis=-1)


def rope_full_adjacent(x: np.ndarray, t, theta_base: float) -> np.ndarray:
    """Full-width rotation of x[..., D] at position(s) t for models that pair NEIGHBOURING dims.

    Pair j couples dims (2j, 2j + 1) counted from 0 (the paper counts from 1: (2x - 1, 2x)); the
    block and the angle t * theta_j are those of Eq. (rope).  The result keeps the input's order.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    phi = np.asarray(t, dtype=np.float64)[..., None] * inv_freq(theta_base, d)
    c, s = np.cos(phi), np.sin(phi)
    a, b = x[..., 0::2], x[..., 1::2]
    out = np.empty(np.broadcast_shapes(x.shape, phi.shape[:-1] + (d,)), dtype=np.float64)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def select_pairs_adjacent(x_full: np.ndarray, keep: np.ndarray) -> np.ndarray:
    """E_k for the neighbouring pairing, in the compact order of this library: the first members
    of the kept pairs (dims 2 keep[c]), then their partners (dims 2 keep[c] + 1)."""
    keep = np.asarray(keep)
    idx = np.concatenate([2 * keep, 2 * keep + 1])
    return np.asarray(x_full)[..., idx]


def select_pairs(x_full: np.ndarray, keep: np.ndarray) -> np.ndarray:
    """E_k applied to a full-width row: gather dims keep and keep + D/2."""
    d = x_full.shape[-1]
    keep = np.asarray(keep)
    idx = np.concatenate([keep, keep + d // 2])
    return np.asarray(x_full)[..., idx]


# --------------------------------------------------------------------------
# Cache append
# --------------------------------------------------------------------------


def append_ref(k_new, v_new, pos, keep, k_cache, v_cache, theta_base, d_head, pair_freq=None):
    """Rotate each new compact K row at its position and store K, V rows.

    k_new   uint16 [B, n_new, H_kv, 2P]  bf16 bits, before rotation
    v_new   uint16 [B, n_new, H_kv, d_v] bf16 bits
    pos     int    [B, n_new]            position == destination row
    keep    int    [H_kv, P]             original pair index per KV head
    k_cache uint16 [B, H_kv, cap, 2P]    modified in place
    v_cache uint16 [B, H_kv, cap, d_v]   modified in place

    The rotated row is rounded to bf16 once, nearest-even, from float64;
    V is a bit copy.
    """
    k_new = np.asarray(k_new)
    v_new = np.asarray(v_new)
    pos = np.asarray(pos)
    keep = np.asarray(keep)
    bsz, n_new, n_kv, _ = k_new.shape
    kf = bf16_bits_to_f64(k_new)
    for b in range(bsz):
        for n in range(n_new):
            t = int(pos[b, n])
            for h in range(n_kv):
                if pair_freq is None:
                    rot = rope_compact(kf[b, n, h], np.float64(t), keep[h], theta_base, d_head)
                else:       # caller's frequency table [H_kv, P] instead of theta_base and keep
                    rot = rope_compact_freq(kf[b, n, h], np.float64(t), pair_freq[h])
                k_cache[b, h, t, :] = f64_to_bf16_bits_rne(rot)
                v_cache[b, h, t, :] = v_new[b, n, h, :]


# --------------------------------------------------------------------------
# Attention
# --------------------------------------------------------------------------


def softmax_ref(s: np.ndarray) -> np.ndarray:
    """softmax over the last axis, max-shifted."""
    s = np.asarray(s, dtype=np.float64)
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def attn_rows_ref(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """One KV head: q [G, d_k], k [S, d_k], v [S, d_v] (float64) -> [G, d_v]."""
    if k.shape[0] == 0:
        return np.zeros((q.shape[0], v.shape[1]), dtype=np.float64)
    s = (q @ k.T) * np.float64(scale)
    return softmax_ref(s) @ v


def attn_ref(q, k_cache, v_cache, seq_lens, scale) -> np.ndarray:
    """GQA decode attention over the compact cache.

    q        uint16 [B, H_q, d_k]        bf16 bits, pruned and already rotated
    k_cache  uint16 [B, H_kv, cap, d_k]
    v_cache  uint16 [B, H_kv, cap, d_v]
    seq_lens int    [B]                  rows [0, len) are attended
    returns  float64 [B, H_q, d_v]; a sequence of length 0 gives zeros.

    Query head a reads KV head a // G (contiguous groups).
    """
    q = np.asarray(q)
    bsz, n_q, _ = q.shape
    n_kv = k_cache.shape[1]
    g = n_q // n_kv
    if g * n_kv != n_q:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    d_v = v_cache.shape[3]
    out = np.zeros((bsz, n_q, d_v), dtype=np.float64)
    qf = bf16_bits_to_f64(q)
    for b in range(bsz):
        n = int(seq_lens[b])
        for h in range(n_kv):
            kf = bf16_bits_to_f64(k_cache[b, h, :n])
            vf = bf16_bits_to_f64(v_cache[b, h, :n])
            out[b, h * g:(h + 1) * g] = attn_rows_ref(qf[b, h * g:(h + 1) * g], kf, vf, scale)
    return out


def prefill_attn_ref(q, k_cache, v_cache, seq_lens, scale) -> np.ndarray:
    """Causal GQA attention of the last n_new tokens of every sequence over the compact cache
    (Eq. (attn) per query token with the decoder-only visibility rule: a token sees itself and
    everything before it; the rule itself is the standard one, the paper does not restate it).

    q        uint16 [B, n_new, H_q, d_k]  bf16 bits, pruned and already rotated; query i of
                                          sequence b sits at position p = seq_lens[b] - n_new + i
    k_cache  uint16 [B, H_kv, cap, d_k]   rows [0, seq_lens[b]) valid (the new tokens' own rows
    v_cache  uint16 [B, H_kv, cap, d_v]   are already in the cache)
    returns  float64 [B, n_new, H_q, d_v]; query i attends rows [0, p]; p < 0 gives zeros.
    """
    q = np.asarray(q)
    bsz, n_new, n_q, _ = q.shape
    n_kv = k_cache.shape[1]
    g = n_q // n_kv
    if g * n_kv != n_q:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    d_v = v_cache.shape[3]
    out = np.zeros((bsz, n_new, n_q, d_v), dtype=np.float64)
    qf = bf16_bits_to_f64(q)
    for b in range(bsz):
        n = int(seq_lens[b])
        for h in range(n_kv):
            kf = bf16_bits_to_f64(k_cache[b, h, :max(n, 0)])
            vf = bf16_bits_to_f64(v_cache[b, h, :max(n, 0)])
            for i in range(n_new):
                p = n - n_new + i
                if p < 0:
                    continue
                out[b, i, h * g:(h + 1) * g] = attn_rows_ref(qf[b, i, h * g:(h + 1) * g], kf[:p + 1], vf[:p + 1], scale)
    return out


def rope_queries_ref(q, q_pos, keep, theta_base, d_head, n_kv_heads, pair_freq=None) -> np.ndarray:
    """Query side of Eq. (latent-score): index-aware rotation of pruned, un-rotated query rows.

    q      uint16 [B, H_q, 2P] bf16 bits; q_pos int [B]; keep int [H_kv, P].
    Query head a uses the kept pairs of KV head a // G.  Returns bf16 bits (one nearest-even
    rounding from float64), i.e. what a rotation stage storing bf16 hands to the attention.
    """
    q = np.asarray(q)
    keep = np.asarray(keep)
    bsz, n_q, _ = q.shape
    g = n_q // n_kv_heads
    qf = bf16_bits_to_f64(q)
    out = np.empty_like(q)
    for b in range(bsz):
        for a_h in range(n_q):
            if pair_freq is None:
                rot = rope_compact(qf[b, a_h], np.float64(int(q_pos[b])), keep[a_h // g], theta_base, d_head)
            else:
                rot = rope_compact_freq(qf[b, a_h], np.float64(int(q_pos[b])), pair_freq[a_h // g])
            out[b, a_h] = f64_to_bf16_bits_rne(rot)
    return out


def attn_full_masked_ref(q_full, k_full, v_full, pos_q, pos_k, keep, keep_v, theta_base, scale):
    """Full-width attention with the removed pairs / channels zeroed.

    q_full float64 [G, D] and k_full [S, D] are UNROTATED full-width rows of one
    KV head; they are rotated here with rope_full at pos_q / pos_k[S], then the
    dims outside the kept pairs are zeroed in q and k, and the channels outside
    keep_v are zeroed in v_full [S, D].  Returns [G, D] (zeros in removed
    channels).
    """
    q_full = np.asarray(q_full, dtype=np.float64)
    k_full = np.asarray(k_full, dtype=np.float64)
    v_full = np.asarray(v_full, dtype=np.float64)
    d = q_full.shape[-1]
    mask = np.zeros(d)
    mask[np.asarray(keep)] = 1.0
    mask[np.asarray(keep) + d // 2] = 1.0
    vmask = np.zeros(d)
    vmask[np.asarray(keep_v)] = 1.0
    qr = rope_full(q_full, np.full(q_full.shape[:-1], pos_q, dtype=np.float64), theta_base) * mask
    kr = rope_full(k_full, np.asarray(pos_k, dtype=np.float64), theta_base) * mask
    return attn_rows_ref(qr, kr, v_full * vmask, scale)


def partial_ref(q, k, v, scale):
    """Un-normalised softmax partial of one row range: (m [G], l [G], acc [G, d_v])."""
    s = (q @ k.T) * np.float64(scale)
    m = np.max(s, axis=-1)
    e = np.exp(s - m[:, None])
    return m, np.sum(e, axis=-1), e @ v


def merge_partials_ref(ms, ls, accs):
    """Combine row-partitioned partials: out = sum_s e^{m_s-m*} acc_s / sum_s e^{m_s-m*} l_s."""
    ms = np.stack(ms)            # [n, G]
    ls = np.stack(ls)            # [n, G]
    accs = np.stack(accs)        # [n, G, d_v]
    mstar = np.max(ms, axis=0)
    w = np.exp(ms - mstar)
    return np.einsum("ng,ngd->gd", w, accs) / np.sum(w * ls, axis=0)[:, None]


# --------------------------------------------------------------------------
# fp8 (E4M3, finite-only "fn" flavour of the OCP 8-bit floating point
# specification) cache codes.  The paper calls KV quantisation orthogonal to
# RAP and composable with it (Sec. "Introduction", "Related Work") without
# fixing a format; this is the 8-bit format gfx950 converts natively.
# --------------------------------------------------------------------------


def e4m3_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint8 codes -> float64.  1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent field 0 is
    subnormal (m / 8 * 2^-6); there is no infinity, and S.1111.111 is NaN, so the largest finite
    magnitude is S.1111.110 = 448."""
    b = np.asarray(bits).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 0xF
    m = (b & 0x7).astype(np.float64)
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    val = np.where((b & 0x7F) == 0x7F, np.nan, val)
    return sign * val


def f64_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """float64 -> nearest E4M3 code, ties to the code with even mantissa, magnitudes above 448
    (infinities included) saturate to 448, NaN -> 0x7F.  Written as a search over the 127 finite
    non-negative codes so that it is the definition, not an algorithm."""
    x = np.asarray(x, dtype=np.float64)
    grid = e4m3_bits_to_f64(np.arange(0x7F, dtype=np.uint8))        # ascending: 0, 2^-9, ..., 448
    a = np.minimum(np.abs(x), 448.0)
    a = np.where(np.isnan(x), 0.0, a)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, 0x7E)    # first code >= a
    lo = np.clip(hi - 1, 0, 0x7E)
    d_hi, d_lo = grid[hi] - a, a - grid[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)


def append_q8_ref(k_new, v_new, pos, keep, k_cache8, v_cache8, k_scale, v_scale, theta_base, d_head, pair_freq=None):
    """append_ref into an fp8 cache: the rotated K row (float64) and the V row are divided by the
    per-KV-head scales k_scale[h], v_scale[h] (float32 values, taken as float64) and rounded once to
    E4M3.  k_cache8, v_cache8: uint8 [B, H_kv, cap, 2P / d_v], modified in place."""
    k_new = np.asarray(k_new)
    v_new = np.asarray(v_new)
    pos = np.asarray(pos)
    bsz, n_new, n_kv, _ = k_new.shape
    kf, vf = bf16_bits_to_f64(k_new), bf16_bits_to_f64(v_new)
    ks = np.asarray(k_scale, dtype=np.float32).astype(np.float64)
    vs = np.asarray(v_scale, dtype=np.float32).astype(np.float64)
    for b in range(bsz):
        for n in range(n_new):
            t = int(pos[b, n])
            for h in range(n_kv):
                if pair_freq is None:
                    rot = rope_compact(kf[b, n, h], np.float64(t), np.asarray(keep)[h], theta_base, d_head)
                else:
                    rot = rope_compact_freq(kf[b, n, h], np.float64(t), pair_freq[h])
                k_cache8[b, h, t, :] = f64_to_e4m3_bits(rot / ks[h])
                v_cache8[b, h, t, :] = f64_to_e4m3_bits(vf[b, n, h] / vs[h])


def attn_q8_ref(q, k_cache8, v_cache8, k_scale, v_scale, seq_lens, scale) -> np.ndarray:
    """attn_ref over an fp8 cache: every code stands for its value times the scale of its KV head."""
    q = np.asarray(q)
    bsz, n_q, _ = q.shape
    n_kv = k_cache8.shape[1]
    g = n_q // n_kv
    d_v = v_cache8.shape[3]
    out = np.zeros((bsz, n_q, d_v), dtype=np.float64)
    qf = bf16_bits_to_f64(q)
    ks = np.asarray(k_scale, dtype=np.float32).astype(np.float64)
    vs = np.asarray(v_scale, dtype=np.float32).astype(np.float64)
    for b in range(bsz):
        n = int(seq_lens[b])
        for h in range(n_kv):
            kf = e4m3_bits_to_f64(k_cache8[b, h, :n]) * ks[h]
            vf = e4m3_bits_to_f64(v_cache8[b, h, :n]) * vs[h]
            out[b, h * g:(h + 1) * g] = attn_rows_ref(qf[b, h * g:(h + 1) * g], kf, vf, scale)
    return out


def prefill_attn_q8_ref(q, k_cache8, v_cache8, k_scale, v_scale, seq_lens, scale) -> np.ndarray:
    """prefill_attn_ref over an fp8 cache: the same causal attention on the values the codes stand
    for (code value times the scale of its KV head).  q uint16 [B, n_new, H_q, d_k] bf16 bits."""
    q = np.asarray(q)
    bsz, n_new, n_q, _ = q.shape
    n_kv = k_cache8.shape[1]
    g = n_q // n_kv
    d_v = v_cache8.shape[3]
    out = np.zeros((bsz, n_new, n_q, d_v), dtype=np.float64)
    qf = bf16_bits_to_f64(q)
    ks = np.asarray(k_scale, dtype=np.float32).astype(np.float64)
    vs = np.asarray(v_scale, dtype=np.float32).astype(np.float64)
    for b in range(bsz):
        n = max(int(seq_lens[b]), 0)
        for h in range(n_kv):
            kf = e4m3_bits_to_f64(k_cache8[b, h, :n]) * ks[h]
            vf = e4m3_bits_to_f64(v_cache8[b, h, :n]) * vs[h]
            for i in range(n_new):
                p = n - n_new + i
                if p < 0:
                    continue
                out[b, i, h * g:(h + 1) * g] = attn_rows_ref(qf[b, i, h * g:(h + 1) * g], kf[:p + 1], vf[:p + 1], scale)
    return out


# --------------------------------------------------------------------------
# 4-bit cache: microscaling FP4 (the "MXFP4" of the OCP Microscaling Formats
# specification): elements are E2M1 codes (1 sign, 2 exponent bits with bias 1,
# 1 mantissa bit: +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}), and every block of 32
# consecutive elements of a row shares one E8M0 scale byte e standing for
# 2^(e - 127).  As for fp8 the paper only says that KV quantisation composes
# with RAP (Sec. "Introduction", "Related Work"); this is the 4-bit format
# gfx950 converts natively.  A row of d elements is stored as ceil(d / 32)
# blocks of 16 code bytes (element 2i of a block in the low nibble of byte i,
# element 2i + 1 in the high nibble; elements at and beyond d are code 0) and
# 4 scale bytes (those beyond the row's blocks hold 127).
# --------------------------------------------------------------------------

MX_BLOCK = 32
MX_SCALE_BYTES = 4


def mx_blocks(d: int) -> int:
    return (d + MX_BLOCK - 1) // MX_BLOCK


def e2m1_code_to_f64(code: np.ndarray) -> np.ndarray:
    """4-bit codes (0..15) -> float64, from the bit layout S.EE.M: exponent field 0 is subnormal
    (M * 0.5), else (1 + M / 2) * 2^(EE - 1); no infinity, no NaN."""
    c = np.asarray(code).astype(np.int64)
    sign = np.where(c & 0x8, -1.0, 1.0)
    e = (c >> 1) & 0x3
    m = (c & 0x1).astype(np.float64)
    val = np.where(e == 0, 0.5 * m, (1.0 + 0.5 * m) * np.exp2((e - 1).astype(np.float64)))
    return sign * val


def f64_to_e2m1_code(y: np.ndarray) -> np.ndarray:
    """float64 -> nearest E2M1 code, ties to the code with mantissa bit 0, magnitudes above 6
    saturate to 6.  A search over the eight magnitudes, so that it is the definition."""
    y = np.asarray(y, dtype=np.float64)
    grid = e2m1_code_to_f64(np.arange(8))                           # ascending: 0 .. 6
    a = np.minimum(np.abs(y), 6.0)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, 7)       # first magnitude >= a
    lo = np.clip(hi - 1, 0, 7)
    d_hi, d_lo = grid[hi] - a, a - grid[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    return np.where(np.signbit(y), code | 0x8, code).astype(np.uint8)


def mx_shared_exponent(amax: np.ndarray) -> np.ndarray:
    """Scale exponent of a block whose largest magnitude is amax: floor(log2 amax) minus the
    exponent of the largest E2M1 binade (2, since 4 <= 6 < 8), so that the block's largest element
    lands in [4, 8) before rounding; limited to [-126, 127]; 0 for a block of zeros."""
    amax = np.asarray(amax, dtype=np.float64)
    with np.errstate(divide="ignore"):
        fl = np.floor(np.log2(np.where(amax > 0, amax, 1.0)))
    # log2 of a double is correctly rounded only near exact powers by luck: repair with exact tests
    fl = np.where(np.exp2(fl) > amax, fl - 1, fl)
    fl = np.where(np.exp2(fl + 1) <= amax, fl + 1, fl)
    e = np.where(amax > 0, fl - 2, 0.0)
    return np.clip(e, -126, 127).astype(np.int64)


def mx4_quantize_rows(x: np.ndarray):
    """x float64 [..., d] -> (codes uint8 [..., 16 * blocks], scales uint8 [..., 4])."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    nb = mx_blocks(d)
    pad = np.zeros(x.shape[:-1] + (nb * MX_BLOCK,), dtype=np.float64)
    pad[..., :d] = x
    blk = pad.reshape(x.shape[:-1] + (nb, MX_BLOCK))
    e = mx_shared_exponent(np.abs(blk).max(axis=-1))                # [..., nb]
    q = f64_to_e2m1_code(blk / np.exp2(e.astype(np.float64))[..., None])    # division by a power of two: exact
    codes = (q[..., 0::2] | (q[..., 1::2] << 4)).astype(np.uint8).reshape(x.shape[:-1] + (nb * 16,))
    scales = np.full(x.shape[:-1] + (MX_SCALE_BYTES,), 127, dtype=np.uint8)
    scales[..., :nb] = (e + 127).astype(np.uint8)
    return codes, scales


def mx4_dequantize_rows(codes: np.ndarray, scales: np.ndarray, d: int) -> np.ndarray:
    """Inverse layout walk: float64 [..., d]; a scale byte of 255 is NaN (the format's rule)."""
    codes = np.asarray(codes)
    nb = mx_blocks(d)
    c = codes.reshape(codes.shape[:-1] + (nb, 16))
    q = np.empty(codes.shape[:-1] + (nb, MX_BLOCK), dtype=np.uint8)
    q[..., 0::2] = c & 0xF
    q[..., 1::2] = c >> 4
    sb = np.asarray(scales)[..., :nb].astype(np.int64)
    sc = np.where(sb == 255, np.nan, np.exp2((sb - 127).astype(np.float64)))
    val = e2m1_code_to_f64(q) * sc[..., None]
    return val.reshape(codes.shape[:-1] + (nb * MX_BLOCK,))[..., :d]


def append_mx4_ref(k_new, v_new, pos, keep, k_codes, k_scales, v_codes, v_scales, theta_base, d_head):
    """append_ref into a 4-bit cache: the rotated K row (float64) and the V row are quantised block
    by block, each block with the scale its own largest magnitude asks for.  k_codes / v_codes:
    uint8 [B, H_kv, cap, 16 * blocks], k_scales / v_scales: uint8 [B, H_kv, cap, 4], in place."""
    k_new = np.asarray(k_new)
    v_new = np.asarray(v_new)
    pos = np.asarray(pos)
    bsz, n_new, n_kv, _ = k_new.shape
    kf, vf = bf16_bits_to_f64(k_new), bf16_bits_to_f64(v_new)
    for b in range(bsz):
        for n in range(n_new):
            t = int(pos[b, n])
            for h in range(n_kv):
                rot = rope_compact(kf[b, n, h], np.float64(t), np.asarray(keep)[h], theta_base, d_head)
                k_codes[b, h, t], k_scales[b, h, t] = mx4_quantize_rows(rot)
                v_codes[b, h, t], v_scales[b, h, t] = mx4_quantize_rows(vf[b, n, h])


def attn_mx4_ref(q, k_codes, k_scales, v_codes, v_scales, seq_lens, scale, d_k: int, d_v: int) -> np.ndarray:
    """attn_ref over a 4-bit cache: every element stands for its code's value times its block's scale."""
    q = np.asarray(q)
    bsz, n_q, _ = q.shape
    n_kv = k_codes.shape[1]
    g = n_q // n_kv
    out = np.zeros((bsz, n_q, d_v), dtype=np.float64)
    qf = bf16_bits_to_f64(q)
    for b in range(bsz):
        n = int(seq_lens[b])
        for h in range(n_kv):
            kf = mx4_dequantize_rows(k_codes[b, h, :n], k_scales[b, h, :n], d_k)
            vf = mx4_dequantize_rows(v_codes[b, h, :n], v_scales[b, h, :n], d_v)
            out[b, h * g:(h + 1) * g] = attn_rows_ref(qf[b, h * g:(h + 1) * g], kf, vf, scale)
    return out


# --------------------------------------------------------------------------
# Paged caches (serving stacks): a pure re-indexing of the dense cache
# --------------------------------------------------------------------------


def paged_to_dense_ref(pool: np.ndarray, block_table: np.ndarray, n_rows) -> np.ndarray:
    """pool [n_pages, H, page_rows, d], block_table [B, max_pages], n_rows int or [B] ->
    dense [B, H, max_pages * page_rows, d] with row t of sequence b = row t % page_rows of page
    block_table[b][t // page_rows] for t < n_rows[b], zeros elsewhere (those table entries are
    not looked at)."""
    pool = np.asarray(pool)
    block_table = np.asarray(block_table)
    n_pages, n_heads, page_rows, d = pool.shape
    bsz, max_pages = block_table.shape
    n_rows = np.broadcast_to(np.asarray(n_rows), (bsz,))
    dense = np.zeros((bsz, n_heads, max_pages * page_rows, d), dtype=pool.dtype)
    for b in range(bsz):
        for t in range(int(n_rows[b])):
            dense[b, :, t, :] = pool[block_table[b, t // page_rows], :, t % page_rows, :]
    return dense


def dense_to_paged_ref(dense: np.ndarray, block_table: np.ndarray, page_rows: int, n_pages: int, n_rows, fill=0) -> np.ndarray:
    """Inverse arrangement: rows [0, n_rows[b]) of dense [B, H, cap, d] stored into a pool of
    n_pages pages through block_table; everything else in the pool holds `fill`."""
    dense = np.asarray(dense)
    block_table = np.asarray(block_table)
    bsz, n_heads, _, d = dense.shape
    n_rows = np.broadcast_to(np.asarray(n_rows), (bsz,))
    pool = np.full((n_pages, n_heads, page_rows, d), fill, dtype=dense.dtype)
    for b in range(bsz):
        for t in range(int(n_rows[b])):
            pool[block_table[b, t // page_rows], :, t % page_rows, :] = dense[b, :, t, :]
    return pool


# --------------------------------------------------------------------------
# Cost model (byte accounting)
# --------------------------------------------------------------------------


def kept_pairs(rho: float, d_head: int) -> int:
    """Budget rounded to whole pairs: m = round(rho * D / 2)."""
    return int(np.floor(rho * d_head / 2.0 + 0.5))


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, d_k: int, d_v: int, bytes_per_el: int = 2) -> int:
    """Resident KV state per token: layers * KV heads * (d_k + d_v) * element size."""
    return n_layers * n_kv_heads * (d_k + d_v) * bytes_per_el


def decode_kv_bytes(seq_lens, n_kv_heads: int, d_k: int, d_v: int, bytes_per_el: int = 2) -> int:
    """Bytes of K and V that one decode step must read once: sum_b H_kv * len_b * (d_k + d_v) * size."""
    return int(sum(int(n) for n in seq_lens)) * n_kv_heads * (d_k + d_v) * bytes_per_el
