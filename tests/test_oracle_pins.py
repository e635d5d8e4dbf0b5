"""Pins for the float64 oracle: everything here runs on the CPU and checks oracle/
against facts fixed by the paper or by mathematics, never against the HIP path.

Each test names the passage it comes from and the mistake it is meant to catch.
"""
import cmath
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import rap_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- bf16 conversion


def _all_finite_bf16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = O.bf16_bits_to_f64(bits)
    ok = np.isfinite(vals)
    return bits[ok], vals[ok]


def test_bf16_decode_against_bit_layout():
    """Value of a bf16 from its fields: (-1)^s 2^(e-127) (1 + f/128), subnormal 2^-126 f/128."""
    for bits in [0x0000, 0x8000, 0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0001, 0x007F, 0x0080, 0x7F7F, 0x4049, 0xC2F7]:
        s, e, f = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
        want = (f / 128.0) * 2.0 ** -126 if e == 0 else (1 + f / 128.0) * 2.0 ** (e - 127)
        want = -want if s else want
        got = O.bf16_bits_to_f64(np.array([bits], dtype=np.uint16))[0]
        assert got == want
    assert np.isinf(O.bf16_bits_to_f64(np.array([0x7F80], dtype=np.uint16))[0])
    assert np.isnan(O.bf16_bits_to_f64(np.array([0x7FC1], dtype=np.uint16))[0])


def test_bf16_round_trip_every_pattern():
    bits, vals = _all_finite_bf16()
    back = O.f64_to_bf16_bits_rne(vals)
    # -0.0 and +0.0 keep their sign bit as well
    assert np.array_equal(back, bits)


def test_bf16_rne_against_exhaustive_nearest_search():
    """Nearest-even by brute force over the sorted list of all finite bf16 values, in exact
    rational arithmetic.  Catches truncation, round-half-up, wrong subnormal quantum."""
    bits, vals = _all_finite_bf16()
    pos = vals >= 0
    pbits, pvals = bits[pos & (bits < 0x8000)], vals[pos & (bits < 0x8000)]
    order = np.argsort(pvals, kind="stable")
    pbits, pvals = pbits[order], pvals[order]
    rng = _rng(7)
    xs = list(np.abs(rng.standard_normal(300)) * 10.0 ** rng.integers(-42, 38, 300))
    # exact ties and near-ties between neighbours, normal and subnormal
    for i in [1, 2, 3, 126, 127, 128, 129, 5000, 16255, 16256, 16257, 20000, len(pvals) - 2]:
        lo, hi = Fraction(float(pvals[i])), Fraction(float(pvals[i + 1]))
        mid = (lo + hi) / 2
        xs += [float(mid), float(np.nextafter(float(mid), 0.0)), float(np.nextafter(float(mid), np.inf))]
    for x in xs:
        if x > float(pvals[-1]):
            continue
        i = int(np.searchsorted(pvals, x, side="right")) - 1
        i = max(i, 0)
        cands = [i] if i + 1 >= len(pvals) else [i, i + 1]
        fx = Fraction(x)
        best = min(cands, key=lambda c: (abs(Fraction(float(pvals[c])) - fx), int(pbits[c]) & 1))
        got = O.f64_to_bf16_bits_rne(np.array([x, -x]))
        assert got[0] == pbits[best], (x, hex(got[0]), hex(pbits[best]))
        assert got[1] == (pbits[best] | 0x8000)


def test_bf16_rne_matches_torch_cast_from_float32():
    """Library routine as a second opinion: torch's float32 -> bfloat16 cast is RNE."""
    rng = _rng(11)
    x32 = (rng.standard_normal(200000) * 10.0 ** rng.integers(-30, 30, 200000)).astype(np.float32)
    x32 = np.concatenate([x32, np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, 6e-41], dtype=np.float32)])
    want = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.f64_to_bf16_bits_rne(x32.astype(np.float64))
    assert np.array_equal(got, want)


def test_bf16_overflow_inf_nan():
    got = O.f64_to_bf16_bits_rne(np.array([1e39, -1e39, np.inf, -np.inf, 3.3961775292304601e38]))
    assert list(got[:4]) == [0x7F80, 0xFF80, 0x7F80, 0xFF80]
    assert got[4] == 0x7F80  # halfway between max finite and 2^128 rounds to even = inf
    assert O.f64_to_bf16_bits_rne(np.array([np.nan]))[0] & 0x7FFF > 0x7F80


# ---------------------------------------------------------------- RoPE


def test_inv_freq_values():
    """theta_j = theta_base^(-2j/D), 0-based j: pair 0 has frequency 1, the last pair
    theta_base^(-(D-2)/D).  Catches 1-based j or an exponent of j/D."""
    f = O.inv_freq(5.0e5, 128)
    assert f.shape == (64,)
    assert f[0] == 1.0
    assert math.isclose(f[63], 5.0e5 ** (-126.0 / 128.0), rel_tol=1e-15)
    assert math.isclose(f[32], 5.0e5 ** -0.5, rel_tol=1e-15)
    assert np.all(np.diff(f) < 0)


def test_rope_full_equals_complex_rotation():
    """Eq. (rope): the 2x2 block is multiplication of (x_j + i x_{j+D/2}) by e^{i t theta_j}.
    Written with cmath, one pair at a time.  Catches a flipped sine sign, adjacent pairing,
    swapped halves."""
    rng = _rng(3)
    d, theta = 16, 1.0e4
    x = rng.standard_normal(d)
    for t in [0, 1, 7, 1000, 131071]:
        y = O.rope_full(x, np.float64(t), theta)
        for j in range(d // 2):
            z = complex(x[j], x[j + d // 2]) * cmath.exp(1j * t * theta ** (-2.0 * j / d))
            assert math.isclose(y[j], z.real, rel_tol=0, abs_tol=1e-12)
            assert math.isclose(y[j + d // 2], z.imag, rel_tol=0, abs_tol=1e-12)


def test_rope_matrix_entries_one_pair():
    """The printed matrix [[cos, -sin], [sin, cos]] at t*theta_j = pi/2 maps (1, 0) to (0, 1)."""
    d, theta = 4, 1.0e4
    # pair 0 has frequency 1: t = pi/2 is not an integer position, so use the function with a float t
    y = O.rope_full(np.array([1.0, 0.0, 0.0, 0.0]), np.float64(math.pi / 2), theta)
    assert abs(y[0]) < 1e-15 and abs(y[2] - 1.0) < 1e-15


def test_rho1_compact_is_full_bit_for_bit():
    """E_k = I: index-aware rotation with keep = 0..D/2-1 is the standard rotation."""
    rng = _rng(4)
    x = rng.standard_normal((5, 128))
    t = np.array([0, 1, 17, 4097, 131071], dtype=np.float64)
    a = O.rope_full(x, t, 5.0e5)
    b = O.rope_compact(x, t, np.arange(64), 5.0e5, 128)
    assert np.array_equal(a, b)


def test_intertwining_identity():
    """App. Method, Eq. (selection-rope-intertwine): E_k R_t = R_{t,S} E_k.
    Catches rotating pair c at frequency c instead of keep[c]."""
    rng = _rng(5)
    d, p = 128, 45
    for trial in range(5):
        keep = np.sort(rng.choice(d // 2, p, replace=False))
        x = rng.standard_normal((3, d))
        t = rng.integers(0, 131072, 3).astype(np.float64)
        lhs = O.select_pairs(O.rope_full(x, t, 1.0e6), keep)
        rhs = O.rope_compact(O.select_pairs(x, keep), t, keep, 1.0e6, d)
        assert np.array_equal(lhs, rhs)
    # and it is NOT what a contiguous re-indexing would give
    wrong = O.rope_compact(O.select_pairs(x, keep), t, np.arange(p), 1.0e6, d)
    assert np.max(np.abs(wrong - rhs)) > 1e-3


def test_selection_matrix_facts():
    """App. Method: E_k E_k^T = I_2m; M_S = E_k^T E_k is a 0/1 diagonal mask; expanding the
    reduced row gives the masked row.  select_pairs is E_k."""
    rng = _rng(6)
    d, p = 16, 3
    keep = np.sort(rng.choice(d // 2, p, replace=False))
    E = O.select_pairs(np.eye(d), keep).T            # [2p, d]: row i picks original dim RAPIndex[i]
    assert np.array_equal(E @ E.T, np.eye(2 * p))
    M = E.T @ E
    assert np.array_equal(M, np.diag(np.diag(M))) and set(np.diag(M)) <= {0.0, 1.0}
    assert int(np.trace(M)) == 2 * p
    x = rng.standard_normal(d)
    assert np.array_equal(O.select_pairs(x, keep) @ E, x * np.diag(M))
    # R_t M_S = M_S R_t
    t = np.float64(37)
    assert np.allclose(O.rope_full(x * np.diag(M), t, 1e4), O.rope_full(x, t, 1e4) * np.diag(M), atol=0)


def test_adjacent_pairing_equals_complex_rotation():
    """Sec. "Motivation", the other pairing named under Eq. (rope): neighbouring dims, (2x - 1, 2x)
    counted from 1, i.e. (2j, 2j + 1) from 0, pair j at theta_j.  One pair at a time with cmath.
    Catches half-apart pairing used by mistake, a 1-based frequency index, a flipped sine."""
    rng = _rng(31)
    d, theta = 16, 1.0e4
    x = rng.standard_normal(d)
    for t in [0, 1, 7, 1000, 131071]:
        y = O.rope_full_adjacent(x, np.float64(t), theta)
        for j in range(d // 2):
            z = complex(x[2 * j], x[2 * j + 1]) * cmath.exp(1j * t * theta ** (-2.0 * j / d))
            assert math.isclose(y[2 * j], z.real, rel_tol=0, abs_tol=1e-12)
            assert math.isclose(y[2 * j + 1], z.imag, rel_tol=0, abs_tol=1e-12)
    # (1, 0) in pair 0 (frequency 1) at angle pi/2 becomes (0, 1): the partner is the NEXT dim
    y = O.rope_full_adjacent(np.array([1.0, 0.0, 0.0, 0.0]), np.float64(math.pi / 2), theta)
    assert abs(y[0]) < 1e-15 and abs(y[1] - 1.0) < 1e-15 and y[2] == 0.0 and y[3] == 0.0
    # and it differs from the half-apart rotation of the same row
    assert np.max(np.abs(O.rope_full_adjacent(x, np.float64(7), theta) - O.rope_full(x, np.float64(7), theta))) > 1e-2


def test_adjacent_pairing_needs_no_other_compact_rotation():
    """A model that pairs neighbouring dims reaches the same compact row: rotate the full row with
    the neighbouring pairing, select the kept pairs into [first members | partners], and the result
    is, bit for bit, rope_compact of the selected un-rotated row (E_k R_t = R_{t,S} E_k for that
    pairing's E_k).  So the library's compact layout and index-aware rotation serve both pairings;
    only the offline selection differs.  Also: scores between two such rows equal the full-width
    scores with the removed pairs zeroed."""
    rng = _rng(32)
    d, p = 128, 45
    for trial in range(5):
        keep = np.sort(rng.choice(d // 2, p, replace=False))
        x = rng.standard_normal((3, d))
        t = rng.integers(0, 131072, 3).astype(np.float64)
        lhs = O.select_pairs_adjacent(O.rope_full_adjacent(x, t, 1.0e6), keep)
        rhs = O.rope_compact(O.select_pairs_adjacent(x, keep), t, keep, 1.0e6, d)
        assert np.array_equal(lhs, rhs)
    # wrong frequency index (position in the compact row instead of the original pair) must differ
    wrong = O.rope_compact(O.select_pairs_adjacent(x, keep), t, np.arange(p), 1.0e6, d)
    assert np.max(np.abs(wrong - rhs)) > 1e-3
    # selection facts for this E_k: a 0/1 matrix with orthonormal rows that keeps pairs together
    E = O.select_pairs_adjacent(np.eye(16), np.array([1, 4, 6])).T
    assert np.array_equal(E @ E.T, np.eye(6))
    kept_dims = sorted(int(np.argmax(r)) for r in E)
    assert kept_dims == [2, 3, 8, 9, 12, 13]
    # masked-logit equivalence for the neighbouring pairing
    q, k = rng.standard_normal(d), rng.standard_normal((6, d))
    tq, tk = np.float64(900), np.arange(6, dtype=np.float64) + 890
    mask = np.zeros(d)
    mask[2 * keep] = 1.0
    mask[2 * keep + 1] = 1.0
    full = (O.rope_full_adjacent(q, tq, 5.0e5) * mask) @ (O.rope_full_adjacent(k, tk, 5.0e5) * mask).T
    comp = O.rope_compact(O.select_pairs_adjacent(q, keep), tq, keep, 5.0e5, d) @ \
        O.rope_compact(O.select_pairs_adjacent(k, keep), tk, keep, 5.0e5, d).T
    assert np.allclose(full, comp, rtol=0, atol=1e-12)


def test_relative_position_invariance():
    """R(t)^T R(u) = R(u - t): the score depends on the offset only, also on the compact row."""
    rng = _rng(8)
    d, p, theta = 128, 45, 5.0e5
    keep = np.sort(rng.choice(d // 2, p, replace=False))
    q = rng.standard_normal(2 * p)
    k = rng.standard_normal(2 * p)
    def score(t, u):
        return float(O.rope_compact(q, np.float64(t), keep, theta, d) @ O.rope_compact(k, np.float64(u), keep, theta, d))
    base = score(900, 123)
    for delta in [1, 64, 4096, 100000]:
        assert abs(score(900 + delta, 123 + delta) - base) < 1e-9
    assert abs(score(901, 123) - base) > 1e-6      # and it does depend on the offset


def test_closed_form_single_pair_score():
    """q-pair = k-pair = (r, 0) on kept pair c only: score = r^2 cos((t-u) theta_keep[c])."""
    d, theta = 128, 1.0e6
    keep = np.array([3, 10, 41])
    r, t, u = 1.75, 5000, 4211
    for c in range(3):
        x = np.zeros(6)
        x[c] = r
        s = float(O.rope_compact(x, np.float64(t), keep, theta, d) @ O.rope_compact(x, np.float64(u), keep, theta, d))
        want = r * r * math.cos((t - u) * theta ** (-2.0 * keep[c] / d))
        assert abs(s - want) < 1e-10


def test_rotation_preserves_pair_norm_and_pos0_is_identity():
    rng = _rng(9)
    keep = np.array([0, 5, 9, 63])
    x = rng.standard_normal(8)
    y = O.rope_compact(x, np.float64(77777), keep, 5e5, 128)
    assert np.allclose(x[:4] ** 2 + x[4:] ** 2, y[:4] ** 2 + y[4:] ** 2, rtol=1e-14)
    assert np.array_equal(O.rope_compact(x, np.float64(0), keep, 5e5, 128), x)


# ---------------------------------------------------------------- append


def _bf16_of(x):
    return O.f64_to_bf16_bits_rne(np.asarray(x, dtype=np.float64))


def test_append_writes_only_its_rows_and_copies_v():
    rng = _rng(10)
    B, n_new, H, P, dv, cap, D = 2, 3, 2, 3, 5, 16, 16
    keep = np.stack([np.sort(rng.choice(D // 2, P, replace=False)) for _ in range(H)])
    k_new = _bf16_of(rng.standard_normal((B, n_new, H, 2 * P)))
    v_new = _bf16_of(rng.standard_normal((B, n_new, H, dv)))
    pos = np.array([[4, 5, 6], [0, 9, 15]])
    kc = _bf16_of(rng.standard_normal((B, H, cap, 2 * P)))
    vc = _bf16_of(rng.standard_normal((B, H, cap, dv)))
    kc0, vc0 = kc.copy(), vc.copy()
    O.append_ref(k_new, v_new, pos, keep, kc, vc, 1e4, D)
    for b in range(B):
        touched = set(pos[b].tolist())
        for r in range(cap):
            if r in touched:
                n = pos[b].tolist().index(r)
                assert np.array_equal(vc[b, :, r], v_new[b, n])
                for h in range(H):
                    want = O.rope_compact(O.bf16_bits_to_f64(k_new[b, n, h]), np.float64(r), keep[h], 1e4, D)
                    assert np.array_equal(kc[b, h, r], _bf16_of(want))
            else:
                assert np.array_equal(kc[b, :, r], kc0[b, :, r]) and np.array_equal(vc[b, :, r], vc0[b, :, r])
    # position 0 rotates by nothing: the stored row is the input row, bit for bit
    assert np.array_equal(kc[1, :, 0], k_new[1, 0])


# ---------------------------------------------------------------- attention


def test_attention_equals_torch_sdpa_float64_with_gqa():
    """Eq. (attn) + GQA remark: a library routine (torch SDPA, float64, CPU) on explicitly
    repeat-interleaved KV heads.  Catches a//G vs a%H_kv, a transposed matmul, a missing scale."""
    rng = _rng(12)
    B, Hq, Hkv, dk, dv, S = 2, 6, 2, 10, 7, 33
    q = _bf16_of(rng.standard_normal((B, Hq, dk)))
    kc = _bf16_of(rng.standard_normal((B, Hkv, S, dk)))
    vc = _bf16_of(rng.standard_normal((B, Hkv, S, dv)))
    scale = 0.37
    got = O.attn_ref(q, kc, vc, np.array([S, S]), scale)
    tq = torch.from_numpy(O.bf16_bits_to_f64(q))[:, :, None, :]
    tk = torch.from_numpy(O.bf16_bits_to_f64(kc)).repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(O.bf16_bits_to_f64(vc)).repeat_interleave(Hq // Hkv, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)[:, :, 0, :].numpy()
    assert np.max(np.abs(got - want)) < 1e-13


def test_attention_respects_seq_lens():
    """Rows at and beyond len must not matter, whatever they hold; len = 1 returns V[0];
    len = 0 returns zeros."""
    rng = _rng(13)
    B, Hq, Hkv, dk, dv, cap = 3, 4, 2, 6, 5, 12
    q = _bf16_of(rng.standard_normal((B, Hq, dk)))
    kc = _bf16_of(rng.standard_normal((B, Hkv, cap, dk)))
    vc = _bf16_of(rng.standard_normal((B, Hkv, cap, dv)))
    lens = np.array([1, 7, 0])
    a = O.attn_ref(q, kc, vc, lens, 0.5)
    kc2, vc2 = kc.copy(), vc.copy()
    for b in range(B):
        kc2[b, :, lens[b]:] = 0x7F00   # huge finite
        vc2[b, :, lens[b]:] = 0xFF00
    assert np.array_equal(a, O.attn_ref(q, kc2, vc2, lens, 0.5))
    for a_h in range(Hq):
        assert np.array_equal(a[0, a_h], O.bf16_bits_to_f64(vc[0, a_h // 2, 0]))
    assert np.all(a[2] == 0)


def test_softmax_invariants():
    rng = _rng(14)
    s = rng.standard_normal((4, 1000)) * 20
    p = O.softmax_ref(s)
    assert np.max(np.abs(p.sum(-1) - 1)) < 1e-14
    assert np.all(p >= 0)
    assert np.max(np.abs(O.softmax_ref(s + 123.0) - p)) < 1e-12
    # equal keys -> mean of V; output inside the per-channel hull of V; row permutation invariance
    q = rng.standard_normal((3, 8))
    k = np.tile(rng.standard_normal(8), (50, 1))
    v = rng.standard_normal((50, 5))
    assert np.max(np.abs(O.attn_rows_ref(q, k, v, 0.3) - v.mean(0))) < 1e-13
    k = rng.standard_normal((50, 8))
    o = O.attn_rows_ref(q, k, v, 0.3)
    assert np.all(o <= v.max(0) + 1e-12) and np.all(o >= v.min(0) - 1e-12)
    perm = rng.permutation(50)
    assert np.max(np.abs(O.attn_rows_ref(q, k[perm], v[perm], 0.3) - o)) < 1e-13


def test_zero_mask_identity():
    """App. Method, Eq. (masked-logit-equivalence): reduced attention == full-width attention
    with removed pairs zeroed in q and k and removed channels zeroed in v, at the same scale."""
    rng = _rng(15)
    D, P, dv, G, S, theta = 128, 45, 90, 4, 40, 5.0e5
    keep = np.sort(rng.choice(D // 2, P, replace=False))
    keep_v = np.sort(rng.choice(D, dv, replace=False))
    qf = rng.standard_normal((G, D))
    kf = rng.standard_normal((S, D))
    vf = rng.standard_normal((S, D))
    pos_k = np.arange(S, dtype=np.float64) + 1000
    pos_q = 1000 + S - 1
    for scale in [1 / math.sqrt(D), 1 / math.sqrt(2 * P)]:
        full = O.attn_full_masked_ref(qf, kf, vf, pos_q, pos_k, keep, keep_v, theta, scale)
        qc = O.rope_compact(O.select_pairs(qf, keep), np.full(G, pos_q, dtype=np.float64), keep, theta, D)
        kc = O.rope_compact(O.select_pairs(kf, keep), pos_k, keep, theta, D)
        red = O.attn_rows_ref(qc, kc, vf[:, keep_v], scale)
        assert np.max(np.abs(full[:, keep_v] - red)) < 1e-12
        dropped = np.setdiff1d(np.arange(D), keep_v)
        assert np.all(full[:, dropped] == 0)
    # masking only q (or only k) already gives the same logits: M_S is idempotent
    mask = np.zeros(D)
    mask[keep] = 1
    mask[keep + D // 2] = 1
    qr = O.rope_full(qf, np.full(G, pos_q, dtype=np.float64), theta)
    kr = O.rope_full(kf, pos_k, theta)
    assert np.max(np.abs((qr * mask) @ kr.T - (qr * mask) @ (kr * mask).T)) < 1e-12
    assert np.max(np.abs(qr @ (kr * mask).T - qc @ kc.T)) < 1e-12


def test_rho1_attention_is_standard_rope_attention():
    """rho = 1: the whole chain (rotate K rows with all pairs, attend) equals textbook RoPE
    attention computed by SDPA on complex-rotated rows."""
    rng = _rng(16)
    D, G, S, theta = 16, 2, 9, 1.0e4
    qf, kf, vf = rng.standard_normal((G, D)), rng.standard_normal((S, D)), rng.standard_normal((S, D))
    keep = np.arange(D // 2)
    pos_k = np.arange(S, dtype=np.float64)
    qc = O.rope_compact(qf, np.full(G, S - 1.0), keep, theta, D)
    kc = O.rope_compact(kf, pos_k, keep, theta, D)
    got = O.attn_rows_ref(qc, kc, vf, 1 / math.sqrt(D))

    def crot(x, t):
        out = np.empty(D)
        for j in range(D // 2):
            z = complex(x[j], x[j + D // 2]) * cmath.exp(1j * t * theta ** (-2.0 * j / D))
            out[j], out[j + D // 2] = z.real, z.imag
        return out
    tq = torch.tensor(np.stack([crot(qf[g], S - 1) for g in range(G)]))[None, :, None, :]
    tk = torch.tensor(np.stack([crot(kf[i], i) for i in range(S)]))[None, None].expand(1, G, S, D)
    tv = torch.tensor(vf)[None, None].expand(1, G, S, D)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    assert np.max(np.abs(got - want)) < 1e-13


def test_query_rotation_pins():
    """rope_queries_ref: position 0 is the identity bit for bit; head a takes the pairs of KV head
    a // G (checked against a per-head scalar rotation with cmath); and rotating q and every key
    by the same extra offset leaves the float64 scores unchanged (relative-position property
    through the whole q-side + k-side chain, before any rounding)."""
    rng = _rng(21)
    B, Hq, Hkv, P, D, theta = 2, 6, 2, 5, 32, 1.0e4
    keep = np.stack([np.sort(rng.choice(D // 2, P, replace=False)) for _ in range(Hkv)])
    q = _bf16_of(rng.standard_normal((B, Hq, 2 * P)))
    assert np.array_equal(O.rope_queries_ref(q, np.zeros(B, dtype=int), keep, theta, D, Hkv), q)
    pos = np.array([7, 1234])
    got = O.rope_queries_ref(q, pos, keep, theta, D, Hkv)
    qf = O.bf16_bits_to_f64(q)
    for b in range(B):
        for a_h in range(Hq):
            kp = keep[a_h // 3]
            want = np.empty(2 * P)
            for c in range(P):
                z = complex(qf[b, a_h, c], qf[b, a_h, c + P]) * cmath.exp(1j * int(pos[b]) * theta ** (-2.0 * kp[c] / D))
                want[c], want[c + P] = z.real, z.imag
            assert np.array_equal(got[b, a_h], _bf16_of(want))
    # offset invariance of scores in float64
    k = rng.standard_normal((9, 2 * P))
    kpos = np.arange(9, dtype=np.float64) + 100
    def scores(delta):
        qr = O.rope_compact(qf[0, 0], np.float64(108 + delta), keep[0], theta, D)
        kr = O.rope_compact(k, kpos + delta, keep[0], theta, D)
        return kr @ qr
    assert np.max(np.abs(scores(0) - scores(54321))) < 1e-9


def _brute_force(k_new_vals, v_vals, q_vals, keep, theta, D, scale, G):
    """Whole path with scalar math only: rotate, round to bf16 by nearest search, attend."""
    bits_all = np.arange(0x7F80, dtype=np.uint32).astype(np.uint16)
    vals_all = O.bf16_bits_to_f64(bits_all).tolist()      # ascending non-negative finite values

    def rne(x):
        a = abs(x)
        import bisect
        i = max(bisect.bisect_right(vals_all, a) - 1, 0)
        cands = [i, i + 1] if i + 1 < len(vals_all) else [i]
        best = min(cands, key=lambda c: (abs(Fraction(vals_all[c]) - Fraction(a)), c & 1))
        return math.copysign(vals_all[best], x)

    S, H, P = len(k_new_vals), len(keep), len(keep[0])
    kc = [[[0.0] * (2 * P) for _ in range(S)] for _ in range(H)]
    for t in range(S):
        for h in range(H):
            for c in range(P):
                phi = t * theta ** (-2.0 * keep[h][c] / D)
                a, b = k_new_vals[t][h][c], k_new_vals[t][h][c + P]
                kc[h][t][c] = rne(a * math.cos(phi) - b * math.sin(phi))
                kc[h][t][c + P] = rne(a * math.sin(phi) + b * math.cos(phi))
    dv = len(v_vals[0][0])
    out = [[0.0] * dv for _ in range(H * G)]
    for a_h in range(H * G):
        h = a_h // G
        s = [scale * sum(q_vals[a_h][c] * kc[h][t][c] for c in range(2 * P)) for t in range(S)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = sum(e)
        for c in range(dv):
            out[a_h][c] = sum(e[t] * v_vals[t][h][c] for t in range(S)) / z
    return kc, out


@pytest.mark.parametrize("P,dv,G,S", [(1, 1, 1, 1), (2, 3, 3, 5), (3, 1, 1, 4), (3, 3, 3, 2), (2, 1, 3, 3)])
def test_brute_force_tiny(P, dv, G, S):
    """D = 8: explicit Python loops with math.cos/sin/exp against append_ref + attn_ref."""
    rng = _rng(100 + P * 31 + dv * 7 + G * 3 + S)
    D, H, theta, scale = 8, 2, 1.0e4, 0.6
    keep = np.stack([np.sort(rng.choice(D // 2, P, replace=False)) for _ in range(H)])
    k_new = _bf16_of(rng.standard_normal((1, S, H, 2 * P)) * 2)
    v_new = _bf16_of(rng.standard_normal((1, S, H, dv)))
    q = _bf16_of(rng.standard_normal((1, H * G, 2 * P)))
    kc = np.zeros((1, H, S + 3, 2 * P), dtype=np.uint16)
    vc = np.zeros((1, H, S + 3, dv), dtype=np.uint16)
    O.append_ref(k_new, v_new, np.arange(S)[None, :], keep, kc, vc, theta, D)
    got = O.attn_ref(q, kc, vc, np.array([S]), scale)[0]
    bk, bo = _brute_force(O.bf16_bits_to_f64(k_new[0]).tolist(), O.bf16_bits_to_f64(v_new[0]).tolist(),
                          O.bf16_bits_to_f64(q[0]).tolist(), keep.tolist(), theta, D, scale, G)
    assert np.array_equal(O.bf16_bits_to_f64(kc[0, :, :S]), np.array(bk))
    assert np.max(np.abs(got - np.array(bo))) < 1e-14


# ---------------------------------------------------------------- causal prefill attention


def test_prefill_equals_torch_sdpa_causal_float64():
    """Full prefill (len == n_new): a library routine (torch SDPA, float64, CPU, is_causal) on
    explicitly repeat-interleaved KV heads.  Catches an off-by-one in the visible range, a
    transposed operand, a wrong head mapping."""
    rng = _rng(41)
    B, Hq, Hkv, dk, dv, S = 2, 6, 2, 10, 7, 29
    q = _bf16_of(rng.standard_normal((B, S, Hq, dk)))
    kc = _bf16_of(rng.standard_normal((B, Hkv, S + 3, dk)))
    vc = _bf16_of(rng.standard_normal((B, Hkv, S + 3, dv)))
    scale = 0.41
    got = O.prefill_attn_ref(q, kc, vc, np.array([S, S]), scale)
    tq = torch.from_numpy(O.bf16_bits_to_f64(q)).permute(0, 2, 1, 3)
    tk = torch.from_numpy(O.bf16_bits_to_f64(kc[:, :, :S])).repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(O.bf16_bits_to_f64(vc[:, :, :S])).repeat_interleave(Hq // Hkv, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale, is_causal=True).permute(0, 2, 1, 3).numpy()
    assert np.max(np.abs(got - want)) < 1e-13


def test_prefill_closed_forms():
    """Identical keys make every visible row equally likely, so query i returns the plain mean of
    V rows [0, p_i] with p_i = len - n_new + i (chunked prefill: len > n_new); position 0 returns
    V[0]; a sequence shorter than n_new gives zero rows for the queries before its start; heads
    read their own KV head."""
    rng = _rng(42)
    B, Hq, Hkv, dk, dv, n_new, cap = 3, 4, 2, 6, 5, 7, 24
    lens = np.array([7, 19, 4])
    krow = rng.standard_normal((Hkv, dk))
    kc = _bf16_of(np.broadcast_to(krow[None, :, None, :], (B, Hkv, cap, dk)).copy())
    vc = _bf16_of(rng.standard_normal((B, Hkv, cap, dv)))
    q = _bf16_of(rng.standard_normal((B, n_new, Hq, dk)))
    got = O.prefill_attn_ref(q, kc, vc, lens, 0.8)
    vf = O.bf16_bits_to_f64(vc)
    for b in range(B):
        for i in range(n_new):
            p = lens[b] - n_new + i
            for a_h in range(Hq):
                want = vf[b, a_h // (Hq // Hkv), :p + 1].mean(axis=0) if p >= 0 else np.zeros(dv)
                assert np.max(np.abs(got[b, i, a_h] - want)) < 1e-14, (b, i, a_h)
    assert np.array_equal(got[0, 0, 0], vf[0, 0, 0])                       # position 0 sees only itself
    assert np.all(got[2, :3] == 0.0) and np.any(got[2, 3] != 0.0)            # len 4 < n_new 7


def test_prefill_causality_and_last_row_is_decode():
    """What lies after a query's position cannot change its output, and the last query of a
    sequence is the decode case (same rows, one query token)."""
    rng = _rng(43)
    B, Hq, Hkv, dk, dv, n_new, cap = 2, 6, 3, 8, 4, 5, 16
    lens = np.array([12, 9])
    q = _bf16_of(rng.standard_normal((B, n_new, Hq, dk)))
    kc = _bf16_of(rng.standard_normal((B, Hkv, cap, dk)))
    vc = _bf16_of(rng.standard_normal((B, Hkv, cap, dv)))
    base = O.prefill_attn_ref(q, kc, vc, lens, 0.5)
    kc2, vc2 = kc.copy(), vc.copy()
    for b in range(B):
        cut = lens[b] - 2                       # rows cut.. are later than query n_new - 3
        kc2[b, :, cut:] = _bf16_of(rng.standard_normal((Hkv, cap - cut, dk)) * 5)
        vc2[b, :, cut:] = _bf16_of(rng.standard_normal((Hkv, cap - cut, dv)) * 5)
    pert = O.prefill_attn_ref(q, kc2, vc2, lens, 0.5)
    assert np.array_equal(base[:, :n_new - 2], pert[:, :n_new - 2])
    assert not np.array_equal(base[:, n_new - 2:], pert[:, n_new - 2:])
    dec = O.attn_ref(q[:, -1], kc, vc, lens, 0.5)
    assert np.array_equal(base[:, -1], dec)


def test_prefill_brute_force_tiny():
    """Explicit Python loops with math.exp over every (query, visible row)."""
    rng = _rng(44)
    B, Hq, Hkv, dk, dv, n_new, cap, scale = 1, 4, 2, 3, 2, 4, 8, 0.7
    lens = np.array([6])
    q = _bf16_of(rng.standard_normal((B, n_new, Hq, dk)))
    kc = _bf16_of(rng.standard_normal((B, Hkv, cap, dk)))
    vc = _bf16_of(rng.standard_normal((B, Hkv, cap, dv)))
    got = O.prefill_attn_ref(q, kc, vc, lens, scale)
    qf, kf, vf = O.bf16_bits_to_f64(q).tolist(), O.bf16_bits_to_f64(kc).tolist(), O.bf16_bits_to_f64(vc).tolist()
    G = Hq // Hkv
    for i in range(n_new):
        p = int(lens[0]) - n_new + i
        for a_h in range(Hq):
            h = a_h // G
            sc = [scale * sum(qf[0][i][a_h][e] * kf[0][h][t][e] for e in range(dk)) for t in range(p + 1)]
            mx = max(sc)
            ex = [math.exp(x - mx) for x in sc]
            z = sum(ex)
            for c in range(dv):
                want = sum(ex[t] * vf[0][h][t][c] for t in range(p + 1)) / z
                assert abs(got[0, i, a_h, c] - want) < 1e-14


def test_frequency_table_rotation_pins():
    """rope_compact_freq: with the table theta^(-2 keep/D) it is rope_compact bit for bit; an entry
    of 0 leaves its pair untouched whatever the position (hybrid rule: un-rotated kept channels);
    any table keeps the relative-position invariant of the scores; one pair in closed form."""
    rng = _rng(77)
    D, P, theta = 128, 45, 5.0e5
    keep = np.sort(rng.choice(D // 2, P, replace=False))
    x = rng.standard_normal((5, 2 * P))
    t = np.array([0, 1, 17, 4095, 131071])
    table = O.inv_freq(theta, D)[keep]
    assert np.array_equal(O.rope_compact_freq(x, t, table), O.rope_compact(x, t, keep, theta, D))
    # a scaled table with some pairs switched off
    scaled = table * np.where(np.arange(P) % 3 == 0, 0.25, 1.0)
    scaled[[2, 7, 40]] = 0.0
    y = O.rope_compact_freq(x, t, scaled)
    for c in (2, 7, 40):
        assert np.array_equal(y[:, c], x[:, c]) and np.array_equal(y[:, c + P], x[:, c + P])
    q, k = rng.standard_normal(2 * P), rng.standard_normal(2 * P)
    s0 = O.rope_compact_freq(q, 1000, scaled) @ O.rope_compact_freq(k, 900, scaled)
    s1 = O.rope_compact_freq(q, 100 + 64, scaled) @ O.rope_compact_freq(k, 64, scaled)
    assert abs(s0 - s1) < 1e-9
    # one pair: (a, b) at position t with frequency f is the complex number (a + i b) e^{i t f}
    z = complex(0.75, -1.5) * cmath.exp(1j * 37 * 0.0123)
    r = O.rope_compact_freq(np.array([0.75, -1.5]), 37, np.array([0.0123]))
    assert abs(r[0] - z.real) < 1e-15 and abs(r[1] - z.imag) < 1e-15


def test_paged_arrangement_pins():
    """Paged caches are a re-indexing: a hand-written 2-page example, the identity table (= a
    reshape), round trips through a shuffled table, and attention over the gathered rows equal to
    attention over the dense cache."""
    pool = np.arange(3 * 1 * 2 * 1).reshape(3, 1, 2, 1)          # 3 pages x 1 head x 2 rows x 1 value: page p holds 2p, 2p+1
    bt = np.array([[2, 0], [1, 2]])
    dense = O.paged_to_dense_ref(pool, bt, [3, 4])
    assert dense[0, 0, :, 0].tolist() == [4, 5, 0, 0]            # rows 0, 1 from page 2, row 2 from page 0, row 3 beyond n_rows
    assert dense[1, 0, :, 0].tolist() == [2, 3, 4, 5]
    rng = _rng(91)
    B, H, page_rows, max_pages, d = 2, 3, 4, 5, 6
    dense = rng.integers(0, 60000, size=(B, H, max_pages * page_rows, d)).astype(np.uint16)
    ident = np.arange(B * max_pages).reshape(B, max_pages)
    pool = O.dense_to_paged_ref(dense, ident, page_rows, B * max_pages, max_pages * page_rows)
    assert np.array_equal(pool.reshape(B, max_pages, H, page_rows, d).transpose(0, 2, 1, 3, 4).reshape(dense.shape), dense)
    table = rng.permutation(B * max_pages + 3)[:B * max_pages].reshape(B, max_pages)
    lens = np.array([17, 9])
    pool = O.dense_to_paged_ref(dense, table, page_rows, B * max_pages + 3, lens, fill=7)
    back = O.paged_to_dense_ref(pool, table, lens)
    for b in range(B):
        assert np.array_equal(back[b, :, :lens[b]], dense[b, :, :lens[b]]) and np.all(back[b, :, lens[b]:] == 0)
    kc = _bf16_of(rng.standard_normal((B, H, max_pages * page_rows, d)))
    vc = _bf16_of(rng.standard_normal((B, H, max_pages * page_rows, 5)))
    q = _bf16_of(rng.standard_normal((B, 2 * H, d)))
    kp = O.dense_to_paged_ref(kc, table, page_rows, B * max_pages + 3, lens)
    vp = O.dense_to_paged_ref(vc, table, page_rows, B * max_pages + 3, lens)
    a1 = O.attn_ref(q, kc, vc, lens, 0.3)
    a2 = O.attn_ref(q, O.paged_to_dense_ref(kp, table, lens), O.paged_to_dense_ref(vp, table, lens), lens, 0.3)
    assert np.array_equal(a1, a2)


def test_e4m3_codes_and_rounding():
    """E4M3 (finite-only) decode against the values the format's specification lists (1.0, the
    largest finite 448, the smallest subnormal 2^-9, the smallest normal 2^-6, NaN) and the bit
    layout; encode against an exhaustive nearest search with ties to even, saturation and sign."""
    assert O.e4m3_bits_to_f64(np.array([0x38]))[0] == 1.0
    assert O.e4m3_bits_to_f64(np.array([0x7E]))[0] == 448.0 and O.e4m3_bits_to_f64(np.array([0xFE]))[0] == -448.0
    assert O.e4m3_bits_to_f64(np.array([0x01]))[0] == 2.0 ** -9 and O.e4m3_bits_to_f64(np.array([0x08]))[0] == 2.0 ** -6
    assert np.isnan(O.e4m3_bits_to_f64(np.array([0x7F, 0xFF]))).all()
    codes = np.arange(256, dtype=np.uint8)
    vals = O.e4m3_bits_to_f64(codes)
    for c in range(256):                                         # bit layout, by hand
        s_, e, m = c >> 7, (c >> 3) & 15, c & 7
        if (c & 0x7F) == 0x7F:
            continue
        want = (m / 8 * 2.0 ** -6) if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
        assert vals[c] == (-want if s_ else want)
    finite = (codes & 0x7F) != 0x7F
    back = O.f64_to_e4m3_bits(vals[finite])
    same = back == codes[finite]
    assert same[codes[finite] != 0x80].all()                     # every code but -0 returns to itself (-0 too, as 0x80)
    assert O.f64_to_e4m3_bits(np.array([-0.0]))[0] == 0x80
    pos = vals[:0x7F]                                            # ascending grid of non-negative finite values
    rng = _rng(5)
    x = np.concatenate([rng.uniform(0, 470, 4000), rng.uniform(0, 0.05, 2000), (pos[:-1] + pos[1:]) / 2, pos, [448.0, 464.0, 1e9, np.inf]])
    got = O.f64_to_e4m3_bits(x)
    for xi, gi in zip(x, got):
        a = min(xi, 448.0)
        d = np.abs(pos - a)
        best = np.flatnonzero(d == d.min())
        want = best[0] if len(best) == 1 else (best[0] if best[0] % 2 == 0 else best[1])   # tie: even mantissa
        assert gi == want, (xi, gi, want)
    assert O.f64_to_e4m3_bits(np.array([-3.3]))[0] == (O.f64_to_e4m3_bits(np.array([3.3]))[0] | 0x80)
    assert O.f64_to_e4m3_bits(np.array([np.nan]))[0] == 0x7F and O.f64_to_e4m3_bits(np.array([-np.inf]))[0] == 0xFE
    # midpoint 1.0625 between 1.0 (mantissa 000) and 1.125 (001) goes to the even one; 1.1875 to 1.25 (010)
    assert O.f64_to_e4m3_bits(np.array([1.0625, 1.1875])).tolist() == [0x38, 0x3A]


def test_q8_cache_pins():
    """The fp8 cache is the dense path on dequantised values: append codes decode to within half a
    code step of the rotated row over the scale, V likewise, and attention over the codes equals
    attn_ref over a bf16 cache holding exactly the dequantised values (every E4M3 value times a
    power-of-two scale is a bf16 number)."""
    rng = _rng(6)
    B, n_new, H, P, dv, cap, D, theta = 2, 3, 2, 4, 5, 16, 16, 1.0e4
    keep = np.stack([np.sort(rng.choice(D // 2, P, replace=False)) for _ in range(H)])
    k_new = _bf16_of(rng.standard_normal((B, n_new, H, 2 * P)) * 3)
    v_new = _bf16_of(rng.standard_normal((B, n_new, H, dv)))
    pos = np.array([[0, 1, 2], [7, 3, 11]])
    ks, vs = np.array([0.25, 0.5], dtype=np.float32), np.array([0.125, 1.0], dtype=np.float32)
    k8 = np.zeros((B, H, cap, 2 * P), dtype=np.uint8); v8 = np.zeros((B, H, cap, dv), dtype=np.uint8)
    O.append_q8_ref(k_new, v_new, pos, keep, k8, v8, ks, vs, theta, D)
    kd = np.zeros((B, H, cap, 2 * P), dtype=np.uint16); vd = np.zeros((B, H, cap, dv), dtype=np.uint16)
    O.append_ref(k_new, v_new, pos, keep, kd, vd, theta, D)       # same rows, bf16
    for b in range(B):
        for n in range(n_new):
            t = pos[b, n]
            for h in range(H):
                exact = O.rope_compact(O.bf16_bits_to_f64(k_new[b, n, h]), np.float64(t), keep[h], theta, D)
                deq = O.e4m3_bits_to_f64(k8[b, h, t]) * ks[h]
                step = np.maximum(np.abs(exact) / ks[h], 2.0 ** -6) * 2.0 ** -3 * ks[h]   # at most one code step
                assert np.all(np.abs(deq - exact) <= step / 2 * 1.0000001)
                assert np.array_equal(v8[b, h, t], O.f64_to_e4m3_bits(O.bf16_bits_to_f64(v_new[b, n, h]) / vs[h]))
    assert np.all(k8[0, :, 3:] == 0) and np.all(v8[1, :, 0] == 0)   # untouched rows
    q = _bf16_of(rng.standard_normal((B, 2 * H, 2 * P)))
    lens = np.array([3, 12])
    got = O.attn_q8_ref(q, k8, v8, ks, vs, lens, 0.4)
    kb = _bf16_of(O.e4m3_bits_to_f64(k8) * ks[None, :, None, None].astype(np.float64))
    vb = _bf16_of(O.e4m3_bits_to_f64(v8) * vs[None, :, None, None].astype(np.float64))
    assert np.array_equal(got, O.attn_ref(q, kb, vb, lens, 0.4))


def test_prefill_q8_pins():
    """Causal prefill over fp8 codes: equal to the bf16 prefill oracle on a cache that holds exactly
    the dequantised values (power-of-two scales), its last row equal to the fp8 decode oracle, and
    rows of a sequence shorter than n_new zero."""
    rng = _rng(23)
    B, n_new, Hq, H, dk, dv, cap = 2, 5, 4, 2, 6, 5, 12
    k8 = rng.integers(0, 0x7E, (B, H, cap, dk)).astype(np.uint8) | (rng.integers(0, 2, (B, H, cap, dk)).astype(np.uint8) << 7)
    v8 = rng.integers(0, 0x7E, (B, H, cap, dv)).astype(np.uint8) | (rng.integers(0, 2, (B, H, cap, dv)).astype(np.uint8) << 7)
    ks, vs = np.array([2.0 ** -5, 2.0 ** -4], dtype=np.float32), np.array([2.0 ** -6, 0.5], dtype=np.float32)
    q = _bf16_of(rng.standard_normal((B, n_new, Hq, dk)))
    lens = np.array([9, 3])
    got = O.prefill_attn_q8_ref(q, k8, v8, ks, vs, lens, 0.3)
    kb = _bf16_of(O.e4m3_bits_to_f64(k8) * ks[None, :, None, None].astype(np.float64))
    vb = _bf16_of(O.e4m3_bits_to_f64(v8) * vs[None, :, None, None].astype(np.float64))
    assert np.array_equal(got, O.prefill_attn_ref(q, kb, vb, lens, 0.3))
    assert np.array_equal(got[:, -1], O.attn_q8_ref(q[:, -1], k8, v8, ks, vs, lens, 0.3))
    assert np.all(got[1, :2] == 0) and np.any(got[1, 2] != 0)      # positions -2, -1 do not exist; position 0 does


# ---------------------------------------------------------------- 4-bit (microscaling FP4) cache


def test_e2m1_codes_and_rounding():
    """E2M1 as the microscaling formats specification lists it (exponent bias 1, largest normal 6,
    smallest normal 1, subnormal 0.5, no infinity or NaN): the eight magnitudes, the sign bit,
    nearest with ties to the even mantissa bit against exact rational arithmetic, saturation."""
    listed = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    vals = O.e2m1_code_to_f64(np.arange(16))
    assert list(vals[:8]) == listed and list(vals[8:]) == [-v for v in listed] and np.signbit(vals[8])
    rng = _rng(21)
    mids = [(a + b) / 2 for a, b in zip(listed[:-1], listed[1:])]
    xs = np.concatenate([np.array(listed), np.array(mids), np.nextafter(mids, 0.0), np.nextafter(mids, 10.0),
                         rng.uniform(0, 7, 4000), [6.0, 6.5, 7.99, 8.0, 1e9, np.inf, 2.0 ** -40]])
    got = O.f64_to_e2m1_code(np.concatenate([xs, -xs]))
    for x, c in zip(np.concatenate([xs, -xs]), got):
        a = Fraction(min(abs(x), 6.0)) if np.isfinite(x) else Fraction(6)
        dist = [abs(Fraction(v) - a) for v in listed]
        best = min(dist)
        cands = [k for k in range(8) if dist[k] == best]
        want = cands[0] if len(cands) == 1 else [k for k in cands if k % 2 == 0][0]
        assert int(c) & 7 == want and bool(int(c) & 8) == bool(np.signbit(x)), (x, c)
    # ties: 0.25 -> 0, 0.75 -> 1, 1.25 -> 1, 1.75 -> 2, 2.5 -> 2, 3.5 -> 4, 5 -> 4
    assert list(O.e2m1_code_to_f64(O.f64_to_e2m1_code(np.array(mids)))) == [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]


def test_mx_shared_exponent_rule():
    """Scale of a block: 2^(floor(log2 amax) - 2), so that amax / scale lies in [4, 8): the top
    binade of E2M1.  Exact at and next to powers of two, limited to [-126, 127], 0 for zeros."""
    for k in range(-120, 120, 7):
        p = 2.0 ** k
        for amax, fl in ((p, k), (np.nextafter(p, 0.0), k - 1), (np.nextafter(p, np.inf), k), (1.75 * p, k), (1.999999 * p, k)):
            e = int(O.mx_shared_exponent(np.array(amax)))
            assert e == fl - 2
            assert 4.0 <= amax / 2.0 ** e < 8.0
    assert int(O.mx_shared_exponent(np.array(0.0))) == 0
    assert int(O.mx_shared_exponent(np.array(2.0 ** -200))) == -126 and int(O.mx_shared_exponent(np.array(1e300))) == 127


def test_mx4_layout_and_round_trip():
    """Where a code and a scale sit in a row (one non-zero element at a time), what the padding
    holds, the error of a round trip, idempotence, and that every stored value is a bf16 number."""
    d = 90
    for i, val in ((0, 1.0), (1, -3.0), (31, 0.5), (32, 6.0), (63, -1.5), (64, 2.0), (89, 96.0)):
        x = np.zeros(d)
        x[i] = val
        codes, scales = O.mx4_quantize_rows(x)
        assert codes.shape == (48,) and scales.shape == (4,)
        blk, within = divmod(i, 32)
        byte = 16 * blk + within // 2
        e = int(np.floor(np.log2(abs(val)))) - 2
        nib = int(O.f64_to_e2m1_code(np.array(val / 2.0 ** e)))
        assert int(codes[byte]) == (nib << 4 if within % 2 else nib), (i, hex(int(codes[byte])))
        assert np.count_nonzero(codes) == 1
        want_scales = [127, 127, 127, 127]
        want_scales[blk] = 127 + e
        assert list(scales) == want_scales
        assert np.array_equal(O.mx4_dequantize_rows(codes, scales, d), x)     # a single element is always exact here
    rng = _rng(22)
    for d in (90, 115, 116, 64, 128, 6, 33):
        x = rng.standard_normal((50, d)) * 10.0 ** rng.integers(-3, 4, (50, 1))
        codes, scales = O.mx4_quantize_rows(x)
        nb = O.mx_blocks(d)
        assert codes.shape == (50, 16 * nb) and np.all(scales[:, nb:] == 127)
        back = O.mx4_dequantize_rows(codes, scales, d)
        full = O.mx4_dequantize_rows(codes, scales, 32 * nb)
        assert np.all(full[:, d:] == 0)                                       # padding elements are code 0
        for r in range(50):
            for b in range(nb):
                sl = slice(32 * b, min(32 * b + 32, d))
                s = 2.0 ** (int(scales[r, b]) - 127)
                y = np.abs(x[r, sl]) / s
                assert 4.0 <= y.max() < 8.0
                # half the spacing of the grid at y (0.5 below 2, 1 below 4, 2 above), 2 where 6 < y < 8 saturates
                half = np.where(y < 2, 0.25, np.where(y < 4, 0.5, 1.0))
                half = np.where(y > 6, 2.0, half)
                assert np.all(np.abs(back[r, sl] - x[r, sl]) <= half * s)
                assert np.abs(back[r, sl]).max() >= 4.0 * s                     # the largest element lands in the top binade
        c2, s2 = O.mx4_quantize_rows(back)
        assert np.array_equal(c2, codes) and np.array_equal(s2, scales)       # stored values are fixed points
        assert np.array_equal(O.bf16_bits_to_f64(O.f64_to_bf16_bits_rne(back)), back)
    assert np.isnan(O.mx4_dequantize_rows(np.full(16, 0x22, dtype=np.uint8), np.array([255, 127, 127, 127], dtype=np.uint8), 32)).all()


def test_mx4_cache_pins():
    """The 4-bit cache is the dense path on dequantised values: the appended rows are the quantised
    rotated rows (position 0: the quantised input row itself), V rows the quantised inputs, other
    rows untouched, and attention over the codes equals attn_ref over a bf16 cache that holds
    exactly the dequantised values."""
    rng = _rng(23)
    B, n_new, H, P, dv, cap, D, theta = 2, 3, 2, 20, 35, 16, 64, 1.0e4
    keep = np.stack([np.sort(rng.choice(D // 2, P, replace=False)) for _ in range(H)])
    k_new = _bf16_of(rng.standard_normal((B, n_new, H, 2 * P)) * 3)
    v_new = _bf16_of(rng.standard_normal((B, n_new, H, dv)))
    pos = np.array([[0, 1, 2], [7, 3, 11]])
    nbk, nbv = O.mx_blocks(2 * P), O.mx_blocks(dv)
    kc = np.zeros((B, H, cap, 16 * nbk), dtype=np.uint8); ks = np.zeros((B, H, cap, 4), dtype=np.uint8)
    vc = np.zeros((B, H, cap, 16 * nbv), dtype=np.uint8); vs = np.zeros((B, H, cap, 4), dtype=np.uint8)
    O.append_mx4_ref(k_new, v_new, pos, keep, kc, ks, vc, vs, theta, D)
    for b in range(B):
        for n in range(n_new):
            t = pos[b, n]
            for h in range(H):
                exact = O.rope_compact(O.bf16_bits_to_f64(k_new[b, n, h]), np.float64(t), keep[h], theta, D)
                c, s = O.mx4_quantize_rows(exact)
                assert np.array_equal(kc[b, h, t], c) and np.array_equal(ks[b, h, t], s)
                c, s = O.mx4_quantize_rows(O.bf16_bits_to_f64(v_new[b, n, h]))
                assert np.array_equal(vc[b, h, t], c) and np.array_equal(vs[b, h, t], s)
    c0, s0 = O.mx4_quantize_rows(O.bf16_bits_to_f64(k_new[0, 0, 1]))
    assert np.array_equal(kc[0, 1, 0], c0) and np.array_equal(ks[0, 1, 0], s0)      # position 0 does not rotate
    assert np.all(kc[0, :, 3:] == 0) and np.all(vs[1, :, 0] == 0)                   # untouched rows
    q = _bf16_of(rng.standard_normal((B, 2 * H, 2 * P)))
    lens = np.array([3, 12])
    # rows never appended hold scale byte 0 = 2^-127 and code 0: value 0
    got = O.attn_mx4_ref(q, kc, ks, vc, vs, lens, 0.4, 2 * P, dv)
    kb = _bf16_of(O.mx4_dequantize_rows(kc, ks, 2 * P))
    vb = _bf16_of(O.mx4_dequantize_rows(vc, vs, dv))
    assert np.array_equal(got, O.attn_ref(q, kb, vb, lens, 0.4))


def test_split_merge_identity():
    """Merging (m, l, acc) partials over any partition of the rows gives the unsplit result."""
    rng = _rng(17)
    G, dk, dv, S = 4, 12, 9, 101
    q, k, v = rng.standard_normal((G, dk)), rng.standard_normal((S, dk)) * 4, rng.standard_normal((S, dv))
    whole = O.attn_rows_ref(q, k, v, 0.4)
    for cuts in [[0, S], [0, 1, S], [0, 32, 64, 96, S], [0, 7, 8, 50, 99, 100, S]]:
        parts = [O.partial_ref(q, k[a:b], v[a:b], 0.4) for a, b in zip(cuts[:-1], cuts[1:])]
        merged = O.merge_partials_ref(*zip(*parts))
        assert np.max(np.abs(merged - whole)) < 1e-13


# ---------------------------------------------------------------- byte accounting


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_kept_pairs_reproduces_counted_fractions():
    """Tab. (effsweep): with D = 128 the counted RAP fraction equals kept_pairs/64 to the three
    printed digits at every retain ratio, which fixes m = round(rho D / 2)."""
    for rho_s, frac_s in _read_table("effsweep.txt"):
        m = O.kept_pairs(float(rho_s), 128)
        assert abs(m / 64.0 - float(frac_s)) < 5.1e-4, (rho_s, m)
    assert [O.kept_pairs(r, 128) for r in (0.9, 0.7, 0.5, 1.0)] == [58, 45, 32, 64]


def test_kv_bytes_per_token_against_serving_table():
    """Tab. (serving): dense Llama-3-8B keeps 128 KiB per token; RAP 0.7 keeps 89.5 KiB, which the
    uniform 45-pair / 90-channel layout (90.0 KiB) matches to 1 % (the deployed budgets are
    layer-adaptive)."""
    t = dict((k, float(v)) for k, v in _read_table("serving.txt"))
    assert O.kv_bytes_per_token(32, 8, 128, 128) == t["dense"] * 1024
    rap = O.kv_bytes_per_token(32, 8, 90, 90) / 1024.0
    assert abs(rap - t["rap0.7"]) / t["rap0.7"] < 0.01
    # cache scales as rho: Cache = rho * 2SD
    assert O.decode_kv_bytes([8192] * 16, 8, 90, 90) == 16 * 8 * 8192 * 180 * 2
    assert abs(O.decode_kv_bytes([100], 8, 90, 90) / O.decode_kv_bytes([100], 8, 128, 128) - 45 / 64) < 1e-15
