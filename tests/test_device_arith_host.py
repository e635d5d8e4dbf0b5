"""CPU tests of the arithmetic and indexing helpers the kernels compile (csrc/rap_arith.h).

The helpers are `__host__ __device__`; tests/host/rap_arith_host.hip is built from the same header
with the host pass of hipcc under AddressSanitizer and UBSan and driven here through stdin/stdout.
What it computes is compared with the float64 oracle (rounding to bf16 and to E4M3), with exact
integer arithmetic (rounding to odd) and with the long-double library routines (sine / cosine).
No GPU is involved.
"""
import os
import subprocess
from fractions import Fraction

import numpy as np
import pytest

from oracle import rap_oracle as O
from paper_2602_02599_amd import build as B


@pytest.fixture(scope="module")
def harness():
    try:
        B.hipcc()
    except RuntimeError:
        pytest.skip("hipcc not available")
    if not os.path.exists("/opt/rocm/bin/hipcc"):
        pytest.skip("hipcc not available")
    return B.build_host_tests()


def _run(harness, cmd, data=None, dtype=None):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    r = subprocess.run([harness, cmd], input=None if data is None else np.ascontiguousarray(data, dtype=np.float64).tobytes(),
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, env=env, timeout=120)
    if dtype is None:
        return r.returncode, r.stdout.decode()
    assert r.returncode == 0, r.stderr.decode()[-2000:]
    return np.frombuffer(r.stdout, dtype=dtype)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _bf16_positive_values():
    bits = np.arange(0x7F80, dtype=np.uint32).astype(np.uint16)       # +0 .. largest finite
    return O.bf16_bits_to_f64(bits)


def test_f64_to_bf16_rne_equals_oracle_rounding(harness):
    """One rounding, nearest even: every bf16 value itself, every midpoint between neighbours (a tie),
    the float64 numbers right next to every midpoint (the cases where a detour through fp32 rounds
    twice), subnormals, the overflow threshold, signed zeros, infinities, random magnitudes."""
    v = _bf16_positive_values()
    mid = (v[:-1] + v[1:]) / 2                                        # exact in float64
    top = float(v[-1])
    over = np.array([top, top * (1 + 2.0 ** -9), np.nextafter(top * (1 + 2.0 ** -9), 0.0),
                     np.nextafter(top * (1 + 2.0 ** -9), np.inf), 2.0 ** 128, 1e39, np.inf])
    rng = _rng(41)
    rnd = rng.standard_normal(200000) * 10.0 ** rng.integers(-45, 39, 200000)
    # float64 values that sit within half an fp32 ulp of a tie: fp32 conversion lands ON the tie
    near = np.concatenate([np.nextafter(mid, 0.0), np.nextafter(mid, np.inf),
                           mid * (1 + 2.0 ** -30), mid * (1 - 2.0 ** -30)])
    x = np.concatenate([v, mid, near, over, rnd, [0.0, 2.0 ** -134, 2.0 ** -133, 1.5 * 2.0 ** -133, 2.0 ** -126]])
    x = np.concatenate([x, -x])
    got = _run(harness, "bf16", x, np.uint16)
    want = O.f64_to_bf16_bits_rne(x)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, [(float(x[i]).hex(), hex(got[i]), hex(want[i])) for i in bad[:5]]
    nan = _run(harness, "bf16", np.array([np.nan, -np.nan]), np.uint16)
    assert np.all((nan & 0x7FFF) > 0x7F80)


def test_sincos_f64_against_long_double_library(harness):
    """|error| <= 2e-16 against sinl / cosl for the angles the rotation meets (position x frequency,
    positions up to 2^31) and for the hard ones: doubles next to multiples of pi/2, where the
    argument reduction cancels."""
    assert np.finfo(np.longdouble).eps < 2e-19, "this platform's long double is not wider than double"
    rng = _rng(42)
    k = np.concatenate([np.arange(0, 4096), rng.integers(0, 2 ** 30, 20000), 2 ** np.arange(1, 31)]).astype(np.float64)
    near_half_pi = k * (np.pi / 2)
    near_half_pi = np.concatenate([near_half_pi, np.nextafter(near_half_pi, 0.0), np.nextafter(near_half_pi, np.inf)])
    pos = rng.integers(0, 2 ** 31, 50000).astype(np.float64)
    freq = np.concatenate([O.inv_freq(5.0e5, 128), O.inv_freq(1.0e6, 128), O.inv_freq(1.0e4, 128)])
    rope = (pos[:, None] * freq[None, :64 * 3:7]).ravel()
    x = np.concatenate([near_half_pi, rope, rng.uniform(-2.0 ** 31, 2.0 ** 31, 100000), rng.uniform(-1, 1, 20000) * 1e-3,
                        [0.0, -0.0, 131071.0, 2.0 ** 31]])
    out = _run(harness, "sincos", x, np.float64).reshape(-1, 2)
    xl = x.astype(np.longdouble)
    es = np.abs(out[:, 0].astype(np.longdouble) - np.sin(xl)).max()
    ec = np.abs(out[:, 1].astype(np.longdouble) - np.cos(xl)).max()
    assert es <= 2e-16 and ec <= 2e-16, (float(es), float(ec))
    assert out[0, 0] == 0.0 and out[0, 1] == 1.0


def _odd_to_f32_bits_exact(y: float) -> int:
    """Definition with integers: clamp to [-448, 448]; write |y| = n * ulp + rest with ulp the fp32
    spacing at |y| (2^(e-23) for 2^e <= |y| < 2^(e+1), never below 2^-149); if rest > 0, force n odd."""
    y = max(-448.0, min(448.0, y))
    sign = 1 if (y < 0 or (y == 0 and np.signbit(y))) else 0
    a = Fraction(abs(y))
    if a == 0:
        return sign << 31
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    ulp = Fraction(2) ** (e - 23)
    n = a // ulp
    if n * ulp != a:
        n |= 1
    # n < 2^24; n >= 2^23 is a normal number with exponent field e + 127
    if n >= 2 ** 23:
        bits = ((e + 127) << 23) | (n - 2 ** 23)
    else:
        bits = n
    return (sign << 31) | bits


def test_round_to_odd_then_nearest_even_is_one_rounding(harness):
    """The software half of fp64 -> E4M3: (a) equals the integer definition of rounding to odd after
    the clamp; (b) rounding ITS result to E4M3 (nearest even, here by the oracle's search over the
    codes) gives the code the oracle finds for the fp64 value directly, also right next to every
    tie between neighbouring codes, which is where a plain fp64 -> fp32 -> E4M3 goes wrong."""
    grid = O.e4m3_bits_to_f64(np.arange(0x7F, dtype=np.uint8))        # 0 .. 448 ascending
    mid = (grid[:-1] + grid[1:]) / 2
    rng = _rng(43)
    tiny = 2.0 ** -30
    x = np.concatenate([grid, mid, np.nextafter(mid, 0.0), np.nextafter(mid, np.inf), mid * (1 + tiny), mid * (1 - tiny),
                        rng.standard_normal(50000) * 10.0 ** rng.integers(-12, 4, 50000),
                        [448.0, 449.0, 464.0, 480.0, 1e6, 1e300, 2.0 ** -149, 2.0 ** -150, 1e-60, 0.0]])
    x = np.concatenate([x, -x])
    got = _run(harness, "odd448", x, np.uint32)
    sample = np.concatenate([np.arange(0, 1200), rng.integers(0, x.size, 3000)])
    for i in sample:
        assert int(got[i]) == _odd_to_f32_bits_exact(float(x[i])), (float(x[i]).hex(), hex(int(got[i])))
    as_f32 = got.view(np.float32).astype(np.float64)
    assert np.array_equal(O.f64_to_e4m3_bits(as_f32), O.f64_to_e4m3_bits(x))
    # the plain detour through nearest-even fp32 does get some of these wrong: the repair matters
    with np.errstate(over="ignore"):
        plain = x.astype(np.float32).astype(np.float64)
    assert np.any(O.f64_to_e4m3_bits(plain) != O.f64_to_e4m3_bits(x))


def test_mx4_block_quantiser_equals_oracle(harness):
    """The 4-bit append's arithmetic (scale exponent of a block from its largest magnitude, division
    by that power of two, rounding to E2M1): codes and scale bytes equal the oracle's for random
    blocks over many magnitudes, blocks whose maximum sits at and next to a power of two, elements at
    and next to every tie between neighbouring codes, zeros, signed zeros and the clamped extremes."""
    rng = _rng(44)
    blocks = [rng.standard_normal((4000, 32)) * 10.0 ** rng.integers(-30, 30, (4000, 1))]
    grid = O.e2m1_code_to_f64(np.arange(8))
    mids = (grid[:-1] + grid[1:]) / 2
    ties = np.concatenate([mids, np.nextafter(mids, 0.0), np.nextafter(mids, 10.0), grid, [5.0, 5.5, 6.5, 7.99]])
    for k in (-140, -126, -40, -1, 0, 3, 77, 127):
        for top in (4.0, np.nextafter(4.0, 0.0), np.nextafter(8.0, 0.0), 6.0, 5.0):
            b = np.zeros(32)
            b[:ties.size] = ties[:32]
            b[31] = top                                   # fixes the block's scale at 2^k (or the binade below)
            b[1::2] *= -1
            blocks.append((b * 2.0 ** k)[None, :])
    blocks.append(np.zeros((1, 32)))
    blocks.append(np.where(np.arange(32) % 2 == 0, 0.0, -0.0)[None, :])
    blocks.append(np.full((1, 32), 3.0e38))
    blocks.append(np.full((1, 32), 2.0 ** -133))
    x = np.concatenate(blocks)
    raw = _run(harness, "mx4", x.ravel(), np.uint8).reshape(-1, 33)
    codes, scales = O.mx4_quantize_rows(x)
    assert np.array_equal(raw[:, 0], scales[:, 0])
    packed = (raw[:, 1::2] | (raw[:, 2::2] << 4)).astype(np.uint8)
    bad = np.nonzero((packed != codes).any(axis=1))[0]
    assert bad.size == 0, (bad[:5], x[bad[0]], raw[bad[0]], codes[bad[0]])


def test_decode_tile_loads_stay_inside_the_tile(harness):
    """Every 16-byte load the decode kernel issues for a K or V tile, for every width the library
    accepts, both element sizes, full and partial tiles: inside the tile's bytes, every byte once."""
    rc, text = _run(harness, "loadplan")
    lines = [ln for ln in text.splitlines() if ln]
    assert rc == 0 and len(lines) == (64 + 128) * (4 + 2), text[-500:]
    seen = set()
    for ln in lines:
        f = dict(kv.split("=") for kv in ln.split()[1:])
        assert int(f["top"]) <= int(f["bytes"]) and f["missed"] == "0" and f["twice"] == "0", ln
        seen.add((ln.split()[0], f["q8"], int(f["d"]), int(f["rows"])))
    for d_k in (34, 38 * 2, 51 * 2, 90, 116, 64, 128):
        assert ("K", "0", d_k, 32) in seen
    # the rule this replaced (only the last load of a run trimmed) reads past bf16 K tiles whose
    # width needs an odd number of loads; the same check must say so
    rc_old, text_old = _run(harness, "loadplan-trim1")
    assert rc_old == 1
    over = {int(dict(kv.split("=") for kv in ln.split()[1:])["d"]) for ln in text_old.splitlines()
            if ln.startswith("K q8=0") and "rows=32" in ln
            and int(dict(kv.split("=") for kv in ln.split()[1:])["top"]) > int(dict(kv.split("=") for kv in ln.split()[1:])["bytes"])}
    assert {34, 76, 102} <= over and not ({64, 90, 116, 128} & over)
