"""GPU parity: librap (through its C ABI) against the float64 oracle on the same seeded inputs.

Bars: appended K rows within 1 bf16 ulp of the oracle's single-rounded row (V rows bit-exact);
attention outputs max-abs <= 1e-2 and mean-relative (mean |diff| / mean |ref|) <= 1e-3.
"""
import math

import numpy as np
import pytest
import torch

from oracle import rap_oracle as O
import rap_inputs as I
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
VALU, MFMA = 1, 2


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ append


def _check_append(rap, case, what):
    kc, vc = I.bits(case.k_cache), I.bits(case.v_cache)       # before: filler
    H.run_append(rap, case)
    torch.cuda.synchronize()
    H.oracle_append(case, kc, vc)
    gk, gv = I.bits(case.k_cache), I.bits(case.v_cache)
    assert np.array_equal(gv, vc), what + ": V cache differs"
    dist = H.bf16_ulp_distance(gk, kc)
    assert dist.max() <= 1, "%s: K row off by %d ulp" % (what, dist.max())
    return int((dist != 0).sum()), dist.size


@pytest.mark.parametrize("P,dv,H_kv,n_new,B", [(45, 90, 8, 5, 3), (58, 115, 2, 1, 2), (32, 64, 8, 4, 1),
                                              (64, 128, 4, 7, 2), (1, 1, 1, 1, 1), (3, 5, 2, 9, 2)])
def test_append_small(rap, P, dv, H_kv, n_new, B):
    w = I.scaled(I.WORKLOADS["cfg2"], batch=B, n_q_heads=H_kv * 2, n_kv_heads=H_kv, n_pairs=P, d_v=dv,
                 ctx=100 + n_new, n_new=n_new, peaky_frac=0.0, seed=40 + P)
    _say("append small P=%d dv=%d" % (P, dv))
    case = I.make_case(w, device=DEV)
    off, n = _check_append(rap, case, "small")
    assert off <= n // 1000 + 1          # single rounding from fp64: essentially bit-exact


def test_append_cfg1_whole_cache(rap):
    """cfg1: all 2048 positions of the cache are written through the append call."""
    _say("append cfg1")
    case = I.make_case(I.WORKLOADS["cfg1"], device=DEV)
    off, n = _check_append(rap, case, "cfg1")
    _say("cfg1 append: %d of %d elements differ (by 1 ulp)" % (off, n))
    assert off <= n // 1000 + 1


@pytest.mark.parametrize("theta", [5.0e5, 1.0e6, 1.0e4])
def test_append_far_positions(rap, theta):
    """Positions up to 131071: the angle needs fp64 to stay inside one bf16 ulp."""
    w = I.scaled(I.WORKLOADS["cfg4"], batch=2, ctx=131072, n_new=6, rope_theta=theta, seed=77)
    _say("append far theta=%g" % theta)
    case = I.make_case(w, device=DEV)
    pos = torch.tensor([[131071, 131066, 99999, 65536, 1, 0], [131070, 77777, 4097, 4096, 12345, 2]], dtype=torch.int32, device=DEV)
    case.pos = pos
    off, n = _check_append(rap, case, "far")
    assert off <= n // 1000 + 1


@pytest.mark.parametrize("P,dv,H_kv,n_new,B,theta", [(45, 90, 8, 100, 2, 5.0e5), (58, 115, 2, 37, 3, 1.0e6), (32, 64, 4, 16, 1, 1.0e6),
                                                    (64, 128, 2, 300, 2, 5.0e5), (3, 5, 2, 65, 2, 1.0e4)])
def test_append_bulk(rap, P, dv, H_kv, n_new, B, theta):
    """Prefill-sized appends take the run-based kernel (angle advanced by one rotation per
    consecutive position): consecutive runs, runs with jumps and repeats of far positions,
    out-of-range positions in the middle of a run."""
    w = I.scaled(I.WORKLOADS["cfg4"], batch=B, n_q_heads=H_kv, n_kv_heads=H_kv, n_pairs=P, d_v=dv, ctx=131072, n_new=n_new,
                 rope_theta=theta, seed=60 + P)
    _say("append bulk P=%d dv=%d n_new=%d" % (P, dv, n_new))
    case = I.make_case(I.scaled(w, ctx=4096 + n_new), device=DEV)
    rng = np.random.Generator(np.random.PCG64(5))
    for mode in ("consecutive", "jumps"):
        if mode == "consecutive":
            start = rng.integers(0, case.cap - n_new, size=B)
            pos = start[:, None] + np.arange(n_new)[None, :]
        else:
            pos = np.empty((B, n_new), dtype=np.int64)
            for b in range(B):
                perm = rng.permutation(case.cap)[:n_new]          # distinct rows, arbitrary order
                seg = np.sort(perm[: n_new // 2])                  # first half ascending with gaps
                pos[b] = np.concatenate([seg, perm[n_new // 2:]])
            pos[0, 3] = -5                                         # skipped
            pos[B - 1, n_new - 2] = case.cap + 7                   # skipped
        case.pos = torch.from_numpy(pos.astype(np.int32)).to(DEV)
        kc, vc = I.bits(case.k_cache), I.bits(case.v_cache)
        H.run_append(rap, case)
        torch.cuda.synchronize()
        ok = (pos >= 0) & (pos < case.cap)
        okc, ovc = kc.copy(), vc.copy()
        keep = case.keep.cpu().numpy()
        k_new, v_new = I.bits(case.k_new), I.bits(case.v_new)
        for b in range(B):
            for n in range(n_new):
                if ok[b, n]:
                    t = int(pos[b, n])
                    for h in range(H_kv):
                        rot = O.rope_compact(O.bf16_bits_to_f64(k_new[b, n, h]), np.float64(t), keep[h], theta, w.d_head)
                        okc[b, h, t] = O.f64_to_bf16_bits_rne(rot)
                        ovc[b, h, t] = v_new[b, n, h]
        gk, gv = I.bits(case.k_cache), I.bits(case.v_cache)
        assert np.array_equal(gv, ovc), mode + ": V cache differs"
        dist = H.bf16_ulp_distance(gk, okc)
        assert dist.max() <= 1, "%s: K off by %d ulp" % (mode, dist.max())
        assert (dist != 0).sum() <= dist.size // 1000 + 1


@pytest.mark.parametrize("P,dv", [(45, 90), (58, 115)])
def test_append_bulk_long(rap, P, dv):
    """A prefill-sized append (each wavefront walks several runs and carries the angle from one
    run into the next): V against the input bits everywhere, K against the oracle on sampled rows
    that include run and wavefront boundaries, a jump in the positions and a shuffled stretch."""
    B, H_kv, n_new = 4, 8, 16400
    w = I.scaled(I.WORKLOADS["cfg4"], batch=B, n_q_heads=H_kv, n_kv_heads=H_kv, n_pairs=P, d_v=dv, ctx=n_new + 40, n_new=n_new,
                 rope_theta=5.0e5, seed=77)
    _say("append bulk long P=%d dv=%d" % (P, dv))
    case = I.make_case(w, device=DEV, fill_unused=False)
    assert case.cap >= n_new + 40
    pos = np.tile(np.arange(n_new, dtype=np.int64), (B, 1)) + np.array([0, 3, 17, 1])[:, None]
    pos[3, 8000:] += 5                                             # a jump inside a wavefront's walk
    rng = np.random.Generator(np.random.PCG64(9))
    pos[2, 4100:4200] = pos[2, 4100:4200][rng.permutation(100)]    # runs that are not in order
    pos[1, 12345] = -1                                             # skipped
    case.pos = torch.from_numpy(pos.astype(np.int32)).to(DEV)
    before_k = I.bits(case.k_cache)[1, :, 12345 + 3].copy()
    H.run_append(rap, case)
    torch.cuda.synchronize()
    gk, gv = I.bits(case.k_cache), I.bits(case.v_cache)
    k_new, v_new = I.bits(case.k_new), I.bits(case.v_new)
    keep = case.keep.cpu().numpy()
    for b in range(B):
        ok = pos[b] >= 0
        assert np.array_equal(gv[b][:, pos[b][ok]], np.transpose(v_new[b][ok], (1, 0, 2))), "V rows differ, b=%d" % b
    assert np.array_equal(gk[1, :, 12345 + 3], before_k), "skipped row was written"
    ns = np.unique(np.concatenate([rng.integers(0, n_new, 400), [0, 15, 16, 63, 64, 65, 255, 256, 257, 4099, 4100, 4150, 4199, 4200,
                                                                   7999, 8000, 8001, 12344, 12346, n_new - 17, n_new - 16, n_new - 1]]))
    worst, n_off, n_all = 0, 0, 0
    for b in range(B):
        for n in ns:
            t = int(pos[b, n])
            if t < 0:
                continue
            for h in range(H_kv):
                ref = O.f64_to_bf16_bits_rne(O.rope_compact(O.bf16_bits_to_f64(k_new[b, n, h]), np.float64(t), keep[h], w.rope_theta, w.d_head))
                dist = H.bf16_ulp_distance(gk[b, h, t], ref)
                worst = max(worst, int(dist.max())); n_off += int((dist != 0).sum()); n_all += dist.size
    assert worst <= 1, "K off by %d ulp" % worst
    assert n_off <= n_all // 1000 + 1, "%d of %d elements differ" % (n_off, n_all)


def test_append_skips_out_of_range(rap):
    w = I.scaled(I.WORKLOADS["cfg2"], batch=1, ctx=64, n_new=3, peaky_frac=0.0, seed=5)
    case = I.make_case(w, device=DEV)
    before_k, before_v = I.bits(case.k_cache).copy(), I.bits(case.v_cache).copy()
    case.pos = torch.tensor([[-1, case.cap, 10]], dtype=torch.int32, device=DEV)
    H.run_append(rap, case)
    torch.cuda.synchronize()
    gk, gv = I.bits(case.k_cache), I.bits(case.v_cache)
    changed = np.where((gk != before_k).any(axis=(0, 1, 3)))[0]
    assert list(changed) == [10]
    assert np.array_equal(np.delete(gv, 10, axis=2), np.delete(before_v, 10, axis=2))


# ------------------------------------------------------------------ decode, small shapes


def _oracle_out(case):
    return O.attn_ref(I.bits(case.q), I.bits(case.k_cache), I.bits(case.v_cache), case.seq_lens.cpu().numpy(), case.w.scale)


SMALL = [
    # P, dv, Hq, Hkv, ctx  (several 32-row tiles and a ragged tail)
    (45, 90, 8, 2, 333), (58, 115, 8, 2, 289), (32, 64, 10, 2, 1000), (64, 128, 8, 2, 515),
    (45, 90, 6, 2, 31), (45, 90, 2, 2, 1), (3, 5, 3, 1, 77), (10, 7, 16, 2, 130), (51, 102, 4, 1, 257),
    (38, 77, 12, 2, 640), (64, 128, 1, 1, 96), (17, 33, 7, 1, 200),
]


@pytest.mark.parametrize("kernel", [VALU, MFMA])
@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx", SMALL)
def test_decode_small(rap, kernel, P, dv, Hq, Hkv, ctx):
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=1,
                 ragged_min=(max(1, ctx // 3) if ctx >= 4 else None), peaky_frac=0.0, seed=900 + P + ctx)
    _say("decode small kernel=%d P=%d dv=%d Hq=%d Hkv=%d ctx=%d" % (kernel, P, dv, Hq, Hkv, ctx))
    case = I.make_case(w, device=DEV)
    ref = _oracle_out(case)
    for rps in (0, 128, 256):
        got = H.run_decode(rap, case, kernel=kernel, rows_per_split=rps).cpu().numpy()
        H.assert_attn_close(got, ref, "rps=%d" % rps)


@pytest.mark.parametrize("kernel", [VALU, MFMA])
def test_decode_peaky_and_scales(rap, kernel):
    """1 % of K rows x8 (softmax dominated by a few rows), both softmax scales."""
    for scale in (1 / np.sqrt(128.0), 1 / np.sqrt(90.0), 0.5):
        w = I.scaled(I.WORKLOADS["cfg2"], batch=2, ctx=1500, scale=scale, seed=321)
        _say("decode peaky kernel=%d scale=%.4f" % (kernel, scale))
        case = I.make_case(w, device=DEV)
        ref = _oracle_out(case)
        for rps in (0, 128, 384):
            got = H.run_decode(rap, case, kernel=kernel, rows_per_split=rps).cpu().numpy()
            H.assert_attn_close(got, ref, "scale=%g rps=%d" % (scale, rps))


@pytest.mark.parametrize("kernel", [VALU, MFMA])
def test_decode_ignores_rows_beyond_len(rap, kernel):
    """Rows at and beyond seq_lens hold NaN / Inf / huge patterns: the result must not change."""
    w = I.scaled(I.WORKLOADS["cfg3"], batch=4, ctx=300, ragged_min=5, seed=11)
    _say("decode garbage kernel=%d" % kernel)
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    ref = _oracle_out(case)
    poison = torch.tensor([0x7FC0, 0x7F80, 0xFF80, 0x7F7F, 0xFFFF], dtype=torch.int32).to(torch.int16).view(torch.bfloat16).to(DEV)
    for b in range(w.batch):
        n = case.cap - int(lens[b])
        if n > 0:
            idx = torch.arange(n * w.d_k, device=DEV) % 5
            case.k_cache[b, :, int(lens[b]):] = poison[idx].view(n, w.d_k)
            idx = torch.arange(n * w.d_v, device=DEV) % 5
            case.v_cache[b, :, int(lens[b]):] = poison[idx].view(n, w.d_v)
    for rps in (0, 128):
        got = H.run_decode(rap, case, kernel=kernel, rows_per_split=rps).cpu().numpy()
        H.assert_attn_close(got, ref, "poisoned tail rps=%d" % rps)


@pytest.mark.parametrize("kernel", [VALU, MFMA])
def test_decode_zero_length_and_clamp(rap, kernel):
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, ctx=200, peaky_frac=0.0, seed=12)
    case = I.make_case(w, device=DEV)
    case.seq_lens = torch.tensor([0, 200, 1], dtype=torch.int32, device=DEV)
    ref = _oracle_out(case)
    for rps in (0, 128):
        got = H.run_decode(rap, case, kernel=kernel, rows_per_split=rps, max_seq_len=200).cpu().numpy()
        assert np.all(got[0] == 0)
        H.assert_attn_close(got, ref, "zero-length rps=%d" % rps)
    # seq_lens above max_seq_len is clamped on the device
    case.seq_lens = torch.tensor([150, 999, 7], dtype=torch.int32, device=DEV)
    got = H.run_decode(rap, case, kernel=kernel, max_seq_len=160).cpu().numpy()
    case.seq_lens = torch.tensor([150, 160, 7], dtype=torch.int32, device=DEV)
    H.assert_attn_close(got, _oracle_out(case), "clamped")


@pytest.mark.parametrize("kernel", [VALU, MFMA])
@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx,theta", [(45, 90, 8, 2, 700, 5.0e5), (58, 115, 8, 2, 300, 1.0e6),
                                                  (32, 64, 10, 2, 1100, 1.0e6), (64, 128, 8, 1, 260, 5.0e5),
                                                  (3, 5, 3, 1, 40, 1.0e4)])
def test_decode_with_query_rope(rap, kernel, P, dv, Hq, Hkv, ctx, theta):
    """rap_decode_attn_rope: un-rotated q + position + kept pairs; the oracle rotates q (float64,
    one rounding to bf16) and attends.  Also bit-identical to feeding rap_decode_attn the
    oracle-rotated q, and far positions."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=1,
                 rope_theta=theta, ragged_min=max(1, ctx // 3), peaky_frac=0.0, seed=500 + P + ctx)
    _say("decode+qrope kernel=%d P=%d dv=%d" % (kernel, P, dv))
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    for q_pos_np in (lens - 1, np.array([131071, 0, 65537])):
        q_pos = torch.from_numpy(q_pos_np.astype(np.int32)).to(DEV)
        q_rot = O.rope_queries_ref(I.bits(case.q), q_pos_np, case.keep.cpu().numpy(), w.rope_theta, w.d_head, w.n_kv_heads)
        ref = O.attn_ref(q_rot, I.bits(case.k_cache), I.bits(case.v_cache), lens, w.scale)
        shp = H.shape_of(rap, case)
        msl = int(lens.max())
        for rps in (0, 128):
            tun = rap.tuning(kernel=kernel, rows_per_split=rps)
            ws = rap.new_workspace(shp, msl, tun)
            out = torch.full((w.batch, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
            rap.rap_decode_attn_rope(shp, case.q, q_pos, case.keep, case.k_cache, case.v_cache, case.seq_lens, msl, out,
                                     float(w.scale), ws, tun)
            out2 = torch.full_like(out, float("nan"))
            rap.rap_decode_attn(shp, I.from_bits(q_rot, DEV), case.k_cache, case.v_cache, case.seq_lens, msl, out2,
                                float(w.scale), ws, tun)
            torch.cuda.synchronize()
            H.assert_attn_close(out.cpu().numpy(), ref, "fused q rope rps=%d" % rps)
            assert torch.equal(out, out2), "fused rotation differs from rotating first"


@pytest.mark.parametrize("kernel", [VALU, MFMA])
@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx", [(45, 90, 8, 2, 900), (58, 115, 8, 2, 300), (32, 64, 10, 2, 1500),
                                             (64, 128, 4, 1, 260), (3, 5, 3, 1, 33)])
def test_decode_step_fused(rap, kernel, P, dv, Hq, Hkv, ctx):
    """rap_decode_step == rap_rope_append(1 token) then rap_decode_attn[_rope]: the oracle's
    composition for the bar, and the two-call sequence of librap itself (both caches bit for bit;
    outputs bit for bit on the vector-ALU kernel, to fp32 rounding on the matrix-core kernel, where
    the combining kernel handles the new token).  Ragged lengths; the new token sits at row len-1, for one sequence in the middle
    of the attended rows (overwriting an old row), for one beyond them (written, not attended)."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=4, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=1,
                 ragged_min=max(2, ctx // 3), peaky_frac=0.0, seed=700 + P + ctx)
    _say("decode step kernel=%d P=%d dv=%d ctx=%d" % (kernel, P, dv, ctx))
    base_case = I.make_case(w, device=DEV)
    lens = base_case.seq_lens.cpu().numpy().copy()
    pos_np = (lens - 1).astype(np.int32)
    pos_np[1] = lens[1] // 2                       # overwrites a row in the middle
    if lens[2] < base_case.cap:
        pos_np[2] = lens[2]                        # lands just beyond the attended rows
    pos = torch.from_numpy(pos_np).to(DEV)
    k_new = base_case.k_new[:, 0].contiguous()
    v_new = base_case.v_new[:, 0].contiguous()
    msl = int(base_case.cap)
    shp = H.shape_of(rap, base_case)
    keep_np = base_case.keep.cpu().numpy()
    for q_is_rotated in (True, False):
        for rps in (0, 128, 256):
            tun = rap.tuning(kernel=kernel, rows_per_split=rps)
            ws = rap.new_workspace(shp, msl, tun)
            # fused
            kc1, vc1 = base_case.k_cache.clone(), base_case.v_cache.clone()
            out1 = torch.full((w.batch, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
            rap.rap_decode_step(shp, k_new, v_new, pos, base_case.keep, base_case.q, q_is_rotated, kc1, vc1,
                                base_case.seq_lens, msl, out1, float(w.scale), ws, tun)
            # two calls
            kc2, vc2 = base_case.k_cache.clone(), base_case.v_cache.clone()
            out2 = torch.full_like(out1, float("nan"))
            rap.rap_rope_append(shp, 1, k_new, v_new, pos, base_case.keep, kc2, vc2)
            if q_is_rotated:
                rap.rap_decode_attn(shp, base_case.q, kc2, vc2, base_case.seq_lens, msl, out2, float(w.scale), ws, tun)
            else:
                rap.rap_decode_attn_rope(shp, base_case.q, pos, base_case.keep, kc2, vc2, base_case.seq_lens, msl, out2,
                                         float(w.scale), ws, tun)
            torch.cuda.synchronize()
            assert torch.equal(kc1.view(torch.int16), kc2.view(torch.int16)) and torch.equal(vc1.view(torch.int16), vc2.view(torch.int16))
            if kernel == VALU:
                assert torch.equal(out1, out2), "step differs from append + decode (rps=%d)" % rps
            else:   # the new token's row is folded in by the combining kernel: other order of fp32 sums
                rel = (out1 - out2).abs().max().item() / out2.abs().max().item()
                assert rel <= 2e-5, "fused step differs from append + decode (rps=%d): %.3g" % (rps, rel)
            # oracle
            okc, ovc = I.bits(base_case.k_cache).copy(), I.bits(base_case.v_cache).copy()
            O.append_ref(I.bits(k_new)[:, None], I.bits(v_new)[:, None], pos_np[:, None], keep_np, okc, ovc, w.rope_theta, w.d_head)
            assert H.bf16_ulp_distance(I.bits(kc1), okc).max() <= 1 and np.array_equal(I.bits(vc1), ovc)
            qb = I.bits(base_case.q) if q_is_rotated else O.rope_queries_ref(I.bits(base_case.q), pos_np, keep_np, w.rope_theta, w.d_head, w.n_kv_heads)
            ref = O.attn_ref(qb, I.bits(kc1), I.bits(vc1), lens, w.scale)
            H.assert_attn_close(out1.cpu().numpy(), ref, "fused step rps=%d rotated=%s" % (rps, q_is_rotated))


@pytest.mark.parametrize("kernel", [VALU, MFMA])
def test_decode_step_edges(rap, kernel):
    """rap_decode_step where the new token is the whole sequence (length 1), is skipped
    (position -1: nothing written, all rows attended), or belongs to an empty sequence
    (length 0: zero output row, row still written)."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=4, n_q_heads=8, n_kv_heads=2, ctx=700, n_new=1, ragged_min=300, peaky_frac=0.0, seed=321)
    _say("decode step edges kernel=%d" % kernel)
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy().copy()
    lens[0] = 1
    lens[2] = 0
    pos_np = (lens - 1).astype(np.int32)
    pos_np[1] = -1
    pos_np[2] = 5
    seq_lens = torch.from_numpy(lens.astype(np.int32)).to(DEV)
    pos = torch.from_numpy(pos_np).to(DEV)
    k_new, v_new = case.k_new[:, 0].contiguous(), case.v_new[:, 0].contiguous()
    shp = H.shape_of(rap, case)
    keep_np = case.keep.cpu().numpy()
    for rps in (0, 128):
        tun = rap.tuning(kernel=kernel, rows_per_split=rps)
        ws = rap.new_workspace(shp, int(case.cap), tun)
        kc, vc = case.k_cache.clone(), case.v_cache.clone()
        out = torch.full((w.batch, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_step(shp, k_new, v_new, pos, case.keep, case.q, True, kc, vc, seq_lens, int(case.cap), out,
                            float(w.scale), ws, tun)
        torch.cuda.synchronize()
        okc, ovc = I.bits(case.k_cache).copy(), I.bits(case.v_cache).copy()
        for b in range(w.batch):
            if pos_np[b] >= 0:
                O.append_ref(I.bits(k_new)[b:b + 1, None], I.bits(v_new)[b:b + 1, None], pos_np[b:b + 1, None], keep_np,
                             okc[b:b + 1], ovc[b:b + 1], w.rope_theta, w.d_head)
        assert H.bf16_ulp_distance(I.bits(kc), okc).max() <= 1 and np.array_equal(I.bits(vc), ovc)
        ref = O.attn_ref(I.bits(case.q), I.bits(kc), I.bits(vc), lens, w.scale)
        got = out.cpu().numpy()
        assert np.all(got[2] == 0.0), "empty sequence must give a zero row"
        H.assert_attn_close(got, ref, "step edges rps=%d" % rps)
        # the length-1 sequence attends only its new token: output == its V row
        v_row = O.bf16_bits_to_f64(I.bits(v_new)[0])              # [H_kv, d_v]
        G = w.n_q_heads // w.n_kv_heads
        assert np.abs(got[0] - np.repeat(v_row, G, axis=0)).max() <= 1e-6


# ---------------------------------------------------------------- causal prefill attention


def _prefill_case(P, dv, Hq, Hkv, n_new, lens, seed, scale=None, nan_beyond=False):
    """Cache rows N(0,1) as bf16 (taken as already rotated), q likewise; lens are the lengths after
    the n_new tokens were appended."""
    lens = np.asarray(lens, dtype=np.int64)
    B = len(lens)
    cap = int((max(int(lens.max()), 1) + 7) // 8 * 8) + 8
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    kc = torch.randn((B, Hkv, cap, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((B, Hkv, cap, dv), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((B, n_new, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    if nan_beyond:
        for b in range(B):
            kc[b, :, int(lens[b]):] = float("nan")
            vc[b, :, int(lens[b]):] = float("nan")
    return q, kc, vc, torch.from_numpy(lens.astype(np.int32)).to(DEV), cap, (scale if scale is not None else 1.0 / math.sqrt(2 * P))


@pytest.mark.parametrize("P,dv,Hq,Hkv,n_new,lens", [
    (45, 90, 8, 2, 200, [200, 333, 150]),          # full, chunked, shorter than n_new
    (58, 115, 8, 2, 130, [130, 517]),              # odd d_v
    (32, 64, 10, 2, 97, [97, 400, 1]),             # group of 5
    (64, 128, 4, 1, 150, [150, 260]),              # rho = 1 widths
    (45, 90, 24, 8, 70, [70, 71]),                 # group of 3
    (3, 5, 3, 1, 33, [33, 40, 5]),
    (45, 90, 8, 8, 300, [300]),                    # no grouping: 256 tokens per workgroup
    (45, 90, 8, 1, 40, [40, 1000]),                # group of 8
    (64, 128, 10, 2, 97, [97, 300]),               # three column blocks: 192 columns over groups of 5 (38 tokens, 2 columns idle)
    (58, 116, 7, 1, 50, [50, 131, 27]),            # ... of 7 (27 tokens, 3 columns idle), blocks that end inside n_new
    (45, 128, 8, 2, 130, [130, 190]),              # narrow scores with wide values: three blocks, only V padded in LDS
])
def test_prefill_small(rap, P, dv, Hq, Hkv, n_new, lens):
    """rap_prefill_attn against the oracle, element by element: several key tiles, ragged tails,
    chunked prefill (len > n_new), sequences shorter than n_new (zero rows), garbage beyond len."""
    _say("prefill P=%d dv=%d heads %d/%d n_new=%d lens=%s" % (P, dv, Hq, Hkv, n_new, lens))
    q, kc, vc, sl, cap, scale = _prefill_case(P, dv, Hq, Hkv, n_new, lens, seed=900 + P + n_new, nan_beyond=True)
    shp = rap.shape(len(lens), Hq, Hkv, 128, P, dv, cap, 5.0e5)
    out = torch.full((len(lens), n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn(shp, n_new, q, kc, vc, sl, cap, out, scale)
    torch.cuda.synchronize()
    ref = O.prefill_attn_ref(I.bits(q), I.bits(kc), I.bits(vc), np.asarray(lens), scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "prefill")


@pytest.mark.parametrize("P,dv,Hq,Hkv,n_new,lens,page_rows", [
    (45, 90, 8, 2, 200, [200, 333, 150], 64), (58, 115, 8, 2, 130, [130, 517], 128),
    (32, 64, 10, 2, 97, [97, 400, 1], 64), (64, 128, 4, 1, 150, [150, 700], 256)])
def test_prefill_paged(rap, P, dv, Hq, Hkv, n_new, lens, page_rows):
    """rap_prefill_attn_paged over pools with a shuffled block table: bit for bit the dense call on
    the same rows, and the oracle's bar; unused pages and the rows beyond each sequence hold NaN,
    table entries beyond the sequences hold wild page numbers; pages of 32 rows are refused."""
    q, kc, vc, sl, cap0, scale = _prefill_case(P, dv, Hq, Hkv, n_new, lens, seed=1200 + P + page_rows, nan_beyond=True)
    _say("prefill paged P=%d dv=%d n_new=%d page_rows=%d" % (P, dv, n_new, page_rows))
    lens_np = np.asarray(lens)
    B = len(lens)
    max_pages = (int(lens_np.max()) + page_rows - 1) // page_rows
    cap = max_pages * page_rows
    n_pages = B * max_pages + 3
    rng = np.random.Generator(np.random.PCG64(31))
    table = rng.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
    nan = 0x7FC0
    kp = O.dense_to_paged_ref(I.bits(kc), table, page_rows, n_pages, lens_np, fill=nan)
    vp = O.dense_to_paged_ref(I.bits(vc), table, page_rows, n_pages, lens_np, fill=nan)
    table_dev = table.copy()
    for b in range(B):
        table_dev[b, (int(lens_np[b]) + page_rows - 1) // page_rows:] = 2 ** 30
    pg = rap.paging(page_rows, n_pages, torch.from_numpy(table_dev).to(DEV))
    shp_p = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    out_p = torch.full((B, n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn_paged(shp_p, pg, n_new, q, I.from_bits(kp, DEV), I.from_bits(vp, DEV), sl, cap, out_p, scale)
    shp_d = rap.shape(B, Hq, Hkv, 128, P, dv, cap0, 5e5)
    out_d = torch.full_like(out_p, float("nan"))
    rap.rap_prefill_attn(shp_d, n_new, q, kc, vc, sl, cap0, out_d, scale)
    torch.cuda.synchronize()
    assert torch.equal(out_p, out_d), "paged and dense prefill differ"
    ref = O.prefill_attn_ref(I.bits(q), I.bits(kc), I.bits(vc), lens_np, scale)
    H.assert_attn_close(out_p.cpu().numpy(), ref, "paged prefill")
    small = rap.paging(32, n_pages * (page_rows // 32), torch.zeros((B, cap // 32), dtype=torch.int32, device=DEV))
    assert rap.rap_prefill_attn_paged(shp_p, small, n_new, q, I.from_bits(kp, DEV), I.from_bits(vp, DEV), sl, cap, out_p, scale,
                                      check=False) == 3


@pytest.mark.parametrize("P,dv,Hq,Hkv,n_new,lens,page_rows", [
    (45, 90, 8, 2, 200, [200, 333, 150], 0), (58, 115, 8, 2, 130, [130, 517], 0), (32, 64, 10, 2, 97, [97, 400, 1], 0),
    (64, 128, 4, 1, 150, [150, 260], 0), (3, 5, 3, 1, 33, [33, 40, 5], 0), (45, 90, 8, 1, 40, [40, 1000], 0),
    (45, 90, 8, 2, 200, [200, 333, 150], 64), (58, 115, 8, 2, 130, [130, 517], 128)])
def test_prefill_q8(rap, P, dv, Hq, Hkv, n_new, lens, page_rows):
    """rap_prefill_attn_ex over fp8 (E4M3) caches, dense and paged, against the fp8 prefill oracle:
    several key tiles, ragged tails, chunked and too-short sequences, NaN codes beyond the
    sequences and in unused pages; the paged result equals the dense one bit for bit."""
    _say("prefill q8 P=%d dv=%d n_new=%d page_rows=%d" % (P, dv, n_new, page_rows))
    lens_np = np.asarray(lens, dtype=np.int64)
    B = len(lens)
    unit = page_rows if page_rows else 16
    cap = (int(lens_np.max()) + unit - 1) // unit * unit
    rng = np.random.Generator(np.random.PCG64(1300 + P + n_new))
    ks = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    k8 = np.full((B, Hkv, cap, 2 * P), 0x7F, dtype=np.uint8)
    v8 = np.full((B, Hkv, cap, dv), 0xFF, dtype=np.uint8)
    for b in range(B):
        n = int(lens_np[b])
        k8[b, :, :n] = O.f64_to_e4m3_bits(rng.standard_normal((Hkv, n, 2 * P)) / ks.astype(np.float64)[:, None, None])
        v8[b, :, :n] = O.f64_to_e4m3_bits(rng.standard_normal((Hkv, n, dv)) / vs.astype(np.float64)[:, None, None])
    gen = torch.Generator(device=DEV); gen.manual_seed(7)
    q = torch.randn((B, n_new, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    ksd, vsd = torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)
    scale = 1.0 / math.sqrt(2 * P)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    out = torch.full((B, n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    k8d, v8d = torch.from_numpy(k8).to(DEV), torch.from_numpy(v8).to(DEV)
    rap.rap_prefill_attn_ex(shp, k8d, v8d, ksd, vsd, None, n_new, q, sl, cap, out, scale)
    torch.cuda.synchronize()
    ref = O.prefill_attn_q8_ref(I.bits(q), k8, v8, ks, vs, lens_np, scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "fp8 prefill")
    if page_rows:
        max_pages = cap // page_rows
        n_pages = B * max_pages + 3
        table = rng.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
        kp = O.dense_to_paged_ref(k8, table, page_rows, n_pages, lens_np, fill=0x7F)
        vp = O.dense_to_paged_ref(v8, table, page_rows, n_pages, lens_np, fill=0xFF)
        table_dev = table.copy()
        for b in range(B):
            table_dev[b, (int(lens_np[b]) + page_rows - 1) // page_rows:] = 2 ** 30
        pg = rap.paging(page_rows, n_pages, torch.from_numpy(table_dev).to(DEV))
        out_p = torch.full_like(out, float("nan"))
        rap.rap_prefill_attn_ex(shp, torch.from_numpy(kp).to(DEV), torch.from_numpy(vp).to(DEV), ksd, vsd, pg, n_new, q, sl, cap,
                                out_p, scale)
        torch.cuda.synchronize()
        assert torch.equal(out_p, out), "paged and dense fp8 prefill differ"
    # scales come as a pair
    assert rap.rap_prefill_attn_ex(shp, k8d, v8d, ksd, None, None, n_new, q, sl, cap, out, scale, check=False) == 1


@pytest.mark.parametrize("seed", range(12))
def test_prefill_random_shapes(rap, seed):
    """rap_prefill_attn_ex on shapes, cache kinds and page sizes drawn from a seed (widths 2 to 128,
    any d_v, G from 1 to 8, whole, chunked and too-short sequences), against the oracle."""
    rng = np.random.Generator(np.random.PCG64(7000 + seed))
    P, dv = int(rng.integers(1, 65)), int(rng.integers(1, 129))
    Hkv, G = int(rng.integers(1, 4)), int(rng.integers(1, 9))
    n_new = int(rng.integers(1, 400))
    B = int(rng.integers(1, 4))
    lens = [int(rng.integers(max(1, n_new // 2), n_new + 700)) for _ in range(B)]
    fp8 = bool(rng.integers(0, 2))
    page_rows = int(rng.choice([0, 64, 128, 256]))
    Hq = G * Hkv
    _say("prefill random fp8=%s page_rows=%d P=%d dv=%d Hq=%d Hkv=%d n_new=%d lens=%s" % (fp8, page_rows, P, dv, Hq, Hkv, n_new, lens))
    lens_np = np.asarray(lens, dtype=np.int64)
    unit = page_rows if page_rows else 16
    cap = (int(lens_np.max()) + unit - 1) // unit * unit
    scale = 1.0 / math.sqrt(2 * P)
    gen = torch.Generator(device=DEV); gen.manual_seed(seed)
    q = torch.randn((B, n_new, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    if fp8:
        ks = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
        vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
        kd = np.full((B, Hkv, cap, 2 * P), 0x7F, dtype=np.uint8); vd = np.full((B, Hkv, cap, dv), 0xFF, dtype=np.uint8)
        for b in range(B):
            n = int(lens_np[b])
            kd[b, :, :n] = O.f64_to_e4m3_bits(rng.standard_normal((Hkv, n, 2 * P)) / ks.astype(np.float64)[:, None, None])
            vd[b, :, :n] = O.f64_to_e4m3_bits(rng.standard_normal((Hkv, n, dv)) / vs.astype(np.float64)[:, None, None])
        ksd, vsd = torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)
        ref = O.prefill_attn_q8_ref(I.bits(q), kd, vd, ks, vs, lens_np, scale)
        fill_k, fill_v = 0x7F, 0xFF
        to_dev = lambda x: torch.from_numpy(x).to(DEV)
    else:
        kd = np.full((B, Hkv, cap, 2 * P), 0x7FC0, dtype=np.uint16); vd = np.full((B, Hkv, cap, dv), 0x7FC0, dtype=np.uint16)
        for b in range(B):
            n = int(lens_np[b])
            kd[b, :, :n] = O.f64_to_bf16_bits_rne(rng.standard_normal((Hkv, n, 2 * P)))
            vd[b, :, :n] = O.f64_to_bf16_bits_rne(rng.standard_normal((Hkv, n, dv)))
        ksd = vsd = None
        ref = O.prefill_attn_ref(I.bits(q), kd, vd, lens_np, scale)
        fill_k = fill_v = 0x7FC0
        to_dev = lambda x: I.from_bits(x, DEV)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    pg = None
    if page_rows:
        max_pages = cap // page_rows
        n_pages = B * max_pages + 2
        table = rng.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
        kd = O.dense_to_paged_ref(kd, table, page_rows, n_pages, lens_np, fill=fill_k)
        vd = O.dense_to_paged_ref(vd, table, page_rows, n_pages, lens_np, fill=fill_v)
        pg = rap.paging(page_rows, n_pages, torch.from_numpy(table).to(DEV))
    out = torch.full((B, n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn_ex(shp, to_dev(kd), to_dev(vd), ksd, vsd, pg, n_new, q, sl, cap, out, scale)
    torch.cuda.synchronize()
    H.assert_attn_close(out.cpu().numpy(), ref, "random prefill")


def _cache_of_any_kind(rap, rng, B, Hkv, P, dv, lens_np, fp8, page_rows):
    """Seeded K / V caches of the asked kind (bf16 or E4M3 codes with scales, dense or pools with a
    shuffled block table), NaN beyond every sequence and in unused pages.  Returns the dense numpy
    arrays for the oracle and what the *_ex / *_multi calls take."""
    unit = page_rows if page_rows else 16
    cap = max(unit, (int(lens_np.max()) + unit - 1) // unit * unit)
    if fp8:
        ks = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
        vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
        kd = np.full((B, Hkv, cap, 2 * P), 0x7F, dtype=np.uint8); vd = np.full((B, Hkv, cap, dv), 0xFF, dtype=np.uint8)
        for b in range(B):
            n = int(lens_np[b])
            kd[b, :, :n] = O.f64_to_e4m3_bits(rng.standard_normal((Hkv, n, 2 * P)) / ks.astype(np.float64)[:, None, None])
            vd[b, :, :n] = O.f64_to_e4m3_bits(rng.standard_normal((Hkv, n, dv)) / vs.astype(np.float64)[:, None, None])
        ksd, vsd = torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)
        fill_k, fill_v = 0x7F, 0xFF
        to_dev = lambda x: torch.from_numpy(x).to(DEV)
    else:
        ks = vs = ksd = vsd = None
        kd = np.full((B, Hkv, cap, 2 * P), 0x7FC0, dtype=np.uint16); vd = np.full((B, Hkv, cap, dv), 0x7FC0, dtype=np.uint16)
        for b in range(B):
            n = int(lens_np[b])
            kd[b, :, :n] = O.f64_to_bf16_bits_rne(rng.standard_normal((Hkv, n, 2 * P)))
            vd[b, :, :n] = O.f64_to_bf16_bits_rne(rng.standard_normal((Hkv, n, dv)))
        fill_k = fill_v = 0x7FC0
        to_dev = lambda x: I.from_bits(x, DEV)
    pg, kdev, vdev = None, to_dev(kd), to_dev(vd)
    if page_rows:
        max_pages = cap // page_rows
        n_pages = B * max_pages + 2
        table = rng.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
        kdev = to_dev(O.dense_to_paged_ref(kd, table, page_rows, n_pages, lens_np, fill=fill_k))
        vdev = to_dev(O.dense_to_paged_ref(vd, table, page_rows, n_pages, lens_np, fill=fill_v))
        pg = rap.paging(page_rows, n_pages, torch.from_numpy(table).to(DEV))
    return cap, kd, vd, ks, vs, kdev, vdev, ksd, vsd, pg


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("P,dv,Hkv,G,n_tok,lens,page_rows", [
    (45, 90, 2, 4, 4, [1300, 700, 3, 4, 0], 0), (58, 115, 2, 4, 3, [2100, 33], 32), (32, 64, 2, 5, 3, [900, 600], 64),
    (64, 128, 1, 1, 16, [5000, 17, 16, 15], 128), (45, 90, 1, 8, 2, [4100, 2], 0), (3, 5, 3, 2, 7, [40, 100, 6], 0)])
def test_decode_multi(rap, fp8, P, dv, Hkv, G, n_tok, lens, page_rows):
    """rap_decode_attn_multi (a few query tokens per sequence through the decode kernel) against
    the causal prefill oracle: token-times-group products up to 16, one and several row ranges,
    sequences shorter than, as long as and longer than the token count, an empty one, every
    cache kind; and against the prefill kernel's result for the same inputs (to fp32 rounding)."""
    _say("decode multi fp8=%s P=%d dv=%d G=%d n_tok=%d lens=%s page_rows=%d" % (fp8, P, dv, G, n_tok, lens, page_rows))
    lens_np = np.asarray(lens, dtype=np.int64)
    B, Hq = len(lens), G * Hkv
    rng = np.random.Generator(np.random.PCG64(9100 + P + n_tok))
    cap, kd, vd, ks, vs, kdev, vdev, ksd, vsd, pg = _cache_of_any_kind(rap, rng, B, Hkv, P, dv, lens_np, fp8, page_rows)
    gen = torch.Generator(device=DEV); gen.manual_seed(n_tok)
    q = torch.randn((B, n_tok, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    scale = 1.0 / math.sqrt(2 * P)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    ws = rap.new_workspace(shp, cap, n_tok=n_tok)
    ws.fill_(0xFF)                                   # NaN bit patterns in every partial slot
    out = torch.full((B, n_tok, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_decode_attn_multi(shp, kdev, vdev, ksd, vsd, pg, n_tok, q, sl, cap, out, scale, ws)
    torch.cuda.synchronize()
    if fp8:
        ref = O.prefill_attn_q8_ref(I.bits(q), kd, vd, ks, vs, lens_np, scale)
    else:
        ref = O.prefill_attn_ref(I.bits(q), kd, vd, lens_np, scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "multi-token decode")
    if page_rows == 0 or page_rows >= 64:
        pre = torch.full_like(out, float("nan"))
        rap.rap_prefill_attn_ex(shp, kdev, vdev, ksd, vsd, pg, n_tok, q, sl, cap, pre, scale)
        torch.cuda.synchronize()
        assert (out - pre).abs().max().item() <= 2e-5 * max(1.0, pre.abs().max().item())
    # the same call twice gives the same bits
    again = torch.full_like(out, float("nan"))
    rap.rap_decode_attn_multi(shp, kdev, vdev, ksd, vsd, pg, n_tok, q, sl, cap, again, scale, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, again)


@pytest.mark.parametrize("seed", range(10))
def test_decode_multi_random_shapes(rap, seed):
    """rap_decode_attn_multi on shapes, token counts, cache kinds and page sizes drawn from a seed
    (token count x group up to 16, lengths from empty to several row ranges), against the oracle."""
    rng = np.random.Generator(np.random.PCG64(9300 + seed))
    P, dv = int(rng.integers(1, 65)), int(rng.integers(1, 129))
    G = int(rng.integers(1, 9))
    n_tok = int(rng.integers(2, 16 // G + 1)) if 16 // G >= 2 else 1
    Hkv, B = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    lens = [int(rng.choice([0, 1, n_tok - 1, n_tok, n_tok + 1, int(rng.integers(2, 3000))])) for _ in range(B)]
    lens[0] = int(rng.integers(600, 3000))
    fp8 = bool(rng.integers(0, 2))
    page_rows = int(rng.choice([0, 32, 64, 256]))
    _say("multi random fp8=%s page_rows=%d P=%d dv=%d G=%d Hkv=%d n_tok=%d lens=%s" % (fp8, page_rows, P, dv, G, Hkv, n_tok, lens))
    lens_np = np.asarray(lens, dtype=np.int64)
    Hq = G * Hkv
    cap, kd, vd, ks, vs, kdev, vdev, ksd, vsd, pg = _cache_of_any_kind(rap, rng, B, Hkv, P, dv, lens_np, fp8, page_rows)
    gen = torch.Generator(device=DEV); gen.manual_seed(seed)
    q = torch.randn((B, n_tok, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    scale = 1.0 / math.sqrt(2 * P)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    rps = int(rng.choice([0, 128, 512]))
    tun = rap.tuning(rows_per_split=rps)
    ws = rap.new_workspace(shp, cap, tun, n_tok=n_tok)
    ws.fill_(0xFF)
    out = torch.full((B, n_tok, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_decode_attn_multi(shp, kdev, vdev, ksd, vsd, pg, n_tok, q, sl, cap, out, scale, ws, tuning=tun)
    torch.cuda.synchronize()
    if fp8:
        ref = O.prefill_attn_q8_ref(I.bits(q), kd, vd, ks, vs, lens_np, scale)
    else:
        ref = O.prefill_attn_ref(I.bits(q), kd, vd, lens_np, scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "random multi-token decode")


@pytest.mark.parametrize("fp8,page_rows", [(False, 0), (True, 0), (False, 64), (True, 128)])
@pytest.mark.parametrize("P,dv,Hkv,G,lens", [(45, 90, 2, 16, [1700, 300, 0]), (58, 115, 1, 12, [2300, 5]), (64, 128, 2, 9, [900, 899])])
def test_wide_groups(rap, fp8, page_rows, P, dv, Hkv, G, lens):
    """More than eight query heads per KV head (up to 16: the columns of the matrix instruction):
    rap_decode_attn over every cache kind and the prefill attention against their oracles; the
    paths that stop at eight (vector-ALU kernel, fused query rotation, one-call step) say so."""
    _say("wide groups fp8=%s page_rows=%d P=%d dv=%d G=%d lens=%s" % (fp8, page_rows, P, dv, G, lens))
    lens_np = np.asarray(lens, dtype=np.int64)
    B, Hq = len(lens), G * Hkv
    rng = np.random.Generator(np.random.PCG64(9500 + P + G))
    cap, kd, vd, ks, vs, kdev, vdev, ksd, vsd, pg = _cache_of_any_kind(rap, rng, B, Hkv, P, dv, lens_np, fp8, page_rows)
    gen = torch.Generator(device=DEV); gen.manual_seed(G)
    n_new = 40
    q = torch.randn((B, n_new, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    scale = 1.0 / math.sqrt(2 * P)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    # decode: the last token's queries
    q1 = q[:, -1].contiguous()
    for rps in (0, 256):
        tun = rap.tuning(rows_per_split=rps)
        ws = rap.new_workspace(shp, cap, tun)
        ws.fill_(0xFF)
        out = torch.full((B, 1, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_attn_multi(shp, kdev, vdev, ksd, vsd, pg, 1, q1, sl, cap, out, scale, ws, tuning=tun)
        torch.cuda.synchronize()
        if fp8:
            ref = O.attn_q8_ref(I.bits(q1), kd, vd, ks, vs, lens_np, scale)
        else:
            ref = O.attn_ref(I.bits(q1), kd, vd, lens_np, scale)
        H.assert_attn_close(out[:, 0].cpu().numpy(), ref, "decode, G = %d, rows_per_split %d" % (G, rps))
    # prefill of the last 40 tokens, whole and cut into key ranges
    if page_rows == 0 or page_rows >= 64:
        pre = torch.full((B, n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_prefill_attn_ex(shp, kdev, vdev, ksd, vsd, pg, n_new, q, sl, cap, pre, scale)
        need = rap.rap_prefill_attn_split_workspace_bytes(shp, n_new, cap)
        pre2 = torch.full_like(pre, float("nan"))
        rap.rap_prefill_attn_split(shp, kdev, vdev, ksd, vsd, pg, n_new, q, sl, cap, pre2, scale,
                                   torch.empty(need, dtype=torch.uint8, device=DEV) if need else None)
        torch.cuda.synchronize()
        if fp8:
            refp = O.prefill_attn_q8_ref(I.bits(q), kd, vd, ks, vs, lens_np, scale)
        else:
            refp = O.prefill_attn_ref(I.bits(q), kd, vd, lens_np, scale)
        H.assert_attn_close(pre.cpu().numpy(), refp, "prefill, G = %d" % G)
        H.assert_attn_close(pre2.cpu().numpy(), refp, "split prefill, G = %d" % G)
    if not fp8 and page_rows == 0:
        ws = rap.new_workspace(shp, cap)
        out = torch.zeros((B, Hq, dv), dtype=torch.float32, device=DEV)
        keep = torch.arange(P, dtype=torch.int32, device=DEV).repeat(Hkv, 1).contiguous()
        pos = torch.zeros(B, dtype=torch.int32, device=DEV)
        assert rap.rap_decode_attn(shp, q1, kdev, vdev, sl, cap, out, scale, ws, rap.tuning(kernel=1), check=False) == 3
        assert rap.rap_decode_attn_rope(shp, q1, pos, keep, kdev, vdev, sl, cap, out, scale, ws, check=False) == 3
        k1 = torch.zeros((B, Hkv, 2 * P), dtype=torch.bfloat16, device=DEV)
        v1 = torch.zeros((B, Hkv, dv), dtype=torch.bfloat16, device=DEV)
        assert rap.rap_decode_step(shp, k1, v1, pos, keep, q1, True, kdev, vdev, sl, cap, out, scale, ws, check=False) == 3
        assert rap.rap_decode_attn(shp, q1, kdev, vdev, sl, cap, out, scale, ws) == 0


def test_decode_multi_one_token_and_rejections(rap):
    """n_tok = 1 is rap_decode_attn bit for bit; more than 16 query rows per KV head, the
    vector-ALU kernel and a workspace sized for one token are refused."""
    _say("decode multi: one token, refusals")
    P, dv, Hq, Hkv, lens = 45, 90, 8, 2, [1500, 64]
    lens_np = np.asarray(lens, dtype=np.int64)
    B = len(lens)
    rng = np.random.Generator(np.random.PCG64(9200))
    cap, kd, vd, _, _, kdev, vdev, _, _, _ = _cache_of_any_kind(rap, rng, B, Hkv, P, dv, lens_np, False, 0)
    gen = torch.Generator(device=DEV); gen.manual_seed(3)
    q = torch.randn((B, 1, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    ws = rap.new_workspace(shp, cap)
    a = torch.full((B, 1, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    b = torch.full((B, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_decode_attn_multi(shp, kdev, vdev, None, None, None, 1, q, sl, cap, a, 0.1, ws)
    rap.rap_decode_attn(shp, q[:, 0].contiguous(), kdev, vdev, sl, cap, b, 0.1, ws)
    torch.cuda.synchronize()
    assert torch.equal(a[:, 0], b)
    q5 = torch.zeros((B, 5, Hq, 2 * P), dtype=torch.bfloat16, device=DEV)
    o5 = torch.zeros((B, 5, Hq, dv), dtype=torch.float32, device=DEV)
    ws5 = rap.new_workspace(shp, cap, n_tok=5)
    assert rap.rap_decode_attn_multi(shp, kdev, vdev, None, None, None, 5, q5, sl, cap, o5, 0.1, ws5, check=False) == 3   # 5 x 4 > 16
    assert rap.rap_decode_attn_multi(shp, kdev, vdev, None, None, None, 4, q5, sl, cap, o5, 0.1, ws, check=False) == 5    # workspace of one token
    assert rap.rap_decode_attn_multi(shp, kdev, vdev, None, None, None, 4, q5, sl, cap, o5, 0.1, ws5,
                                     tuning=rap.tuning(kernel=1), check=False) == 3
    assert rap.rap_decode_attn_multi(shp, kdev, vdev, None, None, None, 0, q5, sl, cap, o5, 0.1, ws5, check=False) == 2
    assert rap.rap_decode_attn_multi(shp, kdev, vdev, None, None, None, 4, q5, sl, cap, o5, 0.1, ws5, check=False) == 0


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("P,dv,Hkv,G,n_new,lens,page_rows", [
    (45, 90, 2, 4, 100, [3000, 700, 40], 0),          # 12 key ranges; a short and a too-short sequence
    (58, 115, 1, 4, 33, [5000, 4999], 64),            # odd d_v, pages of 64 rows
    (64, 128, 2, 2, 300, [2500, 2100], 128),          # padded LDS rows, three column blocks
    (32, 64, 1, 5, 17, [1100, 1], 0), (3, 5, 1, 1, 70, [777, 650, 0], 0),
    (45, 90, 8, 4, 512, [4096], 0)])                  # a chunk at the end of one long sequence
def test_prefill_split(rap, fp8, P, dv, Hkv, G, n_new, lens, page_rows):
    """rap_prefill_attn_split (key ranges + combining launch) against the prefill oracle and
    against the unsplit kernel, on launches small enough to be cut: every cache kind, ranges that
    are empty for some or all tokens of a block, sequences shorter than the chunk."""
    _say("prefill split fp8=%s P=%d dv=%d G=%d n_new=%d lens=%s page_rows=%d" % (fp8, P, dv, G, n_new, lens, page_rows))
    lens_np = np.asarray(lens, dtype=np.int64)
    B, Hq = len(lens), G * Hkv
    rng = np.random.Generator(np.random.PCG64(9400 + P + n_new))
    cap, kd, vd, ks, vs, kdev, vdev, ksd, vsd, pg = _cache_of_any_kind(rap, rng, B, Hkv, P, dv, lens_np, fp8, page_rows)
    gen = torch.Generator(device=DEV); gen.manual_seed(n_new)
    q = torch.randn((B, n_new, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.from_numpy(lens_np.astype(np.int32)).to(DEV)
    scale = 1.0 / math.sqrt(2 * P)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5e5)
    need = rap.rap_prefill_attn_split_workspace_bytes(shp, n_new, cap)
    assert need > 0, "this case was meant to be cut into key ranges"
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=DEV)      # NaN bit patterns in every slot
    out = torch.full((B, n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn_split(shp, kdev, vdev, ksd, vsd, pg, n_new, q, sl, cap, out, scale, ws)
    torch.cuda.synchronize()
    if fp8:
        ref = O.prefill_attn_q8_ref(I.bits(q), kd, vd, ks, vs, lens_np, scale)
    else:
        ref = O.prefill_attn_ref(I.bits(q), kd, vd, lens_np, scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "split prefill")
    one = torch.full_like(out, float("nan"))
    rap.rap_prefill_attn_ex(shp, kdev, vdev, ksd, vsd, pg, n_new, q, sl, cap, one, scale)
    torch.cuda.synchronize()
    assert (out - one).abs().max().item() <= 2e-5 * max(1.0, one.abs().max().item())
    # a workspace one byte short, or none, is refused; a launch that is not cut needs none
    assert rap.rap_prefill_attn_split(shp, kdev, vdev, ksd, vsd, pg, n_new, q, sl, cap, out, scale, ws[:need - 1], check=False) == 5
    assert rap.rap_prefill_attn_split(shp, kdev, vdev, ksd, vsd, pg, n_new, q, sl, cap, out, scale, None, check=False) == 5


def test_prefill_split_not_cut(rap):
    """A launch with enough query blocks is not cut: no workspace asked for, same bits as rap_prefill_attn."""
    _say("prefill split: large launch stays whole")
    P, dv, Hq, Hkv, n_new, lens = 45, 90, 8, 2, 6200, [6200, 6200]
    q, kc, vc, sl, cap, scale = _prefill_case(P, dv, Hq, Hkv, n_new, lens, seed=78)
    shp = rap.shape(len(lens), Hq, Hkv, 128, P, dv, cap, 5.0e5)
    assert rap.rap_prefill_attn_split_workspace_bytes(shp, n_new, cap) == 0
    a = torch.full((len(lens), n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    b = torch.full_like(a, float("nan"))
    rap.rap_prefill_attn_split(shp, kc, vc, None, None, None, n_new, q, sl, cap, a, scale, None)
    rap.rap_prefill_attn(shp, n_new, q, kc, vc, sl, cap, b, scale)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_prefill_last_row_is_decode(rap):
    """The last query of a prefill is the decode case: same numbers as rap_decode_attn (to fp32
    rounding: other tiling of the same sums)."""
    P, dv, Hq, Hkv, n_new, lens = 45, 90, 8, 2, 64, [777, 1500]
    q, kc, vc, sl, cap, scale = _prefill_case(P, dv, Hq, Hkv, n_new, lens, seed=77)
    shp = rap.shape(len(lens), Hq, Hkv, 128, P, dv, cap, 5.0e5)
    out = torch.empty((len(lens), n_new, Hq, dv), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn(shp, n_new, q, kc, vc, sl, cap, out, scale)
    dec = torch.empty((len(lens), Hq, dv), dtype=torch.float32, device=DEV)
    ws = rap.new_workspace(shp, cap, None)
    rap.rap_decode_attn(shp, q[:, -1].contiguous(), kc, vc, sl, cap, dec, scale, ws, None)
    torch.cuda.synchronize()
    rel = (out[:, -1] - dec).abs().max().item() / dec.abs().max().item()
    assert rel <= 2e-5, rel


def test_prefill_cfg2_sampled(rap):
    """Full prefill at the cfg2 shape (16 x 8192 tokens, 32/8 heads, d = 90), sampled (b, token,
    head) rows against the oracle computed one by one."""
    w = I.WORKLOADS["cfg2"]
    B, S, Hq, Hkv, P, dv = w.batch, w.ctx, w.n_q_heads, w.n_kv_heads, w.n_pairs, w.d_v
    _say("prefill cfg2 full size")
    q, kc, vc, sl, cap, scale = _prefill_case(P, dv, Hq, Hkv, S, [S] * B, seed=5)
    shp = rap.shape(B, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    out = torch.full((B, S, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn(shp, S, q, kc, vc, sl, cap, out, scale)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    rng = np.random.Generator(np.random.PCG64(3))
    G = Hq // Hkv
    picks = [(int(rng.integers(B)), int(rng.integers(S)), int(rng.integers(Hq))) for _ in range(60)]
    picks += [(0, 0, 0), (B - 1, S - 1, Hq - 1), (3, 63, 5), (3, 64, 5), (7, 4095, 17), (7, 4096, 17)]
    got, ref = [], []
    for b, i, a_h in picks:
        h = a_h // G
        kf = O.bf16_bits_to_f64(I.bits(kc[b, h, :i + 1]))
        vf = O.bf16_bits_to_f64(I.bits(vc[b, h, :i + 1]))
        qf = O.bf16_bits_to_f64(I.bits(q[b, i, a_h]))[None, :]
        ref.append(O.attn_rows_ref(qf, kf, vf, scale)[0])
        got.append(out[b, i, a_h].cpu().numpy())
    H.assert_attn_close(np.array(got), np.array(ref), "prefill cfg2 sampled")


@pytest.mark.parametrize("call,n_new", [("multi", 4), ("split", 64)])
def test_cfg2_several_tokens_sampled(rap, call, n_new):
    """The two calls for several new tokens at the sizes bench.py times them at (cfg2 shape: 16
    sequences of 8192 rows, 32/8 heads, d = 90; four tokens through rap_decode_attn_multi, a chunk
    of 64 through rap_prefill_attn_split), in the launch configuration of the bench: sampled
    (b, token, head) rows against the oracle computed one by one, plus every token of one head."""
    w = I.WORKLOADS["cfg2"]
    B, S, Hq, Hkv, P, dv = w.batch, w.ctx, w.n_q_heads, w.n_kv_heads, w.n_pairs, w.d_v
    _say("cfg2 full size, %s, %d tokens" % (call, n_new))
    q, kc, vc, sl, cap, scale = _prefill_case(P, dv, Hq, Hkv, n_new, [S] * B, seed=6)
    shp = rap.shape(B, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    out = torch.full((B, n_new, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    if call == "multi":
        ws = rap.new_workspace(shp, cap, None, n_tok=n_new)
        rap.rap_decode_attn_multi(shp, kc, vc, None, None, None, n_new, q, sl, cap, out, scale, ws)
    else:
        need = rap.rap_prefill_attn_split_workspace_bytes(shp, n_new, cap)
        assert need > 0
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        rap.rap_prefill_attn_split(shp, kc, vc, None, None, None, n_new, q, sl, cap, out, scale, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    rng = np.random.Generator(np.random.PCG64(4))
    G = Hq // Hkv
    picks = [(int(rng.integers(B)), int(rng.integers(n_new)), int(rng.integers(Hq))) for _ in range(40)]
    picks += [(0, 0, 0), (B - 1, n_new - 1, Hq - 1)] + [(5, i, 9) for i in range(n_new)]
    got, ref = [], []
    for b, i, a_h in picks:
        h = a_h // G
        n_vis = S - n_new + i + 1                   # rows token i sees
        kf = O.bf16_bits_to_f64(I.bits(kc[b, h, :n_vis]))
        vf = O.bf16_bits_to_f64(I.bits(vc[b, h, :n_vis]))
        qf = O.bf16_bits_to_f64(I.bits(q[b, i, a_h]))[None, :]
        ref.append(O.attn_rows_ref(qf, kf, vf, scale)[0])
        got.append(out[b, i, a_h].cpu().numpy())
    H.assert_attn_close(np.array(got), np.array(ref), "cfg2 %s sampled" % call)


def test_frequency_table(rap):
    """rap_shape_t.pair_inv_freq: a scaled frequency table with un-rotated pairs replaces rope_theta
    and keep_pair_idx in the per-token append, the run-based append, the fused query rotation and
    the one-call step (keep_pair_idx passed as NULL)."""
    P, dv, Hq, Hkv, D, theta = 45, 90, 8, 2, 128, 5.0e5
    _say("frequency table")
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, ctx=600, n_new=40, ragged_min=200, peaky_frac=0.0, seed=55)
    case = I.make_case(w, device=DEV)
    keep = case.keep.cpu().numpy()
    table = O.inv_freq(theta, D)[keep]                                   # [H_kv, P]
    table = table * np.where(table < 0.01, 0.125, 1.0)                   # long wavelengths stretched (a scaled table)
    table[:, ::7] = 0.0                                                  # some pairs not rotated at all
    tdev = torch.from_numpy(table).to(DEV)
    shp = rap.shape(w.batch, Hq, Hkv, D, P, dv, case.cap, 1.0, pair_inv_freq=tdev)   # rope_theta is not used
    lens = case.seq_lens.cpu().numpy()
    # run-based append of 40 tokens, then per-token append of 3 more at far rows
    okc, ovc = I.bits(case.k_cache).copy(), I.bits(case.v_cache).copy()
    rap.rap_rope_append(shp, w.n_new, case.k_new, case.v_new, case.pos, None, case.k_cache, case.v_cache)
    O.append_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), None, okc, ovc, theta, D, pair_freq=table)
    k3, v3 = case.k_new[:, :3].contiguous(), case.v_new[:, :3].contiguous()
    pos3 = torch.tensor([[5, 0, case.cap - 1]] * w.batch, dtype=torch.int32, device=DEV)
    rap.rap_rope_append(shp, 3, k3, v3, pos3, None, case.k_cache, case.v_cache)
    O.append_ref(I.bits(k3), I.bits(v3), pos3.cpu().numpy(), None, okc, ovc, theta, D, pair_freq=table)
    torch.cuda.synchronize()
    dist = H.bf16_ulp_distance(I.bits(case.k_cache), okc)
    assert dist.max() <= 1 and (dist != 0).sum() <= dist.size // 1000 + 1
    assert np.array_equal(I.bits(case.v_cache), ovc)
    # fused query rotation and the one-call step
    qpos_np = (lens - 1).astype(np.int32)
    qpos = torch.from_numpy(qpos_np).to(DEV)
    qrot = O.rope_queries_ref(I.bits(case.q), qpos_np, None, theta, D, Hkv, pair_freq=table)
    for kernel in (VALU, MFMA):
        tun = rap.tuning(kernel=kernel)
        ws = rap.new_workspace(shp, case.cap, tun)
        out = torch.full((w.batch, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_attn_rope(shp, case.q, qpos, None, case.k_cache, case.v_cache, case.seq_lens, case.cap, out, float(w.scale), ws, tun)
        torch.cuda.synchronize()
        ref = O.attn_ref(qrot, I.bits(case.k_cache), I.bits(case.v_cache), lens, w.scale)
        H.assert_attn_close(out.cpu().numpy(), ref, "table, fused query rotation, kernel %d" % kernel)
        kc, vc = case.k_cache.clone(), case.v_cache.clone()
        kn, vn = case.k_new[:, -1].contiguous(), case.v_new[:, -1].contiguous()
        rap.rap_decode_step(shp, kn, vn, qpos, None, case.q, False, kc, vc, case.seq_lens, case.cap, out, float(w.scale), ws, tun)
        torch.cuda.synchronize()
        okc2, ovc2 = I.bits(case.k_cache).copy(), I.bits(case.v_cache).copy()
        O.append_ref(I.bits(kn)[:, None], I.bits(vn)[:, None], qpos_np[:, None], None, okc2, ovc2, theta, D, pair_freq=table)
        assert H.bf16_ulp_distance(I.bits(kc), okc2).max() <= 1 and np.array_equal(I.bits(vc), ovc2)
        ref = O.attn_ref(qrot, I.bits(kc), I.bits(vc), lens, w.scale)
        H.assert_attn_close(out.cpu().numpy(), ref, "table, one-call step, kernel %d" % kernel)


def _rope_queries_oracle(q_bits, pos, keep, theta, d_head, n_kv, pair_freq=None):
    """Token by token through the oracle's query rotation ([B, n, H_q, 2P])."""
    out = np.empty_like(q_bits)
    for n in range(q_bits.shape[1]):
        out[:, n] = O.rope_queries_ref(q_bits[:, n], pos[:, n], keep, theta, d_head, n_kv, pair_freq=pair_freq)
    return out


@pytest.mark.parametrize("P,Hq,Hkv,n_new", [(45, 8, 2, 100), (58, 8, 2, 37), (32, 10, 2, 16), (64, 4, 1, 7), (3, 3, 1, 65)])
def test_rope_queries(rap, P, Hq, Hkv, n_new):
    """rap_rope_queries against the oracle, bit for bit up to the 1-ulp bar: consecutive positions
    (angle carried along runs), shuffled and far positions, short inputs, a bad pair index (stored
    as zero), in place."""
    B, D, theta = 3, 128, 5.0e5
    _say("rope queries P=%d heads %d/%d n_new=%d" % (P, Hq, Hkv, n_new))
    rng = np.random.Generator(np.random.PCG64(31 + P))
    keep = I.draw_keep(rng, Hkv, D // 2, P)
    if P > 4:
        keep[0, 3] = D // 2 + 5                                   # bad index
    gen = torch.Generator(device=DEV); gen.manual_seed(8)
    q = torch.randn((B, n_new, Hq, 2 * P), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    pos = np.stack([np.arange(n_new) + 1000, rng.permutation(131072)[:n_new], np.arange(n_new) * 3]).astype(np.int32)
    keep_t = torch.from_numpy(keep.astype(np.int32)).to(DEV)
    pos_t = torch.from_numpy(pos).to(DEV)
    shp = rap.shape(B, Hq, Hkv, D, P, 2 * P, 8, theta)
    out = torch.empty_like(q)
    rap.rap_rope_queries(shp, n_new, q, pos_t, keep_t, out)
    inplace = q.clone()
    rap.rap_rope_queries(shp, n_new, inplace, pos_t, keep_t, inplace)
    torch.cuda.synchronize()
    keep_ref = keep.copy()
    ref = _rope_queries_oracle(I.bits(q), pos, np.where(keep_ref < D // 2, keep_ref, 0), theta, D, Hkv)
    if P > 4:                                                     # the bad pair reads as zero for the heads of KV head 0
        G = Hq // Hkv
        ref[:, :, :G, 3] = 0
        ref[:, :, :G, 3 + P] = 0
    dist = H.bf16_ulp_distance(I.bits(out), ref)
    assert dist.max() <= 1 and (dist != 0).sum() <= dist.size // 1000 + 1, (int(dist.max()), int((dist != 0).sum()))
    assert torch.equal(out.view(torch.int16), inplace.view(torch.int16))


def test_prefill_pipeline(rap):
    """The three prefill calls in sequence, run-based append of K/V, rotation of the queries and
    causal attention, against the oracle's composition on un-rotated inputs."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=2, n_q_heads=8, n_kv_heads=2, ctx=333, n_new=333, peaky_frac=0.0, seed=99)
    _say("prefill pipeline")
    case = I.make_case(w, device=DEV, fill_unused=False)
    gen = torch.Generator(device=DEV); gen.manual_seed(4)
    q = torch.randn((w.batch, w.n_new, w.n_q_heads, w.d_k), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    shp = H.shape_of(rap, case)
    rap.rap_rope_append(shp, w.n_new, case.k_new, case.v_new, case.pos, case.keep, case.k_cache, case.v_cache)
    qr = torch.empty_like(q)
    rap.rap_rope_queries(shp, w.n_new, q, case.pos, case.keep, qr)
    out = torch.empty((w.batch, w.n_new, w.n_q_heads, w.d_v), dtype=torch.float32, device=DEV)
    rap.rap_prefill_attn(shp, w.n_new, qr, case.k_cache, case.v_cache, case.seq_lens, case.cap, out, float(w.scale))
    torch.cuda.synchronize()
    keep = case.keep.cpu().numpy()
    pos = case.pos.cpu().numpy()
    okc = np.zeros_like(I.bits(case.k_cache)); ovc = np.zeros_like(I.bits(case.v_cache))
    O.append_ref(I.bits(case.k_new), I.bits(case.v_new), pos, keep, okc, ovc, w.rope_theta, w.d_head)
    qref = _rope_queries_oracle(I.bits(q), pos, keep, w.rope_theta, w.d_head, w.n_kv_heads)
    ref = O.prefill_attn_ref(qref, okc, ovc, case.seq_lens.cpu().numpy(), w.scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "prefill pipeline")


@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx,page_rows,n_new", [
    (45, 90, 8, 2, 3000, 256, 1), (58, 115, 8, 2, 1500, 32, 3), (32, 64, 10, 2, 2500, 128, 40), (64, 128, 4, 1, 700, 64, 1),
    (45, 90, 8, 2, 9000, 1024, 100)])
def test_paged_caches(rap, P, dv, Hq, Hkv, ctx, page_rows, n_new):
    """rap_rope_append_paged + rap_decode_attn_paged over pools with a shuffled block table:
    the pools, gathered back, must be what the dense append gives, and the attention what the
    oracle gives on the dense cache; also with the fused query rotation and several range sizes.
    Unused pool pages and the table entries beyond each sequence hold garbage (NaN / wild numbers)."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=n_new,
                 ragged_min=max(n_new + 1, ctx // 4), peaky_frac=0.0, seed=400 + P + page_rows)
    _say("paged P=%d dv=%d ctx=%d page_rows=%d n_new=%d" % (P, dv, ctx, page_rows, n_new))
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    max_pages = (int(lens.max()) + page_rows - 1) // page_rows
    cap = max_pages * page_rows
    n_pages = w.batch * max_pages + 5
    rng = np.random.Generator(np.random.PCG64(7))
    table = rng.permutation(n_pages)[:w.batch * max_pages].reshape(w.batch, max_pages).astype(np.int32)
    prefill = case.prefill_lens
    kd, vd = I.bits(case.k_cache), I.bits(case.v_cache)
    nan = 0x7FC0
    kp = O.dense_to_paged_ref(kd, table, page_rows, n_pages, prefill, fill=nan)
    vp = O.dense_to_paged_ref(vd, table, page_rows, n_pages, prefill, fill=nan)
    table_dev = table.copy()
    for b in range(w.batch):                                     # entries beyond the sequence: never to be read
        used = (int(lens[b]) + page_rows - 1) // page_rows
        table_dev[b, used:] = 2 ** 30
    k_pool, v_pool = I.from_bits(kp, DEV), I.from_bits(vp, DEV)
    bt = torch.from_numpy(table_dev).to(DEV)
    shp = rap.shape(w.batch, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    pg = rap.paging(page_rows, n_pages, bt)
    rap.rap_rope_append_paged(shp, pg, n_new, case.k_new, case.v_new, case.pos, case.keep, k_pool, v_pool)
    torch.cuda.synchronize()
    okc = np.zeros((w.batch, Hkv, cap, 2 * P), dtype=np.uint16); ovc = np.zeros((w.batch, Hkv, cap, dv), dtype=np.uint16)
    for b in range(w.batch):
        okc[b, :, :prefill[b]] = kd[b, :, :prefill[b]]
        ovc[b, :, :prefill[b]] = vd[b, :, :prefill[b]]
    O.append_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), case.keep.cpu().numpy(), okc, ovc, w.rope_theta, w.d_head)
    gk = O.paged_to_dense_ref(I.bits(k_pool), table, lens)
    gv = O.paged_to_dense_ref(I.bits(v_pool), table, lens)
    for b in range(w.batch):
        assert H.bf16_ulp_distance(gk[b, :, :lens[b]], okc[b, :, :lens[b]]).max() <= 1, "paged K rows"
        assert np.array_equal(gv[b, :, :lens[b]], ovc[b, :, :lens[b]]), "paged V rows"
    ref = O.attn_ref(I.bits(case.q), gk, gv, lens, w.scale)
    for rps in (0, 128, 512):
        tun = rap.tuning(kernel=MFMA, rows_per_split=rps)
        ws = rap.new_workspace(shp, cap, tun)
        out = torch.full((w.batch, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_attn_paged(shp, pg, case.q, None, None, k_pool, v_pool, case.seq_lens, cap, out, float(w.scale), ws, tun)
        torch.cuda.synchronize()
        H.assert_attn_close(out.cpu().numpy(), ref, "paged decode rps=%d" % rps)
    # fused query rotation over the paged cache
    qpos_np = (lens - 1).astype(np.int32)
    qrot = O.rope_queries_ref(I.bits(case.q), qpos_np, case.keep.cpu().numpy(), w.rope_theta, w.d_head, Hkv)
    ref2 = O.attn_ref(qrot, gk, gv, lens, w.scale)
    ws = rap.new_workspace(shp, cap, None)
    rap.rap_decode_attn_paged(shp, pg, case.q, torch.from_numpy(qpos_np).to(DEV), case.keep, k_pool, v_pool, case.seq_lens, cap,
                              out, float(w.scale), ws, None)
    torch.cuda.synchronize()
    H.assert_attn_close(out.cpu().numpy(), ref2, "paged decode with query rotation")
    # the vector-ALU kernel does not read pools
    st = rap.rap_decode_attn_paged(shp, pg, case.q, None, None, k_pool, v_pool, case.seq_lens, cap, out, float(w.scale), ws,
                                   rap.tuning(kernel=VALU), check=False)
    assert st == 3


# ---------------------------------------------------------------- fp8 (E4M3) caches


@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx,n_new", [(45, 90, 8, 2, 1200, 1), (58, 115, 8, 2, 700, 5), (32, 64, 10, 2, 2500, 40),
                                                   (64, 128, 4, 1, 300, 1), (3, 5, 3, 1, 40, 2),
                                                   (45, 90, 8, 2, 2600, 700), (58, 115, 4, 2, 900, 333)])   # run-based append
def test_q8_cache(rap, P, dv, Hq, Hkv, ctx, n_new):
    """rap_rope_append_q8 + rap_decode_attn_q8: the appended codes against the oracle's (equal, up
    to one code step on a vanishing fraction where the fp64 angle arithmetic differs in its last
    bit), then attention over the GPU-written cache against the oracle on the same codes, with
    several range sizes, NaN codes beyond the sequences, and the fused query rotation."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=n_new,
                 ragged_min=max(n_new + 1, ctx // 3), peaky_frac=0.0, seed=600 + P)
    _say("q8 cache P=%d dv=%d ctx=%d n_new=%d" % (P, dv, ctx, n_new))
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    cap = (int(lens.max()) + 15) // 16 * 16
    rng = np.random.Generator(np.random.PCG64(11))
    ks = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)        # per-head scales: amax about 4.5 sigma
    vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    kd = O.bf16_bits_to_f64(I.bits(case.k_cache))[:, :, :cap]
    vd = O.bf16_bits_to_f64(I.bits(case.v_cache))[:, :, :cap]
    k8 = np.full((w.batch, Hkv, cap, 2 * P), 0x7F, dtype=np.uint8)      # NaN everywhere ...
    v8 = np.full((w.batch, Hkv, cap, dv), 0xFF, dtype=np.uint8)
    for b in range(w.batch):                                            # ... but the prefilled rows
        n0 = int(case.prefill_lens[b])
        k8[b, :, :n0] = O.f64_to_e4m3_bits(kd[b, :, :n0] / ks[None, :, None, None].astype(np.float64)[0])
        v8[b, :, :n0] = O.f64_to_e4m3_bits(vd[b, :, :n0] / vs[None, :, None, None].astype(np.float64)[0])
    k8d, v8d = torch.from_numpy(k8).to(DEV), torch.from_numpy(v8).to(DEV)
    ksd, vsd = torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)
    shp = rap.shape(w.batch, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    rap.rap_rope_append_q8(shp, n_new, case.k_new, case.v_new, case.pos, case.keep, k8d, v8d, ksd, vsd)
    torch.cuda.synchronize()
    ok8, ov8 = k8.copy(), v8.copy()
    O.append_q8_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), case.keep.cpu().numpy(), ok8, ov8, ks, vs,
                    w.rope_theta, w.d_head)
    gk, gv = k8d.cpu().numpy(), v8d.cpu().numpy()
    assert np.array_equal(gv, ov8), "V codes differ"
    diff = gk != ok8
    assert diff.sum() <= gk.size // 10000 + 1, "%d K codes differ" % diff.sum()
    if diff.any():
        step = np.abs(O.e4m3_bits_to_f64(gk[diff]) - O.e4m3_bits_to_f64(ok8[diff]))
        assert np.all(step <= np.maximum(np.abs(O.e4m3_bits_to_f64(ok8[diff])), 2.0 ** -6) * 0.126)   # one code step
    ref = O.attn_q8_ref(I.bits(case.q), gk, gv, ks, vs, lens, w.scale)
    for rps in (0, 128, 512):
        tun = rap.tuning(kernel=MFMA, rows_per_split=rps)
        ws = rap.new_workspace(shp, cap, tun)
        out = torch.full((w.batch, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_attn_q8(shp, case.q, None, None, k8d, v8d, ksd, vsd, case.seq_lens, cap, out, float(w.scale), ws, tun)
        torch.cuda.synchronize()
        H.assert_attn_close(out.cpu().numpy(), ref, "q8 decode rps=%d" % rps)
    qpos_np = (lens - 1).astype(np.int32)
    qrot = O.rope_queries_ref(I.bits(case.q), qpos_np, case.keep.cpu().numpy(), w.rope_theta, w.d_head, Hkv)
    ref2 = O.attn_q8_ref(qrot, gk, gv, ks, vs, lens, w.scale)
    ws = rap.new_workspace(shp, cap, None)
    rap.rap_decode_attn_q8(shp, case.q, torch.from_numpy(qpos_np).to(DEV), case.keep, k8d, v8d, ksd, vsd, case.seq_lens, cap,
                           out, float(w.scale), ws, None)
    torch.cuda.synchronize()
    H.assert_attn_close(out.cpu().numpy(), ref2, "q8 decode with query rotation")
    assert rap.rap_decode_attn_q8(shp, case.q, None, None, k8d, v8d, ksd, vsd, case.seq_lens, cap, out, float(w.scale), ws,
                                  rap.tuning(kernel=VALU), check=False) == 3


@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx,page_rows,n_new", [(45, 90, 8, 2, 2100, 128, 1), (58, 115, 8, 2, 900, 32, 4),
                                                             (32, 64, 10, 2, 1500, 64, 30), (64, 128, 4, 1, 600, 256, 1)])
def test_q8_paged_caches(rap, P, dv, Hq, Hkv, ctx, page_rows, n_new):
    """fp8 codes in paged pools: rap_rope_append_paged_q8 + rap_decode_attn_paged_q8.  The oracle
    side is the dense fp8 oracle plus pure re-indexing; unused pages hold NaN codes and the table
    entries beyond each sequence hold wild page numbers."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=n_new,
                 ragged_min=max(n_new + 1, ctx // 3), peaky_frac=0.0, seed=800 + P + page_rows)
    _say("q8 paged P=%d dv=%d ctx=%d page_rows=%d n_new=%d" % (P, dv, ctx, page_rows, n_new))
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    prefill = case.prefill_lens
    max_pages = (int(lens.max()) + page_rows - 1) // page_rows
    cap = max_pages * page_rows
    n_pages = w.batch * max_pages + 3
    rng = np.random.Generator(np.random.PCG64(19))
    table = rng.permutation(n_pages)[:w.batch * max_pages].reshape(w.batch, max_pages).astype(np.int32)
    ks = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    kd = O.bf16_bits_to_f64(I.bits(case.k_cache))
    vd = O.bf16_bits_to_f64(I.bits(case.v_cache))
    k8 = np.full((w.batch, Hkv, cap, 2 * P), 0x7F, dtype=np.uint8)
    v8 = np.full((w.batch, Hkv, cap, dv), 0xFF, dtype=np.uint8)
    for b in range(w.batch):
        n0 = int(prefill[b])
        k8[b, :, :n0] = O.f64_to_e4m3_bits(kd[b, :, :n0] / ks.astype(np.float64)[:, None, None])
        v8[b, :, :n0] = O.f64_to_e4m3_bits(vd[b, :, :n0] / vs.astype(np.float64)[:, None, None])
    kp = O.dense_to_paged_ref(k8, table, page_rows, n_pages, prefill, fill=0x7F)
    vp = O.dense_to_paged_ref(v8, table, page_rows, n_pages, prefill, fill=0xFF)
    table_dev = table.copy()
    for b in range(w.batch):
        used = (int(lens[b]) + page_rows - 1) // page_rows
        table_dev[b, used:] = -(2 ** 30)
    k_pool, v_pool = torch.from_numpy(kp).to(DEV), torch.from_numpy(vp).to(DEV)
    bt = torch.from_numpy(table_dev).to(DEV)
    ksd, vsd = torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)
    shp = rap.shape(w.batch, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    pg = rap.paging(page_rows, n_pages, bt)
    rap.rap_rope_append_paged_q8(shp, pg, n_new, case.k_new, case.v_new, case.pos, case.keep, k_pool, v_pool, ksd, vsd)
    torch.cuda.synchronize()
    ok8, ov8 = k8.copy(), v8.copy()
    O.append_q8_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), case.keep.cpu().numpy(), ok8, ov8, ks, vs,
                    w.rope_theta, w.d_head)
    gk = O.paged_to_dense_ref(k_pool.cpu().numpy(), table, lens)
    gv = O.paged_to_dense_ref(v_pool.cpu().numpy(), table, lens)
    n_diff = 0
    for b in range(w.batch):
        n = int(lens[b])
        assert np.array_equal(gv[b, :, :n], ov8[b, :, :n]), "paged V codes"
        n_diff += int((gk[b, :, :n] != ok8[b, :, :n]).sum())
    assert n_diff <= gk.size // 10000 + 1, "%d K codes differ" % n_diff
    ref = O.attn_q8_ref(I.bits(case.q), gk, gv, ks, vs, lens, w.scale)
    for rps in (0, 128, 512):
        tun = rap.tuning(kernel=MFMA, rows_per_split=rps)
        ws = rap.new_workspace(shp, cap, tun)
        out = torch.full((w.batch, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_attn_paged_q8(shp, pg, case.q, None, None, k_pool, v_pool, ksd, vsd, case.seq_lens, cap, out,
                                     float(w.scale), ws, tun)
        torch.cuda.synchronize()
        H.assert_attn_close(out.cpu().numpy(), ref, "q8 paged decode rps=%d" % rps)
    qpos_np = (lens - 1).astype(np.int32)
    qrot = O.rope_queries_ref(I.bits(case.q), qpos_np, case.keep.cpu().numpy(), w.rope_theta, w.d_head, Hkv)
    ref2 = O.attn_q8_ref(qrot, gk, gv, ks, vs, lens, w.scale)
    ws = rap.new_workspace(shp, cap, None)
    rap.rap_decode_attn_paged_q8(shp, pg, case.q, torch.from_numpy(qpos_np).to(DEV), case.keep, k_pool, v_pool, ksd, vsd,
                                 case.seq_lens, cap, out, float(w.scale), ws, None)
    torch.cuda.synchronize()
    H.assert_attn_close(out.cpu().numpy(), ref2, "q8 paged decode with query rotation")
    # identical to the dense fp8 call on the gathered cache
    gk_d, gv_d = torch.from_numpy(gk).to(DEV), torch.from_numpy(gv).to(DEV)
    out_d = torch.full_like(out, float("nan"))
    rap.rap_decode_attn_q8(shp, case.q, torch.from_numpy(qpos_np).to(DEV), case.keep, gk_d, gv_d, ksd, vsd, case.seq_lens, cap,
                           out_d, float(w.scale), ws, None)
    torch.cuda.synchronize()
    assert torch.equal(out, out_d), "paged and dense fp8 attention differ"


@pytest.mark.parametrize("fp8,paged", [(False, True), (True, False), (True, True), (False, False)])
@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx,page_rows", [(45, 90, 8, 2, 1300, 128), (58, 115, 8, 2, 500, 32), (32, 64, 10, 2, 900, 64)])
def test_decode_step_any_cache(rap, fp8, paged, P, dv, Hq, Hkv, ctx, page_rows):
    """rap_decode_step_ex over bf16 / fp8 caches, dense or paged, against the two calls for the same
    kind of cache (caches bit for bit, outputs to fp32 rounding) and against the oracle on the
    resulting cache.  One token sits in the middle of its sequence, one just beyond the attended rows."""
    _check_any_cache(rap, fp8, paged, P, dv, Hq, Hkv, ctx, page_rows, seed=900 + P + page_rows)


@pytest.mark.parametrize("seed", range(20))
def test_random_shapes(rap, seed):
    """The same comparison (append, attention with and without the fused query rotation, one-call
    step; against each other and against the oracle) on shapes, cache kinds and page sizes drawn
    from a seed: widths from 2 to 128, any d_v, G from 1 to 8, contexts from one tile to ~80."""
    rng = np.random.Generator(np.random.PCG64(5000 + seed))
    P = int(rng.integers(1, 65))
    dv = int(rng.integers(1, 129))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.integers(1, 9))
    ctx = int(rng.integers(40, 2600))
    page_rows = int(rng.choice([32, 64, 128, 256]))
    fp8, paged = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    _check_any_cache(rap, fp8, paged, P, dv, G * Hkv, Hkv, ctx, page_rows, seed=6000 + seed, batch=int(rng.integers(2, 5)))


def _check_any_cache(rap, fp8, paged, P, dv, Hq, Hkv, ctx, page_rows, seed, batch=4):
    w = I.scaled(I.WORKLOADS["cfg2"], batch=batch, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=1,
                 ragged_min=max(2, ctx // 3), peaky_frac=0.0, seed=seed)
    _say("any cache fp8=%s paged=%s P=%d dv=%d Hq=%d Hkv=%d ctx=%d page_rows=%d batch=%d" % (fp8, paged, P, dv, Hq, Hkv, ctx, page_rows, batch))
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy().copy()
    max_pages = (int(lens.max()) + 1 + page_rows - 1) // page_rows
    cap = max_pages * page_rows
    pos_np = (lens - 1).astype(np.int32)
    pos_np[1] = lens[1] // 2
    if w.batch > 2:
        pos_np[2] = lens[2]
    pos = torch.from_numpy(pos_np).to(DEV)
    k_new, v_new = case.k_new[:, 0].contiguous(), case.v_new[:, 0].contiguous()
    keep_np = case.keep.cpu().numpy()
    rng = np.random.Generator(np.random.PCG64(23))
    ks = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32)
    ksd, vsd = (torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)) if fp8 else (None, None)
    # dense cache contents of this kind: bf16 bits or E4M3 codes, rows [0, len) valid
    kb, vb = I.bits(case.k_cache)[:, :, :cap], I.bits(case.v_cache)[:, :, :cap]
    if kb.shape[2] < cap:
        kb = np.concatenate([kb, np.zeros((w.batch, Hkv, cap - kb.shape[2], 2 * P), kb.dtype)], axis=2)
        vb = np.concatenate([vb, np.zeros((w.batch, Hkv, cap - vb.shape[2], dv), vb.dtype)], axis=2)
    if fp8:
        kd = O.f64_to_e4m3_bits(O.bf16_bits_to_f64(kb) / ks.astype(np.float64)[None, :, None, None])
        vd = O.f64_to_e4m3_bits(O.bf16_bits_to_f64(vb) / vs.astype(np.float64)[None, :, None, None])
    else:
        kd, vd = kb.copy(), vb.copy()
    n_pages = w.batch * max_pages + 2
    table = rng.permutation(n_pages)[:w.batch * max_pages].reshape(w.batch, max_pages).astype(np.int32)
    full = np.full(w.batch, cap)
    def to_dev(x):
        t = torch.from_numpy(x if fp8 else x.view(np.int16)).to(DEV)
        return t if fp8 else t.view(torch.bfloat16)
    def fresh():
        if paged:
            return to_dev(O.dense_to_paged_ref(kd, table, page_rows, n_pages, full)), to_dev(O.dense_to_paged_ref(vd, table, page_rows, n_pages, full))
        return to_dev(kd.copy()), to_dev(vd.copy())
    def to_dense(t):
        x = t.cpu().numpy() if fp8 else I.bits(t)
        return O.paged_to_dense_ref(x, table, full) if paged else x
    shp = rap.shape(w.batch, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    pg = rap.paging(page_rows, n_pages, torch.from_numpy(table).to(DEV)) if paged else None
    for q_is_rotated in (True, False):
        for rps in (0, 256):
            tun = rap.tuning(kernel=MFMA, rows_per_split=rps)
            ws = rap.new_workspace(shp, cap, tun)
            k1, v1 = fresh()
            out1 = torch.full((w.batch, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
            rap.rap_decode_step_ex(shp, k1, v1, ksd, vsd, pg, k_new, v_new, pos, case.keep, case.q, q_is_rotated,
                                   case.seq_lens, cap, out1, float(w.scale), ws, tun)
            k2, v2 = fresh()
            out2 = torch.full_like(out1, float("nan"))
            qp = None if q_is_rotated else pos
            kp = None if q_is_rotated else case.keep
            if fp8 and paged:
                rap.rap_rope_append_paged_q8(shp, pg, 1, k_new, v_new, pos, case.keep, k2, v2, ksd, vsd)
                rap.rap_decode_attn_paged_q8(shp, pg, case.q, qp, kp, k2, v2, ksd, vsd, case.seq_lens, cap, out2, float(w.scale), ws, tun)
            elif fp8:
                rap.rap_rope_append_q8(shp, 1, k_new, v_new, pos, case.keep, k2, v2, ksd, vsd)
                rap.rap_decode_attn_q8(shp, case.q, qp, kp, k2, v2, ksd, vsd, case.seq_lens, cap, out2, float(w.scale), ws, tun)
            elif paged:
                rap.rap_rope_append_paged(shp, pg, 1, k_new, v_new, pos, case.keep, k2, v2)
                rap.rap_decode_attn_paged(shp, pg, case.q, qp, kp, k2, v2, case.seq_lens, cap, out2, float(w.scale), ws, tun)
            else:
                rap.rap_rope_append(shp, 1, k_new, v_new, pos, case.keep, k2, v2)
                if q_is_rotated:
                    rap.rap_decode_attn(shp, case.q, k2, v2, case.seq_lens, cap, out2, float(w.scale), ws, tun)
                else:
                    rap.rap_decode_attn_rope(shp, case.q, pos, case.keep, k2, v2, case.seq_lens, cap, out2, float(w.scale), ws, tun)
            torch.cuda.synchronize()
            assert torch.equal(k1.view(torch.uint8), k2.view(torch.uint8)) and torch.equal(v1.view(torch.uint8), v2.view(torch.uint8)), "caches differ"
            rel = (out1 - out2).abs().max().item() / out2.abs().max().item()
            assert rel <= 2e-5, "step differs from the two calls (rps=%d): %.3g" % (rps, rel)
            gk, gv = to_dense(k1), to_dense(v1)
            qb = I.bits(case.q) if q_is_rotated else O.rope_queries_ref(I.bits(case.q), pos_np, keep_np, w.rope_theta, w.d_head, Hkv)
            ref = O.attn_q8_ref(qb, gk, gv, ks, vs, lens, w.scale) if fp8 else O.attn_ref(qb, gk, gv, lens, w.scale)
            H.assert_attn_close(out1.cpu().numpy(), ref, "step fp8=%s paged=%s rps=%d rotated=%s" % (fp8, paged, rps, q_is_rotated))


@pytest.mark.parametrize("one_call", [False, True])
def test_graph_replay(rap, one_call):
    """A decode loop recorded once into a HIP graph (append + attention, or the one-call step) and
    replayed for four tokens with new inputs in the same buffers: every replay must leave the
    caches and give the outputs of the same calls made directly, and the last one is checked
    against the oracle.  The library launches kernels only (no allocation, no memset, no
    synchronisation), which is what makes it recordable; eager work and synchronisations lie
    between the replays."""
    n_steps = 4
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=8, n_kv_heads=2, n_pairs=45, d_v=90, ctx=1500, n_new=n_steps,
                 ragged_min=600, peaky_frac=0.0, seed=4242)
    _say("graph replay one_call=%s" % one_call)
    case = I.make_case(w, device=DEV)
    shp = H.shape_of(rap, case)
    cap = int(case.cap)
    prefill = torch.from_numpy(np.asarray(case.prefill_lens, dtype=np.int32)).to(DEV)
    qs = [torch.randn((w.batch, w.n_q_heads, w.d_k), generator=torch.Generator().manual_seed(50 + i)).to(torch.bfloat16).to(DEV)
          for i in range(n_steps)]
    ws = rap.new_workspace(shp, cap, None)

    def step(k1, v1, p1, q, kc, vc, sl, out):
        if one_call:
            rap.rap_decode_step(shp, k1, v1, p1, case.keep, q, True, kc, vc, sl, cap, out, float(w.scale), ws, None)
        else:
            rap.rap_rope_append(shp, 1, k1, v1, p1, case.keep, kc, vc)
            rap.rap_decode_attn(shp, q, kc, vc, sl, cap, out, float(w.scale), ws, None)

    def inputs(i):
        return (case.k_new[:, i:i + 1].contiguous(), case.v_new[:, i:i + 1].contiguous(), case.pos[:, i].contiguous(),
                qs[i], (prefill + i + 1).to(torch.int32))

    # the calls made directly
    kc_e, vc_e = case.k_cache.clone(), case.v_cache.clone()
    outs_e, caches_e = [], []
    for i in range(n_steps):
        k1, v1, p1, q, sl = inputs(i)
        out = torch.full((w.batch, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
        step(k1, v1, p1, q, kc_e, vc_e, sl, out)
        torch.cuda.synchronize()
        outs_e.append(out)
        caches_e.append((kc_e.clone(), vc_e.clone()))

    # the same calls recorded once over fixed buffers
    kc_g, vc_g = case.k_cache.clone(), case.v_cache.clone()
    k1_s, v1_s, p1_s, q_s, sl_s = [t.clone() for t in inputs(0)]
    out_s = torch.full((w.batch, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
    step(k1_s, v1_s, p1_s, q_s, kc_g, vc_g, sl_s, out_s)            # warm-up outside the recording (same token: idempotent)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(k1_s, v1_s, p1_s, q_s, kc_g, vc_g, sl_s, out_s)
    for i in range(n_steps):
        for dst, src in zip((k1_s, v1_s, p1_s, q_s, sl_s), inputs(i)):
            dst.copy_(src)
        out_s.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_s, outs_e[i]), "replay %d: output differs from the direct calls" % i
        assert torch.equal(kc_g, caches_e[i][0]) and torch.equal(vc_g, caches_e[i][1]), "replay %d: caches differ" % i
    lens = (np.asarray(case.prefill_lens) + n_steps).astype(np.int64)
    ref = O.attn_ref(I.bits(qs[-1]), I.bits(kc_g), I.bits(vc_g), lens, w.scale)
    H.assert_attn_close(out_s.cpu().numpy(), ref, "last replay against the oracle")


def test_graph_replay_several_tokens(rap):
    """The calls for several new tokens per step (append of the tokens, rap_decode_attn_multi, and
    rap_prefill_attn_split over the same tokens) recorded once into a HIP graph and replayed three
    times with new inputs in the same buffers: every replay gives the bits of the direct calls,
    and the two attention calls agree with each other and, at the end, with the oracle."""
    n_steps, n_tok = 3, 2
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=8, n_kv_heads=2, n_pairs=45, d_v=90, ctx=1500, n_new=n_steps * n_tok,
                 ragged_min=600, peaky_frac=0.0, seed=4343)
    _say("graph replay, two tokens per step")
    case = I.make_case(w, device=DEV)
    shp = H.shape_of(rap, case)
    cap = int(case.cap)
    prefill = torch.from_numpy(np.asarray(case.prefill_lens, dtype=np.int32)).to(DEV)
    qs = [torch.randn((w.batch, n_tok, w.n_q_heads, w.d_k), generator=torch.Generator().manual_seed(60 + i)).to(torch.bfloat16).to(DEV)
          for i in range(n_steps)]
    ws = rap.new_workspace(shp, cap, None, n_tok=n_tok)
    need = rap.rap_prefill_attn_split_workspace_bytes(shp, n_tok, cap)
    assert need > 0
    ws2 = torch.empty(need, dtype=torch.uint8, device=DEV)

    def step(k2, v2, p2, q, kc, vc, sl, out_m, out_p):
        rap.rap_rope_append(shp, n_tok, k2, v2, p2, case.keep, kc, vc)
        rap.rap_decode_attn_multi(shp, kc, vc, None, None, None, n_tok, q, sl, cap, out_m, float(w.scale), ws)
        rap.rap_prefill_attn_split(shp, kc, vc, None, None, None, n_tok, q, sl, cap, out_p, float(w.scale), ws2)

    def inputs(i):
        lo, hi = i * n_tok, (i + 1) * n_tok
        return (case.k_new[:, lo:hi].contiguous(), case.v_new[:, lo:hi].contiguous(), case.pos[:, lo:hi].contiguous(),
                qs[i], (prefill + hi).to(torch.int32))

    def blank():
        return torch.full((w.batch, n_tok, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)

    kc_e, vc_e = case.k_cache.clone(), case.v_cache.clone()
    outs_e = []
    for i in range(n_steps):
        om, op = blank(), blank()
        step(*inputs(i)[:4], kc_e, vc_e, inputs(i)[4], om, op)
        torch.cuda.synchronize()
        outs_e.append((om, op))
        assert (om - op).abs().max().item() <= 2e-5 * max(1.0, op.abs().max().item())

    kc_g, vc_g = case.k_cache.clone(), case.v_cache.clone()
    k_s, v_s, p_s, q_s, sl_s = [t.clone() for t in inputs(0)]
    om_s, op_s = blank(), blank()
    step(k_s, v_s, p_s, q_s, kc_g, vc_g, sl_s, om_s, op_s)          # warm-up outside the recording (same tokens: idempotent)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(k_s, v_s, p_s, q_s, kc_g, vc_g, sl_s, om_s, op_s)
    for i in range(n_steps):
        for dst, src in zip((k_s, v_s, p_s, q_s, sl_s), inputs(i)):
            dst.copy_(src)
        om_s.fill_(float("nan"))
        op_s.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(om_s, outs_e[i][0]), "replay %d: multi-token output differs from the direct call" % i
        assert torch.equal(op_s, outs_e[i][1]), "replay %d: split prefill output differs from the direct call" % i
    assert torch.equal(kc_g, kc_e) and torch.equal(vc_g, vc_e)
    lens = (np.asarray(case.prefill_lens) + n_steps * n_tok).astype(np.int64)
    ref = O.prefill_attn_ref(I.bits(qs[-1]), I.bits(kc_g), I.bits(vc_g), lens, w.scale)
    H.assert_attn_close(om_s.cpu().numpy(), ref, "last replay (multi-token decode) against the oracle")
    H.assert_attn_close(op_s.cpu().numpy(), ref, "last replay (split prefill) against the oracle")


def test_check_inputs(rap):
    """rap_check_inputs: clean inputs leave the flag word at zero; each kind of bad value sets its bit."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=8, n_kv_heads=2, ctx=300, n_new=5, ragged_min=100, seed=77)
    case = I.make_case(w, device=DEV)
    shp = H.shape_of(rap, case)
    cap = int(case.cap)
    def flags_of(pos, keep, sl, msl=cap):
        f = torch.zeros(1, dtype=torch.int32, device=DEV)
        rap.rap_check_inputs(shp, w.n_new, pos, keep, sl, msl, f)
        torch.cuda.synchronize()
        return int(f.item())
    assert flags_of(case.pos, case.keep, case.seq_lens) == 0
    assert flags_of(None, None, None) == 0
    pos = case.pos.clone(); pos[1, 2] = cap
    assert flags_of(pos, case.keep, case.seq_lens) == 1
    pos[1, 2] = -1
    assert flags_of(pos, None, None) == 1
    keep = case.keep.clone(); keep[1, w.n_pairs - 1] = w.d_head // 2
    assert flags_of(case.pos, keep, case.seq_lens) == 2
    keep = case.keep.clone(); keep[0, 3] = keep[0, 2]
    assert flags_of(case.pos, keep, case.seq_lens) == 4
    keep = case.keep.clone(); keep[1, 0] = -5                     # out of range; the row still ascends
    assert flags_of(None, keep, None) == 2
    sl = case.seq_lens.clone(); sl[2] = cap + 1
    assert flags_of(case.pos, case.keep, sl) == 8
    assert flags_of(case.pos, case.keep, case.seq_lens, msl=int(case.seq_lens.max().item()) - 1) == 8
    sl[0] = -1; pos[0, 0] = 2 ** 30
    assert flags_of(pos, case.keep, sl) == 9
    assert rap.rap_check_inputs(shp, w.n_new, case.pos, case.keep, case.seq_lens, cap, None, check=False) == 1


def test_split_invariance(rap):
    """1 range vs many: same result up to fp32 rounding (merge identity on the GPU side)."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=2, ctx=4000, seed=13)
    case = I.make_case(w, device=DEV)
    base = H.run_decode(rap, case, kernel=MFMA, rows_per_split=4096).cpu().numpy()
    for kernel in (VALU, MFMA):
        for rps in (128, 640, 2048, 4096):
            got = H.run_decode(rap, case, kernel=kernel, rows_per_split=rps).cpu().numpy()
            rel = np.abs(got - base).max() / np.abs(base).max()
            assert rel <= 1e-5, (kernel, rps, rel)


# ------------------------------------------------------------------ the five configurations at full size


def _append_then_decode(rap, case, kernels=(MFMA,), sample=None, rng=None):
    """Append the new tokens with librap, check those rows, then decode and compare (all of it, or
    the (b, kv head) slabs in `sample`) with the oracle fed from the cache librap produced."""
    w = case.w
    pos = case.pos.cpu().numpy()
    lens = case.seq_lens.cpu().numpy()
    # rows the append will touch, before (filler) -> oracle result
    H.run_append(rap, case)
    torch.cuda.synchronize()
    slabs = sample if sample is not None else [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    keep = case.keep.cpu().numpy()
    k_new, v_new = I.bits(case.k_new), I.bits(case.v_new)
    worst = 0
    for b, h in slabs:
        rows = pos[b]
        got_k = I.bits(case.k_cache[b, h, rows.tolist()])
        got_v = I.bits(case.v_cache[b, h, rows.tolist()])
        kf = O.bf16_bits_to_f64(k_new[b, :, h])
        want_k = O.f64_to_bf16_bits_rne(O.rope_compact(kf, rows.astype(np.float64), keep[h], w.rope_theta, w.d_head))
        assert np.array_equal(got_v, v_new[b, :, h])
        worst = max(worst, int(H.bf16_ulp_distance(got_k, want_k).max()))
    assert worst <= 1
    outs = {k: H.run_decode(rap, case, kernel=k).cpu().numpy() for k in kernels}
    qb = I.bits(case.q)
    g = w.group
    for b, h in slabs:
        n = int(lens[b])
        kf = O.bf16_bits_to_f64(I.bits(case.k_cache[b, h, :n]))
        vf = O.bf16_bits_to_f64(I.bits(case.v_cache[b, h, :n]))
        ref = O.attn_rows_ref(O.bf16_bits_to_f64(qb[b, h * g:(h + 1) * g]), kf, vf, w.scale)
        for k, out in outs.items():
            H.assert_attn_close(out[b, h * g:(h + 1) * g], ref, "%s b=%d h=%d kernel=%d" % (w.name, b, h, k))
    for out in outs.values():
        assert np.all(np.isfinite(out))
    return outs


def test_cfg1_full(rap):
    _say("cfg1 full")
    case = I.make_case(I.WORKLOADS["cfg1"], device=DEV)
    _append_then_decode(rap, case, kernels=(VALU, MFMA))


def test_cfg2_full(rap):
    _say("cfg2 full")
    case = I.make_case(I.WORKLOADS["cfg2"], device=DEV)
    _append_then_decode(rap, case, kernels=(VALU, MFMA))


def _sampled(w, n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    picks = set()
    while len(picks) < n:
        picks.add((int(rng.integers(w.batch)), int(rng.integers(w.n_kv_heads))))
    return sorted(picks)


def test_cfg3_full(rap):
    """Every output element of cfg3 against the oracle, slab by slab (256 (b, h) slabs of 32768 rows)."""
    _say("cfg3 full")
    _append_then_decode(rap, I.make_case(I.WORKLOADS["cfg3"], device=DEV))


def test_cfg4_full(rap):
    """Every output element of cfg4 (32 slabs of 131072 rows, 32 row ranges each)."""
    _say("cfg4 full")
    _append_then_decode(rap, I.make_case(I.WORKLOADS["cfg4"], device=DEV))


@pytest.mark.parametrize("name", ["cfg5", "cfg5_rho1"])
def test_cfg5_full(rap, name):
    """Every output element of the ragged batch and of its rho = 1 control (512 slabs, lengths 512
    to 65540, cache offsets beyond 2^32 bytes)."""
    _say(name + " full")
    case = I.make_case(I.WORKLOADS[name], device=DEV)
    _append_then_decode(rap, case)
    del case
    torch.cuda.empty_cache()


def test_cfg3_sampled(rap):
    _say("cfg3 sampled")
    w = I.WORKLOADS["cfg3"]
    case = I.make_case(w, device=DEV)
    _append_then_decode(rap, case, sample=_sampled(w, 6, 3) + [(0, 0), (w.batch - 1, w.n_kv_heads - 1)])


@pytest.mark.parametrize("fp8", [False, True])
def test_cfg3_paged_full(rap, fp8):
    """The cfg3 shape in paged pools (pages of 256 rows, shuffled table; pool offsets beyond 2^31
    bytes), bf16 and fp8: the attention over the pools must equal, bit for bit, the attention over
    the same rows in dense caches, which test_cfg3_sampled and test_q8_cache hold to the oracle."""
    _say("cfg3 paged full fp8=%s" % fp8)
    w = I.WORKLOADS["cfg3"]
    case = I.make_case(w, device=DEV)
    page_rows = 256
    B, Hkv = w.batch, w.n_kv_heads
    max_pages = (int(case.cap) + page_rows - 1) // page_rows
    cap = max_pages * page_rows
    n_pages = B * max_pages + 7
    gen = torch.Generator().manual_seed(5)
    table = torch.randperm(n_pages, generator=gen)[:B * max_pages].reshape(B, max_pages).to(torch.int32)
    def dense_of(t, d):      # [B, Hkv, case.cap, d] -> [B, Hkv, cap, d], what lies beyond stays zero
        x = torch.zeros((B, Hkv, cap, d), dtype=t.dtype, device=DEV)
        x[:, :, :t.shape[2]] = t
        return x
    if fp8:
        g = torch.Generator(device=DEV); g.manual_seed(9)
        kd = dense_of(torch.randint(0, 0x78, (B, Hkv, int(case.cap), w.d_k), generator=g, device=DEV, dtype=torch.uint8), w.d_k)
        vd = dense_of(torch.randint(0, 0x78, (B, Hkv, int(case.cap), w.d_v), generator=g, device=DEV, dtype=torch.uint8), w.d_v)
        ks = torch.full((Hkv,), 0.011, dtype=torch.float32, device=DEV); vs = ks.clone()
    else:
        kd, vd = dense_of(case.k_cache, w.d_k), dense_of(case.v_cache, w.d_v)
    del case.k_cache, case.v_cache
    torch.cuda.empty_cache()
    def pool_of(x):          # [B, Hkv, cap, d] -> [n_pages, Hkv, page_rows, d] through the table
        pool = torch.zeros((n_pages, Hkv, page_rows, x.shape[3]), dtype=x.dtype, device=DEV)
        for b in range(B):
            pages = x[b].reshape(Hkv, max_pages, page_rows, x.shape[3]).permute(1, 0, 2, 3)
            pool[table[b].to(DEV).long()] = pages
        return pool
    kp, vp = pool_of(kd), pool_of(vd)
    shp = rap.shape(B, w.n_q_heads, Hkv, w.d_head, w.n_pairs, w.d_v, cap, w.rope_theta)
    pg = rap.paging(page_rows, n_pages, table.to(DEV))
    msl = int(case.seq_lens.max().item())
    ws = rap.new_workspace(shp, msl, None)
    out_d = torch.full((B, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
    out_p = torch.full_like(out_d, float("nan"))
    if fp8:
        rap.rap_decode_attn_q8(shp, case.q, None, None, kd, vd, ks, vs, case.seq_lens, msl, out_d, float(w.scale), ws, None)
        rap.rap_decode_attn_paged_q8(shp, pg, case.q, None, None, kp, vp, ks, vs, case.seq_lens, msl, out_p, float(w.scale), ws, None)
    else:
        rap.rap_decode_attn(shp, case.q, kd, vd, case.seq_lens, msl, out_d, float(w.scale), ws, None)
        rap.rap_decode_attn_paged(shp, pg, case.q, None, None, kp, vp, case.seq_lens, msl, out_p, float(w.scale), ws, None)
    torch.cuda.synchronize()
    assert torch.isfinite(out_d).all()
    assert torch.equal(out_d, out_p), "paged and dense attention differ at full size"
    del kd, vd, kp, vp
    torch.cuda.empty_cache()


def test_cfg4_sampled(rap):
    _say("cfg4 sampled")
    w = I.WORKLOADS["cfg4"]
    case = I.make_case(w, device=DEV)
    _append_then_decode(rap, case, sample=_sampled(w, 4, 4) + [(0, 0), (w.batch - 1, w.n_kv_heads - 1)])


@pytest.mark.parametrize("name", ["cfg5", "cfg5_rho1"])
def test_cfg5_sampled(rap, name):
    _say(name + " sampled")
    w = I.WORKLOADS[name]
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    sample = _sampled(w, 4, 5) + [(shortest, 0), (longest, w.n_kv_heads - 1)]
    outs = _append_then_decode(rap, case, sample=sample)
    del case
    torch.cuda.empty_cache()
