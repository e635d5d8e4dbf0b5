"""4-bit (microscaling FP4) caches on the GPU: rap_rope_append_mx4 and rap_decode_attn_mx4 through the
C ABI against the float64 oracle (oracle/rap_oracle.py: mx4_quantize_rows, append_mx4_ref,
attn_mx4_ref) on the same seeded inputs."""
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
    print("[mx4] " + msg, flush=True)


def _quantised_caches(case, cap, lens_fill):
    """The case's bf16 caches quantised by the oracle; rows at or beyond lens_fill[b] hold 0xFF in
    codes and scale bytes (a scale byte of 255 is NaN)."""
    w = case.w
    kd = O.bf16_bits_to_f64(I.bits(case.k_cache))[:, :, :cap]
    vd = O.bf16_bits_to_f64(I.bits(case.v_cache))[:, :, :cap]
    kc, ks = O.mx4_quantize_rows(kd)
    vc, vs = O.mx4_quantize_rows(vd)
    for b in range(w.batch):
        n0 = int(lens_fill[b])
        kc[b, :, n0:] = 0xFF
        ks[b, :, n0:] = 0xFF
        vc[b, :, n0:] = 0xFF
        vs[b, :, n0:] = 0xFF
    return kc, ks, vc, vs


def _dev(*arrays):
    return [torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in arrays]


@pytest.mark.parametrize("P,dv,Hq,Hkv,ctx,n_new", [(45, 90, 8, 2, 1200, 1), (58, 115, 8, 2, 700, 5), (32, 64, 10, 2, 2500, 40),
                                                   (64, 128, 4, 1, 300, 1), (3, 5, 3, 1, 40, 2), (17, 33, 4, 2, 260, 3)])
def test_mx4_append_and_decode(rap, P, dv, Hq, Hkv, ctx, n_new):
    """The appended code blocks and scale bytes against the oracle's (V: equal; K: scale bytes and
    codes equal up to one code step on a vanishing fraction of the elements, where the last bit of
    the fp64 angle arithmetic moves a value across a rounding boundary, which can also move a
    block's scale when that element is the block's largest), rows not named by pos untouched; then
    attention over the GPU-written cache against the oracle on the same codes, with several range
    sizes and NaN scales beyond the sequences."""
    w = I.scaled(I.WORKLOADS["cfg2"], batch=3, n_q_heads=Hq, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=n_new,
                 ragged_min=max(n_new + 1, ctx // 3), peaky_frac=0.0, seed=900 + P)
    _say("append + decode P=%d dv=%d ctx=%d n_new=%d" % (P, dv, ctx, n_new))
    case = I.make_case(w, device=DEV)
    lens = case.seq_lens.cpu().numpy()
    cap = (int(lens.max()) + 7) // 8 * 8
    kc, ks, vc, vs = _quantised_caches(case, cap, case.prefill_lens)
    kcd, ksd, vcd, vsd = _dev(kc, ks, vc, vs)
    shp = rap.shape(w.batch, Hq, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    rap.rap_rope_append_mx4(shp, n_new, case.k_new, case.v_new, case.pos, case.keep, kcd, ksd, vcd, vsd)
    torch.cuda.synchronize()
    okc, oks, ovc, ovs = kc.copy(), ks.copy(), vc.copy(), vs.copy()
    O.append_mx4_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), case.keep.cpu().numpy(),
                     okc, oks, ovc, ovs, w.rope_theta, w.d_head)
    gkc, gks, gvc, gvs = (t.cpu().numpy() for t in (kcd, ksd, vcd, vsd))
    assert np.array_equal(gvc, ovc) and np.array_equal(gvs, ovs), "V codes or scales differ"
    rows_off = (gks != oks).any(axis=-1)                                  # rows where a block's scale moved
    assert rows_off.sum() <= gks[..., 0].size // 10000 + 1, "%d K rows with another scale" % rows_off.sum()
    same_scale = ~rows_off
    gnib = np.stack([gkc & 0xF, gkc >> 4], axis=-1)[same_scale]
    onib = np.stack([okc & 0xF, okc >> 4], axis=-1)[same_scale]
    diff = gnib != onib
    assert diff.sum() <= gnib.size // 10000 + 1, "%d K codes differ" % diff.sum()
    if diff.any():
        assert np.all(np.abs((gnib[diff] & 7).astype(int) - (onib[diff] & 7).astype(int)) <= 1)     # one code step
    # attention over what the GPU wrote
    ref = O.attn_mx4_ref(I.bits(case.q), gkc, gks, gvc, gvs, lens, w.scale, 2 * P, dv)
    outs = []
    for rps in (0, 128, 512):
        tun = rap.tuning(kernel=MFMA, rows_per_split=rps)
        gw, ws = H.guarded_workspace(rap, shp, cap, tun, device=DEV)
        go, out = H.guarded_out((w.batch, Hq, dv), DEV)
        rap.rap_decode_attn_mx4(shp, case.q, kcd, ksd, vcd, vsd, case.seq_lens, cap, out, float(w.scale), ws, tun)
        torch.cuda.synchronize()
        gw.check("workspace")
        go.check("out")
        H.assert_attn_close(out.cpu().numpy(), ref, "mx4 decode rps=%d" % rps)
        outs.append(out.clone())
    # the same values as a bf16 cache through the bf16 call: the arithmetic after LDS is the same
    kb = I.from_bits(O.f64_to_bf16_bits_rne(np.nan_to_num(O.mx4_dequantize_rows(gkc, gks, 2 * P))), DEV)
    vb = I.from_bits(O.f64_to_bf16_bits_rne(np.nan_to_num(O.mx4_dequantize_rows(gvc, gvs, dv))), DEV)
    tun = rap.tuning(kernel=MFMA, rows_per_split=128)
    ws = rap.new_workspace(shp, cap, tun)
    out16 = torch.full((w.batch, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_decode_attn(shp, case.q, kb, vb, case.seq_lens, cap, out16, float(w.scale), ws, tun)
    torch.cuda.synchronize()
    assert torch.equal(out16.view(torch.int32), outs[1].view(torch.int32)), "differs from the bf16 call on the dequantised cache"
    # refusals
    ws = rap.new_workspace(shp, cap, None)
    out = torch.zeros((w.batch, Hq, dv), dtype=torch.float32, device=DEV)
    assert rap.rap_decode_attn_mx4(shp, case.q, kcd, ksd, vcd, vsd, case.seq_lens, cap, out, float(w.scale), ws,
                                   rap.tuning(kernel=VALU), check=False) == 3
    assert rap.rap_decode_attn_mx4(shp, case.q, kcd, None, vcd, vsd, case.seq_lens, cap, out, float(w.scale), ws, None, check=False) == 1
    assert rap.rap_rope_append_mx4(shp, n_new, case.k_new, case.v_new, case.pos, case.keep, kcd, ksd, vcd, None, check=False) == 1


def test_mx4_append_edges(rap):
    """Positions outside the cache are skipped, far positions rotate correctly, blocks of zeros get
    the scale byte 127, and nothing but the named rows is written."""
    _say("append edges")
    w = I.scaled(I.WORKLOADS["cfg3"], batch=2, n_q_heads=4, n_kv_heads=2, ctx=64, n_new=6, ragged_min=20, seed=931)
    case = I.make_case(w, device=DEV)
    cap = 131080
    P, dv, Hkv = w.n_pairs, w.d_v, w.n_kv_heads
    nbk, nbv = O.mx_blocks(2 * P), O.mx_blocks(dv)
    pos_np = np.array([[0, 131071, 5, -1, cap, 77777], [131079, 3, 2, 1, 65536, 99999]], dtype=np.int32)
    k_new = case.k_new.clone()
    k_new[0, 2, 0, :] = 0                                                 # a K row of zeros
    v_new = case.v_new.clone()
    v_new[1, 1, 1, 32:64] = 0                                             # a V block of zeros
    kcd = torch.full((2, Hkv, cap, 16 * nbk), 0xAB, dtype=torch.uint8, device=DEV)
    ksd = torch.full((2, Hkv, cap, 4), 0xAB, dtype=torch.uint8, device=DEV)
    vcd = torch.full((2, Hkv, cap, 16 * nbv), 0xAB, dtype=torch.uint8, device=DEV)
    vsd = torch.full((2, Hkv, cap, 4), 0xAB, dtype=torch.uint8, device=DEV)
    shp = rap.shape(2, 4, Hkv, w.d_head, P, dv, cap, w.rope_theta)
    rap.rap_rope_append_mx4(shp, 6, k_new, v_new, torch.from_numpy(pos_np).to(DEV), case.keep, kcd, ksd, vcd, vsd)
    torch.cuda.synchronize()
    keep_np = case.keep.cpu().numpy()
    touched = 0
    for b in range(2):
        for n in range(6):
            t = int(pos_np[b, n])
            if t < 0 or t >= cap:
                continue
            touched += 1
            for h in range(Hkv):
                rot = O.rope_compact(O.bf16_bits_to_f64(I.bits(k_new)[b, n, h]), np.float64(t), keep_np[h], w.rope_theta, w.d_head)
                c, s = O.mx4_quantize_rows(rot)
                gc, gs = kcd[b, h, t].cpu().numpy(), ksd[b, h, t].cpu().numpy()
                assert np.array_equal(gs, s), (b, n, h, gs, s)
                nd = np.count_nonzero((gc & 0xF) != (c & 0xF)) + np.count_nonzero((gc >> 4) != (c >> 4))
                assert nd <= 1, (b, n, h, nd)
                c, s = O.mx4_quantize_rows(O.bf16_bits_to_f64(I.bits(v_new)[b, n, h]))
                assert np.array_equal(vcd[b, h, t].cpu().numpy(), c) and np.array_equal(vsd[b, h, t].cpu().numpy(), s)
    assert np.all(ksd[0, 0, 5].cpu().numpy() == 127) and np.all(kcd[0, 0, 5].cpu().numpy() & 0x77 == 0)   # zeros (of either sign): scale 2^0
    assert int(vsd[1, 1, 3, 1]) == 127
    n_rows = int((ksd[..., 0] != 0xAB).sum().item())
    assert n_rows == touched * Hkv, (n_rows, touched)
    assert int((kcd != 0xAB).any(dim=-1).sum().item()) <= touched * Hkv


@pytest.mark.parametrize("pattern", ["growing", "spike"])
def test_mx4_decode_softmax_edges(rap, pattern):
    """Scores that force the lazily raised softmax reference to move (as in test_gpu_softmax_edges)
    through the 4-bit variant of the kernel."""
    _say("softmax edges: " + pattern)
    rng = np.random.Generator(np.random.PCG64(77))
    B, Hq, Hkv, P, dv, n = 2, 8, 2, 45, 90, 1100
    cap = 1104
    k = rng.standard_normal((B, Hkv, cap, 2 * P))
    v = rng.standard_normal((B, Hkv, cap, dv))
    q = rng.standard_normal((B, Hq, 2 * P))
    if pattern == "growing":
        k *= (1.0 + np.arange(cap) / 6.0)[None, None, :, None]          # norms grow along the sequence
        scale = 1.0
    else:
        k[:, :, n - 3] *= 300.0                                           # one huge key late in the last tile
        scale = 0.7
    kc, ks = O.mx4_quantize_rows(k)
    vc, vs = O.mx4_quantize_rows(v)
    lens = np.array([n, n - 37], dtype=np.int32)
    qb = O.f64_to_bf16_bits_rne(q)
    ref = O.attn_mx4_ref(qb, kc, ks, vc, vs, lens, scale, 2 * P, dv)
    kcd, ksd, vcd, vsd = _dev(kc, ks, vc, vs)
    shp = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5.0e5)
    for rps in (0, 256):
        tun = rap.tuning(rows_per_split=rps)
        ws = rap.new_workspace(shp, cap, tun)
        out = torch.full((B, Hq, dv), float("nan"), dtype=torch.float32, device=DEV)
        rap.rap_decode_attn_mx4(shp, I.from_bits(qb, DEV), kcd, ksd, vcd, vsd, torch.from_numpy(lens).to(DEV), cap, out, scale, ws, tun)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.all(np.isfinite(got))
        mx, mr = H.attn_errors(got, ref)
        assert mx <= 4e-3 and mr <= 7e-4, (pattern, rps, mx, mr)


def test_mx4_cfg2_size_sampled(rap):
    """The cfg2 shape (16 x 8192 rows, d = 90) in the configuration the benchmark times: sampled
    (b, h) slabs against the oracle, everything finite."""
    _say("cfg2 shape, sampled slabs")
    w = I.WORKLOADS["cfg2"]
    case = I.make_case(w, device=DEV)
    cap = case.cap
    lens = case.seq_lens.cpu().numpy()
    P, dv = w.n_pairs, w.d_v
    kc = np.empty((w.batch, w.n_kv_heads, cap, 16 * O.mx_blocks(2 * P)), dtype=np.uint8)
    ks = np.empty((w.batch, w.n_kv_heads, cap, 4), dtype=np.uint8)
    vc = np.empty((w.batch, w.n_kv_heads, cap, 16 * O.mx_blocks(dv)), dtype=np.uint8)
    vs = np.empty((w.batch, w.n_kv_heads, cap, 4), dtype=np.uint8)
    kbits, vbits = I.bits(case.k_cache), I.bits(case.v_cache)
    for b in range(w.batch):
        kc[b], ks[b] = O.mx4_quantize_rows(O.bf16_bits_to_f64(kbits[b]))
        vc[b], vs[b] = O.mx4_quantize_rows(O.bf16_bits_to_f64(vbits[b]))
    kcd, ksd, vcd, vsd = _dev(kc, ks, vc, vs)
    shp = rap.shape(w.batch, w.n_q_heads, w.n_kv_heads, w.d_head, P, dv, cap, w.rope_theta)
    msl = int(lens.max())
    ws = rap.new_workspace(shp, msl, None)
    out = torch.full((w.batch, w.n_q_heads, dv), float("nan"), dtype=torch.float32, device=DEV)
    rap.rap_decode_attn_mx4(shp, case.q, kcd, ksd, vcd, vsd, case.seq_lens, msl, out, float(w.scale), ws, None)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    g = w.n_q_heads // w.n_kv_heads
    qf = O.bf16_bits_to_f64(I.bits(case.q))
    for b, h in ((0, 0), (5, 3), (15, 7), (9, 6)):
        n = int(lens[b])
        kf = O.mx4_dequantize_rows(kc[b, h, :n], ks[b, h, :n], 2 * P)
        vf = O.mx4_dequantize_rows(vc[b, h, :n], vs[b, h, :n], dv)
        ref = O.attn_rows_ref(qf[b, h * g:(h + 1) * g], kf, vf, w.scale)
        H.assert_attn_close(got[b, h * g:(h + 1) * g], ref, "cfg2 shape slab (%d, %d)" % (b, h))


def test_mx4_random_shapes(rap):
    """Twelve seeded draws of widths, group size, heads, batch, context and range size: append of
    one to five tokens per sequence, then attention over the GPU-written 4-bit cache against the
    oracle on the same codes."""
    rng = np.random.Generator(np.random.PCG64(4242))
    for it in range(12):
        P = int(rng.integers(1, 65))
        dv = int(rng.integers(1, 129))
        G = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
        Hkv = int(rng.integers(1, 4))
        B = int(rng.integers(1, 4))
        ctx = int(rng.integers(40, 1500))
        n_new = int(rng.integers(1, 6))
        rps = int(rng.choice([0, 128, 256, 512]))
        _say("random %d: P=%d dv=%d G=%d Hkv=%d B=%d ctx=%d n_new=%d rps=%d" % (it, P, dv, G, Hkv, B, ctx, n_new, rps))
        w = I.scaled(I.WORKLOADS["cfg2"], batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, n_pairs=P, d_v=dv, ctx=ctx, n_new=n_new,
                     ragged_min=max(n_new + 1, ctx // 4), peaky_frac=0.0, seed=5000 + it)
        case = I.make_case(w, device=DEV)
        lens = case.seq_lens.cpu().numpy()
        cap = (int(lens.max()) + 7) // 8 * 8
        kc, ks, vc, vs = _quantised_caches(case, cap, case.prefill_lens)
        kcd, ksd, vcd, vsd = _dev(kc, ks, vc, vs)
        shp = rap.shape(B, G * Hkv, Hkv, w.d_head, P, dv, cap, w.rope_theta)
        rap.rap_rope_append_mx4(shp, n_new, case.k_new, case.v_new, case.pos, case.keep, kcd, ksd, vcd, vsd)
        torch.cuda.synchronize()
        gkc, gks, gvc, gvs = (t.cpu().numpy() for t in (kcd, ksd, vcd, vsd))
        ovc, ovs = vc.copy(), vs.copy()
        okc, oks = kc.copy(), ks.copy()
        O.append_mx4_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), case.keep.cpu().numpy(),
                         okc, oks, ovc, ovs, w.rope_theta, w.d_head)
        assert np.array_equal(gvc, ovc) and np.array_equal(gvs, ovs)
        assert (gks != oks).any(axis=-1).sum() <= 1 and (gkc != okc).sum() <= gkc.size // 5000 + 2
        ref = O.attn_mx4_ref(I.bits(case.q), gkc, gks, gvc, gvs, lens, w.scale, 2 * P, dv)
        tun = rap.tuning(rows_per_split=rps)
        gw, ws = H.guarded_workspace(rap, shp, cap, tun, device=DEV)
        go, out = H.guarded_out((B, G * Hkv, dv), DEV)
        rap.rap_decode_attn_mx4(shp, case.q, kcd, ksd, vcd, vsd, case.seq_lens, cap, out, float(w.scale), ws, tun)
        torch.cuda.synchronize()
        gw.check("workspace")
        go.check("out")
        H.assert_attn_close(out.cpu().numpy(), ref, "random mx4 %d" % it)
