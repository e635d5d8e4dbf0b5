"""GPU parity on adversarial score patterns, through every kernel family.

Every attention kernel of librap keeps a per-wavefront softmax reference that it raises, with a
rescale of the running sums and accumulators, only when a score exceeds it by 2^64.  On N(0,1)
inputs that branch runs on a wavefront's first tile and never again, so the cases here are built
to enter it again and again, and to make a wrong rescale visible:

  growing   element 0 of the K rows climbs one level every 24 rows, and the "hot" query rows
            (heads 0, 3, 6, ... of every group) carry a weight on element 0 that turns a level
            into at least 96 log2 units of score: for them every 32-row group of the cache lies
            more than 2^64 above everything before it.  The other query rows have weight 0 there:
            ordinary scores, in the same wavefront, whose sums must survive the hot rows' rescales.
  spike     one huge key late in the last tile of a row range and one two rows before the end.
  equal     all keys identical and |score| of the order of 1e3: the result is the mean of V.

Before anything is compared, the test PROVES from the oracle's float64 scores that the branch is
entered: it counts the 32-row groups (aligned as every kernel here aligns them) whose maximum lies
more than 72 log2 units above every earlier row of a hot query row and which cannot be the first
group a wavefront sees, and asserts that there are some.  Outputs are then held, element by
element, to the oracle at the spec bar (max-abs 1e-2, mean-relative 1e-3).  Scores here
reach several thousand log2 units, where one fp32 rounding of a score (half an ulp of 4096 is
2.4e-4 log2 units) is a relative error of a few 1e-4 in that row's weight, so the everyday
regression bar of the N(0,1) tests does not apply; these cases carry their own, three times what
the kernels measure (max-abs 1.2e-3, mean-relative 2.3e-4 at worst): max-abs 4e-3, mean-relative
7e-4.  What is measured is printed.
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
LOG2E = 1.4426950408889634

# integers with at most four significant bits: exact in bf16 and as E4M3 code values
LEVELS = [n for n in range(449) if n < 16 or n % (1 << (n.bit_length() - 4)) == 0]
STEP_ROWS = 24           # rows per level of the growing pattern
JUMP = 96.0              # log2 units one level is worth to a hot query row, at least
MARGIN = 72.0            # what the host-side proof asks for (the kernels rescale beyond 64)
LENS = [580, 333]


def _say(msg):
    print(msg, flush=True)


def _pow2_at_least(x):
    return 2.0 ** math.ceil(math.log2(x))


def _hot(head, G):
    return (head % G) % 3 == 0


class Edge:
    """One adversarial case: float64 values, their encodings, and the library-side tensors."""

    def __init__(self, rap, pattern, fp8, page_rows, P, dv, Hkv, G, n_tok, seed, lens=LENS, spikes=(254,)):
        self.pattern, self.fp8, self.P, self.dv, self.Hkv, self.G, self.n_tok = pattern, fp8, P, dv, Hkv, G, n_tok
        rng = np.random.Generator(np.random.PCG64(seed))
        self.lens = np.asarray(lens, dtype=np.int64)
        B, dk, Hq = len(lens), 2 * P, G * Hkv
        self.B, self.dk, self.Hq = B, dk, Hq
        unit_rows = page_rows if page_rows else 16
        self.cap = cap = (int(self.lens.max()) + unit_rows - 1) // unit_rows * unit_rows
        self.scale = 1.0 / math.sqrt(dk)
        # fp8: a code stands for (code value) x scale; a power-of-two K scale keeps the levels exact
        self.ks = np.full(Hkv, 2.0 ** -4, dtype=np.float32) if fp8 else None
        self.vs = (rng.uniform(4.0, 6.0, Hkv) / 448.0).astype(np.float32) if fp8 else None
        unit = 2.0 ** -4 if fp8 else 1.0
        k = rng.standard_normal((B, Hkv, cap, dk))
        v = rng.standard_normal((B, Hkv, cap, dv))
        q = rng.standard_normal((B, n_tok, Hq, dk))
        rows = np.arange(cap)
        if pattern == "growing":
            assert int(self.lens.max()) <= STEP_ROWS * 25
            lev = np.asarray(LEVELS, dtype=np.float64)[np.minimum(rows // STEP_ROWS, 24)]
            k[..., 0] = lev * unit
            weight = _pow2_at_least(JUMP / (self.scale * LOG2E * unit))
        elif pattern == "spike":
            k[..., 0] = 0.0
            for b in range(B):
                for r in list(spikes) + [int(self.lens[b]) - n_tok - 2]:
                    if 0 <= r < int(self.lens[b]):
                        k[b, :, r, 0] = 448.0 * unit
            weight = _pow2_at_least(JUMP / (self.scale * LOG2E * 448.0 * unit))
        elif pattern == "equal":
            k[:] = rng.standard_normal((B, Hkv, 1, dk)) * 8.0
            q *= 128.0
            weight = None
        else:
            raise ValueError(pattern)
        if weight is not None:
            for a in range(Hq):
                q[:, :, a, 0] = weight if _hot(a, G) else 0.0
        self.q_bits = O.f64_to_bf16_bits_rne(q)
        self.q = I.from_bits(self.q_bits, DEV)
        self.kd, self.vd, self.kdev, self.vdev, self.ksd, self.vsd, self.pg = H.encode_cache(
            rap, rng, k, v, self.lens, fp8, page_rows, self.ks, self.vs, device=DEV)
        self.sl = torch.from_numpy(self.lens.astype(np.int32)).to(DEV)
        self.shape = rap.shape(B, Hq, Hkv, 128, P, dv, cap, 5.0e5)

    # ---- what the oracle says
    def k_values(self):
        if self.fp8:
            return O.e4m3_bits_to_f64(self.kd) * self.ks.astype(np.float64)[None, :, None, None]
        return O.bf16_bits_to_f64(self.kd)

    def ref_decode(self):
        qb = self.q_bits[:, 0]
        if self.fp8:
            return O.attn_q8_ref(qb, self.kd, self.vd, self.ks, self.vs, self.lens, self.scale)
        return O.attn_ref(qb, self.kd, self.vd, self.lens, self.scale)

    def ref_causal(self):
        if self.fp8:
            return O.prefill_attn_q8_ref(self.q_bits, self.kd, self.vd, self.ks, self.vs, self.lens, self.scale)
        return O.prefill_attn_ref(self.q_bits, self.kd, self.vd, self.lens, self.scale)

    # ---- proof that the rescale branch is entered
    def rescale_events(self, first_groups_of, walk):
        """Number of (hot query row, 32-row group) pairs whose group maximum lies more than MARGIN
        log2 units above EVERY earlier row of that query row, over the groups that cannot be the
        first one a wavefront sees (first_groups_of(n_rows) returns the group indices that may be
        somebody's first).  A wavefront's reference is at most the maximum of the rows it has seen,
        so each such pair forces a rescale, whatever else shares the wavefront.  Scores come from
        the oracle's float64 values.  walk: rows the kernel walks for token t of a sequence of n
        rows: "decode" all n (one token), "multi" n - n_tok (the scan stops in front of the new
        rows, for every token), "causal" n - n_tok + t + 1 (the prefill kernel, up to the token)."""
        kv = self.k_values()
        qv = O.bf16_bits_to_f64(self.q_bits)
        events = 0
        for b in range(self.B):
            n = int(self.lens[b])
            for t in range(self.n_tok):
                scan = {"decode": n, "multi": n - self.n_tok, "causal": n - self.n_tok + t + 1}[walk]
                if scan <= 32:
                    continue
                firsts = first_groups_of(scan)
                for a in range(self.Hq):
                    if not _hot(a, self.G):
                        continue
                    x = (kv[b, a // self.G, :scan] @ qv[b, t, a]) * self.scale * LOG2E
                    run = np.maximum.accumulate(x)
                    for g in range(1, (scan + 31) // 32):
                        if g not in firsts and x[32 * g:min(32 * g + 32, scan)].max() > run[32 * g - 1] + MARGIN:
                            events += 1
        return events


def _decode_first_groups(rps):
    """Groups that are the first tile of one of the four wavefronts of a row range."""
    def f(n_rows):
        out = set()
        for r0 in range(0, n_rows, rps):
            out.update(range(r0 // 32, r0 // 32 + 4))
        return out
    return f


def _prefill_first_groups(split):
    """Unsplit: only group 0 starts a walk.  Cut into key ranges (whole 64-row tiles, boundaries
    unknown to the test): every group that starts a 64-row tile could start a range."""
    def f(n_rows):
        n_groups = (n_rows + 31) // 32
        return {0} if not split else set(range(0, n_groups, 2))
    return f


def _report(what, got, ref):
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    mx, mr = H.attn_errors(got, ref)
    _say("  %s: max-abs %.3g mean-rel %.3g" % (what, mx, mr))
    assert mx <= H.MAX_ABS and mr <= H.MEAN_REL, "%s: max-abs %.3g mean-rel %.3g outside the bar" % (what, mx, mr)
    assert mx <= 4e-3 and mr <= 7e-4, "%s: max-abs %.3g mean-rel %.3g: worse than fp32 scores of this size explain" % (what, mx, mr)


PATTERNS = ["growing", "spike", "equal"]

DECODE_CASES = [
    # name, fp8, page_rows, P, dv, Hkv, G, n_tok
    ("bf16 d116/115 (KCH 4, single V reads)", False, 0, 58, 115, 2, 4, 1),
    ("bf16 d90/90", False, 0, 45, 90, 2, 4, 1),
    ("bf16 d64/64 G5", False, 0, 32, 64, 2, 5, 1),
    ("fp8 d90/90", True, 0, 45, 90, 2, 4, 1),
    ("fp8 d116/115", True, 0, 58, 115, 1, 4, 1),
    ("paged bf16", False, 64, 45, 90, 2, 4, 1),
    ("paged fp8 G5", True, 32, 32, 64, 2, 5, 1),
    ("bf16 G16", False, 0, 64, 128, 1, 16, 1),
    ("multi 4 tokens x G4 = 16 columns", False, 0, 45, 90, 2, 4, 4),
    ("multi fp8 2 tokens x G8", True, 0, 58, 115, 1, 8, 2),
    ("multi paged 3 tokens x G5", False, 128, 32, 64, 1, 5, 3),
]


@pytest.mark.parametrize("pattern", PATTERNS)
@pytest.mark.parametrize("name,fp8,page_rows,P,dv,Hkv,G,n_tok", DECODE_CASES, ids=[c[0] for c in DECODE_CASES])
def test_decode_families(rap, pattern, name, fp8, page_rows, P, dv, Hkv, G, n_tok):
    """The matrix-core decode kernel in every instantiation family (element size, paging, V read
    width, score steps, 16 columns from several tokens or a wide group) and the combining kernel,
    one range and several."""
    _say("softmax edges, decode: %s, %s" % (name, pattern))
    e = Edge(rap, pattern, fp8, page_rows, P, dv, Hkv, G, n_tok, seed=7000 + P + 13 * n_tok + len(pattern))
    ref = e.ref_causal() if n_tok > 1 else e.ref_decode()[:, None]
    for rps in (256, 1024):
        if pattern != "equal":
            ev = e.rescale_events(_decode_first_groups(rps), "multi" if n_tok > 1 else "decode")
            _say("  rows_per_split %d: %d (query row, tile) pairs must rescale" % (rps, ev))
            assert ev > 0, "this case does not reach the rescale branch"
        tun = rap.tuning(rows_per_split=rps)
        gw, ws = H.guarded_workspace(rap, e.shape, e.cap, tun, DEV, n_tok=n_tok)
        go, out = H.guarded_out((e.B, n_tok, e.Hq, dv), DEV)
        rap.rap_decode_attn_multi(e.shape, e.kdev, e.vdev, e.ksd, e.vsd, e.pg, n_tok, e.q, e.sl, e.cap, out, e.scale, ws, tuning=tun)
        torch.cuda.synchronize()
        gw.check(name)
        go.check(name)
        _report("rows_per_split %d" % rps, out.cpu().numpy(), ref)
        if pattern == "equal":
            # identical keys: every visible row weighs the same, the output is the mean of V
            vv = O.e4m3_bits_to_f64(e.vd) * e.vs.astype(np.float64)[None, :, None, None] if fp8 else O.bf16_bits_to_f64(e.vd)
            for b in range(e.B):
                for t in range(n_tok):
                    vis = int(e.lens[b]) - n_tok + t + 1
                    if vis > 0:
                        want = vv[b, :, :vis].mean(axis=1)             # [Hkv, dv]
                        got = out[b, t].cpu().numpy().reshape(Hkv, G, dv)
                        assert np.abs(got - want[:, None, :]).max() <= 1e-5


@pytest.mark.parametrize("pattern", PATTERNS)
@pytest.mark.parametrize("kernel", [1, 2])
def test_decode_entry_point_both_kernels(rap, pattern, kernel):
    """rap_decode_attn itself (dense bf16), vector-ALU kernel and matrix-core kernel."""
    _say("softmax edges, rap_decode_attn kernel %d, %s" % (kernel, pattern))
    e = Edge(rap, pattern, False, 0, 45, 90, 2, 4, 1, seed=7100 + len(pattern))
    ref = e.ref_decode()
    for rps in (256, 1024):
        if pattern != "equal" and kernel == 2:
            assert e.rescale_events(_decode_first_groups(rps), "decode") > 0
        tun = rap.tuning(kernel=kernel, rows_per_split=rps)
        gw, ws = H.guarded_workspace(rap, e.shape, e.cap, tun, DEV)
        go, out = H.guarded_out((e.B, e.Hq, e.dv), DEV)
        rap.rap_decode_attn(e.shape, e.q[:, 0].contiguous(), e.kdev, e.vdev, e.sl, e.cap, out, e.scale, ws, tun)
        torch.cuda.synchronize()
        gw.check("rap_decode_attn")
        go.check("rap_decode_attn")
        _report("kernel %d rows_per_split %d" % (kernel, rps), out.cpu().numpy(), ref)


@pytest.mark.parametrize("pattern", PATTERNS)
@pytest.mark.parametrize("fp8", [False, True])
def test_one_call_step(rap, pattern, fp8):
    """rap_decode_step_ex: the scan leaves the new token's row out (it holds NaN until the token's
    own workgroup writes it) and the combining kernel folds the token in as one more range.  The
    token sits at the end of one sequence and in the MIDDLE of the other, whose old row there is NaN
    as well: a left-out row must not reach the sums through a zero probability."""
    _say("softmax edges, one-call step fp8=%s, %s" % (fp8, pattern))
    P, dv, Hkv, G = 45, 90, 2, 4
    e = Edge(rap, pattern, fp8, 0, P, dv, Hkv, G, 1, seed=7200 + len(pattern))
    rng = np.random.Generator(np.random.PCG64(5))
    pos_np = np.array([int(e.lens[0]) - 1, 100], dtype=np.int32)
    keep = np.sort(rng.choice(64, P, replace=False)).astype(np.int32)[None, :].repeat(Hkv, 0)
    k_new = rng.standard_normal((e.B, 1, Hkv, 2 * P))
    k_new[..., 0] = 0.0
    k_new[..., P] = 0.0                                   # pair 0 stays (0, 0) under any rotation
    v_new = rng.standard_normal((e.B, 1, Hkv, dv))
    kn_bits, vn_bits = O.f64_to_bf16_bits_rne(k_new), O.f64_to_bf16_bits_rne(v_new)
    # the rows the tokens go to hold NaN beforehand
    kd, vd = e.kd.copy(), e.vd.copy()
    for b in range(e.B):
        kd[b, :, pos_np[b]] = 0x7F if fp8 else 0x7FC0
        vd[b, :, pos_np[b]] = 0xFF if fp8 else 0x7FC0
    to_dev = (lambda x: torch.from_numpy(x).to(DEV)) if fp8 else (lambda x: I.from_bits(x, DEV))
    kdev, vdev = to_dev(kd), to_dev(vd)
    kw, vw = kd.copy(), vd.copy()
    if fp8:
        O.append_q8_ref(kn_bits, vn_bits, pos_np[:, None], keep, kw, vw, e.ks, e.vs, 5.0e5, 128)
        ref = O.attn_q8_ref(e.q_bits[:, 0], kw, vw, e.ks, e.vs, e.lens, e.scale)
    else:
        O.append_ref(kn_bits, vn_bits, pos_np[:, None], keep, kw, vw, 5.0e5, 128)
        ref = O.attn_ref(e.q_bits[:, 0], kw, vw, e.lens, e.scale)
    for rps in (256, 1024):
        tun = rap.tuning(rows_per_split=rps)
        gw, ws = H.guarded_workspace(rap, e.shape, e.cap, tun, DEV)
        go, out = H.guarded_out((e.B, e.Hq, dv), DEV)
        kc, vc = kdev.clone(), vdev.clone()
        rap.rap_decode_step_ex(e.shape, kc, vc, e.ksd, e.vsd, None, I.from_bits(kn_bits[:, 0], DEV), I.from_bits(vn_bits[:, 0], DEV),
                               torch.from_numpy(pos_np).to(DEV), torch.from_numpy(keep).to(DEV), e.q[:, 0].contiguous(), True,
                               e.sl, e.cap, out, e.scale, ws, tun)
        torch.cuda.synchronize()
        gw.check("one-call step")
        go.check("one-call step")
        _report("one-call step rows_per_split %d" % rps, out.cpu().numpy(), ref)
        # and the same bits as append followed by attention over the updated cache
        kc2, vc2 = kdev.clone(), vdev.clone()
        two = torch.full_like(out, float("nan"))
        pos_dev, keep_dev = torch.from_numpy(pos_np[:, None].copy()).to(DEV), torch.from_numpy(keep).to(DEV)
        if fp8:
            rap.rap_rope_append_q8(e.shape, 1, I.from_bits(kn_bits, DEV), I.from_bits(vn_bits, DEV), pos_dev, keep_dev, kc2, vc2, e.ksd, e.vsd)
            rap.rap_decode_attn_q8(e.shape, e.q[:, 0].contiguous(), None, None, kc2, vc2, e.ksd, e.vsd, e.sl, e.cap, two, e.scale, ws, tun)
        else:
            rap.rap_rope_append(e.shape, 1, I.from_bits(kn_bits, DEV), I.from_bits(vn_bits, DEV), pos_dev, keep_dev, kc2, vc2)
            rap.rap_decode_attn(e.shape, e.q[:, 0].contiguous(), kc2, vc2, e.sl, e.cap, two, e.scale, ws, tun)
        torch.cuda.synchronize()
        same = lambda x, y: torch.equal(x.view(torch.uint8), y.view(torch.uint8))      # bit patterns: unused rows hold NaN
        assert same(kc, kc2) and same(vc, vc2), "caches differ from the two-call sequence"
        assert (out - two).abs().max().item() <= 2e-5 * max(1.0, two.abs().max().item())


PREFILL_CASES = [
    # name, fp8, page_rows, P, dv, Hkv, G, n_new, split
    ("bf16 d90/90", False, 0, 45, 90, 2, 4, 70, False),
    ("bf16 d116/115 (row sums from a spare channel)", False, 0, 58, 115, 1, 4, 70, False),
    ("bf16 d128/128 (padded LDS rows, three column blocks)", False, 0, 64, 128, 1, 2, 70, False),
    ("bf16 d64/64 G5", False, 0, 32, 64, 1, 5, 70, False),
    ("fp8 d90/90", True, 0, 45, 90, 2, 4, 70, False),
    ("fp8 paged d116/115", True, 64, 58, 115, 1, 4, 70, False),
    ("key ranges bf16", False, 0, 45, 90, 1, 4, 40, True),
    ("key ranges fp8 paged", True, 64, 58, 115, 1, 4, 40, True),
    ("key ranges G16", False, 0, 45, 90, 1, 16, 24, True),
]


@pytest.mark.parametrize("pattern", PATTERNS)
@pytest.mark.parametrize("name,fp8,page_rows,P,dv,Hkv,G,n_new,split", PREFILL_CASES, ids=[c[0] for c in PREFILL_CASES])
def test_prefill_families(rap, pattern, name, fp8, page_rows, P, dv, Hkv, G, n_new, split):
    """The causal prefill kernel (every staging variant, fp8, pools) whole and cut into key ranges."""
    _say("softmax edges, prefill: %s, %s" % (name, pattern))
    e = Edge(rap, pattern, fp8, page_rows, P, dv, Hkv, G, n_new, seed=7300 + P + n_new + len(pattern), spikes=(254, 125))
    ref = e.ref_causal()
    if pattern != "equal":
        ev = e.rescale_events(_prefill_first_groups(split), "causal")
        _say("  %d (query row, key group) pairs must rescale" % ev)
        assert ev > 0, "this case does not reach the rescale branch"
    go, out = H.guarded_out((e.B, n_new, e.Hq, dv), DEV)
    if split:
        need = rap.rap_prefill_attn_split_workspace_bytes(e.shape, n_new, e.cap)
        assert need > 0, "this case was meant to be cut into key ranges"
        gw = H.Guarded(need, DEV)
        rap.rap_prefill_attn_split(e.shape, e.kdev, e.vdev, e.ksd, e.vsd, e.pg, n_new, e.q, e.sl, e.cap, out, e.scale, gw.bytes)
    else:
        gw = None
        rap.rap_prefill_attn_ex(e.shape, e.kdev, e.vdev, e.ksd, e.vsd, e.pg, n_new, e.q, e.sl, e.cap, out, e.scale)
    torch.cuda.synchronize()
    go.check(name)
    if gw is not None:
        gw.check(name)
    _report(name, out.cpu().numpy(), ref)
