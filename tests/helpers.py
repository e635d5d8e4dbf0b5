"""Shared by the GPU parity tests: run a drawn case through librap and through the oracle."""
from __future__ import annotations

import numpy as np
import torch

from oracle import rap_oracle as O
import rap_inputs as I

# spec tolerances for attention outputs (fp32 accumulation against the float64 oracle)
MAX_ABS = 1e-2
MEAN_REL = 1e-3
# what fp32 accumulation actually delivers on these inputs: bf16 products are exact in fp32, a sum
# of n terms in fp32 carries about sqrt(n) * 6e-8 relative error, and a probability keeps 16 bits
# in its bf16 head + remainder (4e-6): a few 1e-6 relative at n = 1e5, with a margin of ten.  A
# regression past this is a bug even if it is still inside the bar above
TIGHT_MAX_ABS = 2e-4
TIGHT_MEAN_REL = 2e-5


def shape_of(rap, case: I.Case):
    w = case.w
    return rap.shape(w.batch, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, case.cap, w.rope_theta)


def run_append(rap, case: I.Case):
    rap.rap_rope_append(shape_of(rap, case), case.w.n_new, case.k_new, case.v_new, case.pos, case.keep,
                        case.k_cache, case.v_cache)


def run_decode(rap, case: I.Case, kernel=0, rows_per_split=0, max_seq_len=None):
    """rap_decode_attn on the case; the output starts as NaN, the workspace holds NaN bit patterns in
    every slot and is exactly as large as the library asks, and guard bands around both must survive."""
    w = case.w
    shp = shape_of(rap, case)
    tun = rap.tuning(kernel=kernel, rows_per_split=rows_per_split)
    msl = int(case.seq_lens.max().item()) if max_seq_len is None else max_seq_len
    msl = max(msl, 1)
    gw, ws = guarded_workspace(rap, shp, msl, tun, device=case.q.device)
    go, out = guarded_out((w.batch, w.n_q_heads, w.d_v), case.q.device)
    rap.rap_decode_attn(shp, case.q, case.k_cache, case.v_cache, case.seq_lens, msl, out, float(w.scale), ws, tun)
    torch.cuda.synchronize()
    gw.check("workspace of rap_decode_attn")
    go.check("out of rap_decode_attn")
    return out.clone()


def oracle_append(case: I.Case, kc_bits: np.ndarray, vc_bits: np.ndarray):
    w = case.w
    O.append_ref(I.bits(case.k_new), I.bits(case.v_new), case.pos.cpu().numpy(), case.keep.cpu().numpy(),
                 kc_bits, vc_bits, w.rope_theta, w.d_head)


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in representable bf16 values (sign-magnitude patterns mapped to a number line)."""
    def line(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(line(a_bits) - line(b_bits))


def attn_errors(got: np.ndarray, ref: np.ndarray):
    diff = np.abs(got.astype(np.float64) - ref)
    return float(diff.max()) if diff.size else 0.0, float(diff.mean() / max(np.abs(ref).mean(), 1e-30)) if diff.size else 0.0


def assert_attn_close(got: np.ndarray, ref: np.ndarray, what=""):
    assert np.all(np.isfinite(got)), "non-finite output " + what
    mx, mr = attn_errors(got, ref)
    assert mx <= MAX_ABS and mr <= MEAN_REL, "%s: max-abs %.3g mean-rel %.3g outside the bar" % (what, mx, mr)
    assert mx <= TIGHT_MAX_ABS and mr <= TIGHT_MEAN_REL, "%s: max-abs %.3g mean-rel %.3g: worse than fp32 accumulation explains" % (what, mx, mr)
    return mx, mr


# ---- buffers with guard bands: what a call must not touch keeps a known byte pattern


class Guarded:
    """`nbytes` of device memory (256-byte aligned, every byte `fill`; 0xFF reads as NaN in fp32 and
    bf16) with a guard band of 0x5A bytes in front of and behind it.  check() asserts that both
    bands still hold their pattern: a kernel that writes outside the buffer it was handed fails it."""
    BAND = 512

    def __init__(self, nbytes: int, device, fill: int = 0xFF):
        self.n = int(nbytes)
        span = (self.n + 255) // 256 * 256
        self.buf = torch.full((self.BAND + span + self.BAND,), 0x5A, dtype=torch.uint8, device=device)
        self.bytes = self.buf[self.BAND:self.BAND + self.n]
        self.bytes.fill_(fill)

    def as_f32(self, shape):
        return self.bytes.view(torch.float32).view(shape)

    def check(self, what=""):
        head, tail = self.buf[:self.BAND], self.buf[self.BAND + self.n:]
        assert bool((head == 0x5A).all()) and bool((tail == 0x5A).all()), "guard band overwritten: " + what


def guarded_out(shape, device):
    n = 4
    for s in shape:
        n *= int(s)
    g = Guarded(n, device)
    return g, g.as_f32(shape)


def guarded_workspace(rap, shp, max_seq_len, tuning=None, device="cuda:0", n_tok=1):
    """Workspace of exactly the size the library asks for, NaN bit patterns in every slot, guard
    bands around it."""
    need = rap.rap_decode_attn_workspace_bytes(shp, max_seq_len, tuning) * n_tok
    assert need > 0
    g = Guarded(need, device)
    return g, g.bytes


# ---- caches of any kind from float64 values (encoding through the oracle's converters)


def encode_cache(rap, rng, k_vals, v_vals, lens_np, fp8, page_rows, k_scale=None, v_scale=None, device="cuda:0"):
    """k_vals [B, H, cap, d_k], v_vals [B, H, cap, d_v] float64 -> the cache the library reads:
    bf16 bit patterns, or E4M3 codes of value / scale (k_scale, v_scale float32 [H]); dense, or
    pools of page_rows rows behind a shuffled block table.  Rows at and beyond lens_np[b] and unused
    pages hold NaN patterns.  Returns (kd, vd, kdev, vdev, ksd, vsd, paging): the dense host arrays
    for the oracle, the device tensors and scale tensors for the library, and the paging object."""
    B, Hkv, cap, _ = k_vals.shape
    if fp8:
        kd = O.f64_to_e4m3_bits(k_vals / k_scale.astype(np.float64)[None, :, None, None])
        vd = O.f64_to_e4m3_bits(v_vals / v_scale.astype(np.float64)[None, :, None, None])
        fill_k, fill_v = 0x7F, 0xFF
        to_dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(device)
        ksd, vsd = torch.from_numpy(k_scale).to(device), torch.from_numpy(v_scale).to(device)
    else:
        kd, vd = O.f64_to_bf16_bits_rne(k_vals), O.f64_to_bf16_bits_rne(v_vals)
        fill_k = fill_v = 0x7FC0
        to_dev = lambda x: I.from_bits(x, device)
        ksd = vsd = None
    for b in range(B):
        kd[b, :, int(lens_np[b]):] = fill_k
        vd[b, :, int(lens_np[b]):] = fill_v
    pg, kdev, vdev = None, to_dev(kd), to_dev(vd)
    if page_rows:
        assert cap % page_rows == 0
        max_pages = cap // page_rows
        n_pages = B * max_pages + 2
        table = rng.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
        kdev = to_dev(O.dense_to_paged_ref(kd, table, page_rows, n_pages, lens_np, fill=fill_k))
        vdev = to_dev(O.dense_to_paged_ref(vd, table, page_rows, n_pages, lens_np, fill=fill_v))
        pg = rap.paging(page_rows, n_pages, torch.from_numpy(table).to(device))
    return kd, vd, kdev, vdev, ksd, vsd, pg
