"""Shared by the GPU parity tests: run a drawn case through librap and through the oracle."""
from __future__ import annotations

import numpy as np
import torch

from oracle import rap_oracle as O
from paper_2602_02599_amd import inputs as I

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
    w = case.w
    shp = shape_of(rap, case)
    tun = rap.tuning(kernel=kernel, rows_per_split=rows_per_split)
    msl = int(case.seq_lens.max().item()) if max_seq_len is None else max_seq_len
    msl = max(msl, 1)
    ws = rap.new_workspace(shp, msl, tun, device=case.q.device)
    out = torch.full((w.batch, w.n_q_heads, w.d_v), float("nan"), dtype=torch.float32, device=case.q.device)
    rap.rap_decode_attn(shp, case.q, case.k_cache, case.v_cache, case.seq_lens, msl, out, float(w.scale), ws, tun)
    torch.cuda.synchronize()
    return out


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
