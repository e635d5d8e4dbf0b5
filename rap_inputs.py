"""Seeded synthetic inputs for the RAP decode path.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no rotation, no softmax, no rounding rule of its own beyond
torch's float32 -> bfloat16 cast), so both the HIP path and the CPU checker may
be fed from it.  Tensors are created on the requested torch device, so the big
configurations are drawn directly in HBM and only the slices a test inspects
are copied back to the host.

Workload shapes follow the model families the paper evaluates (Llama-3.x,
Mistral-7B, Qwen2.5-14B head counts, d_head = 128, their RoPE bases) and its
retain-ratio grid; activations are i.i.d. N(0,1) cast to bf16 because no trained
weights or text are available offline.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    rope_theta: float
    n_pairs: int                 # P: kept RoPE pairs, d_k = 2P
    d_v: int
    ctx: int                     # rows attended per sequence (max when ragged)
    n_new: int                   # tokens written through rap_rope_append
    scale: float
    ragged_min: Optional[int] = None   # lengths ~ U{ragged_min..ctx} before the appended tokens
    peaky_frac: float = 0.0      # fraction of K rows per (b, h) multiplied by 8
    seed: int = 0

    @property
    def d_k(self) -> int:
        return 2 * self.n_pairs

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


_S128 = 1.0 / np.sqrt(128.0)

WORKLOADS = {
    # Llama-3.2-3B-shaped, every cache row goes through the append call.
    "cfg1": Workload("cfg1", 1, 24, 8, 128, 5.0e5, 45, 90, 2048, 2048, 1.0 / np.sqrt(90.0), seed=1001),
    # Llama-3.1-8B-shaped, 1 % of K rows x8 (peaky softmax); the headline workload.
    "cfg2": Workload("cfg2", 16, 32, 8, 128, 5.0e5, 45, 90, 8192, 1, _S128, peaky_frac=0.01, seed=1002),
    # Mistral-7B-shaped, d_k != d_v.
    "cfg3": Workload("cfg3", 32, 32, 8, 128, 1.0e6, 58, 115, 32768, 1, _S128, seed=1003),
    # Qwen2.5-14B-shaped, GQA group 5, long context.
    "cfg4": Workload("cfg4", 4, 40, 8, 128, 1.0e6, 32, 64, 131072, 1, _S128, seed=1004),
    # Ragged batch on the 8B shape, 4 appended tokens, and its rho = 1 control.
    "cfg5": Workload("cfg5", 64, 32, 8, 128, 5.0e5, 45, 90, 65536 + 4, 4, _S128, ragged_min=512, seed=1005),
    "cfg5_rho1": Workload("cfg5_rho1", 64, 32, 8, 128, 5.0e5, 64, 128, 65536 + 4, 4, _S128, ragged_min=512, seed=1005),
    # rho = 1 control of the headline workload (same lengths, full head).
    "cfg2_rho1": Workload("cfg2_rho1", 16, 32, 8, 128, 5.0e5, 64, 128, 8192, 1, _S128, peaky_frac=0.01, seed=1002),
    # The headline shape at two other budgets of Tab. (effsweep), rho = 0.8 and 0.6: K rows whose tile takes an odd
    # number of 1 KB loads (used for one traffic-counter run; not part of the default benchmark).
    "cfg2_rho08": Workload("cfg2_rho08", 16, 32, 8, 128, 5.0e5, 51, 102, 8192, 1, _S128, peaky_frac=0.01, seed=1002),
    "cfg2_rho06": Workload("cfg2_rho06", 16, 32, 8, 128, 5.0e5, 38, 77, 8192, 1, _S128, peaky_frac=0.01, seed=1002),
}


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (used for reduced-size test cases)."""
    return replace(w, **kw)


def draw_keep(rng: np.random.Generator, n_heads: int, n_total: int, n_keep: int) -> np.ndarray:
    """Per head: n_keep distinct indices from [0, n_total), uniform without replacement, ascending."""
    out = np.empty((n_heads, n_keep), dtype=np.int32)
    for h in range(n_heads):
        out[h] = np.sort(rng.choice(n_total, size=n_keep, replace=False)).astype(np.int32)
    return out


def round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


@dataclass
class Case:
    w: Workload
    cap: int
    keep: torch.Tensor        # int32 [H_kv, P]   (device)
    keep_v: np.ndarray        # int32 [H_kv, d_v] (host; only the zero-mask identity uses it)
    prefill_lens: np.ndarray  # int64 [B] rows present before the appended tokens
    seq_lens: torch.Tensor    # int32 [B] rows attended (device)
    pos: torch.Tensor         # int32 [B, n_new] (device)
    k_new: torch.Tensor       # bf16 [B, n_new, H_kv, d_k] un-rotated
    v_new: torch.Tensor       # bf16 [B, n_new, H_kv, d_v]
    q: torch.Tensor           # bf16 [B, H_q, d_k] already rotated
    k_cache: torch.Tensor     # bf16 [B, H_kv, cap, d_k]
    v_cache: torch.Tensor     # bf16 [B, H_kv, cap, d_v]
    extra: dict = field(default_factory=dict)


def _randn_bf16(shape, gen: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)


def make_case(w: Workload, device="cpu", fill_unused: bool = True, cap_extra: int = 0) -> Case:
    """Draw every tensor of a workload.

    Cache rows [0, prefill_len_b) hold N(0,1) bf16 values taken as already
    rotated keys (a rotation of an isotropic Gaussian row has the same law).
    Rows from prefill_len_b on are what the append call will write; until then,
    and up to cap, they hold a finite filler (also N(0,1)) when fill_unused is
    set, zeros otherwise.  Order of draws is fixed: lengths, keep, keep_v (NumPy
    PCG64), then K, V per batch element, q, k_new, v_new (torch generator).
    """
    dev = torch.device(device)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    # lengths first, so that they depend on the seed alone (a rho = 1 control with the same seed
    # gets the identical length mix)
    if w.ragged_min is not None:
        hi = w.ctx - w.n_new
        prefill = rng.integers(w.ragged_min, hi + 1, size=w.batch).astype(np.int64)
    else:
        prefill = np.full(w.batch, w.ctx - w.n_new, dtype=np.int64)
    keep = draw_keep(rng, w.n_kv_heads, w.d_head // 2, w.n_pairs)
    keep_v = draw_keep(rng, w.n_kv_heads, w.d_head, w.d_v)
    seq_lens = prefill + w.n_new
    cap = round_up(int(seq_lens.max()) + cap_extra, 8)     # cap_extra: spare rows a serving stack would keep

    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    k_cache = torch.empty((w.batch, w.n_kv_heads, cap, w.d_k), dtype=torch.bfloat16, device=dev)
    v_cache = torch.empty((w.batch, w.n_kv_heads, cap, w.d_v), dtype=torch.bfloat16, device=dev)
    n_peaky = int(np.floor(w.peaky_frac * w.ctx))
    for b in range(w.batch):
        kb = torch.randn((w.n_kv_heads, cap, w.d_k), generator=gen, device=dev, dtype=torch.float32)
        if n_peaky > 0:
            # exactly n_peaky distinct rows per (b, h): the top-n of i.i.d. uniforms
            u = torch.rand((w.n_kv_heads, int(prefill[b])), generator=gen, device=dev)
            rows = torch.topk(u, min(n_peaky, int(prefill[b])), dim=1).indices
            for h in range(w.n_kv_heads):
                kb[h, rows[h]] *= 8.0
        k_cache[b] = kb.to(torch.bfloat16)
        del kb
        v_cache[b] = _randn_bf16((w.n_kv_heads, cap, w.d_v), gen, dev)
    if not fill_unused:
        for b in range(w.batch):
            k_cache[b, :, int(prefill[b]):] = 0
            v_cache[b, :, int(prefill[b]):] = 0
    q = _randn_bf16((w.batch, w.n_q_heads, w.d_k), gen, dev)
    k_new = _randn_bf16((w.batch, w.n_new, w.n_kv_heads, w.d_k), gen, dev)
    v_new = _randn_bf16((w.batch, w.n_new, w.n_kv_heads, w.d_v), gen, dev)
    pos = torch.from_numpy((prefill[:, None] + np.arange(w.n_new)[None, :]).astype(np.int32)).to(dev)
    return Case(
        w=w, cap=cap,
        keep=torch.from_numpy(keep).to(dev), keep_v=keep_v,
        prefill_lens=prefill,
        seq_lens=torch.from_numpy(seq_lens.astype(np.int32)).to(dev),
        pos=pos, k_new=k_new, v_new=v_new, q=q, k_cache=k_cache, v_cache=v_cache,
    )


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> host uint16 bit patterns (same shape)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(a: np.ndarray, device="cpu") -> torch.Tensor:
    """host uint16 bit patterns -> bf16 tensor."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
