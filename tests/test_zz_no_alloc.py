"""rap_decode_attn_static, the entry point that allocates nothing (its split partials live in a
fixed array inside the library's device image), against rap_decode_attn with a caller's workspace:
the same kernels, so the outputs must agree bit for bit, and both must meet the oracle's bar.
Two calls in a row, the second with a smaller input: the array keeps what the first call left."""
import numpy as np
import pytest
import torch

from oracle import rap_oracle as O
import rap_inputs as I
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _one(rap, w, rps):
    case = I.make_case(w, device=DEV)
    shp = H.shape_of(rap, case)
    tun = rap.tuning(rows_per_split=rps)
    msl = int(case.seq_lens.max().item())
    want = H.run_decode(rap, case, rows_per_split=rps)
    go, out = H.guarded_out((w.batch, w.n_q_heads, w.d_v), DEV)
    rap.rap_decode_attn_static(shp, case.q, case.k_cache, case.v_cache, case.seq_lens, msl, out, float(w.scale), tun)
    torch.cuda.synchronize()
    go.check("out of rap_decode_attn_static")
    assert torch.equal(out, want), "static-scratch call differs from the workspace call"
    ref = O.attn_ref(I.bits(case.q), I.bits(case.k_cache), I.bits(case.v_cache), case.seq_lens.cpu().numpy(), w.scale)
    H.assert_attn_close(out.cpu().numpy(), ref, "rap_decode_attn_static")


def test_static_scratch_two_calls_second_smaller(rap):
    print("no-alloc entry point: 3 x 2900 rows in 128-row ranges, then 2 x 700 rows", flush=True)
    big = I.scaled(I.WORKLOADS["cfg2"], batch=3, ctx=2900, ragged_min=900, seed=61)
    small = I.scaled(I.WORKLOADS["cfg3"], batch=2, n_q_heads=8, n_kv_heads=2, ctx=700, ragged_min=300, seed=62)
    _one(rap, big, 128)          # 23 ranges per (b, h): partials of every slot are written
    _one(rap, small, 256)        # fewer, narrower slots over what the first call left behind
    _one(rap, small, 0)          # one range: no scratch used at all


def test_static_scratch_limit_and_errors(rap):
    """A shape whose partials exceed the fixed array is refused before any launch; other argument
    errors are those of rap_decode_attn."""
    q = torch.zeros((64, 32, 90), dtype=torch.bfloat16, device=DEV)
    kc = torch.zeros((8,), dtype=torch.bfloat16, device=DEV)      # never read: the call is refused first
    sl = torch.zeros((64,), dtype=torch.int32, device=DEV)
    out = torch.zeros((64, 32, 90), dtype=torch.float32, device=DEV)
    shp = rap.shape(64, 32, 8, 128, 45, 90, 131072, 5.0e5)
    tun = rap.tuning(rows_per_split=128)                          # 1024 ranges: 64 * 32 * 1025 * 92 * 4 bytes
    assert rap.rap_decode_attn_workspace_bytes(shp, 131072, tun) > (16 << 20)
    assert rap.rap_decode_attn_static(shp, q, kc, kc, sl, 131072, out, 0.1, tun, check=False) == 7
    assert "static" in rap.rap_status_str(7)
    ok = rap.shape(2, 8, 2, 128, 45, 90, 1024, 5.0e5)
    assert rap.rap_decode_attn_static(ok, None, kc, kc, sl, 1024, out, 0.1, check=False) == 1        # null q
    assert rap.rap_decode_attn_static(ok, q, kc, kc, sl, 2048, out, 0.1, check=False) == 4           # beyond capacity
    bad = rap.shape(2, 7, 2, 128, 45, 90, 1024, 5.0e5)
    assert rap.rap_decode_attn_static(bad, q, kc, kc, sl, 1024, out, 0.1, check=False) == 2          # 7 / 2 heads
