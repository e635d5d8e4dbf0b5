"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments before launching anything.  No kernel runs here."""
import ctypes as C
import os
import re

import pytest

import paper_2602_02599_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rap():
    if not os.path.exists(pkg.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return pkg.load()


def test_every_declared_symbol_is_exported(rap):
    text = open(os.path.join(ROOT, "include", "rap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(rap_[a-z_0-9]+)\s*\(", text))
    assert {"rap_rope_append", "rap_decode_attn", "rap_decode_attn_workspace_bytes", "rap_status_str"} <= names
    for n in names:
        assert hasattr(rap.lib, n), n


def test_struct_layout_matches_header():
    assert C.sizeof(pkg.RapShape) == 48
    assert pkg.RapShape.cache_cap.offset == 24 and pkg.RapShape.rope_theta.offset == 32
    assert pkg.RapShape.pair_inv_freq.offset == 40
    assert C.sizeof(pkg.RapTuning) == 32 and pkg.RapTuning.ev_main_start.offset == 16


def test_status_strings(rap):
    assert rap.rap_status_str(0) == "ok"
    assert len({rap.rap_status_str(i) for i in range(7)}) == 7
    assert rap.rap_version() >= 100


def _shape(rap, **kw):
    d = dict(batch=2, n_q_heads=8, n_kv_heads=2, d_head=128, n_pairs=45, d_v=90, cache_cap=512, rope_theta=5e5)
    d.update(kw)
    return rap.shape(**d)


def test_append_rejects_bad_arguments(rap):
    f = lambda shp, n=1: rap.rap_rope_append(shp, n, None, None, None, None, None, None, check=False)
    assert f(_shape(rap)) == 1                                   # null pointers
    assert f(_shape(rap), n=0) == 0                              # nothing to do
    assert f(_shape(rap, batch=0)) == 0
    assert f(_shape(rap, n_q_heads=7)) == 2                      # G not integral
    assert f(_shape(rap, n_pairs=65)) == 2                       # P > D/2
    assert f(_shape(rap, cache_cap=510)) == 2                    # cap % 8
    assert f(_shape(rap, rope_theta=0.0)) == 2
    assert f(_shape(rap, d_head=256, n_pairs=100)) == 3          # consistent but not built
    assert f(_shape(rap, d_v=200)) == 3
    assert f(_shape(rap, n_q_heads=34, n_kv_heads=2)) == 3       # G = 17
    assert f(_shape(rap, n_q_heads=32, n_kv_heads=2)) == 1       # G = 16 is within the limits: stops at the null pointers
    assert f(_shape(rap), n=-1) == 2


def test_decode_rejects_bad_arguments(rap):
    f = lambda shp, msl=512, tun=None: rap.rap_decode_attn(shp, None, None, None, None, msl, None, 0.1, None, tun, check=False)
    assert f(_shape(rap)) == 1
    assert f(_shape(rap), msl=513) == 4                          # beyond capacity
    assert f(_shape(rap), msl=0) == 2
    assert f(_shape(rap, n_q_heads=7)) == 2
    assert f(_shape(rap, batch=0)) == 0
    g = lambda shp: rap.rap_decode_attn_rope(shp, None, None, None, None, None, None, 512, None, 0.1, None, None, check=False)
    assert g(_shape(rap)) == 1 and g(_shape(rap, n_q_heads=7)) == 2 and g(_shape(rap, batch=0)) == 0
    st = lambda shp: rap.rap_decode_step(shp, None, None, None, None, None, True, None, None, None, 512, None, 0.1, None, None, check=False)
    assert st(_shape(rap)) == 1 and st(_shape(rap, cache_cap=510)) == 2 and st(_shape(rap, batch=0)) == 0
    assert rap.rap_decode_attn_workspace_bytes(_shape(rap), 512) > 0
    assert rap.rap_decode_attn_workspace_bytes(_shape(rap), 513) == 0
    assert rap.rap_decode_attn_workspace_bytes(_shape(rap, cache_cap=7), 4) == 0
    assert rap.rap_decode_attn_workspace_bytes(_shape(rap), 512, rap.tuning(rows_per_split=100)) == 0
    # workspace grows with the number of row ranges
    a = rap.rap_decode_attn_workspace_bytes(_shape(rap), 512, rap.tuning(rows_per_split=128))
    b = rap.rap_decode_attn_workspace_bytes(_shape(rap), 512, rap.tuning(rows_per_split=256))
    assert a > b


def test_prefill_and_query_rotation_reject_bad_arguments(rap):
    pf = lambda shp, n=4, msl=512: rap.rap_prefill_attn(shp, n, None, None, None, None, msl, None, 0.1, check=False)
    assert pf(_shape(rap)) == 1
    assert pf(_shape(rap), n=0) == 0 and pf(_shape(rap, batch=0)) == 0
    assert pf(_shape(rap), n=-1) == 2 and pf(_shape(rap), msl=0) == 2
    assert pf(_shape(rap), msl=513) == 4
    assert pf(_shape(rap, n_pairs=65)) == 2
    rq = lambda shp, n=4: rap.rap_rope_queries(shp, n, None, None, None, None, check=False)
    assert rq(_shape(rap)) == 1 and rq(_shape(rap), n=0) == 0 and rq(_shape(rap), n=-2) == 2
    assert rq(_shape(rap, rope_theta=-1.0)) == 2


def test_paging_rejects_bad_arguments(rap):
    def pg(page_rows=128, n_pages=10, max_pages=4, table=0):
        return pkg.RapPaging(page_rows, n_pages, max_pages, 0, table)
    ap = lambda shp, paging: rap.rap_rope_append_paged(shp, paging, 1, None, None, None, None, None, None, check=False)
    dc = lambda shp, paging, tun=None: rap.rap_decode_attn_paged(shp, paging, None, None, None, None, None, None, 512, None,
                                                                  0.1, None, tun, check=False)
    ok_shape = _shape(rap, cache_cap=512)
    for f in (ap, dc):
        assert f(ok_shape, pg(table=0)) == 1                       # no block table
        assert f(ok_shape, pg(page_rows=100, table=1)) == 2        # not a power of two
        assert f(ok_shape, pg(page_rows=16, max_pages=32, table=1)) == 2   # below one tile
        assert f(ok_shape, pg(max_pages=5, table=1)) == 2          # capacity != max_pages * page_rows
        assert f(ok_shape, pg(n_pages=0, table=1)) == 2
        assert f(_shape(rap, cache_cap=512, batch=0), pg(table=1)) == 0
    # a plausible table pointer gets past the paging checks and stops at the next null pointer
    assert ap(ok_shape, pg(table=1)) == 1 and dc(ok_shape, pg(table=1)) == 1


def test_later_entry_points_reject_bad_arguments(rap):
    """fp8, paged fp8, paged prefill, the general step, workspace-free helpers: host-side rejections only."""
    def pg(page_rows=128, n_pages=10, max_pages=4, table=1):
        return pkg.RapPaging(page_rows, n_pages, max_pages, 0, table)
    shp = _shape(rap, cache_cap=512)
    # fp8 append / attention: null scales are null pointers, capacity must be a multiple of 16
    a8 = lambda s: rap.rap_rope_append_q8(s, 1, None, None, None, None, None, None, None, None, check=False)
    d8 = lambda s: rap.rap_decode_attn_q8(s, None, None, None, None, None, None, None, None, 8, None, 0.1, None, None, check=False)
    assert a8(shp) == 1 and d8(shp) == 1
    assert a8(_shape(rap, cache_cap=511)) == 2 and d8(_shape(rap, n_q_heads=7)) == 2
    assert a8(_shape(rap, batch=0)) == 0 and d8(_shape(rap, batch=0)) == 0
    # 4-bit append / attention: everything null is a null pointer, bad shapes are seen first, empty batches are no-ops
    a4 = lambda s: rap.rap_rope_append_mx4(s, 1, None, None, None, None, None, None, None, None, check=False)
    d4 = lambda s, msl=8: rap.rap_decode_attn_mx4(s, None, None, None, None, None, None, msl, None, 0.1, None, None, check=False)
    assert a4(shp) == 1 and d4(shp) == 1
    assert a4(_shape(rap, cache_cap=511)) == 2 and d4(_shape(rap, n_q_heads=7)) == 2
    assert a4(_shape(rap, batch=0)) == 0 and d4(_shape(rap, batch=0)) == 0
    assert d4(shp, msl=513) == 4
    # paged fp8
    ap8 = lambda s, p: rap.rap_rope_append_paged_q8(s, p, 1, None, None, None, None, None, None, None, None, check=False)
    dp8 = lambda s, p: rap.rap_decode_attn_paged_q8(s, p, None, None, None, None, None, None, None, None, 512, None, 0.1, None,
                                                    None, check=False)
    assert ap8(shp, pg(page_rows=100)) == 2 and dp8(shp, pg(page_rows=100)) == 2
    assert ap8(shp, pg(table=0)) == 1 and dp8(shp, pg(table=0)) == 1
    assert ap8(shp, pg()) == 1 and dp8(shp, pg()) == 1           # past the paging checks, stops at a null tensor
    # paged prefill: pages below 64 rows are not supported
    pf = lambda s, p, n=4: rap.rap_prefill_attn_paged(s, p, n, None, None, None, None, 512, None, 0.1, check=False)
    assert pf(shp, pg(page_rows=32, max_pages=16)) == 3
    assert pf(shp, pg(page_rows=64, max_pages=8)) == 1
    assert pf(shp, pg(), n=0) == 0 and pf(shp, pg(max_pages=5)) == 2
    # the general step: a cache descriptor is required, scales come as a pair
    lib = rap.lib
    def step_ex(cache, s=shp, msl=512):
        return lib.rap_decode_step_ex(C.byref(s), cache, None, None, None, None, None, 1, None, msl, None, 0.1, None, 0, None, None)
    assert step_ex(None) == 1
    assert step_ex(C.byref(pkg.binding.RapKvCache(None, None, 1, None, None))) == 1
    assert step_ex(C.byref(pkg.binding.RapKvCache(None, None, None, None, None))) == 1
    assert step_ex(C.byref(pkg.binding.RapKvCache(None, None, None, None, None)), s=_shape(rap, n_pairs=65)) == 2
    assert step_ex(C.byref(pkg.binding.RapKvCache(None, None, None, None, None)), s=_shape(rap, batch=0)) == 0
    assert step_ex(C.byref(pkg.binding.RapKvCache(None, None, None, None, None)), msl=0) == 2
    # the general prefill: descriptor required, scales as a pair, fp8 wants cap % 16, small pages refused
    def pf_ex(cache, s=shp, n=4, msl=512):
        return lib.rap_prefill_attn_ex(C.byref(s), cache, n, None, None, msl, None, 0.1, None)
    KV = pkg.binding.RapKvCache
    assert pf_ex(None) == 1
    assert pf_ex(C.byref(KV(None, None, 1, None, None))) == 1
    assert pf_ex(C.byref(KV(None, None, 1, 1, None)), s=_shape(rap, cache_cap=520)) == 2
    assert pf_ex(C.byref(KV(None, None, None, None, None)), n=0) == 0
    assert pf_ex(C.byref(KV(None, None, None, None, C.pointer(pg(page_rows=32, max_pages=16))))) == 3
    assert pf_ex(C.byref(KV(None, None, None, None, None)), msl=513) == 4
    # several query tokens through the decode kernel: descriptor required, token count positive,
    # at most 16 query rows per KV head (the default shape has 4 query heads per KV head)
    def multi(cache, s=shp, n=2, msl=512):
        return lib.rap_decode_attn_multi(C.byref(s), cache, n, None, None, msl, None, 0.1, None, 0, None, None)
    assert multi(None) == 1
    assert multi(C.byref(KV(None, None, 1, None, None))) == 1
    assert multi(C.byref(KV(None, None, None, None, None)), n=0) == 2
    assert multi(C.byref(KV(None, None, None, None, None)), s=_shape(rap, batch=0)) == 0
    assert multi(C.byref(KV(None, None, None, None, None)), msl=513) == 4
    assert multi(C.byref(KV(None, None, None, None, None))) == 1                  # stops at the null tensors
    # prefill with key ranges: descriptor required; the size query answers 0 for what is not cut or not valid
    def pf_split(cache, s=shp, n=4, msl=512, ws=None, nbytes=0):
        return lib.rap_prefill_attn_split(C.byref(s), cache, n, None, None, msl, None, 0.1, ws, nbytes, None)
    assert pf_split(None) == 1
    assert pf_split(C.byref(KV(None, None, None, None, None)), n=0) == 0
    assert pf_split(C.byref(KV(None, None, None, None, None)), msl=513) == 4
    assert pf_split(C.byref(KV(None, None, None, None, None))) == 1                 # null tensors come first
    assert rap.rap_prefill_attn_split_workspace_bytes(shp, 4, 512) > 0             # 2 x 2 query blocks, 8 tiles: cut
    assert rap.rap_prefill_attn_split_workspace_bytes(shp, 4, 256) == 0            # short context: whole
    assert rap.rap_prefill_attn_split_workspace_bytes(shp, 0, 512) == 0
    assert rap.rap_prefill_attn_split_workspace_bytes(shp, 4, 513) == 0            # beyond the capacity
    assert rap.rap_prefill_attn_split_workspace_bytes(_shape(rap, n_pairs=65), 4, 512) == 0
    # input check and workspace of the attention
    ci = lambda s, flags, n=1, msl=512: lib.rap_check_inputs(C.byref(s), n, None, None, None, msl, flags, None)
    assert ci(shp, None) == 1 and ci(_shape(rap, d_v=0), 1) == 2
    assert ci(shp, 4, n=-1) == 2 and ci(shp, 4, msl=513) == 2 and ci(shp, 2) == 2      # misaligned flag word


def test_prefill_split_plan_from_the_outside(rap):
    """rap_prefill_attn_split_workspace_bytes over a grid of shapes: nothing while the query blocks
    alone give at least 384 workgroups or the context is below 8 tiles of 64 rows, else room for
    two or more ranges of partials (d_v + 2 floats per query row and range)."""
    for batch, hq, hkv, n_pairs, dv in [(1, 32, 8, 45, 90), (2, 8, 2, 58, 115), (16, 32, 8, 64, 128), (3, 5, 1, 3, 5)]:
        group = hq // hkv
        nq = 3 if (2 * n_pairs > 96 or dv > 96) else 4            # column blocks per wavefront at these widths
        tok_per_wg = 64 * nq // group
        for n_new in (1, 16, 100, 512, 5000):
            for max_len in (64, 448, 449, 512, 4096, 65536):
                shp = _shape(rap, batch=batch, n_q_heads=hq, n_kv_heads=hkv, n_pairs=n_pairs, d_v=dv, cache_cap=65536)
                need = rap.rap_prefill_attn_split_workspace_bytes(shp, n_new, max_len)
                blocks = -(-n_new // tok_per_wg) * hkv * batch
                tiles = -(-max_len // 64)
                if blocks >= 384 or tiles < 8:
                    assert need == 0, (batch, hq, n_new, max_len, need)
                    continue
                rows = batch * n_new * hq
                per_range = rows * (dv + 2) * 4
                # at most about 512 workgroups, and no range shorter than four tiles
                most = min(-(-512 // blocks), -(-tiles // 4))
                assert need % 256 == 0 and 2 * per_range <= need <= most * per_range + 1024, (batch, hq, n_new, max_len, need)


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(pkg.RapError):
        pkg.Rap(str(tmp_path / "librap.so"))
