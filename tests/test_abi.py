"""The C-ABI library loads, exports what include/ta.h declares, and rejects bad
arguments on the host before anything is launched (so these run without a GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2604_11288_amd import binding as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(tb.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return tb.lib()


def test_exports_match_header(L):
    text = open(os.path.join(ROOT, "include", "ta.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ta_[a-z_]+)\s*\(", text))
    assert declared == set(tb.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_strerror_covers_every_status(L):
    seen = set()
    for code in range(0, -8, -1):
        msg = L.ta_strerror(code).decode()
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 8
    assert L.ta_strerror(-99).decode() == "unknown status"
    assert L.ta_last_hip_error() == 0


FAKE = ctypes.c_void_p(0x7f0000001000)      # never dereferenced: validation fails first


def _lay(**kw):
    lay = tb.CLayout()
    lay.layers, lay.batch, lay.hq, lay.hkv, lay.n, lay.window, lay.d = 2, 1, 32, 8, 4096, 32, 128
    st = [8 * 4096 * 128, 8 * 4096 * 128, 4096 * 128, 128]
    qs = [32 * 32 * 128, 32 * 32 * 128, 32 * 128]
    for i in range(4):
        lay.kv_stride[i] = st[i]
    for i in range(3):
        lay.q_stride[i] = qs[i]
    for k, v in kw.items():
        if k in ("kv_stride", "q_stride"):
            for i, x in enumerate(v):
                getattr(lay, k)[i] = x
        else:
            setattr(lay, k, v)
    return lay


def _table():
    ids = np.array([[5, 6, -1, -1], [7, -1, -1, -1]], np.int32)
    lens = np.array([2, 1], np.int32)
    return ids, lens


def test_match_error_paths(L):
    ids, lens = _table()
    cp = tb.Params().c()
    ok_args = lambda: [FAKE, None, 1, 128, ids.ctypes.data, lens.ctypes.data, 2, None, ctypes.byref(cp),
                       FAKE, FAKE, FAKE, None]
    a = ok_args(); a[0] = None
    assert L.ta_match_anchors(*a) == tb.TA_ERR_NULL
    a = ok_args(); a[11] = None
    assert L.ta_match_anchors(*a) == tb.TA_ERR_NULL
    a = ok_args(); a[8] = None
    assert L.ta_match_anchors(*a) == tb.TA_ERR_NULL
    a = ok_args(); a[3] = 0
    assert L.ta_match_anchors(*a) == tb.TA_ERR_SHAPE
    a = ok_args(); a[6] = tb.TA_MAX_TABLE + 1
    assert L.ta_match_anchors(*a) == tb.TA_ERR_SHAPE
    a = ok_args(); a[4] = None
    assert L.ta_match_anchors(*a) == tb.TA_ERR_NULL
    bad_len = np.array([5, 1], np.int32)
    a = ok_args(); a[5] = bad_len.ctypes.data
    assert L.ta_match_anchors(*a) == tb.TA_ERR_SHAPE
    bad_ids = ids.copy(); bad_ids[0, 1] = -3
    a = ok_args(); a[4] = bad_ids.ctypes.data
    assert L.ta_match_anchors(*a) == tb.TA_ERR_SHAPE
    cp_bad = tb.Params(span_L=tb.TA_MAX_SPAN + 1).c()
    a = ok_args(); a[8] = ctypes.byref(cp_bad)
    assert L.ta_match_anchors(*a) == tb.TA_ERR_SHAPE


def test_score_error_paths(L):
    cp = tb.Params().c()
    lay = _lay()
    need = L.ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp))
    # 2 layers * 8 heads units, 8 chunks of 512 keys, 128 padded rows, (m, Z) floats
    assert need == 16 * 8 * 128 * 2 * 4
    ok = lambda lay_=lay, ws=FAKE, nbytes=need: [FAKE, FAKE, ctypes.byref(lay_), None, ctypes.byref(cp),
                                                 FAKE, ws, nbytes, None]
    a = ok(); a[0] = None
    assert L.ta_score(*a) == tb.TA_ERR_NULL
    assert L.ta_score(*ok(ws=None)) == tb.TA_ERR_WORKSPACE
    assert L.ta_score(*ok(nbytes=need - 1)) == tb.TA_ERR_WORKSPACE
    assert L.ta_score(*ok(_lay(d=64))) == tb.TA_ERR_SHAPE
    assert L.ta_score(*ok(_lay(hq=30))) == tb.TA_ERR_SHAPE
    assert L.ta_score(*ok(_lay(window=0))) == tb.TA_ERR_SHAPE
    assert L.ta_score(*ok(_lay(window=5000))) == tb.TA_ERR_SHAPE
    assert L.ta_score(*ok(_lay(window=256), nbytes=1 << 40)) == tb.TA_ERR_SHAPE      # 4*256 rows > TA_MAX_ROWS
    assert L.ta_score(*ok(_lay(kv_stride=[8 * 4096 * 128, 8 * 4096 * 128, 4096 * 128, 132]))) == tb.TA_ERR_ALIGN
    a = ok(); a[1] = ctypes.c_void_p(0x7f0000001008)
    assert L.ta_score(*a) == tb.TA_ERR_ALIGN
    cp0 = tb.Params(alpha=0.0).c()
    assert L.ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp0)) == 0


def test_select_and_compact_error_paths(L):
    cp = tb.Params(n_sink=4, n_recent=4).c()
    sel = lambda K=16, A=FAKE, prm=cp: [A, FAKE, FAKE, FAKE, None, 1, 1, 8, 4096, K, ctypes.byref(prm),
                                        FAKE, FAKE, None]
    assert L.ta_select(*sel(K=0)) == tb.TA_ERR_BUDGET
    assert L.ta_select(*sel(K=7)) == tb.TA_ERR_BUDGET                 # K < n_sink + n_recent
    assert L.ta_select(*sel(A=None)) == tb.TA_ERR_NULL                # alpha != 0 needs A
    a = sel(); a[7] = 0
    assert L.ta_select(*a) == tb.TA_ERR_SHAPE
    a = sel(); a[11] = None
    assert L.ta_select(*a) == tb.TA_ERR_NULL
    odd = tb.Params(n_sink=4, n_recent=4).c()
    odd.margin = 0x7f0000001002                                       # a float array at an odd address
    assert L.ta_select(*sel(prm=odd)) == tb.TA_ERR_ALIGN
    lay = _lay()
    cmp_ = lambda lay_=lay, K=16: [FAKE, FAKE, FAKE, FAKE, ctypes.byref(lay_), K, 0, FAKE, FAKE, None]
    a = cmp_(); a[7] = None
    assert L.ta_compact(*a) == tb.TA_ERR_NULL
    assert L.ta_compact(*cmp_(K=0)) == tb.TA_ERR_SHAPE
    assert L.ta_compact(*cmp_(_lay(d=96))) == tb.TA_ERR_SHAPE
    a = cmp_(); a[0] = ctypes.c_void_p(0x7f0000001004)
    assert L.ta_compact(*a) == tb.TA_ERR_ALIGN
    # outputs that alias an input or each other are refused (distinct addresses pass this check:
    # with the same fake address everywhere the call above got as far as the alias test)
    assert L.ta_compact(*cmp_()) == tb.TA_ERR_SHAPE


def test_evict_validates_every_stage_before_launching(L):
    ids, lens = _table()
    cp = tb.Params().c()
    lay = _lay()
    need = L.ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp))

    def args(K=16, ws=FAKE, nbytes=need, Q=FAKE, prm=cp, E=2):
        return [FAKE, None, ids.ctypes.data, lens.ctypes.data, E, None, Q, FAKE, FAKE,
                ctypes.byref(lay), ctypes.byref(prm), K, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                ws, nbytes, None]
    assert L.ta_evict(*args(K=3)) == tb.TA_ERR_BUDGET
    assert L.ta_evict(*args(ws=None)) == tb.TA_ERR_WORKSPACE
    assert L.ta_evict(*args(Q=None)) == tb.TA_ERR_NULL
    assert L.ta_evict(*args(E=65)) == tb.TA_ERR_SHAPE
    # TA-Fast needs neither Q nor a workspace, but still a sane budget
    cp0 = tb.Params(alpha=0.0).c()
    assert L.ta_evict(*args(K=3, Q=None, ws=None, nbytes=0, prm=cp0)) == tb.TA_ERR_BUDGET


def test_evict_layers_checks_every_table_entry(L):
    ids, lens = _table()
    cp = tb.Params().c()
    lay = _lay()
    need = L.ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp))
    base = 0x7f0000001000

    def table(vals):
        return (ctypes.c_void_p * len(vals))(*vals)

    def lp(layers=2, **kw):
        # distinct fake addresses per array and layer (never dereferenced)
        arrs = {name: [base + 0x100000 * (5 * l + i) for l in range(layers)]
                for i, name in enumerate(("Q", "K", "V", "Kout", "Vout"))}
        for k, v in kw.items():
            arrs[k] = v
        keep = {k: (None if v is None else table(v)) for k, v in arrs.items()}
        c = tb.CLayerPtrs(*[None if keep[k] is None else ctypes.cast(keep[k], ctypes.c_void_p)
                            for k in ("Q", "K", "V", "Kout", "Vout")])
        c._keep = keep
        return c

    def args(p, lay_=lay, prm=cp, K=16, ws=FAKE, nbytes=need):
        return [FAKE, None, ids.ctypes.data, lens.ctypes.data, 2, None, None if p is None else ctypes.byref(p),
                ctypes.byref(lay_), ctypes.byref(prm), K, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws, nbytes, None]
    assert L.ta_evict_layers(*args(None)) == tb.TA_ERR_NULL
    assert L.ta_evict_layers(*args(lp(V=None))) == tb.TA_ERR_NULL                     # a missing array
    assert L.ta_evict_layers(*args(lp(Q=None))) == tb.TA_ERR_NULL                     # alpha != 0 needs queries
    assert L.ta_evict_layers(*args(lp(K=[base, None]))) == tb.TA_ERR_NULL             # a missing entry
    assert L.ta_evict_layers(*args(lp(Vout=[base + 0x10, base + 0x24]))) == tb.TA_ERR_ALIGN
    k_tab = [base + 0x100000, base + 0x200000]
    assert L.ta_evict_layers(*args(lp(K=k_tab, Kout=[base + 0x300000, k_tab[1]]))) == tb.TA_ERR_SHAPE   # output on its input
    big = _lay(layers=97)
    assert L.ta_evict_layers(*args(lp(layers=97), lay_=big)) == tb.TA_ERR_SHAPE       # more layers than a table holds
    # the stages behind the table are validated as in ta_evict
    assert L.ta_evict_layers(*args(lp(), K=3)) == tb.TA_ERR_BUDGET
    assert L.ta_evict_layers(*args(lp(), ws=None)) == tb.TA_ERR_WORKSPACE
    cp0 = tb.Params(alpha=0.0).c()
    assert L.ta_evict_layers(*args(lp(Q=None), prm=cp0, K=3, ws=None, nbytes=0)) == tb.TA_ERR_BUDGET
    # the table itself needs room in the workspace, also when nothing is scored
    assert L.ta_evict_layers(*args(lp(Q=None), prm=cp0, ws=None, nbytes=0)) == tb.TA_ERR_WORKSPACE
    assert L.ta_evict_layers(*args(lp(), nbytes=need)) == tb.TA_ERR_WORKSPACE
    # one page pool per layer
    pg = tb.CPaged()
    pg.page_size, pg.max_pages, pg.num_pages, pg.block_table = 64, 64, 70, 0x7f0000001000
    for i, x in enumerate((0, 64 * 8 * 128, 8 * 128, 128)):
        pg.stride[i] = x

    def pargs(p, pg_=pg, nbytes=need + 4096 + 256):
        a = args(p, nbytes=nbytes)
        return a[:7] + [None if pg_ is None else ctypes.byref(pg_), None] + a[7:]
    assert L.ta_evict_layers_paged(*pargs(lp(), pg_=None)) == tb.TA_ERR_NULL
    assert L.ta_evict_layers_paged(*pargs(None)) == tb.TA_ERR_NULL
    bad = tb.CPaged.from_buffer_copy(pg)
    bad.page_size = 48
    assert L.ta_evict_layers_paged(*pargs(lp(), pg_=bad)) == tb.TA_ERR_SHAPE          # scoring wants multiples of 64
    assert L.ta_evict_layers_paged(*pargs(lp(K=[base, None]))) == tb.TA_ERR_NULL
    assert L.ta_evict_layers_paged(*pargs(lp(), nbytes=need)) == tb.TA_ERR_WORKSPACE


def _decode_state(**kw):
    st = tb.CDecodeState(2, 3, 32, 8, 128, 256, 5000, *([0x7f0000001000] * 11), None)
    for k, v in kw.items():
        setattr(st, k, v)
    return st


def test_decode_error_paths(L):
    ids, lens = _table()
    cp = tb.Params().c()
    st = _decode_state()
    init = lambda st_=st, n=4096, prm=cp: [ctypes.byref(st_), FAKE, None, n, FAKE, None, None, FAKE, FAKE, FAKE, FAKE,
                                            ctypes.byref(prm), None]
    assert L.ta_decode_init(*init(_decode_state(K=0))) == tb.TA_ERR_SHAPE
    assert L.ta_decode_init(*init(_decode_state(K=2048))) == tb.TA_ERR_SHAPE
    assert L.ta_decode_init(*init(_decode_state(d=64))) == tb.TA_ERR_SHAPE
    assert L.ta_decode_init(*init(_decode_state(hq=30))) == tb.TA_ERR_SHAPE
    assert L.ta_decode_init(*init(_decode_state(pos=None))) == tb.TA_ERR_NULL
    assert L.ta_decode_init(*init(_decode_state(stepped=None))) == tb.TA_ERR_NULL
    assert L.ta_decode_init(*init(n=6000)) == tb.TA_ERR_SHAPE                       # prefill longer than cap
    assert L.ta_decode_init(*init(_decode_state(Kc=0x7f0000001008))) == tb.TA_ERR_ALIGN
    a = init(); a[1] = None
    assert L.ta_decode_init(*a) == tb.TA_ERR_NULL
    step = lambda st_=st, q=FAKE, prm=cp, E=2: [ctypes.byref(st_), FAKE, q, FAKE, FAKE, ids.ctypes.data,
                                                 lens.ctypes.data, E, ctypes.byref(prm), None, None]
    assert L.ta_decode_step(*step(q=None)) == tb.TA_ERR_NULL                        # alpha != 0 needs queries
    assert L.ta_decode_step(*step(E=70)) == tb.TA_ERR_SHAPE
    assert L.ta_decode_step(*step(_decode_state(K=6))) == tb.TA_ERR_BUDGET          # K < n_sink + n_recent
    assert L.ta_decode_step(*step(_decode_state(hq=136))) == tb.TA_ERR_SHAPE        # 17 heads per group
    a = step(); a[3] = ctypes.c_void_p(0x7f0000001004)
    assert L.ta_decode_step(*a) == tb.TA_ERR_ALIGN
    a = step(); a[1] = None
    assert L.ta_decode_step(*a) == tb.TA_ERR_NULL
    # slots in a paged pool: the table must hold K + 1 slots per sequence
    def pages(page_size=16, max_pages=17, num_pages=40, table=FAKE, stride=(40 * 16 * 8 * 128, 16 * 8 * 128, 8 * 128, 128)):
        p = tb.CPaged()
        p.page_size, p.max_pages, p.num_pages = page_size, max_pages, num_pages
        p.block_table = table.value if table is not None else None
        for i in range(4):
            p.stride[i] = stride[i]
        return p
    keep = []
    def paged(p):
        keep.append(p)
        return _decode_state(pages=ctypes.addressof(p))
    assert L.ta_decode_step(*step(paged(pages(max_pages=16)))) == tb.TA_ERR_SHAPE   # 256 slots < K + 1
    assert L.ta_decode_step(*step(paged(pages(table=None)))) == tb.TA_ERR_NULL
    assert L.ta_decode_step(*step(paged(pages(page_size=0)))) == tb.TA_ERR_SHAPE
    assert L.ta_decode_step(*step(paged(pages(stride=(0, 16 * 8 * 128, 8 * 128 + 4, 128))))) == tb.TA_ERR_ALIGN
    assert L.ta_decode_step(*step(paged(pages(stride=(0, 16 * 8 * 64, 64, 128))))) == tb.TA_ERR_SHAPE   # rows overlap
    a = init(); a[9] = None                                 # rows in place (no compacted K/V) only with a paged state
    assert L.ta_decode_init(*a) == tb.TA_ERR_NULL


def test_static_scratch_entry_refuses_oversized_layouts_on_the_host(L):
    # 96 layers x 96 sequences x 8 heads x 128 rows x 8 B = 72 MiB of row statistics: beyond the static buffer
    lay = _lay(layers=96, batch=96, n=1024, kv_stride=[96 * 8 * 1024 * 128, 8 * 1024 * 128, 1024 * 128, 128],
               q_stride=[96 * 32 * 32 * 128, 32 * 32 * 128, 32 * 128])
    cp = tb.Params().c()
    assert L.ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp)) > tb.TA_STATIC_SCRATCH_BYTES
    ids, lens = _table()
    args = [FAKE, None, ids.ctypes.data, lens.ctypes.data, 2, None, FAKE, FAKE, FAKE, ctypes.byref(lay), ctypes.byref(cp), 64,
            FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None]
    assert L.ta_evict_static(*args) == tb.TA_ERR_SCRATCH
    assert "scratch" in L.ta_strerror(tb.TA_ERR_SCRATCH).decode()
    args[9] = None
    assert L.ta_evict_static(*args) == tb.TA_ERR_NULL


def test_layer_budgets_host_function_matches_oracle(L):
    from oracle import ta_oracle as ora
    for layers, K, kmin in ((32, 1024, 64), (32, 16, 4), (5, 100, 1), (1, 50, 10), (28, 333, 17), (2, 7, 7)):
        assert np.array_equal(tb.ta_layer_budgets(layers, K, kmin), ora.layer_budgets(layers, K, kmin))
    out = np.zeros(4, np.int32)
    assert L.ta_layer_budgets(4, 10, 11, out.ctypes.data) == tb.TA_ERR_SHAPE       # k_min > K
    assert L.ta_layer_budgets(0, 10, 1, out.ctypes.data) == tb.TA_ERR_SHAPE
    assert L.ta_layer_budgets(4, 10, 1, None) == tb.TA_ERR_NULL


def test_detector_and_embedding_error_paths(L):
    cp = tb.Params().c()
    f32 = ctypes.c_float
    det = lambda h=FAKE, stride=4096, m=128, dm=4096, thr=0.5, scale=1.0: [
        h, stride, FAKE, FAKE, None, 2, 100, dm, m, f32(thr), 0, f32(scale), ctypes.byref(cp), FAKE, FAKE, FAKE, None]
    assert L.ta_detect_anchors(*det(h=None)) == tb.TA_ERR_NULL
    assert L.ta_detect_anchors(*det(m=96)) == tb.TA_ERR_SHAPE                     # hidden width not 32/64/128/256
    assert L.ta_detect_anchors(*det(dm=4080, stride=4080)) == tb.TA_ERR_SHAPE     # d_model not a multiple of 32
    assert L.ta_detect_anchors(*det(stride=4095)) == tb.TA_ERR_SHAPE              # rows overlap
    assert L.ta_detect_anchors(*det(stride=4100)) == tb.TA_ERR_ALIGN              # rows not 16-byte aligned
    assert L.ta_detect_anchors(*det(thr=float("nan"))) == tb.TA_ERR_SHAPE
    assert L.ta_detect_anchors(*det(scale=float("inf"))) == tb.TA_ERR_SHAPE
    assert L.ta_detect_anchors(*det(h=ctypes.c_void_p(0x7f0000001008))) == tb.TA_ERR_ALIGN
    a = det(); a[12] = None
    assert L.ta_detect_anchors(*a) == tb.TA_ERR_NULL
    emb = lambda E=16, dm=4096, tau=0.5, x=FAKE: [x, dm, FAKE, E, None, 1, 1000, dm, f32(tau), FAKE, FAKE, None]
    assert L.ta_embed_anchors(*emb(x=None)) == tb.TA_ERR_NULL
    assert L.ta_embed_anchors(*emb(E=0)) == tb.TA_ERR_SHAPE
    assert L.ta_embed_anchors(*emb(E=257)) == tb.TA_ERR_SHAPE
    assert L.ta_embed_anchors(*emb(dm=48)) == tb.TA_ERR_SHAPE
    assert L.ta_embed_anchors(*emb(tau=float("nan"))) == tb.TA_ERR_SHAPE
    assert L.ta_lookup_anchors(FAKE, None, 1, 100, None, 10, FAKE, None) == tb.TA_ERR_NULL
    assert L.ta_lookup_anchors(FAKE, None, 1, 100, FAKE, 0, FAKE, None) == tb.TA_ERR_SHAPE
    assert L.ta_expand_vouchers(None, None, None, 1, 100, ctypes.byref(cp), FAKE, FAKE, None) == tb.TA_ERR_NULL
    assert L.ta_expand_vouchers(FAKE, None, None, 0, 100, ctypes.byref(cp), FAKE, FAKE, None) == tb.TA_ERR_SHAPE
    cp_bad = tb.Params(pool_k=4).c()
    assert L.ta_expand_vouchers(FAKE, None, None, 1, 100, ctypes.byref(cp_bad), FAKE, FAKE, None) == tb.TA_ERR_SHAPE


def test_lse_and_paged_error_paths(L):
    cp = tb.Params().c()
    lay = _lay()
    lse = lambda lay_=lay, l=FAKE, K=FAKE: [FAKE, K, ctypes.byref(lay_), None, ctypes.byref(cp), l, FAKE, None]
    assert L.ta_score_lse(*lse(l=None)) == tb.TA_ERR_NULL
    assert L.ta_score_lse(*lse(_lay(d=64))) == tb.TA_ERR_SHAPE
    assert L.ta_score_lse(*lse(K=ctypes.c_void_p(0x7f0000001008))) == tb.TA_ERR_ALIGN

    def pg(page_size=64, max_pages=64, num_pages=70, table=FAKE, stride=(70 * 64 * 8 * 128, 64 * 8 * 128, 8 * 128, 128)):
        p = tb.CPaged()
        p.page_size, p.max_pages, p.num_pages = page_size, max_pages, num_pages
        p.block_table = table.value if table is not None else None
        for i in range(4):
            p.stride[i] = stride[i]
        return p
    need = L.ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp))
    sc = lambda p, lay_=lay: [FAKE, FAKE, ctypes.byref(p), ctypes.byref(lay_), None, ctypes.byref(cp), None,
                              FAKE, FAKE, need, None]
    assert L.ta_score_paged(*sc(pg(page_size=48))) == tb.TA_ERR_SHAPE             # not a multiple of 64
    assert L.ta_score_paged(*sc(pg(max_pages=63))) == tb.TA_ERR_SHAPE             # table too short for n = 4096
    assert L.ta_score_paged(*sc(pg(table=None))) == tb.TA_ERR_NULL
    assert L.ta_score_paged(*sc(pg(stride=(0, 64 * 8 * 128, 8 * 128 + 4, 128)))) == tb.TA_ERR_ALIGN
    assert L.ta_score_paged(*sc(pg(num_pages=0))) == tb.TA_ERR_SHAPE
    a = sc(pg()); a[9] = need - 1
    assert L.ta_score_paged(*a) == tb.TA_ERR_WORKSPACE
    cm = lambda p, K=16: [FAKE, FAKE, ctypes.byref(p), FAKE, FAKE, ctypes.byref(lay), K, 0, FAKE, FAKE, None]
    assert L.ta_compact_paged(*cm(pg(page_size=0))) == tb.TA_ERR_SHAPE
    assert L.ta_compact_paged(*cm(pg(page_size=16, max_pages=255))) == tb.TA_ERR_SHAPE
    assert L.ta_compact_paged(*cm(pg(), K=0)) == tb.TA_ERR_SHAPE
    a = cm(pg()); a[8] = None
    assert L.ta_compact_paged(*a) == tb.TA_ERR_NULL
    # compaction into a page pool: the destination table is sized for K slots, the source for n positions
    F2, F3, F4 = (ctypes.c_void_p(FAKE.value + 4096 * i) for i in (1, 2, 3))
    ci = lambda dst, src=None, K=16, Kd=F3: [FAKE, F2, ctypes.byref(src) if src is not None else None, FAKE, FAKE,
                                                ctypes.byref(lay), K, 0, Kd, F4, ctypes.byref(dst) if dst is not None else None, None]
    assert L.ta_compact_into_pages(*ci(None)) == tb.TA_ERR_NULL
    assert L.ta_compact_into_pages(*ci(pg(page_size=16, max_pages=1), K=17)) == tb.TA_ERR_SHAPE
    assert L.ta_compact_into_pages(*ci(pg(page_size=16, max_pages=1), src=pg(page_size=16, max_pages=255))) == tb.TA_ERR_SHAPE
    assert L.ta_compact_into_pages(*ci(pg(table=None))) == tb.TA_ERR_NULL
    assert L.ta_compact_into_pages(*ci(pg(), K=0)) == tb.TA_ERR_SHAPE
    assert L.ta_compact_into_pages(*ci(pg(), Kd=None)) == tb.TA_ERR_NULL
    assert L.ta_compact_into_pages(*ci(pg(), Kd=FAKE)) == tb.TA_ERR_SHAPE          # dense source: outputs alias the inputs
    # ta_evict_lse: needs an attention term and the log-sum-exps
    ids, lens = _table()
    cp0 = tb.Params(alpha=0.0).c()
    ev = lambda prm, l=FAKE: [FAKE, None, ids.ctypes.data, lens.ctypes.data, 2, None, FAKE, FAKE, FAKE, l,
                              ctypes.byref(lay), ctypes.byref(prm), 16, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None]
    assert L.ta_evict_lse(*ev(cp0)) == tb.TA_ERR_SHAPE
    assert L.ta_evict_lse(*ev(cp, l=None)) == tb.TA_ERR_NULL


def test_decode_rejects_one_shot_options(L):
    st = tb.CDecodeState()
    st.layers, st.batch, st.hq, st.hkv, st.d, st.K, st.cap = 1, 1, 8, 2, 128, 16, 64
    for name in ("tok", "len", "anchor", "budget", "vouch", "spons", "Kc", "Vc", "pos", "A", "stepped"):
        setattr(st, name, FAKE.value)
    ids, lens = _table()
    call = lambda prm: L.ta_decode_step(ctypes.byref(st), FAKE, FAKE, FAKE, FAKE, ids.ctypes.data, lens.ctypes.data, 2,
                                        ctypes.byref(prm), None, None)
    assert call(tb.Params(n_sink=4, n_recent=4, pool_k=5).c()) == tb.TA_ERR_SHAPE
    assert call(tb.Params(n_sink=4, n_recent=4, k_protected=4).c()) == tb.TA_ERR_SHAPE
    assert call(tb.Params(n_sink=10, n_recent=10).c()) == tb.TA_ERR_BUDGET
    bad = tb.Params(n_sink=4, n_recent=4).c()
    bad.last_query = 2                                     # a flag: 0 or 1
    assert call(bad) == tb.TA_ERR_SHAPE


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
