"""GPU parity: every step of the HIP path, called through the C ABI, against the
CPU oracle on the same seeded inputs.

Bars: anchors, sponsor masks, vouchers, selected indices (given the same A) and
compacted K/V are bit-exact; fp32 scores are within 1e-3 relative (+1e-7
absolute for vanishing weights); indices selected from the GPU's own A may
differ from the oracle's only at ties within 1e-3 of the K-th utility, and those
are counted.
"""
import numpy as np
import pytest
import torch

import paper_2604_11288_amd as ta
from oracle import ta_oracle as ora
from paper_2604_11288_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SCORE_RTOL, SCORE_ATOL = 1e-3, 1e-7


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def _prm(w, **kw):
    base = dict(n_sink=w.n_sink, n_recent=w.n_recent, span_L=w.span_L, sponsor_B=w.sponsor_B,
                rho=w.rho, alpha=w.alpha, beta=w.beta, gamma=w.gamma)
    base.update(kw)
    return ta.Params(**base)


def _oracle_seq(td, b, L=6, B=15.0, rho=0.8, anchor_B=None):
    nb = int(td.seq_len[b])
    ab = None if anchor_B is None else anchor_B[b, :nb]
    return ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len, L=L, B=B, rho=rho, anchor_B=ab)


def _score_close(a_gpu, a_ref):
    return np.all(np.abs(a_gpu.astype(np.float64) - a_ref) <= SCORE_RTOL * np.abs(a_ref) + SCORE_ATOL)


# --------------------------------------------------------------------------
# steps 1+2
# --------------------------------------------------------------------------
@pytest.mark.parametrize("n,batch,clean,ragged,L", [
    (4096, 2, True, None, 6),          # vector stores, 4 tiles
    (3001, 3, False, None, 6),         # scalar tail, dirty filler (accidental 1-gram hits, overlaps)
    (5000, 4, False, (100, 5000), 6),  # ragged lengths
    (2048, 2, False, None, 64),        # longest span
    (2048, 2, True, None, 0),          # no span at all
    (7, 2, True, None, 6),             # shorter than a tile, nothing planted
])
def test_match_expand_bit_exact(n, batch, clean, ragged, L):
    w = wl.scaled(wl.CONFIGS["c4_long_context"], n=n, batch=batch, planted=6 if n > 1000 else 0,
                  ragged=ragged, span_L=L if L > 0 else 6)
    td = wl.make_tokens(w, clean=clean)
    prm = _prm(w, span_L=L)
    seq = _dev(td.seq_len) if ragged else None
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm, seq_len=seq)
    torch.cuda.synchronize()
    anchor, spons, vouch = anchor.cpu().numpy(), spons.cpu().numpy(), vouch.cpu().numpy()
    total = 0
    for b in range(batch):
        nb = int(td.seq_len[b])
        a, s, v = _oracle_seq(td, b, L=L)
        assert np.array_equal(anchor[b, :nb], a)
        assert np.array_equal(spons[b, :nb], s)
        assert np.array_equal(vouch[b, :nb].view(np.uint32), v.view(np.uint32))
        assert not anchor[b, nb:].any() and not spons[b, nb:].any() and not vouch[b, nb:].any()
        total += int(a.sum())
    if n > 1000:
        assert total >= batch * 6 - 6


@pytest.mark.parametrize("batch,n,ragged", [
    (16, 1 << 20, False),       # 16 384 tiles: two consecutive tiles per workgroup
    (64, (1 << 20) + 4, True),  # 65 600 tiles: eight per workgroup, ragged ends inside and between tiles
])
def test_match_many_tiles_per_workgroup(batch, n, ragged):
    """Long streams: a workgroup walks through several consecutive tiles (filter built once, the next
    tile's tokens requested ahead).  Unrestricted token IDs over a small vocabulary, so that anchors,
    overlapping spans and matches across tile borders are frequent; sampled sequences go through the oracle."""
    g = torch.Generator(device=DEV).manual_seed(91 + batch)
    tok = torch.randint(0, 200, (batch, n), dtype=torch.int32, device=DEV, generator=g)
    rng = np.random.default_rng(batch)
    tab_len = rng.integers(1, 5, size=24).astype(np.int32)
    tab_ids = np.full((24, 4), -1, np.int32)
    for e in range(24):
        tab_ids[e, :tab_len[e]] = rng.integers(0, 200, size=tab_len[e])
    tab_len[0] = 1                                           # one 1-gram: about n / 200 hits of it alone
    tab_ids[0] = [7, -1, -1, -1]
    lens = np.full(batch, n, np.int32)
    if ragged:
        lens = rng.integers(n // 2, n + 1, size=batch).astype(np.int32)
        lens[0], lens[1], lens[2] = n, 5 * 1024, 5 * 1024 + 1
    prm = ta.Params(n_sink=4, n_recent=4)
    anchor, spons, vouch = ta.ta_match_anchors(tok, tab_ids, tab_len, prm, seq_len=_dev(lens) if ragged else None)
    torch.cuda.synchronize()
    for b in sorted({0, 1, 2, batch // 2, batch - 1}):
        nb = int(lens[b])
        a, s_, v = ora.evict_sequence(tok[b, :nb].cpu().numpy(), tab_ids, tab_len)
        assert a.sum() > nb // 400
        assert np.array_equal(anchor[b, :nb].cpu().numpy(), a), b
        assert np.array_equal(spons[b, :nb].cpu().numpy(), s_), b
        assert np.array_equal(vouch[b, :nb].cpu().numpy().view(np.uint32), v.view(np.uint32)), b
        assert not bool(anchor[b, nb:].any()) and not bool(spons[b, nb:].any()) and not bool(vouch[b, nb:].any())


def test_match_per_anchor_budget_and_empty_table():
    w = wl.scaled(wl.CONFIGS["c2_full_model"], n=2500, batch=2)
    td = wl.make_tokens(w, clean=False)
    rng = np.random.default_rng(1)
    ab = rng.random((w.batch, w.n)).astype(np.float32)            # confidence-like budgets in [0,1)
    prm = _prm(w)
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm, anchor_B=_dev(ab))
    for b in range(w.batch):
        a, s, v = _oracle_seq(td, b, anchor_B=ab)
        assert np.array_equal(anchor[b].cpu().numpy(), a)
        assert np.array_equal(spons[b].cpu().numpy(), s)
        assert np.array_equal(vouch[b].cpu().numpy().view(np.uint32), v.view(np.uint32))
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), np.zeros((0, 4), np.int32),
                                               np.zeros(0, np.int32), prm)
    assert not anchor.any() and not spons.any() and not vouch.any()


@pytest.mark.parametrize("L", [6, 64])
def test_match_nested_table_on_a_tiny_vocabulary(L):
    """Entries that share their last token (a 1-gram inside a 2-gram inside a 3-gram), a full
    64-entry table and a 10-symbol vocabulary: every tile is dense with overlapping, nested and
    tile-straddling matches, and spans of neighbouring anchors pile up."""
    rng = np.random.default_rng(7)
    rows = [[5], [7, 5], [9, 7, 5], [1, 2, 3, 4], [4], [2, 2], [2, 2, 2, 2], [0, 0, 0]]
    while len(rows) < 64:                                   # fill up with random 4-grams (rarely matched)
        rows.append(rng.integers(0, 10, size=4).tolist())
    tab = np.full((64, 4), -1, np.int32)
    lens = np.zeros(64, np.int32)
    for e, r in enumerate(rows):
        tab[e, :len(r)] = r
        lens[e] = len(r)
    n, batch = 5000, 3
    tok = rng.integers(0, 10, size=(batch, n)).astype(np.int32)
    seq_len = np.array([5000, 2049, 3], np.int32)           # one sequence shorter than the longest n-gram
    w = wl.scaled(wl.CONFIGS["c2_full_model"], n=n, batch=batch, span_L=L)
    prm = _prm(w, span_L=L)
    anchor, spons, vouch = ta.ta_match_anchors(_dev(tok), tab, lens, prm, seq_len=_dev(seq_len))
    torch.cuda.synchronize()
    hits = 0
    for b in range(batch):
        nb = int(seq_len[b])
        a, s, v = ora.evict_sequence(tok[b, :nb], tab, lens, L=L)
        assert np.array_equal(anchor[b, :nb].cpu().numpy(), a)
        assert np.array_equal(spons[b, :nb].cpu().numpy(), s)
        assert np.array_equal(vouch[b, :nb].cpu().numpy().view(np.uint32), v.view(np.uint32))
        assert not anchor[b, nb:].any() and not vouch[b, nb:].any()
        hits += int(a.sum())
    assert hits > 1000                                       # roughly one position in five is an anchor


# --------------------------------------------------------------------------
# step 3
# --------------------------------------------------------------------------
def _check_score(w, causal=True, seq_len=None, units=None, scale=1.0):
    Q, K, _ = wl.make_qkv(w, device=DEV, with_v=False)
    if scale != 1.0:
        Q = (Q.float() * scale).to(torch.bfloat16)
    prm = _prm(w, causal=causal)
    seq = None if seq_len is None else _dev(np.asarray(seq_len, np.int32))
    A = ta.ta_score(Q, K, prm, seq_len=seq)
    torch.cuda.synchronize()
    G = w.hq // w.hkv
    all_units = [(l, b, g) for l in range(w.layers) for b in range(w.batch) for g in range(w.hkv)]
    worst = 0.0
    for (l, b, g) in (units or all_units):
        nb = w.n if seq_len is None else int(seq_len[b])
        a_gpu = A[l, b, g].cpu().numpy()
        assert not a_gpu[nb:].any()
        if nb == 0:
            continue
        a_ref = ora.score(wl.bf16_bits(Q[l, b, g * G:(g + 1) * G]), wl.bf16_bits(K[l, b, g, :nb]), causal)
        assert _score_close(a_gpu[:nb], a_ref), (l, b, g)
        live = min(w.window, nb) if causal else w.window
        assert a_gpu.sum(dtype=np.float64) == pytest.approx(G * live, rel=1e-4)   # softmax rows sum to 1
        worst = max(worst, float(np.max(np.abs(a_gpu[:nb] - a_ref) / (np.abs(a_ref) + 1e-7))))
    return worst


def test_score_c1_shape():
    w = wl.CONFIGS["c1_single_layer"]
    _check_score(w, units=[(0, 0, 0), (0, 0, 5), (0, 0, 7)])


@pytest.mark.parametrize("n,hq,hkv,window,causal", [
    (1000, 8, 2, 32, True),       # ragged last stage (n not a multiple of 64), 2 chunks
    (1000, 8, 2, 32, False),      # no mask
    (700, 6, 2, 5, True),         # 15 rows: padded row tile, rows of one tile span several heads
    (1500, 8, 2, 64, True),       # 256 rows: two row tiles per wavefront
    (600, 16, 2, 64, True),       # 512 rows: two passes of 256 rows over each chunk
    (2500, 10, 2, 64, True),      # 320 rows: the second pass has 64 live rows; two chunks
    (64, 4, 1, 64, True),         # window as long as the context
    (33, 4, 4, 1, True),          # one query row per head
    (8192, 4, 1, 32, True),       # 128 rows, 4 chunks of 2048 keys
    (8300, 4, 1, 32, True),       # ragged last chunk and last stage
    (4096, 4, 1, 32, False),      # no mask at the headline context length
])
def test_score_shapes(n, hq, hkv, window, causal):
    w = wl.scaled(wl.CONFIGS["c1_single_layer"], layers=2, batch=2, n=n, hq=hq, hkv=hkv, window=window)
    _check_score(w, causal=causal)


def test_score_ragged_lengths_and_large_logits():
    w = wl.scaled(wl.CONFIGS["c1_single_layer"], layers=1, batch=4, n=900, hq=8, hkv=2, window=16)
    _check_score(w, seq_len=[900, 517, 16, 5])          # 5 < W: some window rows see nothing
    _check_score(w, scale=12.0)                         # sharp softmax: max subtraction must hold


def test_score_chunks_past_the_sequence_end():
    # chunks and stages that lie wholly past a sequence's end contribute empty statistics and zero
    # scores; an empty sequence has only such chunks
    w = wl.scaled(wl.CONFIGS["c1_single_layer"], layers=2, batch=4, n=2000, hq=8, hkv=2, window=32)
    _check_score(w, seq_len=[2000, 130, 0, 1025])


def test_score_long_context_chunking():
    # 40000 keys: chunks of 2048 keys, 20 chunks whose statistics are merged
    w = wl.scaled(wl.CONFIGS["c4_long_context"], layers=1, batch=1, n=40000, hq=4, hkv=1, window=64)
    _check_score(w)


# --------------------------------------------------------------------------
# step 4
# --------------------------------------------------------------------------
def _select_case(n, K, ns, nr, alpha, A, td, b=0, seq_len=None, beta=0.5, gamma=0.3, L=6):
    """Returns (gpu idx, oracle idx) for one unit with the SAME A on both sides."""
    nb = n if seq_len is None else int(seq_len[b])
    a, s, v = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len, L=L)
    A_nb = None if A is None else A[:nb]
    return ora.select(A_nb, a, s, v, K, ns, nr, alpha=alpha, beta=beta, gamma=gamma)


@pytest.mark.parametrize("n,K,ns,nr,planted,mode", [
    (4096, 16, 4, 4, 4, "uniform"),      # pool overflow: 24 sponsored > 8 protected slots
    (4096, 64, 4, 4, 8, "uniform"),
    (4096, 1024, 4, 4, 8, "ties"),       # coarse A: thousands of exact ties broken by position
    (4096, 256, 4, 4, 8, "zeros"),       # A == 0 everywhere: recency decides
    (5000, 300, 0, 0, 8, "uniform"),     # no mandatory class
    (1000, 2000, 4, 4, 4, "uniform"),    # K >= n: keep everything
    (40000, 1024, 4, 128, 60, "uniform"),  # keys do not fit LDS: recomputed per pass
    (33000, 512, 4, 64, 32, "ties"),
])
def test_select_bit_exact_given_same_scores(n, K, ns, nr, planted, mode):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], n=n, batch=2, planted=planted, n_sink=ns, n_recent=nr)
    td = wl.make_tokens(w, clean=False)
    rng = np.random.default_rng(n + K)
    layers, hkv = 2, 3
    if mode == "uniform":
        A = (rng.random((layers, w.batch, hkv, n)) * 4).astype(np.float32)
    elif mode == "ties":
        A = np.round(rng.random((layers, w.batch, hkv, n)) * 4, 1).astype(np.float32)
    else:
        A = np.zeros((layers, w.batch, hkv, n), np.float32)
    margin = torch.full((layers, w.batch, hkv, 2), 123.0, device=DEV)
    prm = _prm(w, n_sink=ns, n_recent=nr, margin=margin)
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm)
    idx, cnt = ta.ta_select(_dev(A), anchor, spons, vouch, K, prm, layers, hkv)
    torch.cuda.synchronize()
    idx, cnt, margin = idx.cpu().numpy(), cnt.cpu().numpy(), margin.cpu().numpy()
    for l in range(layers):
        for b in range(w.batch):
            a, s, v = ora.evict_sequence(td.tok[b], td.tab_ids, td.tab_len)
            for h in range(hkv):
                ref = _select_case(n, K, ns, nr, 1.0, A[l, b, h], td, b=b)
                assert cnt[l, b, h] == len(ref) == min(K, n)
                assert np.array_equal(idx[l, b, h, :len(ref)], ref), (l, b, h)
                want = ora.select_margin(A[l, b, h], a, s, v, K, ns, nr)
                assert margin[l, b, h].tolist() == want.tolist(), (l, b, h, margin[l, b, h], want)


def test_select_ta_fast_ragged_shared():
    w = wl.scaled(wl.CONFIGS["c3_ta_fast"], n=6000, batch=5, planted=12, ragged=(300, 6000))
    td = wl.make_tokens(w)
    prm = _prm(w)
    seq = _dev(td.seq_len)
    K = 512
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm, seq_len=seq)
    prm.margin = torch.full((w.batch, 2), 123.0, device=DEV)
    idx, cnt = ta.ta_select(None, anchor, spons, vouch, K, prm, 1, 1, seq_len=seq)
    torch.cuda.synchronize()
    for b in range(w.batch):
        ref = _select_case(w.n, K, w.n_sink, w.n_recent, 0.0, None, td, b=b, seq_len=td.seq_len)
        assert int(cnt[0, b, 0]) == len(ref)
        nb = int(td.seq_len[b])
        a, s, v = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len)
        want = ora.select_margin(None, a, s, v, K, w.n_sink, w.n_recent, alpha=0.0)
        assert prm.margin[b].cpu().numpy().tolist() == want.tolist(), b
        assert np.array_equal(idx[0, b, 0, :len(ref)].cpu().numpy(), ref)
        planted = [p + k for p in td.planted[b] for k in range(1, 7)]
        assert set(planted) <= set(ref.tolist())            # every sponsored span fits: Thm 2


# --------------------------------------------------------------------------
# step 5
# --------------------------------------------------------------------------
def test_compact_bit_exact_strided_and_shared():
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=2, batch=2, n=700, hkv=3, hq=3, window=0)
    _, K, V = wl.make_qkv(w, device=DEV)
    # a strided view: positions live in a larger allocation (row stride 2*d)
    big = torch.zeros((2, 2, 3, 700, 256), dtype=torch.bfloat16, device=DEV)
    big[..., :128] = K
    Kview = big[..., :128]
    Vbig = torch.zeros_like(big)
    Vbig[..., :128] = V
    Vview = Vbig[..., :128]
    rng = np.random.default_rng(0)
    Kb = 100
    idx = np.full((2, 2, 3, Kb), -1, np.int32)
    cnt = np.zeros((2, 2, 3), np.int32)
    for u in np.ndindex(2, 2, 3):
        c = int(rng.integers(0, Kb + 1)) if u != (0, 0, 0) else Kb
        cnt[u] = c
        idx[u][:c] = np.sort(rng.choice(700, c, replace=False))
    for (Kin, Vin) in ((K, V), (Kview, Vview)):
        Ko, Vo = ta.ta_compact(Kin, Vin, _dev(idx), _dev(cnt), Kb)
        torch.cuda.synchronize()
        for u in np.ndindex(2, 2, 3):
            c = int(cnt[u])
            assert np.array_equal(wl.bf16_bits(Ko[u][:c]), ora.compact(wl.bf16_bits(K[u]), idx[u][:c]))
            assert np.array_equal(wl.bf16_bits(Vo[u][:c]), ora.compact(wl.bf16_bits(V[u]), idx[u][:c]))
            assert not wl.bf16_bits(Ko[u][c:]).any()         # rows past cnt are left untouched
    # one index list per sequence, shared by every layer and head
    sidx, scnt = idx[0, :, 0].copy(), cnt[0, :, 0].copy()
    Ko, Vo = ta.ta_compact(K, V, _dev(sidx), _dev(scnt), Kb, idx_shared=True)
    torch.cuda.synchronize()
    for (l, b, h) in np.ndindex(2, 2, 3):
        c = int(scnt[b])
        assert np.array_equal(wl.bf16_bits(Ko[l, b, h][:c]), ora.compact(wl.bf16_bits(K[l, b, h]), sidx[b][:c]))
        assert np.array_equal(wl.bf16_bits(Vo[l, b, h][:c]), ora.compact(wl.bf16_bits(V[l, b, h]), sidx[b][:c]))


# --------------------------------------------------------------------------
# the fused pass
# --------------------------------------------------------------------------
def _check_evict(w, K, clean=True, units=None, layers=None, lengths=None):
    """Runs ta_evict and checks every output; returns the number of excused tie mismatches."""
    lyr = w.layers if layers is None else layers
    td = wl.make_tokens(w, clean=clean)
    if lengths is not None:                                  # given lengths instead of the drawn ones
        td.seq_len[:] = np.asarray(lengths, np.int32)
        td.planted = [[p for p in pl if p + 7 <= int(nb)] for pl, nb in zip(td.planted, td.seq_len)]
    Q, Kc, Vc = wl.make_qkv(w, device=DEV, layers=lyr)
    prm = _prm(w)
    scored = w.alpha != 0.0
    prm.margin = torch.full((lyr, w.batch, w.hkv, 2) if scored else (w.batch, 2), 123.0, device=DEV)
    seq = _dev(td.seq_len) if w.ragged else None
    plan = ta.ta_evict(_dev(td.tok), td.tab_ids, td.tab_len, Q, Kc, Vc, K, prm, seq_len=seq)
    torch.cuda.synchronize()
    margin = prm.margin.cpu().numpy()
    G = w.hq // w.hkv
    excused = 0
    seqs = {}
    for b in range(w.batch):
        nb = int(td.seq_len[b])
        a, s, v = _oracle_seq(td, b)
        seqs[b] = (a, s, v)
        assert np.array_equal(plan.anchor[b, :nb].cpu().numpy(), a)
        assert np.array_equal(plan.spons[b, :nb].cpu().numpy(), s)
        assert np.array_equal(plan.vouch[b, :nb].cpu().numpy().view(np.uint32), v.view(np.uint32))
    all_units = [(l, b, g) for l in range(lyr) for b in range(w.batch) for g in range(w.hkv)]
    for (l, b, g) in (units or all_units):
        nb = int(td.seq_len[b])
        a, s, v = seqs[b]
        if scored:
            A_gpu = plan.A[l, b, g, :nb].cpu().numpy()
            A_ref = ora.score(wl.bf16_bits(Q[l, b, g * G:(g + 1) * G]), wl.bf16_bits(Kc[l, b, g, :nb]))
            assert _score_close(A_gpu, A_ref), (l, b, g)
            idx_gpu = plan.idx[l, b, g].cpu().numpy()
            cnt = int(plan.cnt[l, b, g])
            # same scores on both sides: the selection itself must be exact
            idx_same = ora.select(A_gpu, a, s, v, K, w.n_sink, w.n_recent, w.alpha, w.beta, w.gamma)
            assert cnt == len(idx_same) and np.array_equal(idx_gpu[:cnt], idx_same), (l, b, g)
            m_same = ora.select_margin(A_gpu, a, s, v, K, w.n_sink, w.n_recent, w.alpha, w.beta, w.gamma)
            assert margin[l, b, g].tolist() == m_same.tolist(), (l, b, g)
            # oracle end to end: differences only at ties within 1e-3 of the K-th utility
            idx_ref = ora.select(A_ref, a, s, v, K, w.n_sink, w.n_recent, w.alpha, w.beta, w.gamma)
            diff = set(idx_ref.tolist()) ^ set(idx_gpu[:cnt].tolist())
            if diff:
                u = ora.utility(A_ref, a, v, w.alpha, w.beta, w.gamma)
                kept_u = u[idx_ref]
                cls = np.where(s.astype(bool), 1, 0)
                p = np.arange(nb)
                cls[(p < w.n_sink) | (p >= nb - w.n_recent)] = 2
                bclass = cls[idx_ref].min()
                kth = kept_u[cls[idx_ref] == bclass].min()
                for p_ in diff:
                    assert cls[p_] == bclass and abs(u[p_] - kth) <= 1e-3 * abs(kth), (l, b, g, p_)
                # a retained set that differs only by rounding has a cut the library itself reports as tight:
                # the swapped pair is ordered one way by each side's scores, so the gap is at most twice
                # the tolerance
                assert margin[l, b, g, 0] - margin[l, b, g, 1] <= 2e-3 * abs(kth), (l, b, g)
                excused += len(diff) // 2
        else:
            idx_gpu = plan.idx[b].cpu().numpy()
            cnt = int(plan.cnt[b])
            idx_ref = ora.select(None, a, s, v, K, w.n_sink, w.n_recent, 0.0, w.beta, w.gamma)
            assert cnt == len(idx_ref) and np.array_equal(idx_gpu[:cnt], idx_ref)
            m_ref = ora.select_margin(None, a, s, v, K, w.n_sink, w.n_recent, 0.0, w.beta, w.gamma)
            assert margin[b].tolist() == m_ref.tolist(), b
        sel = idx_gpu[:cnt]
        assert np.array_equal(wl.bf16_bits(plan.Kout[l, b, g][:cnt]), ora.compact(wl.bf16_bits(Kc[l, b, g]), sel))
        assert np.array_equal(wl.bf16_bits(plan.Vout[l, b, g][:cnt]), ora.compact(wl.bf16_bits(Vc[l, b, g]), sel))
        for pl in td.planted[b]:                                     # the planted credential survives
            if K >= w.n_sink + w.n_recent + 6 * len(td.planted[b]):
                assert set(range(pl + 1, pl + 7)) <= set(sel.tolist())
    return excused


def test_evict_c1_single_layer_all_units():
    w = wl.CONFIGS["c1_single_layer"]
    excused = _check_evict(w, 16)
    print("c1 excused ties:", excused)
    # 4 disjoint anchors, 8 protected slots: offsets 1 and 2 of every anchor survive at K=16
    td = wl.make_tokens(w)
    prm = _prm(w)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    plan = ta.ta_evict(_dev(td.tok), td.tab_ids, td.tab_len, Q, Kc, Vc, 16, prm)
    expect = sorted(set(range(4)) | set(range(w.n - 4, w.n)) | {p + k for p in td.planted[0] for k in (1, 2)})
    for g in range(w.hkv):
        assert plan.idx[0, 0, g].cpu().tolist() == expect


@pytest.mark.parametrize("K", [16, 64, 256, 1024])
def test_evict_c2_budget_sweep_two_layers(K):
    w = wl.CONFIGS["c2_full_model"]
    excused = _check_evict(w, K, layers=2, units=[(0, 0, 0), (0, 0, 3), (1, 0, 6), (1, 0, 7)])
    print("c2 K=%d excused ties: %d" % (K, excused))


def test_evict_c2_dirty_tokens():
    w = wl.CONFIGS["c2_full_model"]
    _check_evict(w, 256, clean=False, layers=1, units=[(0, 0, 1), (0, 0, 4)])


def test_evict_c3_ta_fast_scaled():
    w = wl.scaled(wl.CONFIGS["c3_ta_fast"], layers=2, batch=3, n=32768)
    _check_evict(w, 512, units=[(0, 0, 0), (1, 2, 7), (0, 1, 3)])


def test_evict_c4_long_context_scaled():
    w = wl.scaled(wl.CONFIGS["c4_long_context"], layers=1, batch=1, n=16384, planted=16)
    _check_evict(w, 1024, units=[(0, 0, 0), (0, 0, 5)])


def test_evict_c5_ragged_prefill_scaled():
    w = wl.scaled(wl.CONFIGS["c5_agentic_prefill"], layers=1, batch=6, n=3000, ragged=(500, 3000))
    _check_evict(w, 256, units=[(0, b, b % 8) for b in range(6)])


def test_evict_degenerate_lengths():
    # sequences that are empty, a single token, shorter than the mandatory ranges, shorter than the observation
    # window, exactly the budget and one more than it, next to a full one
    w = wl.scaled(wl.CONFIGS["c5_agentic_prefill"], layers=2, batch=8, n=2048, ragged=(0, 2048))
    K = 64
    lengths = [0, 1, 7, 20, K, K + 1, 2048, 33]
    assert w.n_sink + w.n_recent == 8 and w.window == 32
    excused = _check_evict(w, K, lengths=lengths)
    assert excused == 0


def test_evict_is_deterministic():
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=2)
    td = wl.make_tokens(w)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    prm = _prm(w)
    p1 = ta.ta_evict(_dev(td.tok), td.tab_ids, td.tab_len, Q, Kc, Vc, 64, prm)
    p2 = ta.ta_evict(_dev(td.tok), td.tab_ids, td.tab_len, Q, Kc, Vc, 64, prm)
    torch.cuda.synchronize()
    assert torch.equal(p1.A.view(torch.int32), p2.A.view(torch.int32))
    assert torch.equal(p1.idx, p2.idx) and torch.equal(p1.Kout.view(torch.int16), p2.Kout.view(torch.int16))
