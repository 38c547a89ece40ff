"""GPU parity of scoring and compaction over paged (block-table) caches against the oracle's
paged gather followed by its dense definitions; and against the dense kernels on the same data."""
import numpy as np
import pytest
import torch

import paper_2604_11288_amd as ta
from oracle import ta_oracle as ora
from paper_2604_11288_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _close(got, ref):
    return np.all(np.abs(got - ref) <= 1e-3 * np.abs(ref) + 1e-7)


@pytest.mark.parametrize("page_size,heads_first,n,window,ragged", [
    (64, False, 3000, 32, (700, 3000)),       # smallest page the score kernel takes; last page partly filled
    (256, True, 4096, 32, None),
    (128, False, 9000, 64, (4000, 9000)),     # several chunks, 256 rows per unit
    (64, True, 2600, 128, (150, 2600)),       # 512 rows per unit: two passes over each chunk of pages
])
def test_paged_score_and_compact_match_oracle(page_size, heads_first, n, window, ragged):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=2, batch=2, n=n, hq=8, hkv=2, window=window, ragged=ragged, planted=6)
    td = wl.make_tokens(w, clean=False)
    Q, K, V = wl.make_qkv(w, device=DEV)
    Kp, Vp, table, num_pages, strides = wl.make_paged(K, V, page_size, heads_first=heads_first)
    paged = ta.PagedKV(Kp, Vp, table, page_size, num_pages, strides, w.layers, w.batch, w.hkv, n)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent)
    seq = _dev(td.seq_len)
    A = ta.ta_score_paged(Q, paged, prm, seq_len=seq)
    A_dense = ta.ta_score(Q, K, prm, seq_len=seq)
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm, seq_len=seq)
    Kb = 200
    idx, cnt = ta.ta_select(A, anchor, spons, vouch, Kb, prm, w.layers, w.hkv, seq_len=seq)
    Ko, Vo = ta.ta_compact_paged(paged, idx, cnt, Kb)
    Ko_d, Vo_d = ta.ta_compact(K, V, idx, cnt, Kb)
    torch.cuda.synchronize()
    assert torch.equal(A, A_dense)                          # same kernels, same data, other addresses
    assert torch.equal(Ko, Ko_d) and torch.equal(Vo, Vo_d)
    A_h, idx_h, cnt_h = A.cpu().numpy(), idx.cpu().numpy(), cnt.cpu().numpy()
    Kp_h, Vp_h, Ko_h, Vo_h, tab_h = wl.bf16_bits(Kp), wl.bf16_bits(Vp), wl.bf16_bits(Ko), wl.bf16_bits(Vo), table.cpu().numpy()
    G = w.hq // w.hkv
    for l in range(w.layers):
        for b in range(w.batch):
            nb = int(td.seq_len[b])
            for g in range(w.hkv):
                rows_k = ora.paged_gather(Kp_h[l], tab_h[b], nb, page_size, strides[1], strides[2], strides[3], g, w.d)
                rows_v = ora.paged_gather(Vp_h[l], tab_h[b], nb, page_size, strides[1], strides[2], strides[3], g, w.d)
                ref = ora.score(wl.bf16_bits(Q[l, b, g * G:(g + 1) * G]), rows_k)
                assert _close(A_h[l, b, g, :nb], ref), (l, b, g)
                c = int(cnt_h[l, b, g])
                assert np.array_equal(Ko_h[l, b, g, :c], ora.compact(rows_k, idx_h[l, b, g, :c]))
                assert np.array_equal(Vo_h[l, b, g, :c], ora.compact(rows_v, idx_h[l, b, g, :c]))


def test_paged_one_sweep_score_and_small_pages_for_compaction():
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=1, batch=2, n=2048, hq=8, hkv=2, planted=4)
    Q, K, V = wl.make_qkv(w, device=DEV)
    prm = ta.Params()
    G, W, n = w.hq // w.hkv, w.window, w.n
    S = torch.einsum("lbhwd,lbhnd->lbhwn", Q.float(), K.float().repeat_interleave(G, dim=2)) / w.d ** 0.5
    mask = torch.arange(n, device=DEV)[None, :] > (n - W + torch.arange(W, device=DEV))[:, None]
    lse = torch.logsumexp(S.masked_fill(mask, float("-inf")), dim=-1).contiguous()
    Kp, Vp, table, num_pages, strides = wl.make_paged(K, V, 64)
    paged = ta.PagedKV(Kp, Vp, table, 64, num_pages, strides, w.layers, w.batch, w.hkv, n)
    A1 = ta.ta_score_paged(Q, paged, prm, lse=lse)
    A2 = ta.ta_score_lse(Q, K, lse, prm)
    torch.cuda.synchronize()
    assert torch.equal(A1, A2)
    # compaction has no page-size restriction: 16-position pages (the common serving default)
    Kp, Vp, table, num_pages, strides = wl.make_paged(K, V, 16, heads_first=True)
    paged16 = ta.PagedKV(Kp, Vp, table, 16, num_pages, strides, w.layers, w.batch, w.hkv, n)
    rng = np.random.default_rng(2)
    idx = np.sort(rng.permutation(n)[:100]).astype(np.int32)
    idx_t = _dev(np.broadcast_to(idx, (w.batch, 100)).copy())
    cnt_t = _dev(np.array([100, 37], np.int32))
    Ko, Vo = ta.ta_compact_paged(paged16, idx_t, cnt_t, 100, idx_shared=True)
    torch.cuda.synchronize()
    assert torch.equal(Ko[0, 0, :, :100], K[0, 0][:, idx.tolist()]) and torch.equal(Vo[0, 1, :, :37], V[0, 1][:, idx[:37].tolist()])
    with pytest.raises(ta.TaError):            # scoring needs pages of a multiple of 64 positions
        ta.ta_score_paged(Q, paged16, prm)


def test_corrupt_block_table_cannot_fault():
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=1, batch=1, n=1024, hq=4, hkv=1)
    Q, K, V = wl.make_qkv(w, device=DEV)
    Kp, Vp, table, num_pages, strides = wl.make_paged(K, V, 64)
    bad = table.clone()
    bad[0, 3], bad[0, 5] = -7, 10 ** 6         # clamped to the pool on the device
    paged = ta.PagedKV(Kp, Vp, bad, 64, num_pages, strides, 1, 1, 1, 1024)
    A = ta.ta_score_paged(Q, paged, ta.Params())
    torch.cuda.synchronize()
    assert torch.isfinite(A).all()


@pytest.mark.parametrize("with_lse,alpha", [(False, 1.0), (True, 1.0), (False, 0.0)])
def test_whole_pass_over_a_paged_cache_equals_the_dense_pass(with_lse, alpha):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=2, batch=2, n=2600, hq=8, hkv=2, planted=6, ragged=(900, 2600),
                  alpha=alpha)
    td = wl.make_tokens(w, clean=False)
    Q, K, V = wl.make_qkv(w, device=DEV)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, alpha=alpha)
    seq = _dev(td.seq_len)
    lse = None
    if with_lse:
        G = w.hq // w.hkv
        lse_h = np.full((w.layers, w.batch, w.hq, w.window), -np.inf, np.float32)
        for l in range(w.layers):
            for b in range(w.batch):
                nb = int(td.seq_len[b])
                for g in range(w.hkv):
                    lse_h[l, b, g * G:(g + 1) * G] = ora.row_lse(wl.bf16_bits(Q[l, b, g * G:(g + 1) * G]),
                                                                 wl.bf16_bits(K[l, b, g, :nb]), True)
        lse = _dev(lse_h)
    Kp, Vp, table, num_pages, strides = wl.make_paged(K, V, 128)
    paged = ta.PagedKV(Kp, Vp, table, 128, num_pages, strides, w.layers, w.batch, w.hkv, w.n)
    Kb = 150
    tok = _dev(td.tok)
    Qa = Q if alpha != 0.0 else None
    if with_lse:
        dense = ta.ta_evict_lse(tok, td.tab_ids, td.tab_len, Q, K, V, lse, Kb, prm, seq_len=seq)
    else:
        dense = ta.ta_evict(tok, td.tab_ids, td.tab_len, Qa, K, V, Kb, prm, seq_len=seq)
    pg = ta.ta_evict_paged(tok, td.tab_ids, td.tab_len, Qa, paged, Kb, prm, seq_len=seq, lse=lse)
    torch.cuda.synchronize()
    for name in ("anchor", "spons", "vouch", "idx", "cnt", "Kout", "Vout"):
        assert torch.equal(getattr(dense, name), getattr(pg, name)), name
    if alpha != 0.0:
        assert torch.equal(dense.A, pg.A)
    assert int(pg.cnt.min()) > 0 and pg.Kout.abs().sum() > 0
