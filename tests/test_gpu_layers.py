"""GPU parity of the pass over caches kept as one tensor per layer (ta_evict_layers): against
the oracle on sampled units, and bit for bit against ta_evict on the same data stacked."""
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


def _scatter(stacked, heads_last=False):
    """Per-layer copies of a stacked [Lyr][B][H][rows][d] tensor, each an allocation of its own
    (of a different size, so the distances between layers are irregular); heads_last stores a
    layer as [B][rows][H][d] and hands out the [B][H][rows][d] view of it."""
    out = []
    for l in range(stacked.shape[0]):
        src = stacked[l]
        shape = (src.shape[0], src.shape[2], src.shape[1], src.shape[3]) if heads_last else tuple(src.shape)
        numel = int(np.prod(shape))
        buf = torch.empty(numel + 4096 * (l + 1), dtype=stacked.dtype, device=stacked.device)
        t = buf[8 * (l + 1):8 * (l + 1) + numel].view(shape)      # 16-byte aligned, not at the start of the buffer
        if heads_last:
            t = t.permute(0, 2, 1, 3)
        t.copy_(src)
        out.append(t)
    return out


@pytest.mark.parametrize("n,batch,layers,K,ragged,heads_last", [
    (1000, 2, 3, 64, None, False),
    (4096, 1, 5, 256, None, True),            # rows of a position interleaved over the heads
    (2500, 3, 2, 100, (17, 2500), False),
    (300, 1, 40, 50, None, False),            # more layers than the small form of the address table holds
])
def test_layers_scored_pass_equals_stacked_pass_and_oracle(n, batch, layers, K, ragged, heads_last):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=layers, batch=batch, n=n, hq=8, hkv=2, window=32,
                  ragged=ragged, planted=6)
    td = wl.make_tokens(w, clean=False)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent)
    tok, seq = _dev(td.tok), _dev(td.seq_len)
    ref = ta.ta_evict(tok, td.tab_ids, td.tab_len, Q, Kc, Vc, K, prm, seq_len=seq)
    Ql, Kl, Vl = _scatter(Q), _scatter(Kc, heads_last), _scatter(Vc, heads_last)
    got = ta.ta_evict_layers(tok, td.tab_ids, td.tab_len, Ql, Kl, Vl, K, prm, seq_len=seq)
    torch.cuda.synchronize()
    for name in ("anchor", "spons", "vouch", "A", "idx", "cnt"):
        assert torch.equal(getattr(got, name), getattr(ref, name)), name
    for l in range(layers):
        assert torch.equal(got.Kout[l], ref.Kout[l]) and torch.equal(got.Vout[l], ref.Vout[l]), l
    # and against the oracle, one unit per layer
    G = w.hq // w.hkv
    for l in range(layers):
        b, g = l % batch, l % w.hkv
        nb = int(td.seq_len[b])
        a, s, v = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len)
        k_rows, v_rows = wl.bf16_bits(Kl[l][b, g, :nb]), wl.bf16_bits(Vl[l][b, g, :nb])
        A_ref = ora.score(wl.bf16_bits(Ql[l][b, g * G:(g + 1) * G]), k_rows)
        A_gpu = got.A[l, b, g, :nb].cpu().numpy()
        assert np.all(np.abs(A_gpu - A_ref) <= 1e-3 * np.abs(A_ref) + 1e-7)
        idx_ref = ora.select(A_gpu, a, s, v, K, w.n_sink, w.n_recent)      # same scores on both sides
        c = int(got.cnt[l, b, g])
        assert c == len(idx_ref) and np.array_equal(got.idx[l, b, g, :c].cpu().numpy(), idx_ref)
        assert np.array_equal(wl.bf16_bits(got.Kout[l][b, g, :c]), ora.compact(k_rows, idx_ref))
        assert np.array_equal(wl.bf16_bits(got.Vout[l][b, g, :c]), ora.compact(v_rows, idx_ref))


def test_layers_attention_free_pass_shares_one_retained_set():
    w = wl.scaled(wl.CONFIGS["c3_ta_fast"], layers=4, batch=3, n=3000, hkv=2, ragged=(100, 3000), planted=8)
    td = wl.make_tokens(w)
    _, Kc, Vc = wl.make_qkv(w, device=DEV)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, alpha=0.0)
    tok, seq = _dev(td.tok), _dev(td.seq_len)
    K = 128
    ref = ta.ta_evict(tok, td.tab_ids, td.tab_len, None, Kc, Vc, K, prm, seq_len=seq)
    got = ta.ta_evict_layers(tok, td.tab_ids, td.tab_len, None, _scatter(Kc), _scatter(Vc), K, prm, seq_len=seq)
    torch.cuda.synchronize()
    assert torch.equal(got.idx, ref.idx) and torch.equal(got.cnt, ref.cnt)
    for l in range(w.layers):
        assert torch.equal(got.Kout[l], ref.Kout[l]) and torch.equal(got.Vout[l], ref.Vout[l]), l
    b = 1
    nb = int(td.seq_len[b])
    a, s, v = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len)
    idx_ref = ora.select(None, a, s, v, K, w.n_sink, w.n_recent, alpha=0.0)
    assert np.array_equal(got.idx[b, :int(got.cnt[b])].cpu().numpy(), idx_ref)


@pytest.mark.parametrize("page_size,heads_first,alpha,with_lse", [
    (64, False, 1.0, False),
    (128, True, 1.0, True),        # one sweep from given row log-sum-exps
    (16, False, 0.0, False),       # nothing scored: any page size
])
def test_layers_paged_pass_equals_the_paged_pass_on_a_stacked_pool(page_size, heads_first, alpha, with_lse):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=3, batch=2, n=2000, hq=8, hkv=2, window=32,
                  ragged=(300, 2000), planted=6)
    td = wl.make_tokens(w, clean=False)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    Kp, Vp, table, num_pages, strides = wl.make_paged(Kc, Vc, page_size, heads_first=heads_first)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, alpha=alpha)
    tok, seq = _dev(td.tok), _dev(td.seq_len)
    K = 150
    lse = None
    if with_lse:
        # natural-log normalisers of the window rows, by torch on the device (inputs of the call, not a reference)
        lse = torch.empty((w.layers, w.batch, w.hq, w.window), dtype=torch.float32, device=DEV)
        G = w.hq // w.hkv
        for l in range(w.layers):
            for b in range(w.batch):
                nb = int(td.seq_len[b])
                S = torch.einsum("hwd,hnd->hwn", Q[l, b].float(), Kc[l, b, :, :nb].float().repeat_interleave(G, dim=0))
                S = S / w.d ** 0.5
                vis = torch.arange(nb, device=DEV)[None, :] <= (nb - w.window + torch.arange(w.window, device=DEV))[:, None]
                lse[l, b] = torch.logsumexp(S.masked_fill(~vis[None], float("-inf")), dim=-1)
    stacked = ta.PagedKV(Kp, Vp, table, page_size, num_pages, strides, w.layers, w.batch, w.hkv, w.n)
    Qs = Q if alpha != 0.0 else None
    ref = ta.ta_evict_paged(tok, td.tab_ids, td.tab_len, Qs, stacked, K, prm, seq_len=seq, lse=lse)
    # the same pools, one allocation per layer
    Kl = [Kp[l].clone() for l in range(w.layers)]
    Vl = [Vp[l].clone() for l in range(w.layers)]
    Ql = _scatter(Q) if alpha != 0.0 else None
    desc = ta.PagedKV(None, None, table, page_size, num_pages, strides, w.layers, w.batch, w.hkv, w.n)
    got = ta.ta_evict_layers_paged(tok, td.tab_ids, td.tab_len, Ql, Kl, Vl, desc, K, prm, seq_len=seq, lse=lse)
    torch.cuda.synchronize()
    assert torch.equal(got.idx, ref.idx) and torch.equal(got.cnt, ref.cnt)
    if alpha != 0.0:
        assert torch.equal(got.A, ref.A)
    for l in range(w.layers):
        assert torch.equal(got.Kout[l], ref.Kout[l]) and torch.equal(got.Vout[l], ref.Vout[l]), l
    # one unit against the oracle's paged gather and compaction
    l, b, g = 2, 1, 1
    nb = int(td.seq_len[b])
    rows_k = ora.paged_gather(wl.bf16_bits(Kl[l]), table.cpu().numpy()[b], nb, page_size, strides[1], strides[2], strides[3], g, w.d)
    sel = (b,) if alpha == 0.0 else (l, b, g)
    c = int(got.cnt[sel])
    idx_h = got.idx[sel][:c].cpu().numpy()
    assert np.array_equal(wl.bf16_bits(got.Kout[l][b, g, :c]), ora.compact(rows_k, idx_h))
