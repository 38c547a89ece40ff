"""The streaming form of step 4 (one read of every input, candidate list in LDS) against the oracle.

ta_select picks that form for rows longer than its LDS key cache and for launches of many units;
these cases reach it at sizes the oracle finishes in seconds, on inputs chosen to drive its
branches: repeated cuts of the list (utilities that grow towards the start of the sequence, so
every segment of the walk beats the threshold), thousands of exact ties (position passes), pool
overflow, no mandatory class, ragged lengths below and above the budget, per-layer budgets, and
budgets whose list does not fit (those fall back to the cached kernel and must agree as well).
"""
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


def _inputs(n, batch, planted, ragged, seed):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], n=n, batch=batch, planted=planted, ragged=ragged)
    td = wl.make_tokens(w, clean=False)
    seqs = []
    for b in range(batch):
        nb = int(td.seq_len[b])
        seqs.append(ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len))
    return w, td, seqs


def _scores(mode, shape, rng):
    n = shape[-1]
    if mode == "uniform":
        return (rng.random(shape) * 4).astype(np.float32)
    if mode == "ties":
        return np.round(rng.random(shape) * 4, 1).astype(np.float32)
    if mode == "zeros":
        return np.zeros(shape, np.float32)
    if mode == "early":                # large scores at the start: the walk from the end keeps finding better positions
        return (np.linspace(8.0, 0.0, n, dtype=np.float32)[None, None, None, :] + rng.random(shape).astype(np.float32) * 0.01).astype(np.float32)
    raise ValueError(mode)


def _check(layers, batch, hkv, n, K, ns, nr, mode, planted=8, ragged=None, beta=0.5, layer_K=None, sample=None, seed=0):
    w, td, seqs = _inputs(n, batch, planted, ragged, seed)
    rng = np.random.default_rng(1000 * n + K + seed)
    A = _scores(mode, (layers, batch, hkv, n), rng)
    lk = None if layer_K is None else _dev(np.asarray(layer_K, np.int32))
    margin = torch.full((layers, batch, hkv, 2), 123.0, device=DEV)
    prm = ta.Params(n_sink=ns, n_recent=nr, beta=beta, layer_K=lk, margin=margin)
    seq = _dev(td.seq_len) if ragged else None
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm, seq_len=seq)
    idx, cnt = ta.ta_select(_dev(A), anchor, spons, vouch, K, prm, layers, hkv, seq_len=seq)
    torch.cuda.synchronize()
    idx, cnt, margin = idx.cpu().numpy(), cnt.cpu().numpy(), margin.cpu().numpy()
    units = [(l, b, h) for l in range(layers) for b in range(batch) for h in range(hkv)]
    if sample is not None and sample < len(units):
        pick = np.random.default_rng(seed + 5).choice(len(units), size=sample, replace=False)
        units = [units[i] for i in sorted(pick)] + [units[0], units[-1]]
    for (l, b, h) in units:
        nb = int(td.seq_len[b])
        a, s, v = seqs[b]
        Kl = K if layer_K is None else min(K, max(int(layer_K[l]), ns + nr, 1))
        ref = ora.select(A[l, b, h, :nb], a, s, v, Kl, ns, nr, alpha=1.0, beta=beta, gamma=0.3)
        assert cnt[l, b, h] == len(ref) == min(Kl, nb), (l, b, h)
        assert np.array_equal(idx[l, b, h, :len(ref)], ref), (l, b, h)
        # the margin of the cut: the same two utilities, bit for bit
        want = ora.select_margin(A[l, b, h, :nb], a, s, v, Kl, ns, nr, alpha=1.0, beta=beta, gamma=0.3)
        assert margin[l, b, h].tolist() == want.tolist(), (l, b, h, margin[l, b, h], want)
    return len(units)


@pytest.mark.parametrize("n,K,ns,nr,mode,planted", [
    (1500, 64, 4, 4, "uniform", 8),
    (1500, 16, 4, 4, "uniform", 8),      # pool overflow: more sponsored positions than protected slots
    (2048, 256, 4, 8, "ties", 8),        # exact ties at the threshold: position passes
    (1028, 100, 0, 0, "zeros", 4),       # no mandatory class, recency alone decides
    (3000, 700, 4, 64, "early", 8),      # every segment of the walk beats the threshold: a cut per segment
])
def test_streaming_select_many_units(n, K, ns, nr, mode, planted):
    # 16 x 16 x 8 = 2048 units: enough for ta_select to take the streaming form on short rows
    checked = _check(16, 16, 8, n, K, ns, nr, mode, planted=planted, sample=300)
    assert checked >= 300


def test_streaming_select_ragged_many_units():
    # lengths from below the budget (nothing to evict) to several segments, 4-aligned padded rows
    _check(16, 16, 8, 2600, 128, 4, 16, "uniform", ragged=(40, 2600), sample=400)


def test_streaming_select_negative_recency_weight():
    # beta < 0 reverses the recency order: the walk from the end meets the worst positions first
    _check(16, 16, 8, 2304, 200, 4, 4, "uniform", beta=-0.5, sample=200)


def test_streaming_select_per_layer_budgets():
    layers = 16
    lk = [max(12, 300 - 18 * l) for l in range(layers)]
    _check(layers, 16, 8, 1800, 300, 4, 8, "uniform", layer_K=lk, sample=300)


@pytest.mark.parametrize("n,K,mode", [
    (70000, 1024, "early"),              # long rows, dozens of cuts of the list
    (131072, 1024, "uniform"),           # the long-context row length
    (50000, 4000, "ties"),               # list of more than 4000 entries
    (40000, 7000, "uniform"),            # the list would not fit: cached-kernel fallback, same answer
])
def test_streaming_select_long_rows(n, K, mode):
    _check(1, 2, 3, n, K, 4, 128, mode, planted=40)
