"""Pins of the oracle's incremental (per generation step) form: no GPU involved."""
import numpy as np
import pytest
import torch

from oracle import ta_oracle as ora
from paper_2604_11288_amd import workloads as wl


def _bits(t):
    return wl.bf16_bits(t)


def _rand(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


def _unit_from_prefill(n, K, d, seed, n_keep_idx=None):
    Kall, Vall = _rand((n, d), seed), _rand((n, d), seed + 1)
    idx = np.arange(n - K, n, dtype=np.int32) if n_keep_idx is None else n_keep_idx
    A0 = np.zeros(K, np.float32)
    u = ora.DecodeUnit(_bits(Kall)[idx], _bits(Vall)[idx], idx, A0)
    return u


def test_streaming_window_when_no_attention_and_no_anchors():
    """alpha = 0 and an empty table: the cache is the sinks plus a sliding window (StreamingLLM row
    of the budget-partition table, App. D)."""
    n, K, d, ns = 40, 12, 16, 4
    seq = ora.DecodeSeq(np.arange(n, dtype=np.int32), np.zeros((0, 4), np.int32), np.zeros(0, np.int32), cap=n + 50)
    idx = np.concatenate([np.arange(ns), np.arange(n - (K - ns), n)]).astype(np.int32)
    unit = _unit_from_prefill(n, K, d, 3, idx)
    for t in range(30):
        p = seq.append(1000 + t)
        e, _ = unit.step(seq, _bits(_rand((2, d), 50 + t)), _bits(_rand((d,), 90 + t)), _bits(_rand((d,), 130 + t)),
                         p, n_sink=ns, n_recent=0, alpha=0.0, beta=0.5, gamma=0.3)
        seq.decay()
        kept = sorted(unit.pos[unit.pos >= 0].tolist())
        assert kept == list(range(ns)) + list(range(seq.len - (K - ns), seq.len))
        assert (unit.pos < 0).sum() == 1 and unit.pos[e] == -1


def test_budget_decay_and_fresh_anchor_vouchers():
    tab = np.array([[7, 8, -1, -1]], np.int32)
    ln = np.array([2], np.int32)
    seq = ora.DecodeSeq(np.array([1, 7, 8, 2, 3], np.int32), tab, ln, cap=64, B=15.0)
    assert seq.anchor[:5].tolist() == [0, 0, 1, 0, 0] and seq.budget[2] == 15.0
    V, sp = seq.vouch(3)
    assert sp == 1 and V == np.float32(15.0) * np.float32(0.8)
    for t in range(1, 6):
        seq.decay(0.9)
        assert seq.budget[2] == pytest.approx(15.0 * 0.9 ** t, rel=1e-6)          # B_i <- 0.9 B_i per step
    V, _ = seq.vouch(4)
    assert V == pytest.approx(15.0 * 0.9 ** 5 * 0.8 ** 2, rel=1e-6)
    # an n-gram completed by appended tokens: the anchor is its last token, budget fresh
    p = seq.append(7); assert seq.anchor[p] == 0
    p = seq.append(8); assert seq.anchor[p] == 1 and seq.budget[p] == 15.0
    p2 = seq.append(99)
    V, sp = seq.vouch(p2)
    # the fresh anchor one position back (15 * 0.8) plus the old, decayed one five positions back
    assert sp == 1 and V == pytest.approx(12.0 + 15.0 * 0.9 ** 5 * 0.8 ** 5, rel=1e-6)
    V, sp = seq.vouch(p + 7)                                                      # outside the span L=6
    assert (V, sp) == (0.0, 0)


def test_decode_attention_matches_softmax_and_accumulates():
    n, K, d, G = 30, 10, 64, 3
    seq = ora.DecodeSeq(np.arange(n, dtype=np.int32), np.zeros((0, 4), np.int32), np.zeros(0, np.int32), cap=64)
    unit = _unit_from_prefill(n, K, d, 11)
    A_before = unit.A.copy()
    q, kn, vn = _rand((G, d), 20, 2.0), _rand((d,), 21), _rand((d,), 22)
    p = seq.append(5)
    e, _ = unit.step(seq, _bits(q), _bits(kn), _bits(vn), p, n_sink=1, n_recent=1)
    Kc = torch.from_numpy(unit.Kc.view(np.int16)).view(torch.bfloat16).double()
    ref = torch.softmax(q.double() @ Kc.T / np.sqrt(d), dim=-1).sum(0).numpy()    # all K+1 rows are visible
    free_before = K                                                              # slot K was the free one
    expect = np.zeros(K + 1)
    expect[:K] = A_before[:K]
    expect += ref
    assert np.allclose(unit.A, expect, rtol=1e-6)
    assert unit.A.sum(dtype=np.float64) == pytest.approx(A_before.sum() + G, rel=1e-6)   # softmax rows sum to 1
    assert unit.pos[e] == -1 and np.array_equal(unit.Kc[free_before], _bits(kn))
    assert np.array_equal(unit.Vc[free_before], _bits(vn))


def test_decode_evicts_the_argmin_of_the_order():
    rng = np.random.default_rng(4)
    tab = np.array([[900, -1, -1, -1]], np.int32)
    ln = np.array([1], np.int32)
    for trial in range(20):
        n, K, d, G = 60, 16, 32, 2
        tok = rng.integers(0, 50, n).astype(np.int32)
        tok[rng.integers(5, n - 5, 3)] = 900
        seq = ora.DecodeSeq(tok, tab, ln, cap=128)
        idx = np.sort(rng.choice(n, K, replace=False)).astype(np.int32)
        unit = _unit_from_prefill(n, K, d, 100 + trial, idx)
        unit.A[:K] = np.round(rng.random(K) * 2, 1).astype(np.float32)
        ns, nr = 2, 2
        p = seq.append(int(rng.integers(0, 50)))
        pos_before = unit.pos.copy()
        e, u = unit.step(seq, _bits(_rand((G, d), trial)), _bits(_rand((d,), trial + 1)),
                         _bits(_rand((d,), trial + 2)), p, n_sink=ns, n_recent=nr)
        pos_full = pos_before.copy()
        pos_full[pos_before < 0] = p
        keys = []
        for s in range(K + 1):
            pp = int(pos_full[s])
            V, sp = seq.vouch(pp)
            cls = 2 if (pp < ns or pp >= seq.len - nr) else (1 if sp else 0)
            keys.append((cls, float(u[s]), pp))
        assert e == min(range(K + 1), key=lambda s: keys[s])
        # utilities follow Eq. 1 with the cumulative attention of the slot
        s0 = 0
        pp = int(pos_full[s0])
        V, _ = seq.vouch(pp)
        ref = 1.0 * float(unit.A[s0]) + 0.5 * (pp + 1) / seq.len + 0.3 * int(seq.anchor[pp]) + V
        assert u[s0] == pytest.approx(ref, rel=1e-6)


def test_decode_needle_survives_with_zero_attention():
    """An anchor completed during decode sponsors the next L tokens; with K >= sinks + recent + L
    they stay cached while every other token has far more attention (Thm. 2), until the decayed
    voucher no longer matters - here for 40 steps."""
    n, K, d, G, L = 50, 16, 32, 1, 6
    tab = np.array([[777, 778, -1, -1]], np.int32)
    ln = np.array([2], np.int32)
    seq = ora.DecodeSeq(np.arange(n, dtype=np.int32), tab, ln, cap=256)
    unit = _unit_from_prefill(n, K, d, 5)
    unit.A[:K] = 500.0
    stream = [1, 777, 778] + [2000 + i for i in range(60)]
    span = None
    zero = np.zeros(d, np.uint16)
    for t, tk in enumerate(stream):
        p = seq.append(tk)
        if tk == 778:
            span = set(range(p + 1, p + 1 + L))
        # keys of the value span are orthogonal to the query: they get (almost) no attention
        kn = _rand((d,), 300 + t)
        q = _rand((G, d), 400 + t)
        is_value = span is not None and p in span
        unit.step(seq, _bits(q), zero if is_value else _bits(kn), _bits(kn), p, n_sink=4, n_recent=4, L=L,
                  rank_A=None)
        # every non-value row keeps a large cumulative score
        unit.A[(unit.pos >= 0) & ~np.isin(unit.pos, list(span or []))] += 100.0
        seq.decay(0.9)
        if span is not None and t >= 3 + L and t < 3 + L + 40:
            assert span <= set(unit.pos[unit.pos >= 0].tolist()), t
    assert seq.anchor[n + 2] == 1


def test_sequence_at_capacity_does_not_step():
    """The boundary leaves a sequence at capacity unchanged; the oracle's sequence state refuses the
    append (its arrays end at cap), and a caller that skips the step changes nothing."""
    tab = np.array([[7, 8, -1, -1]], np.int32)
    ln = np.array([2], np.int32)
    seq = ora.DecodeSeq(np.array([1, 7, 8, 2, 3], np.int32), tab, ln, cap=6, B=15.0)
    seq.append(7)
    assert seq.len == seq.cap
    tok, anc, bud = seq.tok.copy(), seq.anchor.copy(), seq.budget.copy()
    with pytest.raises(AssertionError):
        seq.append(8)
    assert seq.len == seq.cap
    assert np.array_equal(seq.tok, tok) and np.array_equal(seq.anchor, anc)
    assert np.array_equal(seq.budget.view(np.uint32), bud.view(np.uint32))


def _attention_f64(q, Krows):
    """Softmax mass of every row, summed over the heads, in float64 (numpy restatement)."""
    qf = torch.from_numpy(q.astype(np.int32) << 16).view(torch.float32).double().numpy()
    kf = torch.from_numpy(Krows.astype(np.int32) << 16).view(torch.float32).double().numpy()
    S = qf @ kf.T / np.sqrt(kf.shape[1])
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    return P.sum(axis=0)


def test_last_query_rule_evicts_the_arg_min_of_the_current_steps_attention():
    """The step-wise minimum-attention rule ascribed to TOVA (Sec. 2; corollary of Thm. 1): with alpha = 1,
    beta = gamma = 0, no anchors and no mandatory positions, the evicted row is the arg-min of the
    attention of THIS step's queries, whatever the rows accumulated before."""
    n, K, d, G = 60, 20, 32, 3
    seq = ora.DecodeSeq(np.arange(n, dtype=np.int32), np.zeros((0, 4), np.int32), np.zeros(0, np.int32), cap=n + 40)
    unit = _unit_from_prefill(n, K, d, 11)
    unit.A[:K] = np.linspace(5.0, 9.0, K).astype(np.float32)          # a history that the rule must ignore
    for t in range(25):
        p = seq.append(500 + t)
        q, kn, vn = _bits(_rand((G, d), 300 + t)), _bits(_rand((d,), 400 + t)), _bits(_rand((d,), 500 + t))
        f = int(np.flatnonzero(unit.pos < 0)[0])
        Kall = unit.Kc.copy()
        Kall[f] = kn
        pos_all = unit.pos.copy()
        pos_all[f] = p
        want = _attention_f64(q, Kall)                                 # every slot is occupied once the row is in
        e, _ = unit.step(seq, q, kn, vn, p, n_sink=0, n_recent=0, alpha=1.0, beta=0.0, gamma=0.0, last_query=True)
        seq.decay()
        assert e == int(np.argmin(want)), t
        occ = np.ones(K + 1, bool)
        assert np.allclose(unit.A[occ], want[occ].astype(np.float32), rtol=1e-6, atol=0)
        assert unit.pos[e] == -1 and (unit.pos < 0).sum() == 1


def test_last_query_and_cumulative_rules_disagree_when_history_matters():
    """One row with a large accumulated mass but (by construction) the smallest current attention: the
    cumulative rule keeps it, the step-wise rule evicts it."""
    n, K, d = 30, 8, 16
    seq_a = ora.DecodeSeq(np.arange(n, dtype=np.int32), np.zeros((0, 4), np.int32), np.zeros(0, np.int32), cap=n + 8)
    seq_b = ora.DecodeSeq(np.arange(n, dtype=np.int32), np.zeros((0, 4), np.int32), np.zeros(0, np.int32), cap=n + 8)
    q = _rand((1, d), 5)
    Krows = _rand((K, d), 6)
    Krows[3] = -4.0 * q[0]                                               # strongly anti-aligned with the query
    Vrows = _rand((K, d), 7)
    idx = np.arange(n - K, n, dtype=np.int32)
    outs = []
    for last_query, seq in ((False, seq_a), (True, seq_b)):
        u = ora.DecodeUnit(_bits(Krows), _bits(Vrows), idx, np.where(np.arange(K) == 3, 50.0, 0.0).astype(np.float32))
        p = seq.append(77)
        e, _ = u.step(seq, _bits(q), _bits(_rand((d,), 8)), _bits(_rand((d,), 9)), p, n_sink=0, n_recent=0,
                      alpha=1.0, beta=0.0, gamma=0.0, last_query=last_query)
        outs.append(e)
    assert outs[1] == 3 and outs[0] != 3
