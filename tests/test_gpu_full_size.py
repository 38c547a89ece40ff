"""Full-size configurations in the launch configuration bench.py times.

The oracle checks sampled units one by one; every other unit is covered by
properties that hold at any size: softmax rows sum to one (sum of A = G * W per
unit), |S| = min(K, len), ascending unique indices that contain the sinks, the
recent window and (when they fit) every sponsored position, and compacted rows
equal to a library gather on the device.
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


def _prm(w):
    return ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, span_L=w.span_L, sponsor_B=w.sponsor_B,
                     rho=w.rho, alpha=w.alpha, beta=w.beta, gamma=w.gamma)


def _check_full(w, K, sample_units, gather_units):
    td = wl.make_tokens(w)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    prm = _prm(w)
    seq = _dev(td.seq_len) if w.ragged else None
    plan = ta.ta_evict(_dev(td.tok), td.tab_ids, td.tab_len, Q, Kc, Vc, K, prm, seq_len=seq)
    torch.cuda.synchronize()
    G = w.hq // w.hkv
    scored = w.alpha != 0.0
    lens = torch.from_numpy(td.seq_len).to(DEV)

    # ---- properties over every unit ------------------------------------------------------
    seqs = {}
    for b in range(w.batch):
        nb = int(td.seq_len[b])
        a, s, v = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len)
        seqs[b] = (a, s, v)
        assert np.array_equal(plan.anchor[b, :nb].cpu().numpy(), a)
        assert np.array_equal(plan.spons[b, :nb].cpu().numpy(), s)
        assert np.array_equal(plan.vouch[b, :nb].cpu().numpy().view(np.uint32), v.view(np.uint32))
        assert sorted(np.flatnonzero(a).tolist()) == sorted(td.planted[b])        # clean stream
    if scored:
        sums = plan.A.double().sum(-1)                                            # [Lyr][B][Hkv]
        live = torch.clamp(lens, max=w.window).double().view(1, -1, 1)
        assert torch.allclose(sums, G * live.expand_as(sums), rtol=2e-4)
        idx_all, cnt_all = plan.idx, plan.cnt
        want_cnt = torch.clamp(lens, max=K).view(1, -1, 1).expand_as(cnt_all)
    else:
        idx_all, cnt_all = plan.idx, plan.cnt
        want_cnt = torch.clamp(lens, max=K)
    assert torch.equal(cnt_all.long(), want_cnt.long())
    if int(td.seq_len.min()) >= K:
        assert bool((idx_all[..., 1:] > idx_all[..., :-1]).all())                 # ascending, unique
        assert bool((idx_all[..., :w.n_sink] == torch.arange(w.n_sink, device=DEV)).all())
        if not w.ragged:
            recent = torch.arange(w.n - w.n_recent, w.n, device=DEV)
            assert bool((idx_all[..., K - w.n_recent:] == recent).all())
    fits = all(w.n_sink + w.n_recent + 6 * len(td.planted[b]) <= K for b in range(w.batch))
    if fits:                                                                      # Thm. 2: spans always kept
        for b in range(w.batch):
            want = torch.tensor(sorted(p + k for p in td.planted[b] for k in range(1, 7)), device=DEV)
            rows = idx_all[:, b] if scored else idx_all[b:b + 1]
            flat = rows.reshape(-1, K)
            for r in flat[:: max(1, flat.shape[0] // 16)]:
                assert bool(torch.isin(want, r).all())

    # ---- compacted rows against a device gather ----------------------------------------------
    for (l, b, g) in gather_units:
        sel = (plan.idx[l, b, g] if scored else plan.idx[b])[: int(td.seq_len[b]) if td.seq_len[b] < K else K].long()
        assert torch.equal(plan.Kout[l, b, g, :len(sel)].view(torch.int16), Kc[l, b, g].index_select(0, sel).view(torch.int16))
        assert torch.equal(plan.Vout[l, b, g, :len(sel)].view(torch.int16), Vc[l, b, g].index_select(0, sel).view(torch.int16))

    # ---- sampled units against the oracle ---------------------------------------------------------
    refs = {}
    for (l, b, g) in sample_units:
        nb = int(td.seq_len[b])
        a, s, v = seqs[b]
        if scored:
            A_gpu = plan.A[l, b, g, :nb].cpu().numpy()
            A_ref = ora.score(wl.bf16_bits(Q[l, b, g * G:(g + 1) * G]), wl.bf16_bits(Kc[l, b, g, :nb]))
            assert np.all(np.abs(A_gpu - A_ref) <= 1e-3 * np.abs(A_ref) + 1e-7), (l, b, g)
            ref = ora.select(A_gpu, a, s, v, K, w.n_sink, w.n_recent, w.alpha, w.beta, w.gamma)
            got = plan.idx[l, b, g, :len(ref)].cpu().numpy()
        else:
            ref = ora.select(None, a, s, v, K, w.n_sink, w.n_recent, 0.0, w.beta, w.gamma)
            got = plan.idx[b, :len(ref)].cpu().numpy()
        assert np.array_equal(got, ref), (l, b, g)
        assert np.array_equal(wl.bf16_bits(plan.Kout[l, b, g, :len(ref)]), ora.compact(wl.bf16_bits(Kc[l, b, g]), ref))
        assert np.array_equal(wl.bf16_bits(plan.Vout[l, b, g, :len(ref)]), ora.compact(wl.bf16_bits(Vc[l, b, g]), ref))
        refs[(l, b, g)] = (A_ref if scored else None, ref, ora.compact(wl.bf16_bits(Kc[l, b, g]), ref),
                           ora.compact(wl.bf16_bits(Vc[l, b, g]), ref))
    return plan, td, refs


@pytest.mark.parametrize("K", [16, 1024])
def test_c2_full_model_all_32_layers(K):
    w = wl.CONFIGS["c2_full_model"]
    units = [(0, 0, 0), (7, 0, 3), (19, 0, 6), (31, 0, 7)]
    _check_full(w, K, units, [(l, 0, g) for l in range(0, 32, 5) for g in (1, 4)])


def test_c3_ta_fast_full():
    w = wl.CONFIGS["c3_ta_fast"]
    print("c3: generating 64 GiB of K/V", flush=True)
    units = [(0, 0, 0), (13, 5, 2), (31, 15, 7)]
    _check_full(w, 512, units, [(l, b, g) for (l, b, g) in [(1, 1, 1), (9, 7, 3), (22, 12, 5), (30, 3, 0)]])


def test_c4_long_context_full():
    w = wl.CONFIGS["c4_long_context"]
    print("c4: generating 64 GiB of K/V", flush=True)
    _check_full(w, 1024, [(0, 0, 0), (31, 3, 7)], [(5, 1, 2), (17, 2, 6)])


def test_c5_agentic_full_prefill_and_decode_steps():
    w = wl.CONFIGS["c5_agentic_prefill"]
    print("c5: generating 128 GiB of K/V", flush=True)
    K = 256
    sample = [(0, 0, 0), (15, 31, 4), (31, 63, 7)]
    plan, td, refs = _check_full(w, K, sample, [(3, 10, 2), (20, 40, 5)])
    prm = _prm(w)
    steps = 3
    cap = w.n + 16
    st = ta.DecodeState(w.layers, w.batch, w.hq, w.hkv, K, cap, DEV)
    ta.ta_decode_init(st, _dev(td.tok), plan.anchor, plan.idx, plan.cnt, plan.Kout, plan.Vout, prm,
                      seq_len=_dev(td.seq_len), A=plan.A)
    torch.cuda.synchronize()
    G = w.hq // w.hkv
    # oracle state of the sampled units, from the oracle's own prefill
    seqs = {b: ora.DecodeSeq(td.tok[b, :int(td.seq_len[b])], td.tab_ids, td.tab_len, cap) for (_, b, _) in sample}
    units = {}
    for key in sample:
        A_ref, idx_ref, Krows, Vrows = refs[key]
        units[key] = ora.DecodeUnit(Krows, Vrows, idx_ref, A_ref[idx_ref])
    stream = wl.make_decode_stream(w, td, steps, p_anchor=0.02)
    evicted = torch.zeros((w.layers, w.batch, w.hkv), dtype=torch.int32, device=DEV)
    for t in range(steps):
        q, kn, vn = wl.make_decode_qkv(w, t, device=DEV)
        ta.ta_decode_step(st, _dev(stream[t]), q, kn, vn, td.tab_ids, td.tab_len, prm, evicted=evicted)
        torch.cuda.synchronize()
        # every unit: exactly one free slot, one eviction, K occupied
        assert bool(((st.pos < 0).sum(-1) == 1).all())
        assert bool((evicted >= 0).all())
        for b in seqs:
            seqs[b].append(int(stream[t, b]))
        for (l, b, g), u in units.items():
            pos_before = u.pos.copy()
            gA = st.A[l, b, g].cpu().numpy()
            e, _ = u.step(seqs[b], wl.bf16_bits(q[l, b, g * G:(g + 1) * G]), wl.bf16_bits(kn[l, b, g]),
                          wl.bf16_bits(vn[l, b, g]), seqs[b].len - 1, w.n_sink, w.n_recent, rank_A=gA)
            ev_pos = seqs[b].len - 1 if pos_before[e] < 0 else int(pos_before[e])
            assert int(evicted[l, b, g]) == ev_pos
            assert np.array_equal(st.pos[l, b, g].cpu().numpy(), u.pos)
            occ = u.pos >= 0
            assert np.all(np.abs(gA[occ] - u.A[occ]) <= 1e-3 * np.abs(u.A[occ]) + 1e-6)
        for b in seqs:
            seqs[b].decay(0.9)


def test_score_run_to_run_identical_with_long_chunks():
    """Many units and one long chunk per workgroup (hundreds of pipelined stages): the column
    sums must not depend on wavefront timing."""
    w = wl.scaled(wl.CONFIGS["c5_agentic_prefill"], layers=8)
    td = wl.make_tokens(w)
    Q, Kc, _ = wl.make_qkv(w, device=DEV, with_v=False)
    seq = _dev(td.seq_len)
    prm = _prm(w)
    first = ta.ta_score(Q, Kc, prm, seq_len=seq).clone()
    for _ in range(3):
        again = ta.ta_score(Q, Kc, prm, seq_len=seq)
        torch.cuda.synchronize()
        assert torch.equal(first.view(torch.int32), again.view(torch.int32))
