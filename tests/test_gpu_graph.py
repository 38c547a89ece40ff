"""The entry points only enqueue work on the given stream (no allocation, no synchronisation,
no memset nodes), so a pass can be captured into a HIP graph and replayed: every replay must
give what the eager call gives."""
import numpy as np
import pytest
import torch

import paper_2604_11288_amd as ta
from paper_2604_11288_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _outputs(plan):
    outs = [plan.anchor, plan.spons, plan.vouch, plan.idx, plan.cnt]
    if plan.A is not None:
        outs.append(plan.A)
    outs += list(plan.Kout) if isinstance(plan.Kout, list) else [plan.Kout]
    outs += list(plan.Vout) if isinstance(plan.Vout, list) else [plan.Vout]
    return outs


@pytest.mark.parametrize("form", ["stacked", "layers", "attention_free"])
def test_captured_pass_replays_to_the_eager_result(form):
    w = wl.scaled(wl.CONFIGS["c2_full_model"], layers=3, batch=2, n=1500, hq=8, hkv=2, window=32,
                  ragged=(400, 1500), planted=6)
    td = wl.make_tokens(w, clean=False)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    alpha = 0.0 if form == "attention_free" else 1.0
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, alpha=alpha)
    tok, seq = _dev(td.tok), _dev(td.seq_len)
    K = 200
    if form == "layers":
        Ql = [Q[l].clone() for l in range(w.layers)]
        Kl = [Kc[l].clone() for l in range(w.layers)]
        Vl = [Vc[l].clone() for l in range(w.layers)]
        plan = ta.LayerEvictPlan(tok, td.tab_ids, td.tab_len, Ql, Kl, Vl, K, prm, seq_len=seq)
    else:
        plan = ta.EvictPlan(tok, td.tab_ids, td.tab_len, Q if alpha else None, Kc, Vc, K, prm, seq_len=seq)
    plan.run()                                              # eager: also the one-time attribute set-up of the launchers
    torch.cuda.synchronize()
    want = [t.clone() for t in _outputs(plan)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            plan.run()                                      # the binding launches on the current (capturing) stream
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in _outputs(plan):                            # eager work between the replays: wipe the outputs
            t.fill_(-1) if t is plan.idx else t.zero_()     # (index rows start as -1, rows past cnt are not written)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(_outputs(plan), want):
            assert torch.equal(got, ref), (form, replay)


@pytest.mark.parametrize("K", [120, 400])                  # 400: more slots than a wavefront's registers hold - four wavefronts per unit
def test_captured_decode_step_replays_like_eager_steps(K):
    # one generation step captured once; before every replay the step's inputs are copied into the
    # captured buffers.  Two states from the same prefill, one stepped eagerly, one by replays.
    w = wl.scaled(wl.CONFIGS["c5_agentic_prefill"], layers=2, batch=3, n=700, hq=8, hkv=2, ragged=(200, 700))
    td = wl.make_tokens(w, clean=False)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent)
    tok, seq = _dev(td.tok), _dev(td.seq_len)
    steps = 6
    plan = ta.ta_evict(tok, td.tab_ids, td.tab_len, Q, Kc, Vc, K, prm, seq_len=seq)
    states = []
    for _ in range(2):
        st = ta.DecodeState(w.layers, w.batch, w.hq, w.hkv, K, w.n + steps + 4, DEV)
        ta.ta_decode_init(st, tok, plan.anchor, plan.idx, plan.cnt, plan.Kout, plan.Vout, prm, seq_len=seq, A=plan.A)
        states.append(st)
    eager, replayed = states
    stream_tok = wl.make_decode_stream(w, td, steps + 1, p_anchor=0.2, clean=False)
    inputs = [(_dev(stream_tok[t]),) + tuple(wl.make_decode_qkv(w, t, device=DEV)) for t in range(steps + 1)]
    ev_e = torch.zeros((w.layers, w.batch, w.hkv), dtype=torch.int32, device=DEV)
    ev_r = torch.zeros_like(ev_e)
    # step 0 eagerly on both (also the launchers' one-time set-up)
    for st, ev in ((eager, ev_e), (replayed, ev_r)):
        t0, q0, k0, v0 = inputs[0]
        ta.ta_decode_step(st, t0, q0, k0, v0, td.tab_ids, td.tab_len, prm, evicted=ev)
    torch.cuda.synchronize()
    buf = [x.clone() for x in inputs[1]]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    snapshot = {k: getattr(replayed, k).clone() for k in ("tok", "len", "anchor", "budget", "vouch", "spons", "Kc", "Vc", "pos", "A")}
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ta.ta_decode_step(replayed, buf[0], buf[1], buf[2], buf[3], td.tab_ids, td.tab_len, prm, evicted=ev_r)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for k, v in snapshot.items():                           # capture records, it does not run: the state is as before
        assert torch.equal(getattr(replayed, k), v), k
    for t in range(1, steps + 1):
        tt, q, kn, vn = inputs[t]
        ta.ta_decode_step(eager, tt, q, kn, vn, td.tab_ids, td.tab_len, prm, evicted=ev_e)
        for dst, src in zip(buf, inputs[t]):
            dst.copy_(src)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ev_r, ev_e), t
        for k in ("len", "anchor", "budget", "vouch", "spons", "pos", "A", "Kc", "Vc"):
            assert torch.equal(getattr(replayed, k), getattr(eager, k)), (k, t)
