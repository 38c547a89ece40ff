#!/usr/bin/env python3
"""Benchmark of the TA eviction pass on one MI355X.

One step = one full eviction pass (anchor match + vouchers, window attention
scores, protected top-K, K/V gather) over all 32 layers of the full-model
workload, through the fused C-ABI entry point.  Inputs are synthetic and
resident in HBM before the timed region starts.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def kv_bytes_per_pass(w, budget, seq_len=None):
    """Bytes of KV the pass must move: K read once for scoring + K/V rows gathered and written.
    Ragged batches count the live positions of each sequence, not the padded length."""
    per_seq = w.layers * w.hkv
    row = w.d * 2
    lens = [w.n] * w.batch if seq_len is None else [min(int(x), w.n) for x in seq_len]
    score = per_seq * sum(lens) * row if w.alpha != 0.0 else 0
    compact = per_seq * sum(min(budget, x) for x in lens) * row * 2 * 2     # two tensors, read + write
    return score, compact


# HBM bytes of one score step (both sweeps) from the FETCH_SIZE / WRITE_SIZE counter runs whose
# summary is profiles/score_two_sweep_c2_full_model_K1024.txt, scaled by the copy-kernel factor.
# The figure belongs to one version of the score kernels: it is reported only while their
# sources still hash to what was profiled, and is null otherwise.
SCORE_TRAFFIC = {
    "workload": "c2_full_model",
    "bytes_per_step": 559.4e6,
    "sources": {
        "ta_score.hip": "3d4c1d0d73c0a6bcc86fbff7ae068b3f33b1357248de3595f22667017ae339f7",
        "ta_score_common.h": "3e4b78495a5669b06b80090303e2ac50ab9622f4b9ead1de520e8aee81424db4",
        "ta_match_device.h": "ea1c659034745b1c86ea139df7a64bd4b0e33ccf9b061b77a80be957bb4e3717",
    },
}


def measured_score_traffic(workload, budget):
    import hashlib
    if workload != SCORE_TRAFFIC["workload"]:
        return None
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2604_11288_amd", "csrc")
    for name, digest in SCORE_TRAFFIC["sources"].items():
        try:
            with open(os.path.join(csrc, name), "rb") as f:
                if hashlib.sha256(f.read()).hexdigest() != digest:
                    return None
        except OSError:
            return None
    return SCORE_TRAFFIC["bytes_per_step"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c2_full_model")
    ap.add_argument("--budget", type=int, default=1024, help="retention budget K of the timed steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the budget sweep (profiling runs)")
    ap.add_argument("--decode-steps", type=int, default=0,
                    help="also time this many generation steps of the incremental form after the pass "
                         "(needs a scored workload; reported as decode_step)")
    ap.add_argument("--score-lse", action="store_true",
                    help="also time the one-sweep score from given row log-sum-exps (what a flash-style prefill "
                         "kernel leaves behind; computed here with torch, outside the timing; reported as score_one_sweep)")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_SIZE",
                    help="also time scoring and compaction over a paged (block-table) copy of the same cache with "
                         "pages of this many positions (a multiple of 64; reported as paged)")
    ap.add_argument("--query-heads", type=int, default=0,
                    help="run the workload with this many query heads instead of its own (more heads per KV head: "
                         "more query rows per unit in the score step); the workload name in the output says so")
    ap.add_argument("--window", type=int, default=0,
                    help="run the workload with this many observation-window rows instead of its own")
    ap.add_argument("--layer-tensors", action="store_true",
                    help="also time the pass over the same cache kept as one tensor per layer (ta_evict_layers), "
                         "and the same work issued as one ta_evict call per layer (reported as layer_tensors)")
    ap.add_argument("--paged-heads-first", action="store_true",
                    help="pages laid out [heads][page_size][d] instead of [page_size][heads][d]")
    ap.add_argument("--detect-positions", type=int, default=0,
                    help="also time the learned anchor detector + voucher expansion on about this many positions "
                         "of synthetic last-layer hidden states (sequences of the workload's length; reported as "
                         "learned_detect)")
    ap.add_argument("--embed-rows", type=int, default=0,
                    help="also time embedding-based anchor detection (largest cosine to --embed-concepts concept "
                         "embeddings) over an embedding table of this many rows, and the per-token lookup of the "
                         "workload's token IDs (reported as embedding_detect)")
    ap.add_argument("--embed-concepts", type=int, default=16)
    ap.add_argument("--detect-dmodel", type=int, default=4096)
    ap.add_argument("--detect-hidden", type=int, default=128)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy kernel (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the eviction pass has no multi-GPU path in this build "
              "(units are independent; see DESIGN.md). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2604_11288_amd as ta
    from paper_2604_11288_amd import workloads as wl

    if not os.path.exists(ta.binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    ta.lib()

    w = wl.CONFIGS[args.workload]
    variant = args.workload
    if args.query_heads > 0 or args.window > 0:
        w = wl.scaled(w, hq=args.query_heads or w.hq, window=args.window or w.window,
                      name="%s with %d query heads, window %d" % (w.name, args.query_heads or w.hq, args.window or w.window))
        variant = w.name                     # not the profiled workload: no stored traffic figure
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    td = wl.make_tokens(w)
    Q, K, V = wl.make_qkv(w, device=dev)
    tok = torch.from_numpy(td.tok).to(dev)
    seq = torch.from_numpy(td.seq_len).to(dev) if w.ragged else None
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, span_L=w.span_L, sponsor_B=w.sponsor_B,
                    rho=w.rho, alpha=w.alpha, beta=w.beta, gamma=w.gamma)
    budget = args.budget
    plan = ta.EvictPlan(tok, td.tab_ids, td.tab_len, Q, K, V, budget, prm, seq_len=seq)
    stream = torch.cuda.current_stream()

    # ---- headline: K steps of the fused pass -----------------------------------------
    for _ in range(args.warmup):
        plan.run(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan.run(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    score_b, compact_b = kv_bytes_per_pass(w, budget, td.seq_len)
    value = (score_b + compact_b) / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel durations: the same steps issued stage by stage, HIP events on the launch stream
    scored = w.alpha != 0.0
    names = ["match_expand"] + (["score"] if scored else []) + ["select", "compact"]
    ev = {k: [] for k in names}

    def timed(name, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        ev[name].append((e0, e1))

    sel_layers, sel_hkv = (w.layers, w.hkv) if scored else (1, 1)
    for it in range(args.warmup + args.steps):
        if it == args.warmup:
            ev = {k: [] for k in names}
        timed("match_expand", lambda: ta.ta_match_anchors(tok, td.tab_ids, td.tab_len, prm, seq_len=seq,
                                                          out=(plan.anchor, plan.spons, plan.vouch), stream=stream))
        if scored:
            timed("score", lambda: ta.ta_score(Q, K, prm, seq_len=seq, A=plan.A, ws=plan.ws, stream=stream))
        timed("select", lambda: ta.ta_select(plan.A, plan.anchor, plan.spons, plan.vouch, budget, prm,
                                             sel_layers, sel_hkv, seq_len=seq, out=(plan.idx, plan.cnt), stream=stream))
        timed("compact", lambda: ta.ta_compact(K, V, plan.idx, plan.cnt, budget, idx_shared=not scored,
                                               out=(plan.Kout, plan.Vout), stream=stream))
    torch.cuda.synchronize()
    # median over the steps: a host hiccup between an event and its launch does not count as kernel time
    kern_us = {k: 1e3 * float(np.median([a.elapsed_time(b) for a, b in v])) for k, v in ev.items()}

    # ---- roofline of the dominant kernel ---------------------------------------------
    units = w.layers * w.batch * w.hkv
    G = w.hq // w.hkv
    if scored:
        # algorithmic traffic of scoring: K once, Q once, A written once
        live = sum(min(int(x), w.n) for x in td.seq_len) * w.layers * w.hkv      # key rows that exist
        alg_bytes = live * (w.d * 2 + 4) + units * G * w.window * w.d * 2
        alg_flops = 2 * G * w.window * live * w.d
        dom, dur = "score (stats sweep + column-sum sweep)", kern_us["score"] * 1e-6
        achieved = alg_bytes / dur / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": measured_score_traffic(variant, budget),
                    "avg_launch_us": round(kern_us["score"], 2),
                    "mfma_tflops": round(alg_flops / dur / 1e12, 1),
                    "mfma_frac": round(alg_flops / dur / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    else:
        alg_bytes = compact_b
        dur = kern_us["compact"] * 1e-6
        achieved = alg_bytes / dur / 1e9
        roofline = {"kernel": "compact", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                    "avg_launch_us": round(kern_us["compact"], 2)}

    # ---- one-sweep score: row normalisers taken from the prefill attention kernel ----------------
    one_sweep = None
    if args.score_lse and scored:
        lse = torch.empty((w.layers, w.batch, w.hq, w.window), dtype=torch.float32, device=dev)
        lens = torch.from_numpy(td.seq_len).to(dev)
        for l in range(w.layers):
            for b in range(w.batch):
                nb = int(td.seq_len[b])
                S = torch.einsum("hwd,hnd->hwn", Q[l, b].float(), K[l, b, :, :nb].float().repeat_interleave(G, dim=0))
                S = S / w.d ** 0.5
                vis = torch.arange(nb, device=dev)[None, :] <= (nb - w.window + torch.arange(w.window, device=dev))[:, None]
                lse[l, b] = torch.logsumexp(S.masked_fill(~vis[None], float("-inf")), dim=-1)
        A2 = torch.empty_like(plan.A)
        for _ in range(10):
            ta.ta_score_lse(Q, K, lse, prm, seq_len=seq, A=A2, stream=stream)
        pairs = []
        for _ in range(max(args.steps, 20)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            ta.ta_score_lse(Q, K, lse, prm, seq_len=seq, A=A2, stream=stream)
            e1.record(stream)
            pairs.append((e0, e1))
        torch.cuda.synchronize()
        us1 = 1e3 * float(np.median([a.elapsed_time(b) for a, b in pairs]))
        rel = float(((A2 - plan.A).abs() / (plan.A.abs() + 1e-7)).max())
        # the whole pass with the one-sweep score (the match tiles ride with the column-sum sweep)
        plan1 = ta.EvictPlan(tok, td.tab_ids, td.tab_len, Q, K, V, budget, prm, seq_len=seq, lse=lse)
        for _ in range(args.warmup):
            plan1.run(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            plan1.run(stream)
        torch.cuda.synchronize()
        pass1_us = (time.perf_counter() - t0) * 1e6 / args.steps
        one_sweep = {"entry_point": "ta_score_lse / ta_evict_lse", "score_us": round(us1, 2),
                     "score_GB/s": round(alg_bytes / us1 / 1e3, 1),
                     "score_hbm_frac": round(alg_bytes / us1 / 1e3 / HBM_PEAK_GBS, 4),
                     "max_rel_diff_to_two_sweep": float("%.2e" % rel),
                     "pass_us": round(pass1_us, 1), "pass_GB/s": round((score_b + compact_b) / pass1_us / 1e3, 1)}
        del lse, A2, plan1

    # ---- the same cache behind a block table -----------------------------------------------------
    paged_out = None
    if args.paged > 0 and scored:
        Kp, Vp, table, num_pages, strides = wl.make_paged(K, V, args.paged, heads_first=args.paged_heads_first)
        pk = ta.PagedKV(Kp, Vp, table, args.paged, num_pages, strides, w.layers, w.batch, w.hkv, w.n)
        Ap = torch.empty_like(plan.A)
        outp = (torch.zeros_like(plan.Kout), torch.zeros_like(plan.Vout))
        evp = {"score": [], "compact": []}
        for it in range(10 + max(args.steps, 20)):
            if it == 10:
                evp = {"score": [], "compact": []}
            # the same sequence of launches as the stage-by-stage timing of the dense cache above
            for name, fn in (("match", lambda: ta.ta_match_anchors(tok, td.tab_ids, td.tab_len, prm, seq_len=seq,
                                                                   out=(plan.anchor, plan.spons, plan.vouch), stream=stream)),
                             ("score", lambda: ta.ta_score_paged(Q, pk, prm, seq_len=seq, A=Ap, ws=plan.ws, stream=stream)),
                             ("select", lambda: ta.ta_select(Ap, plan.anchor, plan.spons, plan.vouch, budget, prm,
                                                             sel_layers, sel_hkv, seq_len=seq, out=(plan.idx, plan.cnt),
                                                             stream=stream)),
                             ("compact", lambda: ta.ta_compact_paged(pk, plan.idx, plan.cnt, budget, out=outp, stream=stream))):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                fn()
                e1.record(stream)
                if name in evp:
                    evp[name].append((e0, e1))
        torch.cuda.synchronize()
        pus = {k: 1e3 * float(np.median([a.elapsed_time(b) for a, b in v])) for k, v in evp.items()}
        paged_out = {"page_size": args.paged, "pages": num_pages,
                     "page_layout": "[heads][page_size][d]" if args.paged_heads_first else "[page_size][heads][d]", "score_us": round(pus["score"], 2),
                     "compact_us": round(pus["compact"], 2),
                     "same_scores_as_dense": bool(torch.equal(Ap, plan.A)),
                     "same_rows_as_dense": bool(torch.equal(outp[0], plan.Kout) and torch.equal(outp[1], plan.Vout))}
        del Kp, Vp, pk, Ap, outp

    # ---- the same cache as one tensor per layer ---------------------------------------------------
    layers_out = None
    if args.layer_tensors:
        Ql = [Q[l].clone() for l in range(w.layers)] if scored else None
        Kl = [K[l].clone() for l in range(w.layers)]
        Vl = [V[l].clone() for l in range(w.layers)]
        lplan = ta.LayerEvictPlan(tok, td.tab_ids, td.tab_len, Ql, Kl, Vl, budget, prm, seq_len=seq)
        # one call per layer: what a caller without the pointer tables would issue
        singles = [ta.EvictPlan(tok, td.tab_ids, td.tab_len, Ql[l][None] if scored else None, Kl[l][None], Vl[l][None],
                                budget, prm, seq_len=seq) for l in range(w.layers)]

        def wall(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e6 / args.steps

        lus = wall(lambda: lplan.run(stream))
        sus = wall(lambda: [p.run(stream) for p in singles])
        same = all(torch.equal(lplan.Kout[l], plan.Kout[l]) and torch.equal(lplan.Vout[l], plan.Vout[l])
                   for l in range(w.layers)) and torch.equal(lplan.idx, plan.idx)
        layers_out = {"entry_point": "ta_evict_layers", "pass_us": round(lus, 1),
                      "pass_GB/s": round((score_b + compact_b) / lus / 1e3, 1),
                      "one_ta_evict_call_per_layer_us": round(sus, 1), "same_output_as_stacked": bool(same)}
        del Ql, Kl, Vl, lplan, singles

    # ---- budget sweep of the same workload (context, outside the headline timing) ----------
    sweep = {}
    if args.calibrate_copy:
        src = torch.empty(1 << 27, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # 256 MiB read + 256 MiB written by one elementwise kernel
        torch.cuda.synchronize()
    for kb in (() if args.no_sweep else w.budgets):
        p = plan if kb == budget else ta.EvictPlan(tok, td.tab_ids, td.tab_len, Q, K, V, kb, prm, seq_len=seq)
        for _ in range(3):
            p.run(stream)
        torch.cuda.synchronize()
        s0 = time.perf_counter()
        for _ in range(20):
            p.run(stream)
        torch.cuda.synchronize()
        us = (time.perf_counter() - s0) * 1e6 / 20
        sb, cb = kv_bytes_per_pass(w, kb, td.seq_len)
        sweep[str(kb)] = {"us_per_pass": round(us, 1), "GB/s": round((sb + cb) / us / 1e3, 1)}

    # ---- incremental form: append / accumulate / evict-one / decay, per generation step ---------
    decode = None
    if args.decode_steps > 0 and scored:
        cap = w.n + args.decode_steps + 16
        st = ta.DecodeState(w.layers, w.batch, w.hq, w.hkv, budget, cap, dev)
        ta.ta_decode_init(st, tok, plan.anchor, plan.idx, plan.cnt, plan.Kout, plan.Vout, prm, seq_len=seq, A=plan.A)
        warm = min(8, args.decode_steps)
        toks = torch.from_numpy(wl.make_decode_stream(w, td, warm + args.decode_steps, p_anchor=0.02)).to(dev)
        q1, k1, v1 = wl.make_decode_qkv(w, 0, device=dev)
        evicted = torch.zeros((w.layers, w.batch, w.hkv), dtype=torch.int32, device=dev)
        for t in range(warm):
            ta.ta_decode_step(st, toks[t], q1, k1, v1, td.tab_ids, td.tab_len, prm, evicted=evicted, stream=stream)
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record(stream)
        for t in range(warm, warm + args.decode_steps):
            ta.ta_decode_step(st, toks[t], q1, k1, v1, td.tab_ids, td.tab_len, prm, evicted=evicted, stream=stream)
        d1.record(stream)
        torch.cuda.synchronize()
        step_us = d0.elapsed_time(d1) * 1e3 / args.decode_steps
        row_bytes = units * (budget + 1) * w.d * 2              # every slot's key row once per step
        decode = {"us_per_step": round(step_us, 1), "steps": args.decode_steps,
                  "key_rows_GB/s": round(row_bytes / step_us / 1e3, 1),
                  "hbm_frac": round(row_bytes / step_us / 1e3 / HBM_PEAK_GBS, 4)}

    # ---- learned anchor detection (the confidence-weighted variant of steps 1+2) ----------------
    detect = None
    if args.detect_positions > 0:
        dB = max(1, args.detect_positions // w.n)
        dm, m = args.detect_dmodel, args.detect_hidden
        h, W1, W2 = wl.make_detector_inputs(dB, w.n, dm, m, device=dev)
        outs = ta.ta_detect_anchors(h, W1, W2, prm, 0.3, True, stream=stream)
        exp = ta.ta_expand_vouchers(outs[1], prm, anchor_B=outs[2], stream=stream)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        reps = 20
        ev[0].record(stream)
        for _ in range(reps):
            ta.ta_detect_anchors(h, W1, W2, prm, 0.3, True, out=outs, stream=stream)
        ev[1].record(stream)
        for _ in range(reps):
            ta.ta_expand_vouchers(outs[1], prm, anchor_B=outs[2], out=exp, stream=stream)
        ev[2].record(stream)
        torch.cuda.synchronize()
        det_us = ev[0].elapsed_time(ev[1]) * 1e3 / reps
        exp_us = ev[1].elapsed_time(ev[2]) * 1e3 / reps
        h_bytes = dB * w.n * dm * 2
        detect = {"positions": dB * w.n, "d_model": dm, "hidden": m, "rule": "TA-LearnRank (conf > 0.3, budget = conf)",
                  "detect_us": round(det_us, 1), "expand_us": round(exp_us, 1),
                  "h_GB/s": round(h_bytes / det_us / 1e3, 1), "hbm_frac": round(h_bytes / det_us / 1e3 / HBM_PEAK_GBS, 4),
                  "TFLOP/s": round(2.0 * dB * w.n * dm * m / det_us / 1e6, 1),
                  "anchors": int(outs[1].sum())}
        if not args.no_cpu_baseline:
            from oracle import ta_oracle as ora
            ora.build()
            rows = 256
            hb, w1b, w2b = wl.bf16_bits(h[0, :rows]), wl.bf16_bits(W1), wl.bf16_bits(W2)
            c0 = time.perf_counter()
            ora.detect(hb, w1b, w2b)
            detect["cpu_oracle_us_per_position"] = round((time.perf_counter() - c0) * 1e6 / rows, 1)
        del h, outs, exp

    # ---- embedding-based detection: the embedding table once, then a lookup per token -------------
    embed = None
    if args.embed_rows > 0:
        dm, E, V = args.detect_dmodel, args.embed_concepts, args.embed_rows
        emb, C = wl.make_embedding_inputs(V, dm, E, device=dev)
        outs = ta.ta_embed_anchors(emb[None], C, 0.5, stream=stream)
        tokv = tok % V
        lk = ta.ta_lookup_anchors(tokv, outs[1].view(-1), seq_len=seq, stream=stream)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        reps = 20
        ev[0].record(stream)
        for _ in range(reps):
            ta.ta_embed_anchors(emb[None], C, 0.5, out=outs, stream=stream)
        ev[1].record(stream)
        for _ in range(reps):
            ta.ta_lookup_anchors(tokv, outs[1].view(-1), seq_len=seq, out=lk, stream=stream)
        ev[2].record(stream)
        torch.cuda.synchronize()
        e_us = ev[0].elapsed_time(ev[1]) * 1e3 / reps
        l_us = ev[1].elapsed_time(ev[2]) * 1e3 / reps
        e_bytes = V * dm * 2
        embed = {"rows": V, "d_model": dm, "concepts": E, "tau": 0.5,
                 "embed_us": round(e_us, 1), "lookup_us": round(l_us, 1),
                 "x_GB/s": round(e_bytes / e_us / 1e3, 1), "hbm_frac": round(e_bytes / e_us / 1e3 / HBM_PEAK_GBS, 4),
                 "anchor_rows": int(outs[1].sum())}
        if not args.no_cpu_baseline:
            from oracle import ta_oracle as ora
            ora.build()
            rows = 256
            c0 = time.perf_counter()
            ora.cosine_sim(wl.bf16_bits(emb[:rows]), wl.bf16_bits(C))
            embed["cpu_oracle_us_per_row"] = round((time.perf_counter() - c0) * 1e6 / rows, 1)
        del emb, outs, lk

    # ---- CPU baseline: the oracle as it stands, one thread, on a bounded sample --------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ta_oracle as ora
        ora.build()
        max_units = min(units, 256)
        Kh = K.cpu() if K.numel() * 2 <= (1 << 30) else None
        sample = []
        for u in range(max_units):
            l, rem = divmod(u, w.batch * w.hkv)
            b, g = divmod(rem, w.hkv)
            sample.append((l, b, g))
        c0 = time.perf_counter()
        seqs = {}
        done = 0
        for (l, b, g) in sample:
            nb = int(td.seq_len[b])
            if b not in seqs:
                seqs[b] = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len, L=w.span_L,
                                             B=w.sponsor_B, rho=w.rho)
            a, s, v = seqs[b]
            Kunit = wl.bf16_bits(Kh[l, b, g, :nb] if Kh is not None else K[l, b, g, :nb])
            Vunit = wl.bf16_bits(V[l, b, g, :nb])
            A = None
            if scored:
                A = ora.score(wl.bf16_bits(Q[l, b, g * G:(g + 1) * G]), Kunit)
            idx = ora.select(A, a, s, v, budget, w.n_sink, w.n_recent, w.alpha, w.beta, w.gamma)
            ora.compact(Kunit, idx)
            ora.compact(Vunit, idx)
            done += 1
            if time.perf_counter() - c0 > 25.0:
                break
        cpu_s = time.perf_counter() - c0
        per_unit_bytes = (score_b + compact_b) / units
        cpu = {"value": round(done * per_unit_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": 1,
               "kind": "oracle",
               "sample": "%d of %d units of %s at K=%d (device->host copies of each unit included), %.1f s"
                         % (done, units, w.name, budget, cpu_s),
               "us_per_unit": round(cpu_s / done * 1e6, 1)}

    out = {
        "metric": "evict+compact GB/s of KV",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: %d layers, batch %d, n=%d, %dq/%dkv heads, d=%d, window %d, sinks %d, recent %d"
                               % (w.name, w.layers, w.batch, w.n, w.hq, w.hkv, w.d, w.window, w.n_sink, w.n_recent),
                   "budget_K": budget, "entry_point": "ta_evict"},
        "us_per_pass": round(ms_per_step * 1e3, 1),
        "hbm_frac": round(value / HBM_PEAK_GBS, 4),
        "kernels_us": {k: round(v, 2) for k, v in kern_us.items()},
        "budget_sweep": sweep,
        "score_one_sweep": one_sweep,
        "paged": paged_out, "layer_tensors": layers_out,
        "decode_step": decode,
        "learned_detect": detect,
        "embedding_detect": embed,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
