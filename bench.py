#!/usr/bin/env python3
"""Benchmark of the TA eviction pass on one MI355X.

One step = one full eviction pass (anchor match + vouchers, window attention
scores, protected top-K, K/V gather) over all 32 layers of a workload, through
the fused C-ABI entry point.  The headline workload is the largest of the five
configurations, the long-context one (4 sequences of 131 072 positions, window
64, K = 1024); the other four and the generation step of the agentic one are
measured after it and reported as named sub-objects of the same line, each with
its own roofline.  Inputs are synthetic and resident in HBM before the timed
region starts.  Prints ONE JSON line.
"""
import argparse
import dataclasses
import gc
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
HEADLINE = "c4_long_context"


def kv_bytes_per_pass(w, budget, seq_len=None):
    """Bytes of KV the pass must move: K read once for scoring + K/V rows gathered and written.
    Ragged batches count the live positions of each sequence, not the padded length."""
    per_seq = w.layers * w.hkv
    row = w.d * 2
    lens = [w.n] * w.batch if seq_len is None else [min(int(x), w.n) for x in seq_len]
    score = per_seq * sum(lens) * row if w.alpha != 0.0 else 0
    compact = per_seq * sum(min(budget, x) for x in lens) * row * 2 * 2     # two tensors, read + write
    return score, compact


# HBM bytes of one score step (both sweeps) from FETCH_SIZE / WRITE_SIZE counter runs (summaries
# under profiles/), scaled by the factor the same counters show for a plain device copy of known
# size.  A figure belongs to one version of the score kernels: it is reported only while their
# sources still hash to what was profiled, and is null otherwise.
SCORE_TRAFFIC = {
    "c4_long_context": {      # profiles/evict_pass_c4_long_context_K1024.txt
        "bytes_per_step": 69.40e9,
        "sources": {
            "ta_score.hip": "d586b676b008b66c77dcd736a4dda21b8437eed7104d9782f522f756f6b1b06c",
            "ta_score_common.h": "3e4b78495a5669b06b80090303e2ac50ab9622f4b9ead1de520e8aee81424db4",
            "ta_match_device.h": "37bdb219a8d33ec055dec043135dc59baa6bb3078a260fc18fd0d5fdc3f6b979",
        },
    },
    "c2_full_model": {        # profiles/score_two_sweep_c2_full_model_K1024.txt
        "bytes_per_step": 559.4e6,
        "sources": {
            "ta_score.hip": "d586b676b008b66c77dcd736a4dda21b8437eed7104d9782f522f756f6b1b06c",
            "ta_score_common.h": "3e4b78495a5669b06b80090303e2ac50ab9622f4b9ead1de520e8aee81424db4",
            "ta_match_device.h": "37bdb219a8d33ec055dec043135dc59baa6bb3078a260fc18fd0d5fdc3f6b979",
        },
    },
}


def measured_score_traffic(workload):
    rec = SCORE_TRAFFIC.get(workload)
    if rec is None:
        return None
    csrc = os.path.join(ROOT, "paper_2604_11288_amd", "csrc")
    for name, digest in rec["sources"].items():
        try:
            with open(os.path.join(csrc, name), "rb") as f:
                if hashlib.sha256(f.read()).hexdigest() != digest:
                    return None
        except OSError:
            return None
    return rec["bytes_per_step"]


def describe(w):
    return ("%s: %d layers, batch %d, n=%d, %dq/%dkv heads, d=%d, window %d, sinks %d, recent %d"
            % (w.name, w.layers, w.batch, w.n, w.hq, w.hkv, w.d, w.window, w.n_sink, w.n_recent))


def free_device_memory(torch):
    gc.collect()
    torch.cuda.empty_cache()


class Bench:
    """Inputs, plan and measurements of one workload."""

    def __init__(self, ta, wl, torch, np, w, budget, dev, copies=1):
        self.ta, self.wl, self.torch, self.np = ta, wl, torch, np
        self.w, self.budget, self.dev = w, budget, dev
        self.td = wl.make_tokens(w)
        self.tok = torch.from_numpy(self.td.tok).to(dev)
        self.seq = torch.from_numpy(self.td.seq_len).to(dev) if w.ragged else None
        self.prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, span_L=w.span_L, sponsor_B=w.sponsor_B,
                             rho=w.rho, alpha=w.alpha, beta=w.beta, gamma=w.gamma)
        self.scored = w.alpha != 0.0
        self.G = w.hq // w.hkv
        self.units = w.layers * w.batch * w.hkv
        # `copies` > 1: the same inputs at several addresses, visited in turn, so that a repeat is
        # not served from the last-level cache (for workloads smaller than that cache)
        self.inputs, self.plans = [], []
        for c in range(copies):
            Q, K, V = wl.make_qkv(w, device=dev)
            self.inputs.append((Q, K, V))
            self.plans.append(ta.EvictPlan(self.tok, self.td.tab_ids, self.td.tab_len, Q, K, V, budget, self.prm,
                                           seq_len=self.seq))
        self.Q, self.K, self.V = self.inputs[0]
        self.plan = self.plans[0]
        self.stream = torch.cuda.current_stream()
        self.score_b, self.compact_b = kv_bytes_per_pass(w, budget, self.td.seq_len)

    # ---- wall time of the fused pass --------------------------------------------------------
    def wall_us(self, warmup, steps, rotate=False):
        torch = self.torch
        plans = self.plans if rotate else [self.plan]
        for i in range(warmup):
            plans[i % len(plans)].run(self.stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            plans[i % len(plans)].run(self.stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / steps

    # ---- per-kernel durations: the same steps issued stage by stage, HIP events on the launch stream
    def stage_us(self, warmup, steps):
        ta, torch, np, w, plan, prm, td = self.ta, self.torch, self.np, self.w, self.plan, self.prm, self.td
        stream, seq, budget, scored = self.stream, self.seq, self.budget, self.scored
        names = ["match_expand"] + (["score"] if scored else []) + ["select", "compact"]
        ev = {k: [] for k in names}

        def timed(name, fn):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            ev[name].append((e0, e1))

        sel_layers, sel_hkv = (w.layers, w.hkv) if scored else (1, 1)
        for it in range(warmup + steps):
            if it == warmup:
                ev = {k: [] for k in names}
            timed("match_expand", lambda: ta.ta_match_anchors(self.tok, td.tab_ids, td.tab_len, prm, seq_len=seq,
                                                              out=(plan.anchor, plan.spons, plan.vouch), stream=stream))
            if scored:
                timed("score", lambda: ta.ta_score(self.Q, self.K, prm, seq_len=seq, A=plan.A, ws=plan.ws, stream=stream))
            timed("select", lambda: ta.ta_select(plan.A, plan.anchor, plan.spons, plan.vouch, budget, prm,
                                                 sel_layers, sel_hkv, seq_len=seq, out=(plan.idx, plan.cnt), stream=stream))
            timed("compact", lambda: ta.ta_compact(self.K, self.V, plan.idx, plan.cnt, budget, idx_shared=not scored,
                                                   out=(plan.Kout, plan.Vout), stream=stream))
        torch.cuda.synchronize()
        # median over the steps: a host hiccup between an event and its launch does not count as kernel time
        return {k: 1e3 * float(np.median([a.elapsed_time(b) for a, b in v])) for k, v in ev.items()}

    # ---- roofline of the dominant kernel ---------------------------------------------
    def score_alg(self):
        w, td = self.w, self.td
        live = sum(min(int(x), w.n) for x in td.seq_len) * w.layers * w.hkv          # key rows that exist
        alg_bytes = live * (w.d * 2 + 4) + self.units * self.G * w.window * w.d * 2  # K once, A written once, Q once
        alg_flops = 2 * self.G * w.window * live * w.d                               # one Q K^T
        return alg_bytes, alg_flops

    def roofline(self, kern_us):
        w = self.w
        if self.scored:
            alg_bytes, alg_flops = self.score_alg()
            dur = kern_us["score"] * 1e-6
            achieved = alg_bytes / dur / 1e9
            return {"kernel": "score (stats sweep + column-sum sweep)", "bound": "hbm", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": measured_score_traffic(w.name),
                    "avg_launch_us": round(kern_us["score"], 2),
                    "mfma_tflops": round(alg_flops / dur / 1e12, 1),
                    "mfma_frac": round(alg_flops / dur / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
        dur = kern_us["compact"] * 1e-6
        achieved = self.compact_b / dur / 1e9
        return {"kernel": "compact", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "avg_launch_us": round(kern_us["compact"], 2)}

    def step_rooflines(self, kern_us):
        """Algorithmic bytes of the other steps over their durations (fractions of the HBM peak)."""
        w, td = self.w, self.td
        live_tok = sum(min(int(x), w.n) for x in td.seq_len)
        sel_units = self.units if self.scored else w.batch
        per_pos = (4 + 4 + 2) if self.scored else (4 + 2)
        live_pos = live_tok * (w.layers * w.hkv if self.scored else 1)
        out = {"match_expand": live_tok * 10, "select": live_pos * per_pos + sel_units * self.budget * 4,
               "compact": self.compact_b}
        return {k: {"GB/s": round(b / kern_us[k] / 1e3, 1), "hbm_frac": round(b / kern_us[k] / 1e3 / HBM_PEAK_GBS, 4)}
                for k, b in out.items()}

    # ---- one-sweep score: row normalisers taken from the prefill attention kernel ----------------
    def one_sweep(self, warmup, steps):
        ta, torch, np, w, td = self.ta, self.torch, self.np, self.w, self.td
        dev, stream, seq, prm, plan = self.dev, self.stream, self.seq, self.prm, self.plan
        G, W = self.G, w.window
        lse = torch.empty((w.layers, w.batch, w.hq, W), dtype=torch.float32, device=dev)
        for l in range(w.layers):
            for b in range(w.batch):
                nb = int(td.seq_len[b])
                hidden = torch.arange(nb, device=dev)[None, :] > (nb - W + torch.arange(W, device=dev))[:, None]
                tail = max(0, nb - W)                       # keys before `tail` are visible to every row
                for g in range(w.hkv):
                    q = self.Q[l, b, g * G:(g + 1) * G].float().reshape(G * W, w.d)
                    S = (q @ self.K[l, b, g, :nb].float().T) / w.d ** 0.5
                    S = S.view(G, W, nb)
                    S[:, :, tail:].masked_fill_(hidden[None, :, tail:], float("-inf"))
                    lse[l, b, g * G:(g + 1) * G] = torch.logsumexp(S, dim=-1)
                    del S
        A2 = torch.empty_like(plan.A)
        for _ in range(max(2, warmup)):
            ta.ta_score_lse(self.Q, self.K, lse, prm, seq_len=seq, A=A2, stream=stream)
        pairs = []
        for _ in range(max(steps, 5)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            ta.ta_score_lse(self.Q, self.K, lse, prm, seq_len=seq, A=A2, stream=stream)
            e1.record(stream)
            pairs.append((e0, e1))
        torch.cuda.synchronize()
        us1 = 1e3 * float(np.median([a.elapsed_time(b) for a, b in pairs]))
        live = torch.arange(w.n, device=dev).view(1, 1, 1, -1) < torch.from_numpy(td.seq_len).to(dev).view(1, -1, 1, 1)
        rel = float((((A2 - plan.A).abs() / (plan.A.abs() + 1e-7)) * live).max())
        # the whole pass with the one-sweep score (the match tiles ride with the column-sum sweep)
        plan1 = ta.EvictPlan(self.tok, td.tab_ids, td.tab_len, self.Q, self.K, self.V, self.budget, prm, seq_len=seq, lse=lse)
        for _ in range(warmup):
            plan1.run(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan1.run(stream)
        torch.cuda.synchronize()
        pass1_us = (time.perf_counter() - t0) * 1e6 / steps
        alg_bytes, alg_flops = self.score_alg()
        return {"entry_point": "ta_score_lse / ta_evict_lse", "score_us": round(us1, 2),
                "score_GB/s": round(alg_bytes / us1 / 1e3, 1),
                "score_hbm_frac": round(alg_bytes / us1 / 1e3 / HBM_PEAK_GBS, 4),
                "score_mfma_frac": round(alg_flops / us1 / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                "max_rel_diff_to_two_sweep": float("%.2e" % rel),
                "pass_us": round(pass1_us, 1), "pass_GB/s": round((self.score_b + self.compact_b) / pass1_us / 1e3, 1)}

    # ---- incremental form: append / accumulate / evict-one / decay, per generation step ---------
    def decode_step(self, nsteps, page_size=0):
        """Generation steps after a pass.  page_size > 0: the K + 1 slots of every unit live in a page pool
        (pages of `page_size` slots behind a block table); the pass's retained rows are compacted straight
        into those pages (timed, reported as compact_into_pages_us) and the state takes them in place."""
        ta, torch, wl, w, td, plan = self.ta, self.torch, self.wl, self.w, self.td, self.plan
        dev, stream, budget = self.dev, self.stream, self.budget
        cap = w.n + nsteps + 16
        into_us = None
        if page_size > 0:
            Kp, Vp, table, num_pages, strides = wl.make_slot_pool(w.layers, w.batch, w.hkv, w.d, budget + 1, page_size, dev)
            pool = ta.PagedKV(Kp, Vp, torch.from_numpy(table).to(dev), page_size, num_pages, strides, w.layers, w.batch,
                              w.hkv, budget + 1)
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 5
            ta.ta_compact_into_pages(self.K, self.V, plan.idx, plan.cnt, budget, pool, stream=stream)
            c0.record(stream)
            for _ in range(reps):
                ta.ta_compact_into_pages(self.K, self.V, plan.idx, plan.cnt, budget, pool, stream=stream)
            c1.record(stream)
            torch.cuda.synchronize()
            into_us = c0.elapsed_time(c1) * 1e3 / reps
            st = ta.DecodeState(w.layers, w.batch, w.hq, w.hkv, budget, cap, dev, pages=pool)
            ta.ta_decode_init(st, self.tok, plan.anchor, plan.idx, plan.cnt, None, None, self.prm, seq_len=self.seq, A=plan.A)
        else:
            st = ta.DecodeState(w.layers, w.batch, w.hq, w.hkv, budget, cap, dev)
            ta.ta_decode_init(st, self.tok, plan.anchor, plan.idx, plan.cnt, plan.Kout, plan.Vout, self.prm, seq_len=self.seq, A=plan.A)
        warm = min(8, nsteps)
        toks = torch.from_numpy(wl.make_decode_stream(w, td, warm + nsteps, p_anchor=0.02)).to(dev)
        q1, k1, v1 = wl.make_decode_qkv(w, 0, device=dev)
        evicted = torch.zeros((w.layers, w.batch, w.hkv), dtype=torch.int32, device=dev)
        for t in range(warm):
            ta.ta_decode_step(st, toks[t], q1, k1, v1, td.tab_ids, td.tab_len, self.prm, evicted=evicted, stream=stream)
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record(stream)
        for t in range(warm, warm + nsteps):
            ta.ta_decode_step(st, toks[t], q1, k1, v1, td.tab_ids, td.tab_len, self.prm, evicted=evicted, stream=stream)
        d1.record(stream)
        torch.cuda.synchronize()
        step_us = d0.elapsed_time(d1) * 1e3 / nsteps
        row_bytes = self.units * (budget + 1) * w.d * 2              # every slot's key row once per step
        paged = {} if page_size <= 0 else {"slot_page_size": page_size, "compact_into_pages_us": round(into_us, 1),
                                           "compact_into_pages_GB/s": round(self.compact_b / into_us / 1e3, 1)}
        return {**paged, "us_per_step": round(step_us, 1), "steps": nsteps, "units": self.units, "slots": budget + 1,
                "key_rows_GB/s": round(row_bytes / step_us / 1e3, 1),
                "hbm_frac": round(row_bytes / step_us / 1e3 / HBM_PEAK_GBS, 4),
                "roofline": {"kernel": "decode_unit_kernel (+ the per-sequence kernels of the step)", "bound": "hbm",
                             "achieved": round(row_bytes / step_us / 1e3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(row_bytes / step_us / 1e3 / HBM_PEAK_GBS, 4), "traffic": None}}

    # ---- how close every unit's cut is to flipping: the margin output of the selection, all units -------
    def cut_margins(self):
        """Selects once more with the margin output on (not timed) and counts, over ALL units of the workload,
        those whose smallest retained and largest evicted utility lie within the parity tolerance of each
        other: the units where a retained set may legitimately differ from the oracle's."""
        ta, torch, w, plan = self.ta, self.torch, self.w, self.plan
        layers, hkv = (w.layers, w.hkv) if self.scored else (1, 1)
        prm = dataclasses.replace(self.prm, margin=torch.empty((layers * w.batch * hkv, 2), device=self.dev))
        ta.ta_select(plan.A if self.scored else None, plan.anchor, plan.spons, plan.vouch, self.budget, prm,
                     layers, hkv, seq_len=self.seq)
        torch.cuda.synchronize()
        m = prm.margin.double().cpu().numpy()
        cut = self.np.isfinite(m).all(axis=1)                  # units that evict and keep something of the cut's class
        gap = (m[cut, 0] - m[cut, 1]) / self.np.abs(m[cut, 0])
        return {"units": int(m.shape[0]), "units_with_a_cut": int(cut.sum()),
                "near_tie_units_rel_gap_le_1e-3": int((gap <= 1e-3).sum()),
                "exact_tie_units": int((gap == 0).sum()),
                "median_rel_gap": float("%.3e" % self.np.median(gap)) if gap.size else None}

    # ---- the oracle: timed on the host cores and compared with the GPU's outputs -------------------
    def oracle_leg(self, single_s, multi_s):
        """Runs the CPU oracle on a bounded, seeded sample of this workload's units.
        Timing: one unit at a time on one core for about `single_s` seconds, then one unit per worker on
        all cores of this process for about `multi_s` seconds (the oracle itself is single-threaded).
        Every unit the oracle finished is also compared with the GPU's outputs of the pass."""
        from oracle import ta_oracle as ora
        ora.build()
        np, wl, w, td, plan, budget = self.np, self.wl, self.w, self.td, self.plan, self.budget
        G, scored = self.G, self.scored
        rng = np.random.default_rng(w.seed)
        order = [int(x) for x in rng.permutation(self.units)]
        seqs = {}
        for b in range(w.batch):
            nb = int(td.seq_len[b])
            seqs[b] = ora.evict_sequence(td.tok[b, :nb], td.tab_ids, td.tab_len, L=w.span_L, B=w.sponsor_B, rho=w.rho)

        def fetch(u):                                        # device -> host copies, outside the timing
            l, rem = divmod(u, w.batch * w.hkv)
            b, g = divmod(rem, w.hkv)
            nb = int(td.seq_len[b])
            return ((l, b, g), wl.bf16_bits(self.Q[l, b, g * G:(g + 1) * G]) if scored else None,
                    wl.bf16_bits(self.K[l, b, g, :nb]), wl.bf16_bits(self.V[l, b, g, :nb]),
                    plan.A[l, b, g, :nb].cpu().numpy() if scored else None,
                    (plan.idx[l, b, g] if scored else plan.idx[b]).cpu().numpy(),
                    wl.bf16_bits(plan.Kout[l, b, g]), wl.bf16_bits(plan.Vout[l, b, g]))

        def run(job):
            (l, b, g), Qb, Kb, Vb, A_gpu, idx_gpu, Ko, Vo = job
            nb = Kb.shape[0]
            a, s, v = seqs[b]
            c0 = time.perf_counter()
            A = ora.score(Qb, Kb) if scored else None
            idx = ora.select(A, a, s, v, budget, w.n_sink, w.n_recent, w.alpha, w.beta, w.gamma)
            Kr, Vr = ora.compact(Kb, idx), ora.compact(Vb, idx)
            dt = time.perf_counter() - c0
            # comparison with the GPU (not timed): scores, then the end-to-end selection with excused near-ties
            rel, excused, ok = 0.0, 0, True
            got = idx_gpu[:len(idx)]
            if scored:
                err = np.abs(A_gpu.astype(np.float64) - A)
                rel = float(np.max(err / (np.abs(A) + 1e-4)))     # the tolerance is 1e-3 |A| + 1e-7
                ok = bool(np.all(err <= 1e-3 * np.abs(A) + 1e-7))
                diff = set(idx.tolist()) ^ set(got.tolist())
                if diff:
                    u = ora.utility(A, a, v, w.alpha, w.beta, w.gamma)
                    cls = np.where(s.astype(bool), 1, 0)
                    p = np.arange(nb)
                    cls[(p < w.n_sink) | (p >= nb - w.n_recent)] = 2
                    bclass = cls[idx].min()
                    kth = u[idx][cls[idx] == bclass].min()
                    ok = ok and all(cls[q] == bclass and abs(u[q] - kth) <= 1e-3 * abs(kth) for q in diff)
                    excused = len(diff) // 2
                ok = ok and np.array_equal(Ko[:len(got)], ora.compact(Kb, got)) and np.array_equal(Vo[:len(got)], ora.compact(Vb, got))
            else:
                ok = np.array_equal(got, idx) and np.array_equal(Ko[:len(idx)], Kr) and np.array_equal(Vo[:len(idx)], Vr)
            return dt, rel, excused, bool(ok)

        results, pos = [], 0
        # one core
        t_single, n_single = 0.0, 0
        while pos < len(order) and (n_single == 0 or t_single < single_s):
            r = run(fetch(order[pos]))
            pos += 1
            results.append(r)
            t_single += r[0]
            n_single += 1
        per_unit = t_single / n_single
        per_unit_bytes = (self.score_b + self.compact_b) / self.units
        # every core: one unit per worker
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cores = max(1, min(cores, 16))
        n_multi = int(min(len(order) - pos, max(cores, multi_s * cores / max(per_unit, 1e-6))))
        multi = None
        if n_multi > 0 and cores > 1:
            jobs = [fetch(u) for u in order[pos:pos + n_multi]]
            c0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=cores) as pool:
                rs = list(pool.map(run, jobs))
            wall = time.perf_counter() - c0
            results += rs
            del jobs
            multi = {"value": round(n_multi * per_unit_bytes / wall / 1e9, 4), "unit": "GB/s", "cores": cores,
                     "sample": "%d units, one per worker thread, %.1f s wall" % (n_multi, wall)}
        cpu = {"value": round(n_single * per_unit_bytes / t_single / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "%d of %d units of %s at K=%d, one after the other on one core, %.1f s (copies to the host not timed)"
                         % (n_single, self.units, w.name, budget, t_single),
               "us_per_unit": round(per_unit * 1e6, 1),
               "us_per_pass_extrapolated": round(per_unit * 1e6 * self.units, 0),
               "all_cores": multi}
        parity = {"units_compared_with_oracle": len(results), "all_within_criteria": all(r[3] for r in results),
                  "excused_near_tie_selections": int(sum(r[2] for r in results)),
                  "max_rel_score_error": float("%.2e" % max(r[1] for r in results)) if scored else None}
        return cpu, parity


def measure_extra(ta, wl, torch, np, name, budget, dev, steps, warmup, copies=1, decode_steps=0, oracle_s=0.0,
                  decode_page_size=0):
    """One of the other workloads as a sub-object of the line."""
    w = wl.CONFIGS[name]
    b = Bench(ta, wl, torch, np, w, budget, dev, copies=copies)
    us = b.wall_us(warmup, steps)
    kern = b.stage_us(warmup, steps)
    out = {"workload": describe(w), "budget_K": budget, "us_per_pass": round(us, 1),
           "GB/s": round((b.score_b + b.compact_b) / us / 1e3, 1),
           "hbm_frac": round((b.score_b + b.compact_b) / us / 1e3 / HBM_PEAK_GBS, 4),
           "kernels_us": {k: round(v, 2) for k, v in kern.items()},
           "roofline": b.roofline(kern), "steps_vs_hbm": b.step_rooflines(kern)}
    if copies > 1:
        cold = b.wall_us(warmup, steps, rotate=True)
        out["us_per_pass_rotating_%d_input_copies" % copies] = round(cold, 1)
    extra = None
    if decode_steps > 0 and b.scored:
        b.plan.run(b.stream)
        torch.cuda.synchronize()
        extra = b.decode_step(decode_steps)
        if decode_page_size > 0:
            extra["paged_slots"] = b.decode_step(decode_steps, decode_page_size)
    if oracle_s > 0:
        b.plan.run(b.stream)
        torch.cuda.synchronize()
        _, parity = b.oracle_leg(oracle_s / 2, oracle_s / 2)
        parity["cut_margins_all_units"] = b.cut_margins()
        out["parity"] = parity
    del b
    free_device_memory(torch)
    return out, extra


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--budget", type=int, default=0, help="retention budget K of the timed steps (default: the workload's largest)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the named workload: skip the sub-objects of the other configurations (profiling runs)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the budget sweeps of the full-model workload")
    ap.add_argument("--rotate", type=int, default=0, metavar="COPIES",
                    help="time the named workload over this many copies of its inputs visited in turn (a repeat is "
                         "then not served from the last-level cache); the sub-objects of the small workloads do so anyway")
    ap.add_argument("--decode-steps", type=int, default=0,
                    help="also time this many generation steps of the incremental form after the pass "
                         "(needs a scored workload; reported as decode_step)")
    ap.add_argument("--decode-paged", type=int, default=0, metavar="PAGE_SIZE",
                    help="with --decode-steps: keep the state's K/V slots in a page pool of this page size (rows "
                         "compacted straight into the pages, state initialised in place)")
    ap.add_argument("--score-lse", action="store_true",
                    help="also time the one-sweep score from given row log-sum-exps (what a flash-style prefill "
                         "kernel leaves behind; computed here with torch, outside the timing; reported as score_one_sweep; "
                         "always on for the headline workload unless --no-extras)")
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
    ap.add_argument("--match-stress-tokens", type=int, default=0,
                    help="also time the anchor match + voucher expansion alone on this many tokens of unrestricted "
                         "IDs (256 sequences; the shape on which that step is bound by memory; reported as match_stress)")
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
    if args.query_heads > 0 or args.window > 0:
        w = wl.scaled(w, hq=args.query_heads or w.hq, window=args.window or w.window,
                      name="%s with %d query heads, window %d" % (w.name, args.query_heads or w.hq, args.window or w.window))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ta.ta_init()
    budget = args.budget or max(w.budgets)
    bench = Bench(ta, wl, torch, np, w, budget, dev, copies=max(1, args.rotate))
    td, Q, K, V, tok, seq, prm, plan, stream = (bench.td, bench.Q, bench.K, bench.V, bench.tok, bench.seq, bench.prm,
                                                bench.plan, bench.stream)
    scored = bench.scored
    score_b, compact_b = bench.score_b, bench.compact_b

    # ---- headline: K steps of the fused pass -----------------------------------------
    us_per_pass = bench.wall_us(args.warmup, args.steps, rotate=args.rotate > 1)
    ms_per_step = us_per_pass * 1e-3
    value = (score_b + compact_b) / (ms_per_step * 1e-3) / 1e9
    kern_us = bench.stage_us(args.warmup, args.steps)
    roofline = bench.roofline(kern_us)
    step_fracs = bench.step_rooflines(kern_us)
    sel_layers, sel_hkv = (w.layers, w.hkv) if scored else (1, 1)
    full_run = args.workload == HEADLINE and not args.no_extras

    one_sweep = None
    if scored and (args.score_lse or full_run):
        one_sweep = bench.one_sweep(min(args.warmup, 3), min(args.steps, 10))

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

    if args.calibrate_copy:
        src = torch.empty(1 << 27, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # 256 MiB read + 256 MiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst

    # ---- budget sweep of the named workload when it has several budgets ---------------------------
    sweep = {}
    for kb in (() if (args.no_sweep or len(w.budgets) < 2) else w.budgets):
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

    decode = None
    decode_steps = args.decode_steps if args.decode_steps > 0 else (0 if args.no_extras else 32)   # the headline reports its step too
    if decode_steps > 0 and scored:
        plan.run(stream)                                        # the state starts from the outputs of a pass at this budget
        torch.cuda.synchronize()
        decode = bench.decode_step(decode_steps, args.decode_paged)

    # ---- anchor match + voucher expansion alone on a shape that is bound by memory ---------------
    match_stress = None
    if args.match_stress_tokens > 0:
        sB = 256
        sn = max(1024, args.match_stress_tokens // sB)
        g = torch.Generator(device=dev).manual_seed(w.seed + 17)
        stok = torch.randint(0, wl.VOCAB, (sB, sn), dtype=torch.int32, device=dev, generator=g)
        outs = ta.ta_match_anchors(stok, td.tab_ids, td.tab_len, prm, stream=stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record(stream)
        for _ in range(reps):
            ta.ta_match_anchors(stok, td.tab_ids, td.tab_len, prm, out=outs, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        m_us = e0.elapsed_time(e1) * 1e3 / reps
        m_bytes = sB * sn * 10                                 # 4 B read, 1 + 1 + 4 B written per token
        match_stress = {"tokens": sB * sn, "sequences": sB, "table_entries": int(len(td.tab_len)), "us": round(m_us, 1),
                        "anchors": int(outs[0].sum()),
                        "roofline": {"kernel": "match_expand_kernel", "bound": "hbm", "achieved": round(m_bytes / m_us / 1e3, 1),
                                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(m_bytes / m_us / 1e3 / HBM_PEAK_GBS, 4),
                                     "traffic": None}}
        del stok, outs

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
        dm, E, Vr = args.detect_dmodel, args.embed_concepts, args.embed_rows
        emb, C = wl.make_embedding_inputs(Vr, dm, E, device=dev)
        outs = ta.ta_embed_anchors(emb[None], C, 0.5, stream=stream)
        tokv = tok % Vr
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
        e_bytes = Vr * dm * 2
        embed = {"rows": Vr, "d_model": dm, "concepts": E, "tau": 0.5,
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

    # ---- CPU baseline: the oracle as it stands on a bounded sample, and the parity of that sample ----
    cpu, parity = None, None
    if not args.no_cpu_baseline:
        plan.run(stream)                                        # the outputs of the fused pass at this budget
        torch.cuda.synchronize()
        cpu, parity = bench.oracle_leg(single_s=10.0, multi_s=8.0)
        parity["cut_margins_all_units"] = bench.cut_margins()

    config = {"workload": describe(w), "budget_K": budget, "entry_point": "ta_evict"}
    if args.rotate > 1:
        config["input_copies_visited_in_turn"] = args.rotate

    # ---- the other configurations as sub-objects (the headline's tensors are released first) --------
    workloads = None
    if full_run:
        del bench, plan, Q, K, V, tok, seq, td
        free_device_memory(torch)
        st, wu = min(args.steps, 10), min(args.warmup, 3)
        ora_s = 0.0 if args.no_cpu_baseline else 1.0
        workloads = {}
        workloads["c1_single_layer"], _ = measure_extra(ta, wl, torch, np, "c1_single_layer", 16, dev, max(st, 20), max(wu, 5),
                                                        copies=3, oracle_s=2 * ora_s)
        c2 = {}
        for kb in ((1024,) if args.no_sweep else wl.CONFIGS["c2_full_model"].budgets):
            # at the largest budget also the generation step of one sequence: 256 units of 1025 slots, which run
            # several wavefronts per unit
            c2["K=%d" % kb], c2_step = measure_extra(ta, wl, torch, np, "c2_full_model", kb, dev, max(st, 20), max(wu, 5), copies=3,
                                                     oracle_s=4 * ora_s if kb == 1024 else 0.0,
                                                     decode_steps=32 if kb == 1024 else 0, decode_page_size=0)
            if c2_step is not None:
                workloads["c2_full_model_decode_step"] = c2_step
        workloads["c2_full_model"] = c2
        workloads["c3_ta_fast"], _ = measure_extra(ta, wl, torch, np, "c3_ta_fast", 512, dev, st, wu, oracle_s=2 * ora_s)
        workloads["c5_agentic_prefill"], workloads["c5_agentic_decode_step"] = measure_extra(
            ta, wl, torch, np, "c5_agentic_prefill", 256, dev, st, wu, decode_steps=32, oracle_s=4 * ora_s, decode_page_size=16)

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
        "config": config,
        "us_per_pass": round(ms_per_step * 1e3, 1),
        "hbm_frac": round(value / HBM_PEAK_GBS, 4),
        "kernels_us": {k: round(v, 2) for k, v in kern_us.items()},
        "steps_vs_hbm": step_fracs,
        "budget_sweep": sweep,
        "score_one_sweep": one_sweep,
        "paged": paged_out, "layer_tensors": layers_out,
        "decode_step": decode,
        "match_stress": match_stress,
        "learned_detect": detect,
        "embedding_detect": embed,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
        "workloads": workloads,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
