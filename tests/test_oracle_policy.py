"""Pins of the oracle's policy options: SnapKV-style max-pooling of the scores, the fixed budget
partition K = K_main + K_protected of Sec. 3.3, PyramidKV-style per-layer budgets, allowlist
filtering (Sec. 5.2), and the baselines of Sec. 4 as settings of the same selection."""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import ta_oracle as ora


def _ref_partition(u, spons, K, kp, ns, nr):
    """The partition written a second way: python sorts on (u, position) tuples."""
    n = len(u)
    mand = [p for p in range(n) if p < ns or p >= n - nr]
    rest = [p for p in range(n) if not (p < ns or p >= n - nr)]
    sp = sorted([p for p in rest if spons[p]], key=lambda p: (u[p], p), reverse=True)
    prot = sp[:max(0, min(kp, len(sp), K - len(mand)))]
    others = sorted([p for p in rest if p not in set(prot)], key=lambda p: (u[p], p), reverse=True)
    keep = mand + prot + others[:K - len(mand) - len(prot)]
    return sorted(keep[:K]) if K < n else list(range(n))


def test_maxpool_equals_torch_max_pool1d_and_hand_case():
    rng = np.random.default_rng(1)
    A = rng.random(257).astype(np.float32)
    for k in (1, 3, 5, 7, 9):
        ref = torch.nn.functional.max_pool1d(torch.tensor(A)[None, None], kernel_size=k, stride=1, padding=k // 2)[0, 0]
        assert np.array_equal(ora.maxpool(A, k), ref.numpy())
    assert np.array_equal(ora.maxpool(A, 1), A)
    hand = np.array([0, 5, 0, 0, 0, 0, 2, 0], np.float32)
    assert ora.maxpool(hand, 3).tolist() == [5, 5, 5, 0, 0, 2, 2, 2]
    assert ora.maxpool(hand, 5).tolist() == [5, 5, 5, 5, 2, 2, 2, 2]
    neg = np.array([-3, -1, -2], np.float32)                 # the padding never wins
    assert ora.maxpool(neg, 3).tolist() == [-1, -1, -1]


def test_partition_large_pool_equals_elastic_selection():
    rng = np.random.default_rng(2)
    n, K, ns, nr = 300, 64, 4, 6
    anchor = (rng.random(n) < 0.02).astype(np.uint8)
    spons, V = ora.expand(anchor)
    assert 0 < spons[ns:n - nr].sum() <= K - ns - nr            # the sponsored tokens fit
    A = (rng.random(n) * 30).astype(np.float32)                # some plain tokens outrank sponsored ones by u
    elastic = ora.select(A, anchor, spons, V, K, ns, nr)
    assert np.array_equal(ora.select_partition(A, anchor, spons, V, K, n, ns, nr), elastic)
    assert np.array_equal(ora.select_partition(A, anchor, spons, V, K, int(spons.sum()), ns, nr), elastic)
    # a smaller pool lets high-attention tokens displace the sponsored ones that are not protected
    small = ora.select_partition(A, anchor, spons, V, K, 2, ns, nr)
    assert not np.array_equal(small, elastic)


def test_partition_zero_pool_is_plain_topk_with_mandatory_tokens():
    rng = np.random.default_rng(3)
    n, K, ns, nr = 200, 24, 3, 5
    anchor = (rng.random(n) < 0.03).astype(np.uint8)
    spons, V = ora.expand(anchor)
    A = (rng.random(n) * 20).astype(np.float32)
    got = ora.select_partition(A, anchor, spons, V, K, 0, ns, nr)
    # the same as the elastic selection told that nothing is sponsored (vouchers still count in u)
    assert np.array_equal(got, ora.select(A, anchor, np.zeros(n, np.uint8), V, K, ns, nr))


@pytest.mark.parametrize("seed", range(6))
def test_partition_against_python_sort(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(12, 60))
    ns, nr = int(rng.integers(0, 3)), int(rng.integers(0, 4))
    K = int(rng.integers(ns + nr + 1, n + 3))
    anchor = (rng.random(n) < 0.15).astype(np.uint8)
    spons, V = ora.expand(anchor, L=3)
    A = (rng.integers(0, 6, n) * 2.0).astype(np.float32)       # many ties: the position breaks them
    u = np.zeros(n, np.float32)
    ora._load().ta_oracle_utility(ora._p(A), ora._p(anchor), ora._p(V), n, 1.0, 0.5, 0.3, ora._p(u))
    for kp in (0, 1, 2, 5, n):
        got = ora.select_partition(A, anchor, spons, V, K, kp, ns, nr).tolist()
        assert got == _ref_partition(u, spons, K, kp, ns, nr), (kp, K, ns, nr)


def test_partition_reproduces_the_budget_table_and_the_strict_configuration(golden_dir):
    # App. D: 4 sinks + 6 window + 6 protected at K = 16.  With K_protected = 4 (Sec. 3.3) four
    # sponsored tokens are protected and the other two win main-pool slots by utility; with
    # K_protected = 0 (the strict configuration of the ablation) all six do: same retained set.
    rows = [l.split() for l in open(os.path.join(golden_dir, "budget_partition_K16.txt")) if not l.startswith("#")]
    ta = [r for r in rows if r and r[0] == "TA-Fast"][0]
    sinks, win, L = int(ta[1]), int(ta[2]), int(ta[3])
    n = 4090
    anchor = np.zeros(n, np.uint8)
    anchor[2047] = 1
    spons, V = ora.expand(anchor, L=L)
    expect = [0, 1, 2, 3] + list(range(2048, 2054)) + list(range(4084, 4090))
    for kp in (4, 0, 6, 16):
        idx = ora.select_partition(None, anchor, spons, V, 16, kp, sinks, win, alpha=0.0)
        assert idx.tolist() == expect
    # with attention in play and a dormant span, the strict configuration loses what the pool keeps
    A = np.full(n, 50.0, np.float32)
    A[2048:2054] = 0
    kept4 = set(ora.select_partition(A, anchor, spons, V, 16, 4, sinks, win).tolist())
    kept0 = set(ora.select_partition(A, anchor, spons, V, 16, 0, sinks, win).tolist())
    assert set(range(2048, 2052)) <= kept4 and not (set(range(2048, 2054)) & kept0)


def test_layer_budgets():
    for layers, K, kmin in ((32, 1024, 64), (32, 16, 4), (5, 100, 1), (2, 7, 7), (28, 333, 17)):
        b = ora.layer_budgets(layers, K, kmin)
        assert b.sum() == layers * K
        assert np.all(np.diff(b) <= 0) and b[-1] == kmin
        assert abs(int(b[0]) - (2 * K - kmin)) <= layers          # the rounding residue sits in layer 0
        step = np.diff(b[1:].astype(np.int64))
        assert len(step) == 0 or step.max() - step.min() <= 1     # arithmetic up to rounding
    assert ora.layer_budgets(1, 50, 10).tolist() == [50]
    assert ora.layer_budgets(3, 10, 4).tolist() == [16, 10, 4]
    assert ora.layer_budgets(4, 9, 9).tolist() == [9, 9, 9, 9]


def test_allow_filter_and_injection_scenario():
    # anchors injected into an untrusted span would use up the protected slots; with the span
    # disallowed the legitimate span is retained again (Sec. 5.2)
    n, K, ns, nr = 400, 16, 4, 6
    anchor = np.zeros(n, np.uint8)
    anchor[100] = 1                                             # legitimate anchor, its value in 101..106
    anchor[200:260:3] = 1                                       # injected anchors, closer to the end
    allow = np.ones(n, np.uint8)
    allow[180:300] = 0
    assert ora.allow_filter(anchor, allow).nonzero()[0].tolist() == [100]
    assert ora.allow_filter(anchor * 9, allow * 3).tolist() == ora.allow_filter(anchor, allow).tolist()
    spons, V = ora.expand(anchor)
    lost = set(ora.select(None, anchor, spons, V, K, ns, nr, alpha=0.0).tolist())
    assert not set(range(101, 107)) <= lost                     # the pool overflowed with injected spans
    fa = ora.allow_filter(anchor, allow)
    spons, V = ora.expand(fa)
    kept = set(ora.select(None, fa, spons, V, K, ns, nr, alpha=0.0).tolist())
    assert set(range(101, 107)) <= kept


def test_baselines_as_settings():
    rng = np.random.default_rng(8)
    n, K = 500, 32
    z8, zf = np.zeros(n, np.uint8), np.zeros(n, np.float32)
    A = rng.random(n).astype(np.float32)
    # StreamingLLM / TOVA window: no table, no attention term: sinks + the most recent tokens
    idx = ora.select(None, z8, z8, zf, K, 4, 0, alpha=0.0, beta=0.5, gamma=0.0)
    assert idx.tolist() == [0, 1, 2, 3] + list(range(n - (K - 4), n))
    # H2O: heavy hitters by attention plus a recent window of K / 2, nothing else in the utility
    idx = ora.select(A, z8, z8, zf, K, 0, K // 2, alpha=1.0, beta=0.0, gamma=0.0)
    heavy = np.argsort(-A[:n - K // 2], kind="stable")[:K // 2]
    assert sorted(idx.tolist()) == sorted(heavy.tolist() + list(range(n - K // 2, n)))
    # SnapKV: the observation window is kept, the prefix is ranked by max-pooled attention
    W = 8
    pooled = ora.maxpool(A, 5)
    idx = ora.select(pooled, z8, z8, zf, K, 0, W, alpha=1.0, beta=0.0, gamma=0.0)
    order = sorted(range(n - W), key=lambda p: (pooled[p], p), reverse=True)[:K - W]
    assert idx.tolist() == sorted(order + list(range(n - W, n)))
