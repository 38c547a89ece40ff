"""Pins of the learned-detector part of the oracle (Sec. 5.1): the detector equation
f(h) = sigmoid(W2 . GELU(W1 . h)) and the TA-Learned / TA-LearnRank rules.

Nothing here calls the GPU.  The pins: closed forms of GELU and of the logistic function,
a one-hidden-unit special case worked by hand with math.erf, a library evaluation of the
same network in float64 (torch's own matmul / gelu / sigmoid), the threshold rules, and
the voucher equation of TA-LearnRank written out for a tiny case.
"""
import math

import numpy as np
import torch

from oracle import ta_oracle as ora


def _bf16(a):
    """float array -> (bf16 bit patterns uint16, the exactly representable values as float64)."""
    t = torch.as_tensor(np.asarray(a, np.float32)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    return bits, t.to(torch.float64).numpy()


def test_detector_zero_weights_give_one_half_and_saturation():
    h, _ = _bf16(np.random.default_rng(0).normal(size=(5, 16)))
    W1, _ = _bf16(np.zeros((4, 16)))
    W2, _ = _bf16(np.ones(4))
    assert np.all(ora.detect(h, W1, W2) == 0.5)                   # GELU(0) = 0, sigmoid(0) = 1/2
    # one hidden unit that copies h[0] * 8: GELU(x) -> x for large x, -> 0 for very negative x
    hb, hv = _bf16([[4.0], [-4.0], [0.0]])
    W1, _ = _bf16([[8.0]])
    W2, _ = _bf16([1.0])
    c = ora.detect(hb, W1, W2)
    assert c[0] == 1.0                                             # sigmoid(32) rounds to 1 in fp32
    assert abs(float(c[1]) - 0.5) < 1e-6 and c[1] <= 0.5           # GELU(-32) = -0 -> sigmoid = 1/2
    assert c[2] == 0.5


def test_detector_one_unit_worked_by_hand():
    # f = sigmoid(w2 * GELU(w1 . h)) with GELU(z) = z/2 (1 + erf(z / sqrt 2)), values exact in bf16
    hb, hv = _bf16([[0.5, -1.0, 2.0, 0.25]])
    W1b, W1v = _bf16([[1.0, 0.5, 0.75, -2.0]])
    W2b, W2v = _bf16([-1.5])
    z = float(np.dot(hv[0], W1v[0]))                              # 0.5 - 0.5 + 1.5 - 0.5 = 1.0
    assert z == 1.0
    gelu = 0.5 * z * (1.0 + math.erf(z / math.sqrt(2.0)))         # 0.8413447...
    want = 1.0 / (1.0 + math.exp(1.5 * gelu))
    got = float(ora.detect(hb, W1b, W2b)[0])
    assert abs(got - want) < 1e-7
    assert abs(gelu - 0.8413447460685429) < 1e-12                 # Phi(1) = 0.84134474...


def test_detector_against_torch_float64():
    rng = np.random.default_rng(3)
    n, dm, m = 37, 96, 24
    hb, hv = _bf16(rng.normal(size=(n, dm)))
    W1b, W1v = _bf16(rng.normal(size=(m, dm)) / np.sqrt(dm))
    W2b, W2v = _bf16(rng.normal(size=m))
    ref = torch.sigmoid(torch.nn.functional.gelu(torch.from_numpy(hv) @ torch.from_numpy(W1v).T)
                        @ torch.from_numpy(W2v)).numpy()
    got = ora.detect(hb, W1b, W2b)
    assert np.max(np.abs(got - ref)) < 1e-7
    # a transposed W1 or a dropped GELU would not pass: check that they differ from the reference
    lin = torch.sigmoid((torch.from_numpy(hv) @ torch.from_numpy(W1v).T) @ torch.from_numpy(W2v)).numpy()
    assert np.max(np.abs(lin - ref)) > 1e-3


def test_threshold_rules_of_learned_and_learnrank():
    conf = np.array([0.2, 0.3, 0.30000004, 0.5, 0.50000006, 0.9], np.float32)
    a, b = ora.confidence_anchors(conf, thr=0.5, rank=False, B=15.0)       # TA-Learned: conf > 0.5, budget B
    assert a.tolist() == [0, 0, 0, 0, 1, 1] and b.tolist() == [0, 0, 0, 0, 15.0, 15.0]
    a, b = ora.confidence_anchors(conf, thr=0.3, rank=True)                # TA-LearnRank: conf > 0.3, budget conf
    assert a.tolist() == [0, 0, 1, 1, 1, 1]
    assert np.array_equal(b[2:], conf[2:]) and not b[:2].any()
    a, b = ora.confidence_anchors(conf, thr=0.3, rank=True, scale=15.0)
    assert np.array_equal(b[2:], np.float32(15.0) * conf[2:])


def test_learnrank_vouchers_are_the_printed_sum():
    # V_j = sum_i f(h_i) 0.8^(j-i) 1[f(h_i) > 0.3, i < j <= i + L]: two competing anchors, the more
    # confident one protects its followers more
    conf = np.zeros(20, np.float32)
    conf[3], conf[5], conf[12] = 0.9, 0.4, 0.25                            # the last one is below 0.3
    a, b = ora.confidence_anchors(conf, thr=0.3, rank=True)
    s, V = ora.expand(a, L=6, rho=0.8, anchor_B=b)
    for j in range(20):
        want = sum(float(conf[i]) * 0.8 ** (j - i) for i in (3, 5) if i < j <= i + 6)
        assert abs(float(V[j]) - want) < 1e-6
        assert s[j] == (1 if want > 0 else 0)
    assert abs(float(V[4]) - 0.72) < 1e-6 and abs(float(V[6]) - 0.7808) < 1e-6 and V[13] == 0
