"""GPU parity of the learned anchor detector and of the voucher expansion from given anchors
(Sec. 5.1: detector f(h) = sigmoid(W2 . GELU(W1 . h)), TA-Learned, TA-LearnRank) against the oracle.

The confidence is floating point: it is compared within a tolerance.  The anchor decision
conf > thr is an integer decided by a float, so both sides take it from the same fp32
confidences (the GPU's): flags, budgets, sponsor flags and vouchers are then bit-exact.  The
oracle's own confidences must lead to the same flags wherever they are not within the
tolerance of the threshold.
"""
import numpy as np
import pytest
import torch

import paper_2604_11288_amd as ta
from oracle import ta_oracle as ora
from paper_2604_11288_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# fp32 accumulation of exact bf16 products over d_model terms, fp32 erf / exp: the logit carries
# an absolute error of about 1e-5, and d conf / d logit = conf (1 - conf) <= conf
RTOL, ATOL = 1e-3, 1e-12


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _conf_ref(h, W1, W2, seq_len=None, rows=None):
    B, n, _ = h.shape
    hb, w1, w2 = wl.bf16_bits(h), wl.bf16_bits(W1), wl.bf16_bits(W2)
    out = np.zeros((B, n), np.float32)
    for b in range(B):
        nb = n if seq_len is None else int(seq_len[b])
        if nb:
            out[b, :nb] = ora.detect(hb[b, :nb], w1, w2)
    return out


def _close(got, ref):
    return np.abs(got.astype(np.float64) - ref) <= RTOL * np.abs(ref) + ATOL


def _check_decisions(conf, conf_ref, anchor, anchor_B, thr, rank, B, scale):
    for b in range(conf.shape[0]):
        a_ref, ab_ref = ora.confidence_anchors(conf[b], thr, rank, B=B, scale=scale)
        assert np.array_equal(anchor[b], a_ref)
        assert np.array_equal(anchor_B[b].view(np.uint32), ab_ref.view(np.uint32))
        a_own, _ = ora.confidence_anchors(conf_ref[b], thr, rank, B=B, scale=scale)
        clear = np.abs(conf_ref[b] - thr) > RTOL * thr + 1e-6
        assert np.array_equal(anchor[b][clear], a_own[clear])


@pytest.mark.parametrize("m", [32, 64, 128, 256])
@pytest.mark.parametrize("rank", [False, True])
def test_detect_matches_oracle(m, rank):
    B, n, dm = 2, 700, 256                     # 1400 positions: five full tiles of 256 and a ragged one
    h, W1, W2 = wl.make_detector_inputs(B, n, dm, m, seed=wl.BASE_SEED + m, p_anchor=0.1, device=DEV)
    seq_len = np.array([700, 431], np.int32)
    prm = ta.Params(n_sink=4, n_recent=4)
    thr, scale = (0.3, 1.0) if rank else (0.5, 1.0)
    conf, anchor, anchor_B = ta.ta_detect_anchors(h, W1, W2, prm, thr, rank, scale, seq_len=_dev(seq_len))
    torch.cuda.synchronize()
    conf, anchor, anchor_B = conf.cpu().numpy(), anchor.cpu().numpy(), anchor_B.cpu().numpy()
    ref = _conf_ref(h, W1, W2, seq_len)
    assert _close(conf, ref).all(), np.abs(conf - ref).max()
    assert 10 < anchor.sum() < 0.2 * B * n
    assert not conf[1, 431:].any() and not anchor[1, 431:].any() and not anchor_B[1, 431:].any()
    _check_decisions(conf, ref, anchor, anchor_B, thr, rank, 15.0, scale)


def test_detect_wide_model_strided_rows_and_scaled_budgets():
    # d_model of an 8B model, rows padded to a larger stride, LearnRank with a budget scale
    B, n, dm, m = 1, 515, 4096, 128
    h, W1, W2 = wl.make_detector_inputs(B, n, dm, m, p_anchor=0.1, device=DEV, row_stride=dm + 64)
    assert h.stride(1) == dm + 64
    prm = ta.Params(n_sink=4, n_recent=4, sponsor_B=11.0)
    conf, anchor, anchor_B = ta.ta_detect_anchors(h, W1, W2, prm, 0.3, True, 15.0)
    conf2, anchor2, anchor_B2 = ta.ta_detect_anchors(h, W1, W2, prm, 0.5, False)
    torch.cuda.synchronize()
    ref = _conf_ref(h, W1, W2)
    for c, a, ab, thr, rank, scale in ((conf, anchor, anchor_B, 0.3, True, 15.0), (conf2, anchor2, anchor_B2, 0.5, False, 1.0)):
        c, a, ab = c.cpu().numpy(), a.cpu().numpy(), ab.cpu().numpy()
        assert _close(c, ref).all(), np.abs(c - ref).max()
        _check_decisions(c, ref, a, ab, thr, rank, 11.0, scale)
    assert set(np.unique(anchor_B2.cpu().numpy())) == {0.0, 11.0}


def test_detect_tiny_inputs():
    prm = ta.Params(n_sink=0, n_recent=0)
    for B, n, dm, m in ((1, 1, 32, 32), (3, 5, 64, 64), (1, 257, 32, 256)):
        h, W1, W2 = wl.make_detector_inputs(B, n, dm, m, p_anchor=0.3, device=DEV)
        conf, anchor, anchor_B = ta.ta_detect_anchors(h, W1, W2, prm, 0.5, False)
        torch.cuda.synchronize()
        ref = _conf_ref(h, W1, W2)
        assert _close(conf.cpu().numpy(), ref).all()
    # every sequence empty: all outputs zero
    h, W1, W2 = wl.make_detector_inputs(2, 40, 64, 32, device=DEV)
    conf, anchor, anchor_B = ta.ta_detect_anchors(h, W1, W2, prm, 0.5, False, seq_len=_dev(np.zeros(2, np.int32)))
    torch.cuda.synchronize()
    assert not conf.any() and not anchor.any() and not anchor_B.any()


def test_detect_rejects_unsupported_shapes():
    prm = ta.Params(n_sink=4, n_recent=4)
    h, W1, W2 = wl.make_detector_inputs(1, 64, 64, 32, device=DEV)
    with pytest.raises(ta.TaError):            # hidden width outside {32, 64, 128, 256}
        ta.ta_detect_anchors(h, torch.zeros((48, 64), dtype=torch.bfloat16, device=DEV),
                             torch.zeros(48, dtype=torch.bfloat16, device=DEV), prm, 0.5, False)
    with pytest.raises(ta.TaError):            # d_model not a multiple of 32
        ta.ta_detect_anchors(h[:, :, :48], W1[:, :48].contiguous(), W2, prm, 0.5, False)
    with pytest.raises(ta.TaError):            # threshold not finite
        ta.ta_detect_anchors(h, W1, W2, prm, float("nan"), False)
    hp = torch.zeros((1, 64, 72), dtype=torch.bfloat16, device=DEV)[:, :, 4:68]
    with pytest.raises(ta.TaError):            # rows not 16-byte aligned
        ta.ta_detect_anchors(hp, W1, W2, prm, 0.5, False)


@pytest.mark.parametrize("L", [0, 6, 64])
def test_expand_from_given_anchors_matches_oracle(L):
    rng = np.random.default_rng(77 + L)
    B, n = 3, 2333                              # three tiles per sequence, n not a multiple of 4
    seq_len = np.array([2333, 1024, 7], np.int32)
    anchor = (rng.random((B, n)) < 0.04).astype(np.uint8)
    anchor[0, 1000:1040] = 1                    # a dense run across a tile border
    anchor[:, 0] = 1
    anchor[0, n - 1] = 1
    anchor *= rng.integers(1, 256, size=(B, n)).astype(np.uint8)     # any non-zero byte is a flag
    budgets = (rng.random((B, n)) * 20).astype(np.float32)
    prm = ta.Params(n_sink=4, n_recent=4, span_L=L, sponsor_B=15.0)
    for ab in (None, budgets):
        spons, vouch = ta.ta_expand_vouchers(_dev(anchor), prm, anchor_B=None if ab is None else _dev(ab),
                                             seq_len=_dev(seq_len))
        torch.cuda.synchronize()
        spons, vouch = spons.cpu().numpy(), vouch.cpu().numpy()
        for b in range(B):
            nb = int(seq_len[b])
            s_ref, v_ref = ora.expand((anchor[b, :nb] != 0).astype(np.uint8), L=L, B=15.0,
                                      anchor_B=None if ab is None else ab[b, :nb])
            assert np.array_equal(spons[b, :nb], s_ref)
            assert np.array_equal(vouch[b, :nb].view(np.uint32), v_ref.view(np.uint32))
            assert not spons[b, nb:].any() and not vouch[b, nb:].any()


def test_expand_equals_table_match_on_its_own_anchors():
    # step 2 from the flags the table match produced gives the match's own sponsor flags and vouchers
    w = wl.scaled(wl.CONFIGS["c5_agentic_prefill"], layers=1, batch=4, n=5000, ragged=(1500, 5000))
    td = wl.make_tokens(w, clean=False)
    prm = ta.Params(n_sink=w.n_sink, n_recent=w.n_recent)
    seq_len = _dev(td.seq_len)
    anchor, spons, vouch = ta.ta_match_anchors(_dev(td.tok), td.tab_ids, td.tab_len, prm, seq_len=seq_len)
    spons2, vouch2 = ta.ta_expand_vouchers(anchor, prm, seq_len=seq_len)
    torch.cuda.synchronize()
    assert torch.equal(spons, spons2) and torch.equal(vouch.view(torch.int32), vouch2.view(torch.int32))


@pytest.mark.parametrize("rank", [False, True])
def test_learned_detection_through_selection(rank):
    # detector -> vouchers -> protected top-K, against the same chain of the oracle on the GPU's confidences
    B, n, dm, m, K = 2, 900, 128, 64, 48
    h, W1, W2 = wl.make_detector_inputs(B, n, dm, m, seed=wl.BASE_SEED + 91, p_anchor=0.03, device=DEV)
    seq_len = np.array([900, 640], np.int32)
    prm = ta.Params(n_sink=4, n_recent=4, alpha=0.0)
    thr = 0.3 if rank else 0.5
    conf, anchor, anchor_B = ta.ta_detect_anchors(h, W1, W2, prm, thr, rank, seq_len=_dev(seq_len))
    spons, vouch = ta.ta_expand_vouchers(anchor, prm, anchor_B=anchor_B, seq_len=_dev(seq_len))
    idx, cnt = ta.ta_select(None, anchor, spons, vouch, K, prm, 1, 1, seq_len=_dev(seq_len))
    torch.cuda.synchronize()
    conf, idx, cnt = conf.cpu().numpy(), idx.cpu().numpy(), cnt.cpu().numpy()
    for b in range(B):
        nb = int(seq_len[b])
        a_ref, ab_ref = ora.confidence_anchors(conf[b, :nb], thr, rank)
        s_ref, v_ref = ora.expand(a_ref, anchor_B=ab_ref)
        if rank:                                 # vouchers are confidence * 0.8^k here: below 1
            assert 0 < v_ref.max() < 3.0
        idx_ref = ora.select(None, a_ref, s_ref, v_ref, K, 4, 4, 0.0, 0.5, 0.3)
        assert cnt[0, b, 0] == len(idx_ref)
        assert np.array_equal(idx[0, b, 0, :len(idx_ref)], idx_ref)
