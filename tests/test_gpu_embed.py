"""GPU parity of embedding-based anchor detection (Sec. 3.2, third detector; TA-Fast-Embedding)
against the oracle: largest cosine within a tolerance; flags exact given the GPU's similarities
(and equal to the oracle's own wherever those are clear of the threshold); lookup by token ID,
voucher expansion and selection behind it bit-exact."""
import numpy as np
import pytest
import torch

import paper_2604_11288_amd as ta
from oracle import ta_oracle as ora
from paper_2604_11288_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# dot products and squared norms are fp32 sums of exact bf16 products over d_model terms
# (relative error about sqrt(d_model) * 2^-24 of |x||c|), then one division and one square root
RTOL, ATOL = 1e-3, 1e-5


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _check(sim, anchor, x, C, tau, valid=None):
    ref = ora.cosine_sim(wl.bf16_bits(x), wl.bf16_bits(C))
    sim, anchor = sim.cpu().numpy().reshape(-1), anchor.cpu().numpy().reshape(-1)
    if valid is not None:
        assert not sim[~valid].any() and not anchor[~valid].any()
        sim, anchor, ref = sim[valid], anchor[valid], ref[valid]
    assert np.all(np.abs(sim - ref) <= RTOL * np.abs(ref) + ATOL), np.abs(sim - ref).max()
    assert np.array_equal(anchor, ora.threshold_anchors(sim, tau))
    clear = np.abs(ref - tau) > RTOL * abs(tau) + ATOL
    assert np.array_equal(anchor[clear], ora.threshold_anchors(ref, tau)[clear])
    return sim, anchor


@pytest.mark.parametrize("E", [1, 5, 32, 33, 64, 100, 129, 256])
def test_largest_cosine_matches_oracle(E):
    V, dm = 1400, 256                          # five full tiles of 256 rows and a ragged one
    x, C = wl.make_embedding_inputs(V, dm, E, seed=wl.BASE_SEED + E, p_near=0.2, device=DEV)
    sim, anchor = ta.ta_embed_anchors(x[None], C, 0.6)
    torch.cuda.synchronize()
    sim, anchor = _check(sim, anchor, x, C, 0.6)
    assert 20 < anchor.sum() < 0.3 * V
    assert sim.max() > 0.95 and np.all(np.abs(sim) <= 1.0 + 1e-5)


def test_wide_rows_strided_and_ragged_sequences():
    B, n, dm, E = 3, 300, 4096, 24
    x, C = wl.make_embedding_inputs(B * n, dm, E, p_near=0.1, device=DEV, row_stride=dm + 32)
    assert x.stride(0) == dm + 32
    seq_len = np.array([300, 0, 77], np.int32)
    sim, anchor = ta.ta_embed_anchors(x.view(B, n, dm), C, 0.5, seq_len=_dev(seq_len))
    torch.cuda.synchronize()
    valid = (np.arange(n)[None, :] < seq_len[:, None]).reshape(-1)
    _check(sim, anchor, x, C, 0.5, valid=valid)


def test_degenerate_vectors():
    dm = 64
    rng = np.random.default_rng(3)
    base = torch.tensor(rng.standard_normal((6, dm)).astype(np.float32)).to(torch.bfloat16).to(DEV)
    x = base.clone()
    x[1] = 0                                   # zero input row: similarity 0
    x[2] = -base[0] * 2                        # opposite of concept 0
    C = torch.stack([base[0], torch.zeros(dm, dtype=torch.bfloat16, device=DEV)])   # one concept is the zero vector
    sim, anchor = ta.ta_embed_anchors(x[None], C, 0.9)
    torch.cuda.synchronize()
    s, a = _check(sim, anchor, x, C, 0.9)
    assert abs(s[0] - 1.0) < 1e-6 and s[1] == 0.0 and s[2] == 0.0 and a.tolist() == [1, 0, 0, 0, 0, 0]
    # without the zero concept the opposite row keeps its negative cosine (the maximum is not clamped at 0)
    sim, anchor = ta.ta_embed_anchors(x[None], C[:1].contiguous(), 0.9)
    torch.cuda.synchronize()
    s, _ = _check(sim, anchor, x, C[:1], 0.9)
    assert abs(s[2] + 1.0) < 1e-6


def test_lookup_by_token_id_matches_oracle():
    rng = np.random.default_rng(11)
    V, B, n = 5000, 3, 1111
    vocab = (rng.random(V) < 0.03).astype(np.uint8) * rng.integers(1, 256, size=V).astype(np.uint8)
    tok = rng.integers(0, V, size=(B, n)).astype(np.int32)
    tok[0, 5], tok[0, 6], tok[1, 0] = -1, V, 2 ** 31 - 1          # IDs outside the vocabulary
    seq_len = np.array([1111, 600, 1], np.int32)
    anchor = ta.ta_lookup_anchors(_dev(tok), _dev(vocab), seq_len=_dev(seq_len))
    torch.cuda.synchronize()
    anchor = anchor.cpu().numpy()
    for b in range(B):
        nb = int(seq_len[b])
        assert np.array_equal(anchor[b, :nb], ora.lookup_anchors(tok[b, :nb], vocab))
        assert not anchor[b, nb:].any()


def test_vocabulary_route_equals_per_position_route_and_feeds_selection():
    # flags of the embedding table once + lookup  ==  flags of each position's embedding; then
    # vouchers and the protected top-K of TA-Fast-Embedding against the oracle's chain
    V, dm, E, K = 3000, 128, 6, 40
    emb, C = wl.make_embedding_inputs(V, dm, E, p_near=0.03, device=DEV)
    rng = np.random.default_rng(21)
    B, n = 2, 800
    tok = rng.integers(0, V, size=(B, n)).astype(np.int32)
    seq_len = np.array([800, 513], np.int32)
    prm = ta.Params(n_sink=4, n_recent=4, alpha=0.0)
    sim_v, flag_v = ta.ta_embed_anchors(emb[None], C, 0.55)
    anchor = ta.ta_lookup_anchors(_dev(tok), flag_v.view(-1), seq_len=_dev(seq_len))
    x_pos = emb[_dev(tok).long().view(-1)].view(B, n, dm).contiguous()
    sim_p, anchor_p = ta.ta_embed_anchors(x_pos, C, 0.55, seq_len=_dev(seq_len))
    spons, vouch = ta.ta_expand_vouchers(anchor, prm, seq_len=_dev(seq_len))
    idx, cnt = ta.ta_select(None, anchor, spons, vouch, K, prm, 1, 1, seq_len=_dev(seq_len))
    torch.cuda.synchronize()
    assert torch.equal(anchor, anchor_p) and anchor.sum() > 10
    flags = flag_v.view(-1).cpu().numpy()
    idx, cnt = idx.cpu().numpy(), cnt.cpu().numpy()
    for b in range(B):
        nb = int(seq_len[b])
        a_ref = ora.lookup_anchors(tok[b, :nb], flags)
        s_ref, v_ref = ora.expand(a_ref)
        idx_ref = ora.select(None, a_ref, s_ref, v_ref, K, 4, 4, 0.0, 0.5, 0.3)
        assert cnt[0, b, 0] == len(idx_ref) and np.array_equal(idx[0, b, 0, :len(idx_ref)], idx_ref)


def test_embed_rejects_unsupported_shapes():
    x, C = wl.make_embedding_inputs(64, 64, 4, device=DEV)
    with pytest.raises(ta.TaError):            # more concepts than a tile holds
        ta.ta_embed_anchors(x[None], torch.zeros((257, 64), dtype=torch.bfloat16, device=DEV), 0.5)
    with pytest.raises(ta.TaError):            # d_model not a multiple of 32
        ta.ta_embed_anchors(x[None, :, :48], C[:, :48].contiguous(), 0.5)
    with pytest.raises(ta.TaError):
        ta.ta_embed_anchors(x[None], C, float("inf"))
