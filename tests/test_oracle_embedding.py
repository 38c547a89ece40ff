"""Pins of the oracle's embedding-based anchor detection (Sec. 3.2, third detector; TA-Fast-Embedding):
largest cosine between an input embedding and the anchor-concept embeddings, threshold, and
the per-vocabulary lookup.  Each pin fails for a plausible mistake: a missing norm, the norm of
the wrong operand, min instead of max, a non-strict threshold, an off-by-one in the lookup."""
import numpy as np
import torch

from oracle import ta_oracle as ora


def _bits(a):
    """bf16 bit patterns of an array whose values are exactly representable in bf16."""
    t = torch.tensor(np.asarray(a, np.float32)).to(torch.bfloat16)
    assert torch.equal(t.to(torch.float32), torch.tensor(np.asarray(a, np.float32)))
    return t.view(torch.int16).numpy().view(np.uint16)


def _rand_bf16(rng, shape):
    t = torch.tensor(rng.standard_normal(shape).astype(np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16), t.to(torch.float64).numpy()


def test_closed_forms_identical_orthogonal_opposite_zero():
    C = _bits([[3.0, 4.0, 0.0, 0.0]])
    x = _bits([[3.0, 4.0, 0.0, 0.0],      # the concept itself: 1
               [6.0, 8.0, 0.0, 0.0],      # a multiple of it: 1 (norm of x divides out)
               [0.0, 0.0, 5.0, 0.0],      # orthogonal: 0
               [-3.0, -4.0, 0.0, 0.0],    # opposite: -1
               [4.0, 3.0, 0.0, 0.0],      # 24 / 25
               [0.0, 0.0, 0.0, 0.0]])     # zero vector: counted as 0
    sim = ora.cosine_sim(x, C)
    assert np.array_equal(sim, np.array([1.0, 1.0, 0.0, -1.0, 0.96, 0.0], np.float32))


def test_largest_cosine_over_the_concepts_and_concept_norms_divide_out():
    # concept 1 has the larger norm but the smaller cosine: a dot-product maximum would pick it
    C = _bits([[1.0, 0.0], [8.0, 8.0]])
    x = _bits([[2.0, 0.5]])
    sim = ora.cosine_sim(x, C)
    c0 = 2.0 / np.sqrt(4.25)
    c1 = 20.0 / (np.sqrt(4.25) * np.sqrt(128.0))
    assert c0 > c1 and sim[0] == np.float32(c0)
    # all cosines negative: the maximum is the least negative one, not 0
    sim = ora.cosine_sim(_bits([[-1.0, -1.0]]), C)
    assert sim[0] == np.float32(-1.0 / np.sqrt(2.0))
    # a zero concept counts as cosine 0
    sim = ora.cosine_sim(_bits([[-1.0, -1.0]]), _bits([[1.0, 0.0], [0.0, 0.0]]))
    assert sim[0] == 0.0


def test_against_numpy_float64_and_invariances():
    rng = np.random.default_rng(5)
    xb, x = _rand_bf16(rng, (40, 96))
    Cb, C = _rand_bf16(rng, (7, 96))
    ref = ((x @ C.T) / np.linalg.norm(x, axis=1)[:, None] / np.linalg.norm(C, axis=1)[None, :]).max(axis=1)
    sim = ora.cosine_sim(xb, Cb)
    assert np.array_equal(sim, ref.astype(np.float32)) or np.abs(sim - ref).max() < 1e-7
    # permuting the concepts, or doubling every vector (exact in bf16), changes nothing
    assert np.array_equal(ora.cosine_sim(xb, Cb[::-1]), sim)
    x2 = torch.tensor(x * 2.0).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    C4 = torch.tensor(C * 4.0).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.abs(ora.cosine_sim(x2, C4) - sim).max() <= 1e-7
    # Cauchy-Schwarz
    assert np.all(np.abs(sim) <= 1.0)


def test_threshold_is_strict_and_lookup_indexes_by_token_id():
    sim = np.array([0.25, 0.5, np.nextafter(np.float32(0.5), np.float32(1.0)), -0.7, 1.0], np.float32)
    assert ora.threshold_anchors(sim, 0.5).tolist() == [0, 0, 1, 0, 1]
    vocab = np.zeros(10, np.uint8)
    vocab[[0, 3, 9]] = [1, 7, 1]
    tok = np.array([3, 4, 9, 0, 10, -1, 2], np.int32)
    assert ora.lookup_anchors(tok, vocab).tolist() == [1, 0, 1, 1, 0, 0, 0]


def test_detection_over_the_vocabulary_equals_detection_per_position():
    # input embeddings are rows of the embedding table: thresholding the table once and looking the
    # flags up per token gives the flags of thresholding each position's embedding
    rng = np.random.default_rng(9)
    Eb, _ = _rand_bf16(rng, (50, 32))
    Cb = Eb[[4, 17]]                             # two vocabulary entries serve as concepts
    tok = rng.integers(0, 50, size=200).astype(np.int32)
    per_pos = ora.threshold_anchors(ora.cosine_sim(Eb[tok], Cb), 0.6)
    per_vocab = ora.threshold_anchors(ora.cosine_sim(Eb, Cb), 0.6)
    assert per_vocab[4] == 1 and per_vocab[17] == 1
    assert np.array_equal(ora.lookup_anchors(tok, per_vocab), per_pos)
