"""ctypes front end of the CPU oracle (test infrastructure only).

Loads ``libta_oracle.so`` built from ``ta_oracle.c`` with gcc; arguments are
numpy arrays in host memory.  bf16 tensors are passed as ``uint16`` bit
patterns.  Nothing here is part of the product path: only tests, the smoke
check and the benchmark's CPU-baseline leg import this module, and it imports
nothing from the GPU package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ta_oracle.c")
# TA_ORACLE_SANITIZE=1: the same source built with AddressSanitizer and UndefinedBehaviorSanitizer
# (any report aborts the process).  The interpreter must then be started with the sanitizer
# runtime preloaded (LD_PRELOAD=$(gcc -print-file-name=libasan.so)); tests/test_sanitizers.py does.
SANITIZE = os.environ.get("TA_ORACLE_SANITIZE", "") not in ("", "0")
_SO = os.path.join(_HERE, "libta_oracle_san.so" if SANITIZE else "libta_oracle.so")

_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain C11, no contraction, no fast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] if SANITIZE else ["-O2"]
        cmd = ["gcc", "-std=c11", *opt, "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        vp, i32, f32, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_double
        lib.ta_oracle_match.argtypes = [vp, i32, vp, i32, vp, i32, vp]
        lib.ta_oracle_match.restype = None
        lib.ta_oracle_expand.argtypes = [vp, vp, i32, i32, f32, f64, vp, vp]
        lib.ta_oracle_expand.restype = None
        lib.ta_oracle_score.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        lib.ta_oracle_score.restype = None
        lib.ta_oracle_utility.argtypes = [vp, vp, vp, i32, f32, f32, f32, vp]
        lib.ta_oracle_utility.restype = None
        lib.ta_oracle_select.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, f32, f32, f32, vp]
        lib.ta_oracle_select.restype = i32
        lib.ta_oracle_select_margin.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, f32, f32, f32, vp]
        lib.ta_oracle_select_margin.restype = None
        lib.ta_oracle_compact.argtypes = [vp, vp, i32, i32, vp]
        lib.ta_oracle_compact.restype = None
        lib.ta_oracle_decode_append.argtypes = [vp, vp, vp, i32, i32, vp, i32, vp, i32, f32]
        lib.ta_oracle_decode_append.restype = None
        lib.ta_oracle_decode_vouch.argtypes = [vp, vp, i32, i32, f64, vp, vp]
        lib.ta_oracle_decode_vouch.restype = None
        lib.ta_oracle_decode_decay.argtypes = [vp, i32, f32]
        lib.ta_oracle_decode_decay.restype = None
        lib.ta_oracle_decode_unit.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, i32, vp, vp, i32,
                                              i32, i32, i32, f64, f32, f32, f32, vp, vp, i32]
        lib.ta_oracle_decode_unit.restype = i32
        lib.ta_oracle_detect.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        lib.ta_oracle_detect.restype = None
        lib.ta_oracle_confidence_anchors.argtypes = [vp, i32, f32, i32, f32, f32, vp, vp]
        lib.ta_oracle_confidence_anchors.restype = None
        i64 = ctypes.c_int64
        lib.ta_oracle_paged_gather.argtypes = [vp, vp, i32, i32, i64, i64, i64, i32, i32, vp]
        lib.ta_oracle_paged_gather.restype = None
        lib.ta_oracle_paged_scatter.argtypes = [vp, i32, vp, i32, i64, i64, i64, i32, i32, vp]
        lib.ta_oracle_paged_scatter.restype = None
        lib.ta_oracle_row_lse.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        lib.ta_oracle_row_lse.restype = None
        lib.ta_oracle_score_lse.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp]
        lib.ta_oracle_score_lse.restype = None
        lib.ta_oracle_maxpool.argtypes = [vp, i32, i32, vp]
        lib.ta_oracle_maxpool.restype = None
        lib.ta_oracle_select_partition.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, f32, vp]
        lib.ta_oracle_select_partition.restype = i32
        lib.ta_oracle_select_partition_margin.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, f32, vp]
        lib.ta_oracle_select_partition_margin.restype = None
        lib.ta_oracle_layer_budgets.argtypes = [i32, i32, i32, vp]
        lib.ta_oracle_layer_budgets.restype = None
        lib.ta_oracle_allow_filter.argtypes = [vp, vp, i32, vp]
        lib.ta_oracle_allow_filter.restype = None
        lib.ta_oracle_cosine_sim.argtypes = [vp, vp, i32, i32, i32, vp]
        lib.ta_oracle_cosine_sim.restype = None
        lib.ta_oracle_threshold_anchors.argtypes = [vp, i32, f32, vp]
        lib.ta_oracle_threshold_anchors.restype = None
        lib.ta_oracle_lookup_anchors.argtypes = [vp, i32, vp, i32, vp]
        lib.ta_oracle_lookup_anchors.restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def match(tok, tab_ids, tab_len):
    """anchor[p] = 1 iff a table n-gram ends at p.  tok int32 [n]."""
    tok = _c(tok, np.int32)
    tab_ids = _c(tab_ids, np.int32).reshape(len(tab_len), -1) if len(tab_len) else np.zeros((0, 4), np.int32)
    tab_len = _c(tab_len, np.int32)
    anchor = np.zeros(tok.shape[0], np.uint8)
    _load().ta_oracle_match(_p(tok), tok.shape[0], _p(tab_ids), tab_ids.shape[1],
                            _p(tab_len), tab_len.shape[0], _p(anchor))
    return anchor


def expand(anchor, L=6, B=15.0, rho=0.8, anchor_B=None):
    """Sponsor mask and voucher V of Eq. 2.  Returns (spons u8 [n], V f32 [n])."""
    anchor = _c(anchor, np.uint8)
    n = anchor.shape[0]
    ab = None if anchor_B is None else _c(anchor_B, np.float32)
    spons = np.zeros(n, np.uint8)
    V = np.zeros(n, np.float32)
    _load().ta_oracle_expand(_p(anchor), _p(ab), n, int(L), float(B), float(rho), _p(spons), _p(V))
    return spons, V


def score(Q, K, causal=True):
    """A[i] = sum over the group's heads and window rows of softmax weights.

    Q uint16 (bf16 bits) [G][W][d]; K uint16 [n][d].  Returns f32 [n].
    """
    Q = _c(Q, np.uint16)
    K = _c(K, np.uint16)
    G, W, d = Q.shape
    n = K.shape[0]
    assert K.shape[1] == d
    A = np.zeros(n, np.float32)
    _load().ta_oracle_score(_p(Q), _p(K), n, G, W, d, 1 if causal else 0, _p(A))
    return A


def paged_gather(pool, table, n, page_size, stride_page, stride_pos, stride_head, head, d):
    """Dense [n][d] rows (uint16) of one (sequence, head) of a paged cache pool of one layer.
    pool: flat uint16 array; table int32 [pages of the sequence]; strides in elements."""
    pool = _c(pool, np.uint16).reshape(-1)
    table = _c(table, np.int32)
    assert table.shape[0] * page_size >= n
    out = np.zeros((n, d), np.uint16)
    _load().ta_oracle_paged_gather(_p(pool), _p(table), int(n), int(page_size), int(stride_page), int(stride_pos),
                                   int(stride_head), int(head), int(d), _p(out))
    return out


def paged_scatter(pool, rows, table, page_size, stride_page, stride_pos, stride_head, head):
    """Writes rows [cnt][d] (uint16) to slots 0..cnt-1 of one (sequence, head) of a paged cache pool of one
    layer, in place.  pool: flat, contiguous uint16 array (modified); strides in elements."""
    assert pool.dtype == np.uint16 and pool.flags["C_CONTIGUOUS"]
    rows = _c(rows, np.uint16)
    table = _c(table, np.int32)
    cnt, d = rows.shape
    assert table.shape[0] * page_size >= cnt
    _load().ta_oracle_paged_scatter(_p(rows), int(cnt), _p(table), int(page_size), int(stride_page), int(stride_pos),
                                    int(stride_head), int(head), int(d), _p(pool.reshape(-1)))
    return pool


def row_lse(Q, K, causal=True):
    """Log-sum-exp of the scaled logits of every window row: the by-product of a flash-style
    prefill attention kernel.  Q uint16 [G][W][d], K uint16 [n][d].  Returns f32 [G][W]."""
    Q, K = _c(Q, np.uint16), _c(K, np.uint16)
    G, W, d = Q.shape
    n = K.shape[0]
    lse = np.zeros((G, W), np.float32)
    _load().ta_oracle_row_lse(_p(Q), _p(K), n, G, W, d, int(bool(causal)), _p(lse))
    return lse


def score_lse(Q, K, lse, causal=True):
    """Attention column sums from given row log-sum-exps (one sweep over the keys)."""
    Q, K, lse = _c(Q, np.uint16), _c(K, np.uint16), _c(lse, np.float32)
    G, W, d = Q.shape
    n = K.shape[0]
    assert lse.shape == (G, W)
    A = np.zeros(n, np.float32)
    _load().ta_oracle_score_lse(_p(Q), _p(K), _p(lse), n, G, W, d, int(bool(causal)), _p(A))
    return A


def utility(A, anchor, V, alpha=1.0, beta=0.5, gamma=0.3):
    anchor = _c(anchor, np.uint8)
    V = _c(V, np.float32)
    n = anchor.shape[0]
    a = None if A is None else _c(A, np.float32)
    if a is None:
        assert alpha == 0.0
    u = np.zeros(n, np.float32)
    _load().ta_oracle_utility(_p(a), _p(anchor), _p(V), n, float(alpha), float(beta), float(gamma), _p(u))
    return u


def select(A, anchor, spons, V, K, n_sink, n_recent, alpha=1.0, beta=0.5, gamma=0.3):
    """Retained positions (ascending) under the (class, u, position) order."""
    anchor = _c(anchor, np.uint8)
    spons = _c(spons, np.uint8)
    V = _c(V, np.float32)
    n = anchor.shape[0]
    a = None if A is None else _c(A, np.float32)
    if a is None:
        assert alpha == 0.0
    idx = np.zeros(max(min(K, n), 1), np.int32)
    cnt = _load().ta_oracle_select(_p(a), _p(anchor), _p(spons), _p(V), n, int(K),
                                   int(n_sink), int(n_recent),
                                   float(alpha), float(beta), float(gamma), _p(idx))
    return idx[:cnt].copy()


def select_margin(A, anchor, spons, V, K, n_sink, n_recent, alpha=1.0, beta=0.5, gamma=0.3, k_protected=-1):
    """(smallest retained u, largest evicted u) of the class - with k_protected >= 0: of the main pool -
    that the cut of select / select_partition falls in; (+inf, -inf) when nothing is evicted."""
    anchor = _c(anchor, np.uint8)
    spons = _c(spons, np.uint8)
    V = _c(V, np.float32)
    n = anchor.shape[0]
    a = None if A is None else _c(A, np.float32)
    if a is None:
        assert alpha == 0.0
    out = np.zeros(2, np.float32)
    if k_protected < 0:
        _load().ta_oracle_select_margin(_p(a), _p(anchor), _p(spons), _p(V), n, int(K), int(n_sink), int(n_recent),
                                        float(alpha), float(beta), float(gamma), _p(out))
    else:
        _load().ta_oracle_select_partition_margin(_p(a), _p(anchor), _p(spons), _p(V), n, int(K), int(k_protected),
                                                  int(n_sink), int(n_recent), float(alpha), float(beta),
                                                  float(gamma), _p(out))
    return out


def compact(rows, idx):
    """out[r,:] = rows[idx[r],:] for 16-bit row elements (bf16 bits)."""
    rows = _c(rows, np.uint16)
    idx = _c(idx, np.int32)
    out = np.zeros((idx.shape[0], rows.shape[1]), np.uint16)
    _load().ta_oracle_compact(_p(rows), _p(idx), idx.shape[0], rows.shape[1], _p(out))
    return out


def detect(h, W1, W2):
    """Detector confidence sigmoid(W2 . GELU(W1 . h)) per position (Sec. 5.1).
    h uint16 [n][dm], W1 uint16 [m][dm], W2 uint16 [m] (bf16 bit patterns).  Returns f32 [n]."""
    h, W1, W2 = _c(h, np.uint16), _c(W1, np.uint16), _c(W2, np.uint16)
    n, dm = h.shape
    m = W1.shape[0]
    assert W1.shape == (m, dm) and W2.shape == (m,)
    conf = np.zeros(n, np.float32)
    _load().ta_oracle_detect(_p(h), _p(W1), _p(W2), n, dm, m, _p(conf))
    return conf


def confidence_anchors(conf, thr, rank, B=15.0, scale=1.0):
    """Anchor flags (conf > thr) and per-anchor budgets: B when rank is false (TA-Learned), else
    scale * conf (TA-LearnRank).  Returns (anchor u8 [n], anchor_B f32 [n])."""
    conf = _c(conf, np.float32)
    n = conf.shape[0]
    anchor = np.zeros(n, np.uint8)
    ab = np.zeros(n, np.float32)
    _load().ta_oracle_confidence_anchors(_p(conf), n, float(thr), int(bool(rank)), float(B), float(scale),
                                         _p(anchor), _p(ab))
    return anchor, ab


def cosine_sim(x, C):
    """Largest cosine between each row of x and the concept rows of C (embedding-based anchor
    detection, Sec. 3.2).  x uint16 [n][dm], C uint16 [E][dm] (bf16 bit patterns).  Returns f32 [n]."""
    x, C = _c(x, np.uint16), _c(C, np.uint16)
    n, dm = x.shape
    E = C.shape[0]
    assert C.shape == (E, dm) and E >= 1
    sim = np.zeros(n, np.float32)
    _load().ta_oracle_cosine_sim(_p(x), _p(C), n, dm, E, _p(sim))
    return sim


def threshold_anchors(sim, tau):
    """anchor[p] = sim[p] > tau."""
    sim = _c(sim, np.float32)
    anchor = np.zeros(sim.shape[0], np.uint8)
    _load().ta_oracle_threshold_anchors(_p(sim), sim.shape[0], float(tau), _p(anchor))
    return anchor


def lookup_anchors(tok, vocab_anchor):
    """anchor[p] = vocab_anchor[tok[p]] (0 for IDs outside the vocabulary)."""
    tok = _c(tok, np.int32)
    va = _c(vocab_anchor, np.uint8)
    anchor = np.zeros(tok.shape[0], np.uint8)
    _load().ta_oracle_lookup_anchors(_p(tok), tok.shape[0], _p(va), va.shape[0], _p(anchor))
    return anchor


def maxpool(A, k):
    """out[p] = max of A over the k positions centred on p (clipped to the sequence); k odd."""
    A = _c(A, np.float32)
    assert k >= 1 and k % 2 == 1
    out = np.zeros_like(A)
    _load().ta_oracle_maxpool(_p(A), A.shape[0], int(k), _p(out))
    return out


def select_partition(A, anchor, spons, V, K, k_protected, n_sink, n_recent, alpha=1.0, beta=0.5, gamma=0.3):
    """Retained positions (ascending) under the fixed partition K = K_main + K_protected (Sec. 3.3)."""
    anchor = _c(anchor, np.uint8)
    spons = _c(spons, np.uint8)
    V = _c(V, np.float32)
    n = anchor.shape[0]
    a = None if A is None else _c(A, np.float32)
    if a is None:
        assert alpha == 0.0
    idx = np.zeros(max(min(K, n), 1), np.int32)
    cnt = _load().ta_oracle_select_partition(_p(a), _p(anchor), _p(spons), _p(V), n, int(K), int(k_protected),
                                             int(n_sink), int(n_recent), float(alpha), float(beta), float(gamma),
                                             _p(idx))
    return idx[:cnt].copy()


def layer_budgets(layers, K, k_min):
    """Per-layer budgets falling arithmetically from 2K - k_min to k_min with mean K."""
    out = np.zeros(layers, np.int32)
    _load().ta_oracle_layer_budgets(int(layers), int(K), int(k_min), _p(out))
    return out


def allow_filter(anchor, allow):
    """Anchors that lie on allowed positions."""
    anchor, allow = _c(anchor, np.uint8), _c(allow, np.uint8)
    out = np.zeros_like(anchor)
    _load().ta_oracle_allow_filter(_p(anchor), _p(allow), anchor.shape[0], _p(out))
    return out


def evict_sequence(tok, tab_ids, tab_len, L=6, B=15.0, rho=0.8, anchor_B=None):
    """Steps 1-2 for one sequence: (anchor, spons, V)."""
    anchor = match(tok, tab_ids, tab_len)
    spons, V = expand(anchor, L=L, B=B, rho=rho, anchor_B=anchor_B)
    return anchor, spons, V


# ---------------------------------------------------------------------------
# incremental (per generation step) form
# ---------------------------------------------------------------------------
class DecodeSeq:
    """Per-sequence state of the incremental pass: tokens, anchor flags, current budgets."""

    def __init__(self, tok, tab_ids, tab_len, cap, B=15.0):
        tok = _c(tok, np.int32)
        self.len = int(tok.shape[0])
        self.cap = int(cap)
        self.tok = np.zeros(cap, np.int32)
        self.tok[:self.len] = tok
        self.tab_len = _c(tab_len, np.int32)
        E = len(self.tab_len)
        self.tab_ids = _c(tab_ids, np.int32).reshape(E, -1) if E else np.zeros((0, 4), np.int32)
        self.B = float(B)
        self.anchor = np.zeros(cap, np.uint8)
        self.anchor[:self.len] = match(tok, self.tab_ids, self.tab_len)
        self.budget = np.where(self.anchor == 1, np.float32(B), np.float32(0)).astype(np.float32)

    def append(self, new_tok):
        assert self.len < self.cap
        _load().ta_oracle_decode_append(_p(self.tok), _p(self.anchor), _p(self.budget), self.len, int(new_tok),
                                        _p(self.tab_ids), self.tab_ids.shape[1], _p(self.tab_len),
                                        self.tab_len.shape[0], self.B)
        self.len += 1
        return self.len - 1

    def vouch(self, p, L=6, rho=0.8):
        V = np.zeros(1, np.float32)
        sp = np.zeros(1, np.uint8)
        _load().ta_oracle_decode_vouch(_p(self.anchor), _p(self.budget), int(p), int(L), float(rho), _p(V), _p(sp))
        return float(V[0]), int(sp[0])

    def decay(self, factor=0.9):
        _load().ta_oracle_decode_decay(_p(self.budget), self.len, float(factor))


class DecodeUnit:
    """Per-unit cache state: K+1 slots of K/V rows, their positions and cumulative attention."""

    def __init__(self, Krows, Vrows, idx, A_kept):
        Krows, Vrows = _c(Krows, np.uint16), _c(Vrows, np.uint16)
        K, d = Krows.shape
        self.slots, self.d = K + 1, d
        self.Kc = np.zeros((K + 1, d), np.uint16)
        self.Vc = np.zeros((K + 1, d), np.uint16)
        self.Kc[:K], self.Vc[:K] = Krows, Vrows
        self.pos = np.full(K + 1, -1, np.int32)
        self.pos[:K] = _c(idx, np.int32)
        self.A = np.zeros(K + 1, np.float32)
        self.A[:K] = _c(A_kept, np.float32)

    def step(self, seq, q, k_new, v_new, p_new, n_sink, n_recent, L=6, rho=0.8,
             alpha=1.0, beta=0.5, gamma=0.3, rank_A=None, last_query=False):
        """q uint16 [G][d].  Returns (evicted slot, utilities [slots]).  last_query: the attention term is
        this step's softmax mass alone (TOVA's step-wise rule), not the running sum."""
        q = _c(q, np.uint16)
        k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
        ra = None if rank_A is None else _c(rank_A, np.float32)
        u = np.zeros(self.slots, np.float32)
        e = _load().ta_oracle_decode_unit(_p(self.Kc), _p(self.Vc), _p(self.pos), _p(self.A), self.slots, self.d,
                                          _p(q), q.shape[0], _p(k_new), _p(v_new), int(p_new),
                                          _p(seq.anchor), _p(seq.budget), seq.len,
                                          int(n_sink), int(n_recent), int(L), float(rho),
                                          float(alpha), float(beta), float(gamma), _p(ra), _p(u),
                                          1 if last_query else 0)
        return int(e), u
