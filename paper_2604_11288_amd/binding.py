"""ctypes binding of libta.so: argument marshalling only.

Every step of the eviction pass runs in the HIP kernels behind the C ABI
declared in include/ta.h; torch is used for device memory and the current
stream.  There is no CPU fallback: a missing library or a failing call raises.
"""
import ctypes
import os
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TA_LIBTA_PATH names another build of the same library (the host-sanitizer build of the tests)
LIB_PATH = os.environ.get("TA_LIBTA_PATH") or os.path.join(_HERE, "libta.so")

TA_MAX_TABLE = 64
TA_MAX_GRAM = 4
TA_MAX_SPAN = 64
TA_HEAD_DIM = 128
TA_MAX_ROWS = 512
TA_MAX_LAYER_PTRS = 96
TA_LAYER_WS_BYTES = 4096

TA_OK, TA_ERR_NULL, TA_ERR_SHAPE, TA_ERR_BUDGET = 0, -1, -2, -3
TA_ERR_WORKSPACE, TA_ERR_ALIGN, TA_ERR_HIP, TA_ERR_SCRATCH = -4, -5, -6, -7
TA_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ("ta_workspace_bytes", "ta_match_anchors", "ta_detect_anchors", "ta_expand_vouchers", "ta_embed_anchors",
           "ta_lookup_anchors", "ta_layer_budgets", "ta_score", "ta_score_lse", "ta_score_paged", "ta_select", "ta_compact", "ta_compact_paged", "ta_compact_into_pages",
           "ta_evict", "ta_evict_static", "ta_evict_lse", "ta_evict_paged", "ta_evict_layers", "ta_evict_layers_paged", "ta_decode_init", "ta_decode_step", "ta_init", "ta_strerror", "ta_last_hip_error")


class TaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().ta_strerror(status).decode()
        if status == TA_ERR_HIP:
            msg += " (hipError %d)" % lib().ta_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, status))


class CParams(ctypes.Structure):
    _fields_ = [("n_sink", ctypes.c_int32), ("n_recent", ctypes.c_int32), ("span_L", ctypes.c_int32),
                ("sponsor_B", ctypes.c_float), ("rho", ctypes.c_double),
                ("alpha", ctypes.c_float), ("beta", ctypes.c_float), ("gamma", ctypes.c_float),
                ("causal", ctypes.c_int32), ("budget_decay", ctypes.c_float),
                ("pool_k", ctypes.c_int32), ("k_protected", ctypes.c_int32), ("last_query", ctypes.c_int32),
                ("layer_K", ctypes.c_void_p), ("allow", ctypes.c_void_p), ("margin", ctypes.c_void_p)]


class CDecodeState(ctypes.Structure):
    _fields_ = [("layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("hq", ctypes.c_int32),
                ("hkv", ctypes.c_int32), ("d", ctypes.c_int32), ("K", ctypes.c_int32), ("cap", ctypes.c_int32),
                ("tok", ctypes.c_void_p), ("len", ctypes.c_void_p), ("anchor", ctypes.c_void_p),
                ("budget", ctypes.c_void_p), ("vouch", ctypes.c_void_p), ("spons", ctypes.c_void_p),
                ("Kc", ctypes.c_void_p), ("Vc", ctypes.c_void_p),
                ("pos", ctypes.c_void_p), ("A", ctypes.c_void_p), ("stepped", ctypes.c_void_p),
                ("pages", ctypes.c_void_p)]


class CLayout(ctypes.Structure):
    _fields_ = [("layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("hq", ctypes.c_int32),
                ("hkv", ctypes.c_int32), ("n", ctypes.c_int32), ("window", ctypes.c_int32),
                ("d", ctypes.c_int32),
                ("kv_stride", ctypes.c_int64 * 4), ("q_stride", ctypes.c_int64 * 3)]


class CPaged(ctypes.Structure):
    _fields_ = [("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32), ("num_pages", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("stride", ctypes.c_int64 * 4)]


@dataclass
class Params:
    """Hyper-parameters (defaults: the paper's Full-TA values, Eq. 1-2)."""
    n_sink: int = 4
    n_recent: int = 4
    span_L: int = 6
    sponsor_B: float = 15.0
    rho: float = 0.8
    alpha: float = 1.0
    beta: float = 0.5
    gamma: float = 0.3
    causal: bool = True
    budget_decay: float = 0.9
    pool_k: int = 1                              # max-pool window over A (SnapKV clustering), 1 = none
    k_protected: int = -1                        # K_protected of Sec. 3.3, negative = elastic pool
    last_query: bool = False                     # per-step form: rank by the current step's attention (TOVA's rule)
    layer_K: Optional[torch.Tensor] = None       # device int32 [layers]: per-layer budgets
    allow: Optional[torch.Tensor] = None         # device uint8 [B][n]: allowlist of positions
    margin: Optional[torch.Tensor] = None        # device float [units][2] (out): margin of every unit's cut

    def c(self) -> CParams:
        for t, dt in ((self.layer_K, torch.int32), (self.allow, torch.uint8), (self.margin, torch.float32)):
            assert t is None or (t.dtype == dt and t.is_contiguous())
        return CParams(self.n_sink, self.n_recent, self.span_L, self.sponsor_B, self.rho,
                       self.alpha, self.beta, self.gamma, 1 if self.causal else 0, self.budget_decay,
                       self.pool_k, self.k_protected, 1 if self.last_query else 0,
                       None if self.layer_K is None else self.layer_K.data_ptr(),
                       None if self.allow is None else self.allow.data_ptr(),
                       None if self.margin is None else self.margin.data_ptr())


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libta.so is not built: run paper_2604_11288_amd/build.py "
                               "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.ta_workspace_bytes.argtypes = [vp, vp]
        L.ta_workspace_bytes.restype = sz
        L.ta_match_anchors.argtypes = [vp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.ta_match_anchors.restype = i32
        L.ta_detect_anchors.argtypes = [vp, ctypes.c_int64, vp, vp, vp, i32, i32, i32, i32,
                                        ctypes.c_float, i32, ctypes.c_float, vp, vp, vp, vp, vp]
        L.ta_detect_anchors.restype = i32
        L.ta_layer_budgets.argtypes = [i32, i32, i32, vp]
        L.ta_layer_budgets.restype = i32
        L.ta_embed_anchors.argtypes = [vp, ctypes.c_int64, vp, i32, vp, i32, i32, i32, ctypes.c_float, vp, vp, vp]
        L.ta_embed_anchors.restype = i32
        L.ta_lookup_anchors.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp]
        L.ta_lookup_anchors.restype = i32
        L.ta_expand_vouchers.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp]
        L.ta_expand_vouchers.restype = i32
        L.ta_score.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.ta_score.restype = i32
        L.ta_score_lse.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
        L.ta_score_lse.restype = i32
        L.ta_score_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.ta_score_paged.restype = i32
        L.ta_compact_paged.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.ta_compact_paged.restype = i32
        L.ta_select.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        L.ta_select.restype = i32
        L.ta_compact_into_pages.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        L.ta_compact_into_pages.restype = i32
        L.ta_compact.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.ta_compact.restype = i32
        L.ta_evict.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32,
                               vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.ta_evict.restype = i32
        L.ta_evict_static.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32,
                                      vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.ta_evict_static.restype = i32
        L.ta_evict_lse.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, i32,
                                   vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.ta_evict_lse.restype = i32
        L.ta_evict_paged.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                     vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.ta_evict_paged.restype = i32
        L.ta_evict_layers.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, i32,
                                      vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ta_evict_layers.restype = i32
        L.ta_evict_layers_paged.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32,
                                            vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ta_evict_layers_paged.restype = i32
        L.ta_decode_init.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.ta_decode_init.restype = i32
        L.ta_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
        L.ta_decode_step.restype = i32
        L.ta_init.argtypes = []
        L.ta_init.restype = i32
        L.ta_strerror.argtypes = [i32]
        L.ta_strerror.restype = ctypes.c_char_p
        L.ta_last_hip_error.argtypes = []
        L.ta_last_hip_error.restype = i32
        _lib = L
    return _lib


def ta_init():
    """One-time set-up on the current device (kernel attributes); optional except before a stream capture."""
    _check(lib().ta_init(), "ta_init")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc, where):
    if rc != TA_OK:
        raise TaError(rc, where)


def _table(tab_ids, tab_len):
    """Host copies of the anchor table in the ABI's [E][TA_MAX_GRAM] / [E] int32 form."""
    tab_len = np.ascontiguousarray(np.asarray(tab_len, dtype=np.int32))
    E = int(tab_len.shape[0])
    ids = np.full((max(E, 1), TA_MAX_GRAM), -1, np.int32)
    if E:
        src = np.asarray(tab_ids, dtype=np.int32).reshape(E, -1)
        ids[:E, :min(src.shape[1], TA_MAX_GRAM)] = src[:, :TA_MAX_GRAM]
    return ids, tab_len, E


def layout_of(K: torch.Tensor, Q: Optional[torch.Tensor] = None, window: Optional[int] = None) -> CLayout:
    """ta_layout of a [Lyr][B][Hkv][n][d] cache tensor (and its [Lyr][B][Hq][W][d] queries)."""
    assert K.dim() == 5 and K.dtype == torch.bfloat16 and K.stride(4) == 1
    lay = CLayout()
    lay.layers, lay.batch, lay.hkv, lay.n, lay.d = K.shape
    for i in range(4):
        lay.kv_stride[i] = K.stride(i)
    if Q is not None:
        assert Q.dim() == 5 and Q.dtype == torch.bfloat16 and Q.stride(4) == 1
        assert Q.stride(3) == Q.shape[4], "rows of a query head must be contiguous"
        lay.hq, lay.window = Q.shape[2], Q.shape[3]
        for i in range(3):
            lay.q_stride[i] = Q.stride(i)
    else:
        lay.hq, lay.window = lay.hkv, (window or 0)
    return lay


def ta_workspace_bytes(lay: CLayout, params: Params) -> int:
    cp = params.c()
    return int(lib().ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(cp)))


def ta_match_anchors(tok, tab_ids, tab_len, params: Params, seq_len=None, anchor_B=None,
                     out=None, stream=None):
    """Steps 1+2.  tok int32 [B][n] (device).  Returns (anchor u8, spons u8, vouch f32), each [B][n]."""
    assert tok.dtype == torch.int32 and tok.dim() == 2 and tok.is_contiguous()
    B, n = tok.shape
    ids, lens, E = _table(tab_ids, tab_len)
    if out is None:
        anchor = torch.empty((B, n), dtype=torch.uint8, device=tok.device)
        spons = torch.empty((B, n), dtype=torch.uint8, device=tok.device)
        vouch = torch.empty((B, n), dtype=torch.float32, device=tok.device)
    else:
        anchor, spons, vouch = out
    cp = params.c()
    rc = lib().ta_match_anchors(_ptr(tok), _ptr(seq_len), B, n, ids.ctypes.data, lens.ctypes.data, E,
                                _ptr(anchor_B), ctypes.byref(cp), _ptr(anchor), _ptr(spons), _ptr(vouch),
                                _stream(stream))
    _check(rc, "ta_match_anchors")
    return anchor, spons, vouch


def ta_detect_anchors(h, W1, W2, params: Params, thr: float, rank: bool, scale: float = 1.0, seq_len=None,
                      out=None, stream=None):
    """Learned detector.  h bf16 [B][n][d_model] (rows may be strided), W1 bf16 [m][d_model], W2 bf16 [m].
    Returns (conf f32, anchor u8, anchor_B f32), each [B][n]."""
    assert h.dtype == torch.bfloat16 and h.dim() == 3 and h.stride(2) == 1
    B, n, dm = h.shape
    assert B == 1 or h.stride(0) == n * h.stride(1), "sequences must follow each other row after row"
    assert W1.dtype == torch.bfloat16 and W1.dim() == 2 and W1.is_contiguous() and W1.shape[1] == dm
    m = W1.shape[0]
    assert W2.dtype == torch.bfloat16 and W2.is_contiguous() and W2.numel() == m
    if out is None:
        conf = torch.empty((B, n), dtype=torch.float32, device=h.device)
        anchor = torch.empty((B, n), dtype=torch.uint8, device=h.device)
        anchor_B = torch.empty((B, n), dtype=torch.float32, device=h.device)
    else:
        conf, anchor, anchor_B = out
    cp = params.c()
    rc = lib().ta_detect_anchors(_ptr(h), h.stride(1), _ptr(W1), _ptr(W2), _ptr(seq_len), B, n, dm, m,
                                 float(thr), int(bool(rank)), float(scale), ctypes.byref(cp),
                                 _ptr(conf), _ptr(anchor), _ptr(anchor_B), _stream(stream))
    _check(rc, "ta_detect_anchors")
    return conf, anchor, anchor_B


def ta_layer_budgets(layers: int, K: int, k_min: int) -> np.ndarray:
    """Pyramidal per-layer budgets (host int32 [layers]) with mean K that fall to k_min."""
    out = np.zeros(layers, np.int32)
    _check(lib().ta_layer_budgets(layers, K, k_min, out.ctypes.data), "ta_layer_budgets")
    return out


def ta_embed_anchors(x, C, tau: float, seq_len=None, out=None, stream=None):
    """Embedding-based detection.  x bf16 [B][n][d_model] (rows may be strided; the embedding table is
    B = 1, n = vocabulary size), C bf16 [E][d_model].  Returns (sim f32, anchor u8), each [B][n]."""
    assert x.dtype == torch.bfloat16 and x.dim() == 3 and x.stride(2) == 1
    B, n, dm = x.shape
    assert B == 1 or x.stride(0) == n * x.stride(1), "sequences must follow each other row after row"
    assert C.dtype == torch.bfloat16 and C.dim() == 2 and C.is_contiguous() and C.shape[1] == dm
    if out is None:
        sim = torch.empty((B, n), dtype=torch.float32, device=x.device)
        anchor = torch.empty((B, n), dtype=torch.uint8, device=x.device)
    else:
        sim, anchor = out
    rc = lib().ta_embed_anchors(_ptr(x), x.stride(1), _ptr(C), C.shape[0], _ptr(seq_len), B, n, dm, float(tau),
                                _ptr(sim), _ptr(anchor), _stream(stream))
    _check(rc, "ta_embed_anchors")
    return sim, anchor


def ta_lookup_anchors(tok, vocab_anchor, seq_len=None, out=None, stream=None):
    """anchor[b][p] = vocab_anchor[tok[b][p]] != 0.  tok int32 [B][n], vocab_anchor u8 [V].  Returns u8 [B][n]."""
    assert tok.dtype == torch.int32 and tok.dim() == 2 and tok.is_contiguous()
    assert vocab_anchor.dtype == torch.uint8 and vocab_anchor.dim() == 1 and vocab_anchor.is_contiguous()
    B, n = tok.shape
    anchor = torch.empty((B, n), dtype=torch.uint8, device=tok.device) if out is None else out
    rc = lib().ta_lookup_anchors(_ptr(tok), _ptr(seq_len), B, n, _ptr(vocab_anchor), vocab_anchor.numel(),
                                 _ptr(anchor), _stream(stream))
    _check(rc, "ta_lookup_anchors")
    return anchor


def ta_expand_vouchers(anchor, params: Params, anchor_B=None, seq_len=None, out=None, stream=None):
    """Step 2 from given anchor flags u8 [B][n].  Returns (spons u8, vouch f32), each [B][n]."""
    assert anchor.dtype == torch.uint8 and anchor.dim() == 2 and anchor.is_contiguous()
    B, n = anchor.shape
    if out is None:
        spons = torch.empty((B, n), dtype=torch.uint8, device=anchor.device)
        vouch = torch.empty((B, n), dtype=torch.float32, device=anchor.device)
    else:
        spons, vouch = out
    cp = params.c()
    rc = lib().ta_expand_vouchers(_ptr(anchor), _ptr(anchor_B), _ptr(seq_len), B, n, ctypes.byref(cp),
                                  _ptr(spons), _ptr(vouch), _stream(stream))
    _check(rc, "ta_expand_vouchers")
    return spons, vouch


def ta_score(Q, K, params: Params, seq_len=None, A=None, ws=None, stream=None):
    """Step 3.  Returns A f32 [Lyr][B][Hkv][n]."""
    lay = layout_of(K, Q)
    if A is None:
        A = torch.empty((lay.layers, lay.batch, lay.hkv, lay.n), dtype=torch.float32, device=K.device)
    need = ta_workspace_bytes(lay, replace(params, alpha=1.0))   # sized as for a scored pass
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=K.device)
    cp = params.c()
    rc = lib().ta_score(_ptr(Q), _ptr(K), ctypes.byref(lay), _ptr(seq_len), ctypes.byref(cp),
                        _ptr(A), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "ta_score")
    return A


def ta_score_lse(Q, K, lse, params: Params, seq_len=None, A=None, stream=None):
    """Step 3 in one sweep from the row log-sum-exps of a prefill attention kernel.
    lse f32 [Lyr][B][Hq][W].  Returns A f32 [Lyr][B][Hkv][n]."""
    lay = layout_of(K, Q)
    assert lse.dtype == torch.float32 and lse.is_contiguous()
    assert tuple(lse.shape) == (lay.layers, lay.batch, lay.hq, lay.window)
    if A is None:
        A = torch.empty((lay.layers, lay.batch, lay.hkv, lay.n), dtype=torch.float32, device=K.device)
    cp = params.c()
    rc = lib().ta_score_lse(_ptr(Q), _ptr(K), ctypes.byref(lay), _ptr(seq_len), ctypes.byref(cp),
                            _ptr(lse), _ptr(A), _stream(stream))
    _check(rc, "ta_score_lse")
    return A


class PagedKV:
    """A paged (block-table) cache: pools of pages, the block table and the element strides
    {layer, page, position, head} of ta_paged_kv.  Kpool / Vpool: bf16 tensors of any shape whose
    storage the strides index; table: device int32 [batch][max_pages]."""

    def __init__(self, Kpool, Vpool, table, page_size, num_pages, strides, layers, batch, hkv, n, d=TA_HEAD_DIM):
        assert table.dtype == torch.int32 and table.dim() == 2 and table.is_contiguous() and table.shape[0] == batch
        self.Kpool, self.Vpool, self.table = Kpool, Vpool, table
        self.page_size, self.num_pages, self.strides = int(page_size), int(num_pages), tuple(int(x) for x in strides)
        self.layers, self.batch, self.hkv, self.n, self.d = layers, batch, hkv, n, d

    def c(self) -> CPaged:
        pg = CPaged()
        pg.page_size, pg.max_pages, pg.num_pages = self.page_size, self.table.shape[1], self.num_pages
        pg.block_table = self.table.data_ptr()
        for i in range(4):
            pg.stride[i] = self.strides[i]
        return pg

    def layout(self, Q=None) -> CLayout:
        lay = CLayout()
        lay.layers, lay.batch, lay.hkv, lay.n, lay.d = self.layers, self.batch, self.hkv, self.n, self.d
        if Q is not None:
            assert Q.dim() == 5 and Q.dtype == torch.bfloat16 and Q.stride(4) == 1 and Q.stride(3) == Q.shape[4]
            lay.hq, lay.window = Q.shape[2], Q.shape[3]
            for i in range(3):
                lay.q_stride[i] = Q.stride(i)
        else:
            lay.hq, lay.window = self.hkv, 0
        return lay


def ta_score_paged(Q, paged: PagedKV, params: Params, seq_len=None, lse=None, A=None, ws=None, stream=None):
    """Step 3 over a paged cache (two sweeps, or one with lse).  Returns A f32 [Lyr][B][Hkv][n]."""
    lay, pg = paged.layout(Q), paged.c()
    if A is None:
        A = torch.empty((lay.layers, lay.batch, lay.hkv, lay.n), dtype=torch.float32, device=Q.device)
    if ws is None and lse is None:
        dense = CLayout.from_buffer_copy(lay)
        dense.kv_stride[3] = lay.d
        need = ta_workspace_bytes(dense, replace(params, alpha=1.0))
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    cp = params.c()
    rc = lib().ta_score_paged(_ptr(Q), _ptr(paged.Kpool), ctypes.byref(pg), ctypes.byref(lay), _ptr(seq_len),
                              ctypes.byref(cp), _ptr(lse), _ptr(A), _ptr(ws),
                              0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "ta_score_paged")
    return A


def ta_compact_paged(paged: PagedKV, idx, cnt, K: int, idx_shared: bool = False, out=None, stream=None):
    """Step 5 over a paged cache.  Returns dense (Kout, Vout) bf16 [Lyr][B][Hkv][K][d]."""
    lay, pg = paged.layout(), paged.c()
    if out is None:
        shape = (lay.layers, lay.batch, lay.hkv, K, lay.d)
        Kout = torch.zeros(shape, dtype=torch.bfloat16, device=paged.Kpool.device)
        Vout = torch.zeros(shape, dtype=torch.bfloat16, device=paged.Kpool.device)
    else:
        Kout, Vout = out
    rc = lib().ta_compact_paged(_ptr(paged.Kpool), _ptr(paged.Vpool), ctypes.byref(pg), _ptr(idx), _ptr(cnt),
                                ctypes.byref(lay), K, 1 if idx_shared else 0, _ptr(Kout), _ptr(Vout), _stream(stream))
    _check(rc, "ta_compact_paged")
    return Kout, Vout


def ta_compact_into_pages(Kin, Vin, idx, cnt, K: int, dst: PagedKV, src: Optional[PagedKV] = None,
                          idx_shared: bool = False, stream=None):
    """Step 5 straight into a page pool: row r of a unit goes to slot r of its sequence's pages in
    dst.Kpool / dst.Vpool.  The source is the dense pair (Kin, Vin), or the paged cache `src`
    (then Kin and Vin are ignored)."""
    if src is not None:
        lay, spg = src.layout(), src.c()
        Kin, Vin = src.Kpool, src.Vpool
    else:
        lay, spg = layout_of(Kin), None
    dpg = dst.c()
    rc = lib().ta_compact_into_pages(_ptr(Kin), _ptr(Vin), None if spg is None else ctypes.byref(spg), _ptr(idx), _ptr(cnt),
                                     ctypes.byref(lay), K, 1 if idx_shared else 0, _ptr(dst.Kpool), _ptr(dst.Vpool),
                                     ctypes.byref(dpg), _stream(stream))
    _check(rc, "ta_compact_into_pages")
    return dst


def ta_select(A, anchor, spons, vouch, K: int, params: Params, layers: int, hkv: int,
              seq_len=None, out=None, stream=None):
    """Step 4.  Returns (idx i32 [layers][B][hkv][K], cnt i32 [layers][B][hkv])."""
    B, n = anchor.shape
    if out is None:
        idx = torch.full((layers, B, hkv, K), -1, dtype=torch.int32, device=anchor.device)
        cnt = torch.zeros((layers, B, hkv), dtype=torch.int32, device=anchor.device)
    else:
        idx, cnt = out
    cp = params.c()
    rc = lib().ta_select(_ptr(A), _ptr(anchor), _ptr(spons), _ptr(vouch), _ptr(seq_len),
                         layers, B, hkv, n, K, ctypes.byref(cp), _ptr(idx), _ptr(cnt), _stream(stream))
    _check(rc, "ta_select")
    return idx, cnt


def ta_compact(Kin, Vin, idx, cnt, K: int, idx_shared: bool = False, out=None, stream=None):
    """Step 5.  Returns (Kout, Vout) bf16 [Lyr][B][Hkv][K][d]."""
    lay = layout_of(Kin)
    assert Vin.shape == Kin.shape and Vin.stride() == Kin.stride()
    if out is None:
        shape = (lay.layers, lay.batch, lay.hkv, K, lay.d)
        Kout = torch.zeros(shape, dtype=torch.bfloat16, device=Kin.device)
        Vout = torch.zeros(shape, dtype=torch.bfloat16, device=Kin.device)
    else:
        Kout, Vout = out
    rc = lib().ta_compact(_ptr(Kin), _ptr(Vin), _ptr(idx), _ptr(cnt), ctypes.byref(lay), K,
                          1 if idx_shared else 0, _ptr(Kout), _ptr(Vout), _stream(stream))
    _check(rc, "ta_compact")
    return Kout, Vout


class EvictPlan:
    """Pre-allocated outputs and marshalled arguments of one ta_evict configuration.

    run() only performs the C call, so it can sit inside a timed loop.
    """

    def __init__(self, tok, tab_ids, tab_len, Q, Kin, Vin, K: int, params: Params,
                 seq_len=None, anchor_B=None, lse=None, paged=None, static_scratch=False):
        self.paged = paged                 # PagedKV: Kin / Vin are then its pools (pass None for both)
        self.static_scratch = static_scratch   # ta_evict_static: no workspace tensor, the library's own scratch
        assert not (static_scratch and (lse is not None or paged is not None))
        if paged is not None:
            Kin, Vin = paged.Kpool, paged.Vpool
        dev = Kin.device
        self.params, self.K = params, int(K)
        self.lse = lse                     # row log-sum-exps of the prefill attention kernel: ta_evict_lse
        self.scored = params.alpha != 0.0
        if paged is not None:
            self.lay = paged.layout(Q if self.scored else None)
            self._pg = paged.c()
        else:
            self.lay = layout_of(Kin, Q if self.scored else None)
        lay = self.lay
        self.tok, self.seq_len, self.anchor_B = tok, seq_len, anchor_B
        self.Q, self.Kin, self.Vin = (Q if self.scored else None), Kin, Vin
        self.ids, self.lens, self.E = _table(tab_ids, tab_len)
        B, n = lay.batch, lay.n
        self.anchor = torch.empty((B, n), dtype=torch.uint8, device=dev)
        self.spons = torch.empty((B, n), dtype=torch.uint8, device=dev)
        self.vouch = torch.empty((B, n), dtype=torch.float32, device=dev)
        if self.scored:
            self.A = torch.empty((lay.layers, B, lay.hkv, n), dtype=torch.float32, device=dev)
            self.idx = torch.full((lay.layers, B, lay.hkv, self.K), -1, dtype=torch.int32, device=dev)
            self.cnt = torch.zeros((lay.layers, B, lay.hkv), dtype=torch.int32, device=dev)
            sized = lay
            if paged is not None:                                # workspace size depends on the sizes only
                sized = CLayout.from_buffer_copy(lay)
                sized.kv_stride[3] = lay.d
            nbytes = ta_workspace_bytes(sized, params) if lse is None else 0
            self.ws = None if static_scratch else torch.empty(max(nbytes, 16), dtype=torch.uint8, device=dev)
            if lse is not None:
                assert lse.dtype == torch.float32 and lse.is_contiguous()
                assert tuple(lse.shape) == (lay.layers, B, lay.hq, lay.window)
        else:
            self.A, self.ws = None, None
            self.idx = torch.full((B, self.K), -1, dtype=torch.int32, device=dev)
            self.cnt = torch.zeros((B,), dtype=torch.int32, device=dev)
        shape = (lay.layers, B, lay.hkv, self.K, lay.d)
        self.Kout = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
        self.Vout = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
        self._cp = params.c()

    def run(self, stream=None):
        ws_bytes = 0 if self.ws is None else self.ws.numel()
        if self.paged is not None:
            rc = lib().ta_evict_paged(_ptr(self.tok), _ptr(self.seq_len), self.ids.ctypes.data, self.lens.ctypes.data,
                                      self.E, _ptr(self.anchor_B), _ptr(self.Q), _ptr(self.Kin), _ptr(self.Vin),
                                      ctypes.byref(self._pg), _ptr(self.lse), ctypes.byref(self.lay),
                                      ctypes.byref(self._cp), self.K,
                                      _ptr(self.anchor), _ptr(self.spons), _ptr(self.vouch), _ptr(self.A),
                                      _ptr(self.idx), _ptr(self.cnt), _ptr(self.Kout), _ptr(self.Vout),
                                      _ptr(self.ws), ws_bytes, _stream(stream))
            _check(rc, "ta_evict_paged")
            return self
        if self.lse is not None:
            rc = lib().ta_evict_lse(_ptr(self.tok), _ptr(self.seq_len), self.ids.ctypes.data, self.lens.ctypes.data,
                                    self.E, _ptr(self.anchor_B), _ptr(self.Q), _ptr(self.Kin), _ptr(self.Vin),
                                    _ptr(self.lse), ctypes.byref(self.lay), ctypes.byref(self._cp), self.K,
                                    _ptr(self.anchor), _ptr(self.spons), _ptr(self.vouch), _ptr(self.A),
                                    _ptr(self.idx), _ptr(self.cnt), _ptr(self.Kout), _ptr(self.Vout), _stream(stream))
            _check(rc, "ta_evict_lse")
            return self
        if self.static_scratch:
            rc = lib().ta_evict_static(_ptr(self.tok), _ptr(self.seq_len), self.ids.ctypes.data, self.lens.ctypes.data,
                                       self.E, _ptr(self.anchor_B), _ptr(self.Q), _ptr(self.Kin), _ptr(self.Vin),
                                       ctypes.byref(self.lay), ctypes.byref(self._cp), self.K,
                                       _ptr(self.anchor), _ptr(self.spons), _ptr(self.vouch), _ptr(self.A),
                                       _ptr(self.idx), _ptr(self.cnt), _ptr(self.Kout), _ptr(self.Vout), _stream(stream))
            _check(rc, "ta_evict_static")
            return self
        rc = lib().ta_evict(_ptr(self.tok), _ptr(self.seq_len), self.ids.ctypes.data, self.lens.ctypes.data,
                            self.E, _ptr(self.anchor_B), _ptr(self.Q), _ptr(self.Kin), _ptr(self.Vin),
                            ctypes.byref(self.lay), ctypes.byref(self._cp), self.K,
                            _ptr(self.anchor), _ptr(self.spons), _ptr(self.vouch), _ptr(self.A),
                            _ptr(self.idx), _ptr(self.cnt), _ptr(self.Kout), _ptr(self.Vout),
                            _ptr(self.ws), ws_bytes, _stream(stream))
        _check(rc, "ta_evict")
        return self


def ta_evict(tok, tab_ids, tab_len, Q, Kin, Vin, K: int, params: Params, seq_len=None, anchor_B=None,
             stream=None) -> EvictPlan:
    """The whole pass in one call; returns the plan object holding every output tensor."""
    return EvictPlan(tok, tab_ids, tab_len, Q, Kin, Vin, K, params, seq_len, anchor_B).run(stream)


def ta_evict_static(tok, tab_ids, tab_len, Q, Kin, Vin, K: int, params: Params, seq_len=None, anchor_B=None,
                    stream=None) -> EvictPlan:
    """ta_evict with the library's static scratch in place of a workspace (the outputs are still
    allocated here, by the binding; build an EvictPlan(static_scratch=True) once to call without that)."""
    return EvictPlan(tok, tab_ids, tab_len, Q, Kin, Vin, K, params, seq_len, anchor_B, static_scratch=True).run(stream)


def ta_evict_paged(tok, tab_ids, tab_len, Q, paged: "PagedKV", K: int, params: Params, seq_len=None, anchor_B=None,
                   lse=None, stream=None) -> EvictPlan:
    """The whole pass over a paged cache (two sweeps, or one with lse)."""
    return EvictPlan(tok, tab_ids, tab_len, Q, None, None, K, params, seq_len, anchor_B, lse=lse, paged=paged).run(stream)


def ta_evict_lse(tok, tab_ids, tab_len, Q, Kin, Vin, lse, K: int, params: Params, seq_len=None, anchor_B=None,
                 stream=None) -> EvictPlan:
    """The whole pass with the one-sweep score from given row log-sum-exps (f32 [Lyr][B][Hq][W])."""
    return EvictPlan(tok, tab_ids, tab_len, Q, Kin, Vin, K, params, seq_len, anchor_B, lse=lse).run(stream)


class CLayerPtrs(ctypes.Structure):
    _fields_ = [("Q", ctypes.c_void_p), ("K", ctypes.c_void_p), ("V", ctypes.c_void_p),
                ("Kout", ctypes.c_void_p), ("Vout", ctypes.c_void_p)]


class LayerEvictPlan:
    """ta_evict_layers on caches kept as one tensor per layer.

    Q_layers: list of bf16 [B][Hq][W][d] (or None when params.alpha == 0); K_layers, V_layers: lists
    of bf16 [B][Hkv][n][d] with the same strides in every layer.  Kout / Vout are lists of dense
    [B][Hkv][K][d] tensors; the other outputs are as in EvictPlan.  run() only performs the C call.
    """

    def __init__(self, tok, tab_ids, tab_len, Q_layers, K_layers, V_layers, K: int, params: Params,
                 seq_len=None, anchor_B=None, paged: Optional["PagedKV"] = None, lse=None):
        layers = len(K_layers)
        assert layers >= 1 and len(V_layers) == layers
        K0 = K_layers[0]
        dev = K0.device
        self.params, self.K = params, int(K)
        self.scored = params.alpha != 0.0
        self.paged, self.lse = paged, lse
        for t in list(K_layers) + list(V_layers):
            assert t.dtype == torch.bfloat16 and t.shape == K0.shape and t.stride() == K0.stride()
        lay = CLayout()
        lay.layers = layers
        if paged is not None:
            # K_layers / V_layers are the page pools of the layers; sizes and addressing come from `paged`
            # (a PagedKV whose own pools may be None and whose layer stride is not used)
            assert paged.layers == layers
            lay.batch, lay.hkv, lay.n, lay.d = paged.batch, paged.hkv, paged.n, paged.d
            self._pg = paged.c()
            self._pg.stride[0] = 0
        else:
            assert K0.dim() == 4 and K0.stride(3) == 1
            lay.batch, lay.hkv, lay.n, lay.d = K0.shape
            lay.kv_stride[0] = 0
            for i in range(3):
                lay.kv_stride[i + 1] = K0.stride(i)
        if self.scored:
            assert len(Q_layers) == layers
            Q0 = Q_layers[0]
            for t in Q_layers:
                assert t.dim() == 4 and t.dtype == torch.bfloat16 and t.shape == Q0.shape and t.stride() == Q0.stride()
            assert Q0.stride(3) == 1 and Q0.stride(2) == Q0.shape[3], "rows of a query head must be contiguous"
            lay.hq, lay.window = Q0.shape[1], Q0.shape[2]
            lay.q_stride[0] = 0
            lay.q_stride[1], lay.q_stride[2] = Q0.stride(0), Q0.stride(1)
        else:
            lay.hq, lay.window = lay.hkv, 0
        self.lay = lay
        self.tok, self.seq_len, self.anchor_B = tok, seq_len, anchor_B
        self.Q_layers = list(Q_layers) if self.scored else None
        self.K_layers, self.V_layers = list(K_layers), list(V_layers)
        self.ids, self.lens, self.E = _table(tab_ids, tab_len)
        B, n = lay.batch, lay.n
        self.anchor = torch.empty((B, n), dtype=torch.uint8, device=dev)
        self.spons = torch.empty((B, n), dtype=torch.uint8, device=dev)
        self.vouch = torch.empty((B, n), dtype=torch.float32, device=dev)
        if self.scored:
            self.A = torch.empty((layers, B, lay.hkv, n), dtype=torch.float32, device=dev)
            self.idx = torch.full((layers, B, lay.hkv, self.K), -1, dtype=torch.int32, device=dev)
            self.cnt = torch.zeros((layers, B, lay.hkv), dtype=torch.int32, device=dev)
            sized = lay
            if paged is not None:                                # workspace size depends on the sizes only
                sized = CLayout.from_buffer_copy(lay)
                sized.kv_stride[3] = lay.d
            nbytes = (0 if lse is not None else (ta_workspace_bytes(sized, params) + 255) // 256 * 256) + TA_LAYER_WS_BYTES
            if lse is not None:
                assert lse.dtype == torch.float32 and lse.is_contiguous()
                assert tuple(lse.shape) == (layers, B, lay.hq, lay.window)
        else:
            self.A = None
            nbytes = TA_LAYER_WS_BYTES
            self.idx = torch.full((B, self.K), -1, dtype=torch.int32, device=dev)
            self.cnt = torch.zeros((B,), dtype=torch.int32, device=dev)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)      # score scratch + the address table
        self.Kout = [torch.zeros((B, lay.hkv, self.K, lay.d), dtype=torch.bfloat16, device=dev) for _ in range(layers)]
        self.Vout = [torch.zeros((B, lay.hkv, self.K, lay.d), dtype=torch.bfloat16, device=dev) for _ in range(layers)]
        table = lambda ts: (ctypes.c_void_p * layers)(*[t.data_ptr() for t in ts])
        self._tables = [table(self.Q_layers) if self.scored else None, table(self.K_layers), table(self.V_layers),
                        table(self.Kout), table(self.Vout)]     # host arrays, kept alive with the plan
        addr = lambda a: None if a is None else ctypes.cast(a, ctypes.c_void_p)
        self._lp = CLayerPtrs(*[addr(a) for a in self._tables])
        self._cp = params.c()

    def run(self, stream=None):
        ws_bytes = self.ws.numel()
        if self.paged is not None:
            rc = lib().ta_evict_layers_paged(_ptr(self.tok), _ptr(self.seq_len), self.ids.ctypes.data,
                                             self.lens.ctypes.data, self.E, _ptr(self.anchor_B), ctypes.byref(self._lp),
                                             ctypes.byref(self._pg), _ptr(self.lse), ctypes.byref(self.lay),
                                             ctypes.byref(self._cp), self.K,
                                             _ptr(self.anchor), _ptr(self.spons), _ptr(self.vouch), _ptr(self.A),
                                             _ptr(self.idx), _ptr(self.cnt), _ptr(self.ws), ws_bytes, _stream(stream))
            _check(rc, "ta_evict_layers_paged")
            return self
        assert self.lse is None, "row log-sum-exps are taken by the paged form only"
        rc = lib().ta_evict_layers(_ptr(self.tok), _ptr(self.seq_len), self.ids.ctypes.data, self.lens.ctypes.data,
                                   self.E, _ptr(self.anchor_B), ctypes.byref(self._lp), ctypes.byref(self.lay),
                                   ctypes.byref(self._cp), self.K,
                                   _ptr(self.anchor), _ptr(self.spons), _ptr(self.vouch), _ptr(self.A),
                                   _ptr(self.idx), _ptr(self.cnt), _ptr(self.ws), ws_bytes, _stream(stream))
        _check(rc, "ta_evict_layers")
        return self


def ta_evict_layers_paged(tok, tab_ids, tab_len, Q_layers, Kpool_layers, Vpool_layers, paged: "PagedKV", K: int,
                          params: Params, seq_len=None, anchor_B=None, lse=None, stream=None) -> LayerEvictPlan:
    """The whole pass over one page pool per layer behind a shared block table (`paged` describes
    the table, the page geometry and the sizes; its own pools are not used)."""
    return LayerEvictPlan(tok, tab_ids, tab_len, Q_layers, Kpool_layers, Vpool_layers, K, params, seq_len, anchor_B,
                          paged=paged, lse=lse).run(stream)


def ta_evict_layers(tok, tab_ids, tab_len, Q_layers, K_layers, V_layers, K: int, params: Params, seq_len=None,
                    anchor_B=None, stream=None) -> LayerEvictPlan:
    """The whole pass over per-layer cache tensors; returns the plan object holding every output."""
    return LayerEvictPlan(tok, tab_ids, tab_len, Q_layers, K_layers, V_layers, K, params, seq_len, anchor_B).run(stream)


class DecodeState:
    """Device tensors of the incremental pass (see ta_decode_state in include/ta.h)."""

    def __init__(self, layers, batch, hq, hkv, K, cap, device, d=TA_HEAD_DIM, pages: Optional["PagedKV"] = None):
        """pages: a PagedKV whose pools hold the K/V slots (slot s of a unit is position s of its addressing;
        max_pages * page_size >= K + 1); None: dense [layers][batch][hkv][K+1][d] tensors allocated here."""
        self.layers, self.batch, self.hq, self.hkv, self.K, self.cap, self.d = layers, batch, hq, hkv, K, cap, d
        self.pages = pages
        self._cpages = None if pages is None else pages.c()
        i32, dev = torch.int32, device
        self.tok = torch.zeros((batch, cap), dtype=i32, device=dev)
        self.len = torch.zeros((batch,), dtype=i32, device=dev)
        self.anchor = torch.zeros((batch, cap), dtype=torch.uint8, device=dev)
        self.budget = torch.zeros((batch, cap), dtype=torch.float32, device=dev)
        self.vouch = torch.zeros((batch, cap), dtype=torch.float32, device=dev)
        self.spons = torch.zeros((batch, cap), dtype=torch.uint8, device=dev)
        if pages is None:
            self.Kc = torch.zeros((layers, batch, hkv, K + 1, d), dtype=torch.bfloat16, device=dev)
            self.Vc = torch.zeros((layers, batch, hkv, K + 1, d), dtype=torch.bfloat16, device=dev)
        else:
            self.Kc, self.Vc = pages.Kpool, pages.Vpool
        self.pos = torch.full((layers, batch, hkv, K + 1), -1, dtype=i32, device=dev)
        self.A = torch.zeros((layers, batch, hkv, K + 1), dtype=torch.float32, device=dev)
        self.stepped = torch.zeros((batch,), dtype=i32, device=dev)

    def c(self) -> CDecodeState:
        return CDecodeState(self.layers, self.batch, self.hq, self.hkv, self.d, self.K, self.cap,
                            self.tok.data_ptr(), self.len.data_ptr(), self.anchor.data_ptr(),
                            self.budget.data_ptr(), self.vouch.data_ptr(), self.spons.data_ptr(),
                            self.Kc.data_ptr(), self.Vc.data_ptr(),
                            self.pos.data_ptr(), self.A.data_ptr(), self.stepped.data_ptr(),
                            None if self._cpages is None else ctypes.addressof(self._cpages))


def ta_decode_init(state: DecodeState, tok, anchor, idx, cnt, Kout, Vout, params: Params,
                   seq_len=None, anchor_B=None, A=None, stream=None):
    """Fill a decode state from the outputs of a prefill eviction (per-unit idx / cnt)."""
    cs, cp = state.c(), params.c()
    rc = lib().ta_decode_init(ctypes.byref(cs), _ptr(tok), _ptr(seq_len), tok.shape[1], _ptr(anchor),
                              _ptr(anchor_B), _ptr(A), _ptr(idx), _ptr(cnt), _ptr(Kout), _ptr(Vout),
                              ctypes.byref(cp), _stream(stream))
    _check(rc, "ta_decode_init")
    return state


def ta_decode_step(state: DecodeState, new_tok, q_new, k_new, v_new, tab_ids, tab_len, params: Params,
                   evicted=None, stream=None):
    """One generation step: append, accumulate attention, evict one row per unit, decay budgets."""
    ids, lens, E = _table(tab_ids, tab_len)
    cs, cp = state.c(), params.c()
    rc = lib().ta_decode_step(ctypes.byref(cs), _ptr(new_tok), _ptr(q_new), _ptr(k_new), _ptr(v_new),
                              ids.ctypes.data, lens.ctypes.data, E, ctypes.byref(cp), _ptr(evicted),
                              _stream(stream))
    _check(rc, "ta_decode_step")
    return evicted
