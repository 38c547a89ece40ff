"""Seeded synthetic workloads shaped like the paper's evaluation settings.

This module only draws inputs (token streams with planted anchor n-grams,
anchor tables, N(0,1) bf16 K/V/Q); it contains none of the method's arithmetic
and is the one piece of code that both the GPU tests and the CPU oracle tests
use.  The shapes follow the needle-in-haystack setting (Sec. 4.1: a credential
after an anchor at depths 0.1-0.9 of a 4K context, budgets K from 16 upward),
the TA-Fast long-context runs (Sec. 4.7) and agentic multi-turn decode
(Sec. 4.4); no text, prompt, dataset item or model weight is involved.
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np
import torch

VOCAB = 32000
RESERVED = 1024          # table IDs are drawn from the top RESERVED ids
TABLE_WIDTH = 4          # max n-gram length; unused slots hold -1
BASE_SEED = 20260411


@dataclass(frozen=True)
class Workload:
    """One configuration of the eviction pass."""
    name: str
    layers: int
    batch: int
    n: int
    hq: int
    hkv: int
    d: int = 128
    window: int = 32            # observation-window queries W (0: attention-free)
    n_sink: int = 4
    n_recent: int = 4
    budgets: Tuple[int, ...] = (16,)
    table_entries: int = 16
    gram_min: int = 2
    gram_max: int = 2
    planted: int = 4
    value_min: int = 8
    value_max: int = 8
    alpha: float = 1.0
    beta: float = 0.5
    gamma: float = 0.3
    span_L: int = 6
    sponsor_B: float = 15.0
    rho: float = 0.8
    seed: int = BASE_SEED
    ragged: Optional[Tuple[int, int]] = None   # (min_len, max_len) or None


# The five benchmark configurations.
CONFIGS = {
    "c1_single_layer": Workload("c1_single_layer", layers=1, batch=1, n=4096, hq=32, hkv=8,
                                window=32, n_sink=4, n_recent=4, budgets=(16,),
                                table_entries=16, gram_min=2, gram_max=2, planted=4,
                                seed=BASE_SEED + 1),
    "c2_full_model": Workload("c2_full_model", layers=32, batch=1, n=4096, hq=32, hkv=8,
                              window=32, n_sink=4, n_recent=4, budgets=(16, 64, 256, 1024),
                              table_entries=16, gram_min=1, gram_max=3, planted=8,
                              seed=BASE_SEED + 2),
    "c3_ta_fast": Workload("c3_ta_fast", layers=32, batch=16, n=32768, hq=32, hkv=8,
                           window=0, n_sink=4, n_recent=64, budgets=(512,),
                           table_entries=64, gram_min=1, gram_max=4, planted=32,
                           alpha=0.0, seed=BASE_SEED + 3),
    "c4_long_context": Workload("c4_long_context", layers=32, batch=4, n=131072, hq=32, hkv=8,
                                window=64, n_sink=4, n_recent=128, budgets=(1024,),
                                table_entries=64, gram_min=1, gram_max=4, planted=128,
                                value_min=4, value_max=32, seed=BASE_SEED + 4),
    "c5_agentic_prefill": Workload("c5_agentic_prefill", layers=32, batch=64, n=16384, hq=32, hkv=8,
                                   window=32, n_sink=4, n_recent=4, budgets=(256,),
                                   table_entries=16, gram_min=1, gram_max=3, planted=8,
                                   ragged=(2048, 16384), seed=BASE_SEED + 5),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a configuration with some sizes replaced (for oracle-sized tests)."""
    return replace(w, **kw)


@dataclass
class TokenData:
    tok: np.ndarray            # int32 [B][n] (rows padded with filler past seq_len)
    seq_len: np.ndarray        # int32 [B]
    tab_ids: np.ndarray        # int32 [E][TABLE_WIDTH], -1 padded
    tab_len: np.ndarray        # int32 [E]
    planted: List[List[int]] = field(default_factory=list)   # per sequence: anchor positions


def make_table(w: Workload, rng: np.random.Generator):
    """E n-grams whose IDs are all distinct and come from the reserved id range."""
    E = w.table_entries
    lens = rng.integers(w.gram_min, w.gram_max + 1, size=E).astype(np.int32)
    ids = rng.permutation(RESERVED)[: E * TABLE_WIDTH].astype(np.int32) + (VOCAB - RESERVED)
    tab = ids.reshape(E, TABLE_WIDTH).copy()
    for e in range(E):
        tab[e, lens[e]:] = -1
    return tab, lens


def make_tokens(w: Workload, clean: bool = True) -> TokenData:
    """Token streams with w.planted anchor n-grams per sequence.

    clean: filler IDs never touch the reserved range, so the planted positions
    are exactly the anchors.  dirty: filler is uniform over the whole vocabulary,
    so accidental (mostly 1-gram) matches and overlapping spans occur.
    """
    rng = np.random.default_rng(w.seed)
    tab, lens = make_table(w, rng)
    hi = VOCAB - RESERVED if clean else VOCAB
    tok = rng.integers(0, hi, size=(w.batch, w.n)).astype(np.int32)
    if w.ragged is None:
        seq_len = np.full(w.batch, w.n, np.int32)
    else:
        seq_len = rng.integers(w.ragged[0], w.ragged[1] + 1, size=w.batch).astype(np.int32)
        seq_len = np.minimum(seq_len, w.n)
    planted = []
    for b in range(w.batch):
        nb = int(seq_len[b])
        lo = w.n_sink + 2
        hi_pos = nb - w.n_recent - 2
        foot = w.gram_max + w.value_max + w.span_L + 1
        P = w.planted
        seg = (hi_pos - lo) // max(P, 1)
        pos_list = []
        if P > 0 and seg >= foot:
            for s in range(P):
                e = int(rng.integers(0, w.table_entries))
                start = lo + s * seg + int(rng.integers(0, seg - foot + 1))
                ln = int(lens[e])
                tok[b, start:start + ln] = tab[e, :ln]
                pos_list.append(start + ln - 1)          # anchor = last token of the n-gram
        planted.append(pos_list)
    return TokenData(tok=tok, seq_len=seq_len, tab_ids=tab, tab_len=lens, planted=planted)


def make_qkv(w: Workload, device="cpu", layers: Optional[int] = None, with_v: bool = True):
    """bf16 N(0,1) tensors: Q [Lyr][B][Hq][W][d], K and V [Lyr][B][Hkv][n][d]."""
    lyr = w.layers if layers is None else layers
    g = torch.Generator(device=device)
    g.manual_seed(w.seed)

    def draw(shape):
        out = torch.empty(shape, dtype=torch.bfloat16, device=device)
        flat = out.view(-1)
        step = 1 << 26
        for s in range(0, flat.numel(), step):
            e = min(s + step, flat.numel())
            flat[s:e] = torch.randn(e - s, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
        return out

    K = draw((lyr, w.batch, w.hkv, w.n, w.d))
    V = draw((lyr, w.batch, w.hkv, w.n, w.d)) if with_v else None
    Q = draw((lyr, w.batch, w.hq, w.window, w.d)) if w.window > 0 else None
    return Q, K, V


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of a bf16 tensor as a numpy uint16 array (host)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def make_decode_stream(w: Workload, td: TokenData, steps: int, p_anchor: float = 0.02, clean: bool = True):
    """Token IDs appended during decode: int32 [steps][B].

    Per step and sequence: if an n-gram emission is pending, its next token; else with
    probability p_anchor a table entry is picked uniformly and its emission starts (it
    completes len-1 steps later); else a filler ID.
    """
    rng = np.random.default_rng(w.seed + 7919)
    hi = VOCAB - RESERVED if clean else VOCAB
    out = np.zeros((steps, w.batch), np.int32)
    pending = [[] for _ in range(w.batch)]
    for t in range(steps):
        for b in range(w.batch):
            if pending[b]:
                out[t, b] = pending[b].pop(0)
            elif w.table_entries > 0 and rng.random() < p_anchor:
                e = int(rng.integers(0, w.table_entries))
                gram = td.tab_ids[e, :td.tab_len[e]].tolist()
                out[t, b] = gram[0]
                pending[b] = gram[1:]
            else:
                out[t, b] = int(rng.integers(0, hi))
    return out


def make_decode_qkv(w: Workload, step: int, device="cpu", layers: Optional[int] = None):
    """bf16 N(0,1) rows of one decode step: q [Lyr][B][Hq][d], k and v [Lyr][B][Hkv][d]."""
    lyr = w.layers if layers is None else layers
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 1000003 + step)
    def draw(shape):
        return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    return draw((lyr, w.batch, w.hq, w.d)), draw((lyr, w.batch, w.hkv, w.d)), draw((lyr, w.batch, w.hkv, w.d))


def make_detector_inputs(batch: int, n: int, d_model: int, m: int, seed: int = BASE_SEED + 11, p_anchor: float = 0.05,
                         device="cpu", row_stride: Optional[int] = None):
    """Inputs of the learned anchor detector (Sec. 5.1): hidden states h bf16 [B][n][d_model]
    (rows row_stride elements apart), first-layer weights W1 bf16 [m][d_model], output weights
    W2 bf16 [m].

    No trained detector or model is involved.  The weights are built so that the confidences
    spread over (0, 1) the way a trained detector's do: half of the hidden units look along one
    random direction u, the other half are random background units with negative output weight
    (the detector has no bias, so they supply the negative resting logit).  h is N(0,1) noise;
    a fraction p_anchor of the positions gets a component along u whose strength is uniform, so
    their confidences land on both sides of the 0.3 and 0.5 thresholds and the rest stay near 0.
    """
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    stride = d_model if row_stride is None else row_stride
    u = torch.randn(d_model, generator=g, device=device, dtype=torch.float32)
    u = u / u.norm()
    half = m // 2
    W1 = torch.randn((m, d_model), generator=g, device=device, dtype=torch.float32) / d_model ** 0.5
    W1[:half] = 0.25 * u + 0.02 * W1[:half]
    W2 = torch.empty(m, device=device, dtype=torch.float32)
    W2[:half] = 0.25 * 64.0 / half
    W2[half:] = -0.5 * 64.0 / (m - half)
    hbuf = torch.empty((batch * n, stride), dtype=torch.bfloat16, device=device)
    step = max(1, (1 << 26) // stride)
    for s in range(0, batch * n, step):
        e = min(s + step, batch * n)
        x = torch.randn((e - s, d_model), generator=g, device=device, dtype=torch.float32)
        is_anchor = torch.rand(e - s, generator=g, device=device) < p_anchor
        strength = torch.rand(e - s, generator=g, device=device) * 7.2
        x += (is_anchor * strength)[:, None] * u[None, :]
        hbuf[s:e, :d_model] = x.to(torch.bfloat16)
        if stride > d_model:
            hbuf[s:e, d_model:] = 7.0                      # padding a correct kernel never reads
    h = hbuf.view(batch, n, stride)[:, :, :d_model]
    return h, W1.to(torch.bfloat16), W2.to(torch.bfloat16)


def make_embedding_inputs(V: int, d_model: int, E: int, seed: int = BASE_SEED + 13, p_near: float = 0.05,
                          device="cpu", row_stride: Optional[int] = None):
    """Inputs of embedding-based anchor detection (Sec. 3.2): an input-embedding table bf16
    [V][d_model] (rows row_stride elements apart) and E anchor-concept embeddings bf16 [E][d_model].

    No model's embedding table is involved.  Rows are N(0, 0.02^2) noise; a fraction p_near of
    them is a mix t * c_e / |c_e| + (1 - t) * noise / |noise| with a random concept e and t uniform
    on (0, 1), so their largest cosine spreads over (0, 1); the other rows have cosines of order
    1 / sqrt(d_model).  Concepts are N(0,1) scaled by random factors (norms must divide out).
    """
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    stride = d_model if row_stride is None else row_stride
    C = torch.randn((E, d_model), generator=g, device=device, dtype=torch.float32)
    C *= torch.rand((E, 1), generator=g, device=device) * 3.0 + 0.25
    buf = torch.empty((V, stride), dtype=torch.bfloat16, device=device)
    step = max(1, (1 << 26) // stride)
    Cn = C / C.norm(dim=1, keepdim=True)
    for s in range(0, V, step):
        e = min(s + step, V)
        noise = torch.randn((e - s, d_model), generator=g, device=device, dtype=torch.float32)
        near = torch.rand(e - s, generator=g, device=device) < p_near
        which = torch.randint(0, E, (e - s,), generator=g, device=device)
        t = torch.rand(e - s, generator=g, device=device)[:, None]
        mixed = t * Cn[which] + (1.0 - t) * noise / noise.norm(dim=1, keepdim=True)
        rows = torch.where(near[:, None], mixed * 0.5, noise * 0.02)
        buf[s:e, :d_model] = rows.to(torch.bfloat16)
        if stride > d_model:
            buf[s:e, d_model:] = 7.0                       # padding a correct kernel never reads
    return buf[:, :d_model], C.to(torch.bfloat16)


def make_paged(K: torch.Tensor, V: torch.Tensor, page_size: int, heads_first: bool = False, spare_pages: int = 3,
               seed: int = BASE_SEED + 17):
    """Scatters dense caches [Lyr][B][Hkv][n][d] into paged pools the way a serving engine's
    allocator leaves them: every sequence's pages sit at random places of a pool that also holds
    a few unused pages.  Pools are [Lyr][pages][page_size][Hkv][d], or [Lyr][pages][Hkv][page_size][d]
    with heads_first.  Returns (Kpool, Vpool, table int32 [B][max_pages] on the device, num_pages,
    element strides (layer, page, position, head)).  Pure data movement."""
    lyr, B, H, n, d = K.shape
    max_pages = (n + page_size - 1) // page_size
    num_pages = B * max_pages + spare_pages
    rng = np.random.default_rng(seed)
    table = rng.permutation(num_pages)[: B * max_pages].astype(np.int32).reshape(B, max_pages)
    shape = (lyr, num_pages, H, page_size, d) if heads_first else (lyr, num_pages, page_size, H, d)
    pools = []
    for src in (K, V):
        pool = torch.full(shape, 3.0, dtype=torch.bfloat16, device=K.device)   # unused pages and tails hold junk
        for b in range(B):
            for j in range(max_pages):
                lo, hi = j * page_size, min((j + 1) * page_size, n)
                rows = src[:, b, :, lo:hi]                                      # [Lyr][H][rows][d]
                if heads_first:
                    pool[:, table[b, j], :, : hi - lo] = rows
                else:
                    pool[:, table[b, j], : hi - lo] = rows.transpose(1, 2)
        pools.append(pool)
    if heads_first:
        strides = (num_pages * H * page_size * d, H * page_size * d, d, page_size * d)
    else:
        strides = (num_pages * page_size * H * d, page_size * H * d, H * d, d)
    return pools[0], pools[1], torch.from_numpy(table).to(K.device), num_pages, strides


def make_slot_pool(layers: int, batch: int, hkv: int, d: int, slots: int, page_size: int, device, heads_first: bool = False,
                   spare_pages: int = 5, seed: int = BASE_SEED + 19):
    """Empty page pools for `slots` cache slots per (sequence, head): every sequence's pages at random
    places of a pool that also holds spare pages, junk values everywhere.  Pools are
    [Lyr][pages][page_size][Hkv][d], or [Lyr][pages][Hkv][page_size][d] with heads_first.  Returns
    (Kpool, Vpool, table int32 [B][max_pages] as a numpy array, num_pages, element strides
    (layer, page, position, head)).  Pure allocation."""
    max_pages = (slots + page_size - 1) // page_size
    num_pages = batch * max_pages + spare_pages
    table = np.random.default_rng(seed).permutation(num_pages)[: batch * max_pages].astype(np.int32).reshape(batch, max_pages)
    shape = (layers, num_pages, hkv, page_size, d) if heads_first else (layers, num_pages, page_size, hkv, d)
    Kp = torch.full(shape, 3.0, dtype=torch.bfloat16, device=device)
    Vp = torch.full(shape, -5.0, dtype=torch.bfloat16, device=device)
    if heads_first:
        strides = (num_pages * hkv * page_size * d, hkv * page_size * d, d, page_size * d)
    else:
        strides = (num_pages * page_size * hkv * d, page_size * hkv * d, hkv * d, d)
    return Kp, Vp, table, num_pages, strides
