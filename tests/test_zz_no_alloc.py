"""ta_evict_static (the entry point that allocates nothing: static device scratch) against ta_evict.

Same kernels, so every output must be bit-identical; two calls in a row on the one buffer, the
second on a smaller input, and a layout beyond the buffer's size is refused before any launch.
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2604_11288_amd as ta
from paper_2604_11288_amd import binding as tb
from paper_2604_11288_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _prm(w):
    return ta.Params(n_sink=w.n_sink, n_recent=w.n_recent, span_L=w.span_L, sponsor_B=w.sponsor_B,
                     rho=w.rho, alpha=w.alpha, beta=w.beta, gamma=w.gamma)


def _pair(w, K):
    td = wl.make_tokens(w, clean=False)
    Q, Kc, Vc = wl.make_qkv(w, device=DEV)
    seq = _dev(td.seq_len) if w.ragged else None
    tok = _dev(td.tok)
    ref = ta.EvictPlan(tok, td.tab_ids, td.tab_len, Q, Kc, Vc, K, _prm(w), seq_len=seq)
    got = ta.EvictPlan(tok, td.tab_ids, td.tab_len, Q, Kc, Vc, K, _prm(w), seq_len=seq, static_scratch=True)
    assert got.ws is None
    return ref, got, td


def _same(ref, got, td, K):
    for name in ("anchor", "spons"):
        assert torch.equal(getattr(ref, name), getattr(got, name)), name
    assert torch.equal(ref.vouch.view(torch.int32), got.vouch.view(torch.int32))
    lens = torch.from_numpy(td.seq_len).to(DEV)
    live = torch.arange(ref.A.shape[-1], device=DEV).view(1, 1, 1, -1) < lens.view(1, -1, 1, 1)
    assert torch.equal(ref.A.view(torch.int32)[live.expand_as(ref.A)], got.A.view(torch.int32)[live.expand_as(got.A)])
    assert torch.equal(ref.cnt, got.cnt) and torch.equal(ref.idx, got.idx)
    assert torch.equal(ref.Kout.view(torch.int16), got.Kout.view(torch.int16))
    assert torch.equal(ref.Vout.view(torch.int16), got.Vout.view(torch.int16))


def test_static_scratch_pass_equals_workspace_pass_twice_second_smaller():
    ta.ta_init()
    big = wl.scaled(wl.CONFIGS["c2_full_model"], layers=4)                     # 32 units x 2 chunks of statistics
    small = wl.scaled(wl.CONFIGS["c5_agentic_prefill"], layers=1, batch=3, n=1500, hq=8, hkv=2, ragged=(600, 1500))
    for w, K in ((big, 256), (small, 64)):
        ref, got, td = _pair(w, K)
        ref.run()
        got.run()
        torch.cuda.synchronize()
        _same(ref, got, td, K)
    # and once more on the first shape: the buffer now holds the smaller call's statistics
    ref, got, td = _pair(big, 64)
    ref.run()
    got.run()
    torch.cuda.synchronize()
    _same(ref, got, td, 64)


def test_static_scratch_attention_free_pass():
    w = wl.scaled(wl.CONFIGS["c3_ta_fast"], layers=2, batch=2, n=4096)
    ref, got, td = _pair(w, 512)
    ref.run()
    got.run()
    torch.cuda.synchronize()
    for name in ("anchor", "spons", "idx", "cnt"):
        assert torch.equal(getattr(ref, name), getattr(got, name)), name
    assert torch.equal(ref.Kout.view(torch.int16), got.Kout.view(torch.int16))


def test_static_scratch_refuses_a_layout_beyond_its_size():
    # 96 layers x 96 sequences x 8 heads x 128 rows x 8 B = 72 MiB of row statistics
    lay = tb.CLayout()
    lay.layers, lay.batch, lay.hq, lay.hkv, lay.n, lay.window, lay.d = 96, 96, 32, 8, 1024, 32, 128
    st = [96 * 8 * 1024 * 128, 8 * 1024 * 128, 1024 * 128, 128]
    for i in range(4):
        lay.kv_stride[i] = st[i]
    qs = [96 * 32 * 32 * 128, 32 * 32 * 128, 32 * 128]
    for i in range(3):
        lay.q_stride[i] = qs[i]
    prm = ta.Params(n_sink=4, n_recent=4).c()
    need = tb.lib().ta_workspace_bytes(ctypes.byref(lay), ctypes.byref(prm))
    assert need > tb.TA_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x7f0000001000)                 # never dereferenced: the size check comes first
    ids = np.zeros((1, 4), np.int32)
    lens = np.ones(1, np.int32)
    rc = tb.lib().ta_evict_static(fake, None, ids.ctypes.data, lens.ctypes.data, 1, None, fake, fake, fake,
                                  ctypes.byref(lay), ctypes.byref(prm), 64, fake, fake, fake, fake, fake, fake,
                                  fake, fake, None)
    assert rc == tb.TA_ERR_SCRATCH
    assert "scratch" in tb.lib().ta_strerror(rc).decode()
