"""The beam top-b entry point that allocates nothing (its scratch is a device array inside the library) against the
entry point that takes a context's workspace: same inputs, identical outputs, two calls in a row, the second smaller."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _engine(batch, gamma, beam, V):
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    shape = si.ModelShape(1, 64, 1, 1, 64, 96, V, "fp32")
    m = DeviceModel(shape, si.make_weights(shape, 1, "target", threads=1), DEV)
    return Engine(m, m, batch=batch, gamma=gamma, beam=beam, mode="mmtad", max_context=256, prefill_rows=8, device=DEV)


def _case(B, gamma, beam, V, step, sample, seed):
    from paper_2407_09722_amd import binding as mb
    g = np.random.default_rng(seed)
    R = gamma + 1 if step == 0 else beam
    logits = (g.standard_normal((B, R, V)) * 3).astype(np.float32)
    if step > 0 and beam > 1:
        logits[:, 1] = logits[:, 0]                            # equal rows: ties between beams
    lse = np.log(np.exp(logits.astype(np.float64)).sum(-1)).astype(np.float32)
    cnt = torch.from_numpy(g.integers(1, 3, B).astype(np.int32)).to(DEV)
    length = torch.from_numpy(g.integers(20, 60, B).astype(np.int32)).to(DEV)
    prev = torch.from_numpy(-np.abs(g.standard_normal((B, gamma, beam))).astype(np.float32)).to(DEV)
    dl, dlse = torch.from_numpy(logits).to(DEV), torch.from_numpy(lse).to(DEV)

    eng = _engine(B, gamma, beam, V)
    eng.h_cum.copy_(prev)
    mb.mtad_k_beam_topb(eng.ctx, dl, dlse, eng.hist, step, cnt, length, R, V, int(sample), seed)
    torch.cuda.synchronize()
    want = [x.clone() for x in (eng.h_tok, eng.h_parent, eng.h_cum)]
    eng.close()

    i32 = dict(dtype=torch.int32, device=DEV)
    tok, par = torch.full((B, gamma, beam), -7, **i32), torch.full((B, gamma, beam), -7, **i32)
    cum = prev.clone()
    hist = mb.mtad_beam(mb.ptr(tok), mb.ptr(par), mb.ptr(cum))
    before = torch.cuda.memory_allocated()
    mb.mtad_k_beam_topb_static(dl, dlse, hist, B, gamma, beam, step, cnt, length, R, V, int(sample), seed)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for got, ref in zip((tok, par, cum), want):
        assert torch.equal(got[:, step], ref[:, step]), (B, gamma, beam, V, step, sample)
    assert torch.equal(cum[:, :step], prev[:, :step]) and torch.equal(cum[:, step + 1:], prev[:, step + 1:])


def test_static_scratch_entry_point_matches_workspace_entry_point():
    # two calls in a row on the library's one scratch array; the second is smaller in every dimension
    _case(5, 4, 4, 32000, 2, True, 3)
    _case(2, 3, 2, 1024, 0, False, 4)
    _case(3, 3, 8, 4096, 1, True, 5)


def test_static_scratch_entry_point_rejects_what_it_cannot_hold():
    from paper_2407_09722_amd import binding as mb
    L = mb.lib()
    p = C.c_void_p(256)
    hist = mb.mtad_beam(p, p, p)
    args = lambda batch, gamma, beam, step, R, V: (p, p, C.byref(hist), batch, gamma, beam, step, p, p, R, V, 0, 0, None)
    assert L.mtad_k_beam_topb_static(*args(mb.MTAD_STATIC_TOPB_MAX_BATCH + 1, 4, 4, 0, 5, 1024)) == mb.MTAD_ECAP
    assert L.mtad_k_beam_topb_static(*args(2, 4, 9, 0, 5, 1024)) == mb.MTAD_ESHAPE
    assert L.mtad_k_beam_topb_static(*args(2, 4, 4, 4, 5, 1024)) == mb.MTAD_EINVAL     # step out of range
    assert L.mtad_k_beam_topb_static(*args(2, 4, 4, 0, 4, 1024)) == mb.MTAD_EINVAL     # fewer rows than step 0 may read
    assert L.mtad_k_beam_topb_static(*args(2, 4, 4, 1, 3, 1024)) == mb.MTAD_EINVAL
    assert L.mtad_k_beam_topb_static(None, p, C.byref(hist), 2, 4, 4, 0, p, p, 5, 1024, 0, 0, None) == mb.MTAD_EINVAL
