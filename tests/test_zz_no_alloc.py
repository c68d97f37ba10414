"""The entry point that allocates nothing (hola_verify_ex_static: the library's static scratch array instead of
a caller's workspace) against hola_verify_ex through the C ABI.  The two enqueue the same kernels, so every
output must be bit-identical; two calls in a row, the second on a smaller input, show that nothing a call reads
was left by the one before.  Collected last so that a failure here hides no other test."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2506_18952_amd import binding as hb, workloads as wl
from parity import DEV, to_dev

pytestmark = pytest.mark.gpu


def _both(w, tau, **kw):
    B, g, V = w.B, w.gamma, w.V
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    outs = []
    for entry in ("ex", "static"):
        acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        ent = torch.full((B, g), -7.0, dtype=torch.float32, device=DEV)
        common = dict(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                      temperature=w.temperature, entropy_threshold=tau, out_accept_len=acc, out_next_token=nxt,
                      out_entropy=ent, **kw)
        if entry == "ex":
            ws = hb.alloc_workspace(hb.hola_workspace_bytes_ex(B, g, V, kw.get("top_k", 0), kw.get("top_p", 0.0)), DEV)
            hb.hola_verify_ex(workspace=ws, **common)
        else:
            hb.hola_verify_ex_static(**common)
        torch.cuda.synchronize()
        outs.append((acc.cpu().numpy(), nxt.cpu().numpy(), ent.cpu().numpy()))
    return outs


def test_static_scratch_entry_matches_the_workspace_entry_twice_in_a_row():
    big = wl.config2()                                          # B=64, gamma=5, V=32000 bf16: 704 rows
    small = wl.small_case(7, 3, 5003, dtype="bf16", temperature=0.9, case_id=950)
    for w, taus in ((big, [big.taus[0], 0.0]), (small, [small.taus[0], 0.0])):   # the second input is the smaller one
        for tau in taus:
            ex, st = _both(w, tau)
            for a, b in zip(ex, st):
                np.testing.assert_array_equal(a, b)
            assert np.all(st[0] >= 0) and np.all(st[0] <= w.gamma) and np.all(st[1] >= 0)
    assert len(set(ex[0].tolist())) > 1                          # not a degenerate case
    # float rows with ragged lengths and per-row temperatures, then a filtered call that still fits the array
    f = wl.small_case(9, 4, 4099, dtype="f32", temperature=0.8, greedy_below=3, case_id=951)
    dl = to_dev(np.array([0, 1, 2, 3, 4, 4, 2, 0, 4], np.int32))
    ex, st = _both(f, f.taus[0], draft_len=dl, row_temperature=to_dev(f.row_temperature))
    for a, b in zip(ex, st):
        np.testing.assert_array_equal(a, b)
    ex, st = _both(small, 0.0, top_k=40, top_p=0.9)
    for a, b in zip(ex, st):
        np.testing.assert_array_equal(a, b)
    # a small batch of wide rows: several workgroups share a sequence's tail, their tickets lie in the static array,
    # which by now holds whatever the calls above left there; twice, so that the second call meets the first one's
    wide = wl.config3(B=6)
    for _ in range(2):
        ex, st = _both(wide, wide.taus[0])
        for a, b in zip(ex, st):
            np.testing.assert_array_equal(a, b)
    assert (st[0] < wide.gamma).any()                            # residual draws took part


def test_static_scratch_entry_refuses_what_does_not_fit():
    B, g, V = 1024, 8, 32000                                    # 17 408 rows: 34 MB of partial sums
    assert hb.hola_workspace_bytes_ex(B, g, V) > hb.HOLA_STATIC_SCRATCH_BYTES
    a = hb.VerifyArgs()
    fake = 0x1000                                               # never dereferenced: the size check comes first
    a.target_logits = a.draft_logits = a.draft_tokens = a.out_accept_len = a.out_next_token = fake
    a.dtype, a.B, a.gamma, a.V = hb.HOLA_DTYPE_BF16, B, g, V
    a.temperature, a.entropy_threshold = 1.0, 2.0
    assert hb.lib().hola_verify_ex_static(C.byref(a)) == hb.HOLA_ERR_WORKSPACE
    a.B, a.top_k = 256, 50                                      # filtered headline-sized batch: candidate lists do not fit
    assert hb.lib().hola_verify_ex_static(C.byref(a)) == hb.HOLA_ERR_WORKSPACE
    a.B, a.top_k, a.gamma = 4, 0, 0                             # argument errors as in hola_verify_ex
    assert hb.lib().hola_verify_ex_static(C.byref(a)) == hb.HOLA_ERR_INVALID_ARG
    assert hb.lib().hola_verify_ex_static(None) == hb.HOLA_ERR_INVALID_ARG
    a.gamma, a.B = 3, 0
    assert hb.lib().hola_verify_ex_static(C.byref(a)) == hb.HOLA_OK     # empty batch: nothing to do


def test_static_scratch_entry_in_a_hip_graph():
    """The use it exists for: captured once, replayed with eager work in between; no allocation may happen."""
    w = wl.small_case(24, 4, 20011, dtype="bf16", temperature=0.8, case_id=952)
    B, g, V = w.B, w.gamma, w.V
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    outs = [torch.zeros(B, dtype=torch.int32, device=DEV), torch.zeros(B, dtype=torch.int32, device=DEV),
            torch.zeros((B, g), dtype=torch.float32, device=DEV)]

    def call(stream=None):
        hb.hola_verify_ex_static(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                                 temperature=w.temperature, entropy_threshold=0.0, out_accept_len=outs[0],
                                 out_next_token=outs[1], out_entropy=outs[2], stream=stream)

    call()                                                       # the first call on the device looks the array up
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call(stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for o in outs:
            o.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), f"replay {rep} differs from the eager call"
        call()
        torch.cuda.synchronize()
