"""Pins of the oracle's paper-literal mode (Equation (1) without stopping), CPU only."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import hola_oracle as orc
from paper_2506_18952_amd import workloads as wl


def _softmax(x, T=1.0):
    return scipy.special.softmax(np.asarray(x, np.float64) / T, axis=-1)


def test_literal_gate_keeps_draft_else_draws_from_target():
    w = wl.small_case(12, 5, 211, dtype="bf16", temperature=0.8, case_id=400)
    T = float(np.float32(0.8))
    tau = 0.55 * math.log(w.V)
    tau32 = float(np.float32(tau))
    r = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, tau)
    n_gate = 0
    for b in range(w.B):
        calls = 0
        for t in range(w.gamma):
            H = scipy.stats.entropy(_softmax(wl.as_f32(w.draft[b, t]), T))
            assert r.entropy64[b, t] == pytest.approx(H, rel=1e-12)
            if abs(H - tau32) < 1e-9:
                continue
            if H < tau32:                                   # Equation (1), first case: the draft token
                assert r.gate[b, t] == 1 and r.tokens[b, t] == w.tokens[b, t]
                n_gate += 1
            else:                                           # otherwise: f_ver = a draw from the target row
                calls += 1
                p = _softmax(wl.as_f32(w.target[b, t]), T)
                C = np.cumsum(p)
                u2 = orc.hsd_uniforms(w.seed, b, t, 0)[1]
                if r.sample_margin[b, t] > 1e-9:
                    assert r.tokens[b, t] == int(np.searchsorted(C, u2 * C[-1], side="right"))
        assert r.calls[b] == calls == int((r.gate[b] == 0).sum())
    assert 0 < n_gate < w.B * w.gamma                        # both branches were exercised


def test_literal_extremes_ragged_and_greedy():
    w = wl.small_case(8, 4, 97, greedy_below=4, temperature=0.7, case_id=401)
    lens = np.array([4, 0, 2, 3, 4, 1, 0, 4], np.int32)
    all_gate = orc.verify_literal(w.target, w.draft, w.tokens, 1, 0.7, float("inf"), draft_len=lens,
                                  row_temperature=w.row_temperature)
    none = orc.verify_literal(w.target, w.draft, w.tokens, 1, 0.7, 0.0, draft_len=lens,
                              row_temperature=w.row_temperature)
    for b in range(w.B):
        L = lens[b]
        assert np.array_equal(all_gate.tokens[b, :L], w.tokens[b, :L]) and np.all(all_gate.tokens[b, L:] == -1)
        assert all_gate.calls[b] == 0 and none.calls[b] == L      # O(k) verifier calls: k = non-gated positions
        assert np.all(none.entropy[b, L:] == -1.0)
        if b < 4:                                                # greedy rows: the verifier's argmax
            assert np.array_equal(none.tokens[b, :L], np.argmax(w.target[b, :L], axis=-1))
    # positions are independent: changing one target row changes only that position
    P = w.target.copy()
    P[7, 2] = P[7, 2][::-1].copy()
    moved = orc.verify_literal(P, w.draft, w.tokens, 1, 0.7, 0.0, draft_len=lens, row_temperature=w.row_temperature)
    same = np.ones_like(none.tokens, bool)
    same[7, 2] = False
    assert np.array_equal(moved.tokens[same], none.tokens[same])


def test_literal_sampled_positions_follow_the_target_distribution():
    rng = np.random.default_rng(3)
    V, N = 5, 100_000
    P1 = (1.3 * rng.standard_normal((2, V))).astype(np.float32)
    D1 = (1.3 * rng.standard_normal((1, V))).astype(np.float32)
    P = np.broadcast_to(P1, (N, 2, V)).copy()
    D = np.broadcast_to(D1, (N, 1, V)).copy()
    tok = np.zeros((N, 1), np.int32)
    r = orc.verify_literal(P, D, tok, 99, 1.0, 0.0)
    p = _softmax(P1[0])
    assert scipy.stats.chisquare(np.bincount(r.tokens[:, 0], minlength=V), N * p).pvalue > 1e-3


def test_forced_gates_and_the_row_interval_aid():
    """Test aids: a forced gate only swaps the branch of Equation (1) at that position; the CDF interval of a token
    under softmax(row / T) is numpy's cumsum, and the oracle's own draw lies inside its interval."""
    w = wl.small_case(10, 4, 151, dtype="bf16", temperature=0.9, case_id=402)
    T = float(np.float32(0.9))
    tau = 0.5 * math.log(w.V)
    base = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, tau)
    all_draft = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, tau, force_gate=np.ones((w.B, w.gamma), np.int8))
    all_drawn = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, tau, force_gate=np.zeros((w.B, w.gamma), np.int8))
    never = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, -1.0)
    np.testing.assert_array_equal(all_draft.tokens, w.tokens)
    assert np.all(all_draft.calls == 0)
    np.testing.assert_array_equal(all_drawn.tokens, never.tokens)
    np.testing.assert_array_equal(all_drawn.calls, never.calls)
    unforced = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, tau, force_gate=np.full((w.B, w.gamma), -1, np.int8))
    np.testing.assert_array_equal(unforced.tokens, base.tokens)
    one = np.full((w.B, w.gamma), -1, np.int8)
    b, t = 3, 2
    one[b, t] = 0 if base.gate[b, t] else 1
    flipped = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, T, tau, force_gate=one)
    same = np.ones((w.B, w.gamma), bool); same[b, t] = False
    np.testing.assert_array_equal(flipped.tokens[same], base.tokens[same])
    assert flipped.tokens[b, t] == (never.tokens[b, t] if base.gate[b, t] else w.tokens[b, t])
    for b in range(w.B):
        for t in range(w.gamma):
            p = _softmax(wl.as_f32(w.target[b, t]), T)
            C = np.cumsum(p)
            k = int(never.tokens[b, t])
            lo, hi = orc.row_interval(w.target[b, t], T, k)
            assert lo == pytest.approx((C[k - 1] if k else 0.0) / C[-1], abs=1e-13) and hi == pytest.approx(C[k] / C[-1], abs=1e-13)
            u2 = orc.hsd_uniforms(w.seed, b, t, 0)[1]
            assert lo <= u2 < hi or never.sample_margin[b, t] < 1e-12
    assert orc.row_interval(w.target[0, 0], T, w.V) is None and orc.row_interval(w.target[0, 0], T, -1) is None
