"""Pins of the oracle's whole verify step and of the hierarchical driver (CPU only).

The step is a randomised procedure, so it is pinned by what must hold whatever the seed:
invariants the paper's gate fixes (Section 3.1, Equation (1), Algorithm 1 Step 1), the
defining property of the draft-and-verify rule (gate off: output marginal = target p), brute
force over the per-position booleans, and reductions to library routines.
"""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import hola_oracle as orc
from paper_2506_18952_amd import workloads as wl


def _softmax(x, T=1.0):
    return scipy.special.softmax(np.asarray(x, np.float64) / T, axis=-1)


def _case(B=6, g=4, V=97, dtype="f32", T=1.0, seed=11, **kw):
    return wl.small_case(B, g, V, dtype=dtype, temperature=T, seed=seed, **kw)


# ----------------------------------------------------------------------------- gate (the paper's part)
def test_gate_is_strict_and_uses_draft_entropy():
    w = _case()
    r = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, 0.0)
    for b in range(w.B):
        for j in range(w.gamma):
            H = scipy.stats.entropy(_softmax(w.draft[b, j], w.temperature))
            assert r.entropy64[b, j] == pytest.approx(H, rel=1e-12)         # entropy of the DRAFT row
    # tau exactly equal to an entropy does not fire (strict <); the next float above does
    H00 = float(np.float32(r.entropy64[0, 0]))
    up = float(np.nextafter(np.float32(H00), np.float32(np.inf)))
    dn = float(np.nextafter(np.float32(H00), np.float32(-np.inf)))
    for tau, want in ((up, r.entropy64[0, 0] < up), (dn, r.entropy64[0, 0] < dn)):
        rr = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, tau)
        assert bool(rr.gate[0, 0]) == bool(want)
    x = np.zeros((1, 2, 8), np.float32)                                       # uniform rows: H = ln 8 exactly
    tau = float(np.float32(math.log(8)))
    rr = orc.verify(x, x[:, :1], np.zeros((1, 1), np.int32), 0, 1.0, tau)
    assert bool(rr.gate[0, 0]) == (rr.entropy64[0, 0] < tau)


def test_gate_off_and_gate_always():
    w = _case(B=16, g=5)
    off = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, 0.0)     # H >= 0: never fires
    assert not off.gate.any()
    neg = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, -1.0)
    assert np.array_equal(neg.accept_len, off.accept_len) and np.array_equal(neg.next_token, off.next_token)
    inf = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, float("inf"))
    assert inf.gate.all() and np.all(inf.accept_len == w.gamma)               # everything kept: bonus token
    for b in range(w.B):                                                      # bonus = categorical draw from p
        u2 = orc.hsd_uniforms(w.seed, b, w.gamma, 0)[1]
        p = _softmax(w.target[b, w.gamma], w.temperature)
        C = np.cumsum(p)
        assert inf.next_token[b] == int(np.searchsorted(C, u2 * C[-1], side="right"))


def test_gate_accepts_even_when_target_probability_is_zero():
    """'Directly accepted': the gate does not look at the verifier (Section 3.1)."""
    w = _case(B=4, g=3)
    P = w.target.copy()
    for b in range(w.B):
        P[b, 0, w.tokens[b, 0]] = -np.inf                                     # p(x) = 0 at position 0
    on = orc.verify(P, w.draft, w.tokens, w.seed, w.temperature, float("inf"))
    assert np.all(on.accept_len == w.gamma)
    off = orc.verify(P, w.draft, w.tokens, w.seed, w.temperature, 0.0)
    assert np.all(off.accept_len == 0)                                        # gate off: always rejected


def test_accept_len_is_monotone_in_tau():
    w = _case(B=40, g=6, V=211, seed=5)
    prev = None
    for tau in np.linspace(0.0, math.log(w.V) + 0.1, 25):
        r = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, float(tau))
        if prev is not None:
            assert np.all(r.accept_len >= prev)
        prev = r.accept_len


# ----------------------------------------------------------------------------- ratio test / first reject
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identical_models_accept_everything(dtype):
    w = _case(B=12, g=5, V=300, dtype=dtype, T=0.8)
    D = w.target[:, :w.gamma]
    for seed in range(20):
        r = orc.verify(w.target, D, w.tokens, seed, w.temperature, 0.0)
        assert np.all(r.accept_len == w.gamma) and r.ratio_ok.all()


def test_zero_target_probability_always_rejected_gate_off():
    w = _case(B=8, g=4, V=64)
    P = w.target.copy()
    for b in range(w.B):
        P[b, 2, w.tokens[b, 2]] = -np.inf
    for seed in range(50):
        r = orc.verify(P, w.draft, w.tokens, seed, w.temperature, 0.0)
        assert np.all(r.accept_len <= 2) and not r.ratio_ok[:, 2].any()


def test_out_of_range_token_is_rejected_gate_off():
    w = _case(B=3, g=3, V=50)
    tok = w.tokens.copy()
    tok[0, 1], tok[1, 0], tok[2, 2] = -1, w.V, 10 ** 6
    r = orc.verify(w.target, w.draft, tok, w.seed, w.temperature, 0.0)
    assert r.accept_len[0] <= 1 and r.accept_len[1] == 0 and r.accept_len[2] <= 2


def test_decisions_recomputed_by_brute_force():
    """Every boolean, the scan and the sample rebuilt in Python from scipy probabilities."""
    for dtype, T in (("f32", 1.0), ("bf16", 0.8)):
        w = _case(B=10, g=6, V=401, dtype=dtype, T=T, seed=21)
        T32 = float(np.float32(T))
        tau = 0.6 * math.log(w.V)
        r = orc.verify(w.target, w.draft, w.tokens, w.seed, T32, tau)
        tau32 = float(np.float32(tau))
        for b in range(w.B):
            a = w.gamma
            for j in range(w.gamma):
                q = _softmax(wl.as_f32(w.draft[b, j]), T32)
                p = _softmax(wl.as_f32(w.target[b, j]), T32)
                H = scipy.stats.entropy(q)
                u = orc.hsd_uniforms(w.seed, b, j, 0)[0]
                x = w.tokens[b, j]
                gate, ok = H < tau32, u * q[x] < p[x]
                if min(abs(H - tau32), abs(u - p[x] / q[x])) > 1e-9:
                    assert bool(r.gate[b, j]) == gate and bool(r.ratio_ok[b, j]) == ok
                assert r.gate_margin[b, j] == pytest.approx(abs(H - tau32), abs=1e-10)
                assert r.ratio_margin[b, j] == pytest.approx(abs(u - p[x] / q[x]), rel=1e-9, abs=1e-12)
            acc = np.logical_or(r.gate[b], r.ratio_ok[b])
            rej = np.flatnonzero(~acc)
            a = int(rej[0]) if len(rej) else w.gamma                          # first-reject: python scan
            assert r.accept_len[b] == a
            u2 = orc.hsd_uniforms(w.seed, b, a, 0)[1]
            p = _softmax(wl.as_f32(w.target[b, a]), T32)
            wts = p if a == w.gamma else np.maximum(0.0, p - _softmax(wl.as_f32(w.draft[b, a]), T32))
            C = np.cumsum(wts)
            if r.sample_margin[b] > 1e-9:
                assert r.next_token[b] == int(np.searchsorted(C, u2 * C[-1], side="right"))
            assert r.Z[b] == pytest.approx(C[-1], rel=1e-10)


def test_identical_rows_rejected_token_falls_back_to_target():
    """Z = 0 at a rejection (p == q and p(x) = 0 through an out-of-range token): sample from p."""
    w = _case(B=1, g=2, V=40)
    D = w.target[:, :2].copy()
    tok = np.array([[w.V + 3, 1]], np.int32)
    r = orc.verify(w.target, D, tok, 9, 1.0, 0.0)
    assert r.accept_len[0] == 0
    p = _softmax(w.target[0, 0])
    C = np.cumsum(p)
    u2 = orc.hsd_uniforms(9, 0, 0, 0)[1]
    assert r.next_token[0] == int(np.searchsorted(C, u2 * C[-1], side="right"))


def test_ragged_draft_len_and_seq_base():
    w = _case(B=9, g=5, V=120)
    lens = np.array([0, 1, 2, 3, 4, 5, 5, 2, 0], np.int32)
    tau = 0.3 * math.log(w.V)
    r = orc.verify(w.target, w.draft, w.tokens, 3, 1.0, tau, draft_len=lens)
    assert np.all(r.accept_len <= lens)
    for b in range(w.B):
        assert np.all(r.entropy[b, lens[b]:] == -1.0)
        # row b of the batch equals a B=1 call with seq_base = b
        one = orc.verify(w.target[b:b + 1], w.draft[b:b + 1], w.tokens[b:b + 1], 3, 1.0, tau,
                         draft_len=lens[b:b + 1], seq_base=b)
        assert one.accept_len[0] == r.accept_len[b] and one.next_token[0] == r.next_token[b]
        # a sequence cut to len drafts equals the same sequence given only those drafts
        L = int(lens[b])
        if 0 < L < w.gamma:
            cut = orc.verify(w.target[b:b + 1, :L + 1], w.draft[b:b + 1, :L], w.tokens[b:b + 1, :L],
                             3, 1.0, tau, seq_base=b)
            assert cut.accept_len[0] == r.accept_len[b] and cut.next_token[0] == r.next_token[b]
    # determinism, and independence from the thread count
    r1 = orc.verify(w.target, w.draft, w.tokens, 3, 1.0, tau, draft_len=lens, num_threads=1)
    r3 = orc.verify(w.target, w.draft, w.tokens, 3, 1.0, tau, draft_len=lens, num_threads=3)
    for f in ("accept_len", "next_token", "entropy"):
        assert np.array_equal(getattr(r1, f), getattr(r3, f)) and np.array_equal(getattr(r1, f), getattr(r, f))


# ----------------------------------------------------------------------------- greedy rows
def test_greedy_rows_follow_argmax():
    w = wl.small_case(12, 4, 150, greedy_below=6, temperature=0.7, seed=2)
    assert np.all(w.row_temperature[:6] == 0) and np.all(w.row_temperature[6:] > 0)
    r = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, 0.0, row_temperature=w.row_temperature)
    for b in range(6):
        am = np.argmax(w.target[b], axis=-1)
        match = w.tokens[b] == am[:w.gamma]
        a = int(np.flatnonzero(~match)[0]) if (~match).any() else w.gamma
        assert r.accept_len[b] == a and r.next_token[b] == am[a]
        for j in range(w.gamma):                                             # gate entropy at T = 1
            assert r.entropy64[b, j] == pytest.approx(scipy.stats.entropy(_softmax(w.draft[b, j])), rel=1e-12)
    # stochastic rows are unaffected by the greedy ones next to them
    s = orc.verify(w.target[6:], w.draft[6:], w.tokens[6:], w.seed, w.temperature, 0.0, seq_base=6)
    assert np.array_equal(s.accept_len, r.accept_len[6:]) and np.array_equal(s.next_token, r.next_token[6:])


def test_greedy_equals_stochastic_on_one_hot_like_logits():
    rng = np.random.default_rng(8)
    B, g, V = 6, 3, 30
    P = rng.standard_normal((B, g + 1, V)).astype(np.float32)
    hot = rng.integers(0, V, (B, g + 1))
    for b in range(B):
        for j in range(g + 1):
            P[b, j, hot[b, j]] += 1e4
    D = P[:, :g].copy()
    tok = hot[:, :g].astype(np.int32)
    tok[1, 1] = (tok[1, 1] + 1) % V                                          # one wrong draft
    st = orc.verify(P, D, tok, 1, 1.0, 0.0)
    gr = orc.verify(P, D, tok, 1, 1.0, 0.0, row_temperature=np.zeros(B, np.float32))
    assert np.array_equal(st.accept_len, gr.accept_len) and np.array_equal(st.next_token, gr.next_token)
    assert gr.accept_len[1] == 1 and gr.next_token[1] == hot[1, 1]


# ----------------------------------------------------------------------------- output marginal = p (gate off)
def _exact_output_marginal(P_row, D_row, T):
    """sum_x q_x [ acc(x) 1(y = x) + (1 - acc(x)) res(y) ] from the oracle's own parts, with the
    accept and selection frequencies counted over the whole uniform lattice."""
    V = P_row.shape[0]
    lseP, _, _ = orc.row_stats(P_row, T)
    lseD, _, _ = orc.row_stats(D_row, T)
    p = np.exp(P_row.astype(np.float64) / T - lseP)
    q = np.exp(D_row.astype(np.float64) / T - lseD)
    res_w = orc.residual_weights(P_row, D_row, T)
    res = orc.inverse_cdf_lattice_hist(res_w, 16) / (2 ** 24 / 16)
    out = np.zeros(V)
    for x in range(V):
        acc = orc.ratio_accept_lattice_count(p[x], q[x], 16) / (2 ** 24 / 16)
        out[x] += q[x] * acc
        out += q[x] * (1.0 - acc) * res
    return out, p


@pytest.mark.parametrize("V", [3, 4, 6])
def test_single_position_output_marginal_equals_target(V):
    rng = np.random.default_rng(V)
    for T in (1.0, 0.5):
        P = (1.5 * rng.standard_normal(V)).astype(np.float32)
        D = (1.5 * rng.standard_normal(V)).astype(np.float32)
        out, p = _exact_output_marginal(P, D, T)
        np.testing.assert_allclose(out, p, atol=4 * V * 16 * 2.0 ** -24)


def test_emitted_tokens_follow_target_through_the_entry_point():
    """Monte Carlo through oracle_verify itself (gate off): with drafts drawn from q, the token
    emitted at position 0 is distributed as p_0, and the one at position 1 (given position 0 was
    accepted) as p_1.  Chi-square at fixed seeds."""
    rng = np.random.default_rng(99)
    V, g, N = 5, 2, 200_000
    P1 = (1.2 * rng.standard_normal((g + 1, V))).astype(np.float32)
    D1 = (1.2 * rng.standard_normal((g, V))).astype(np.float32)
    P = np.broadcast_to(P1, (N, g + 1, V)).copy()
    D = np.broadcast_to(D1, (N, g, V)).copy()
    q = _softmax(D1)
    tok = np.stack([rng.choice(V, size=N, p=q[j]) for j in range(g)], axis=1).astype(np.int32)
    r = orc.verify(P, D, tok, 12345, 1.0, 0.0)
    p = _softmax(P1)
    first = np.where(r.accept_len >= 1, tok[:, 0], r.next_token)
    chi0 = scipy.stats.chisquare(np.bincount(first, minlength=V), N * p[0])
    assert chi0.pvalue > 1e-3
    sel = r.accept_len >= 1
    second = np.where(r.accept_len[sel] >= 2, tok[sel, 1], r.next_token[sel])
    chi1 = scipy.stats.chisquare(np.bincount(second, minlength=V), sel.sum() * p[1])
    assert chi1.pvalue > 1e-3
    # acceptance rate at position 0 = sum_i min(p_i, q_i)
    rate = np.minimum(p[0], q[0]).sum()
    assert abs((r.accept_len >= 1).mean() - rate) < 5 * math.sqrt(rate * (1 - rate) / N)
    # a wrong residual (e.g. sampling the rejection from p itself) would fail chi0: check the test has teeth
    bad = np.where(r.accept_len >= 1, tok[:, 0], rng.choice(V, size=N, p=p[0]))
    assert scipy.stats.chisquare(np.bincount(bad, minlength=V), N * p[0]).pvalue < 1e-6


# ----------------------------------------------------------------------------- sample_interval helper
def test_sample_interval_brackets_the_sampling_uniform():
    w = _case(B=10, g=4, V=83, seed=4)
    call = orc.VerifyCall(w.target, w.draft, w.tokens, w.seed, 1.0, 0.0)
    r = call.run()
    for b in range(w.B):
        lo, hi = call.sample_interval(b, int(r.accept_len[b]), int(r.next_token[b]))
        u2 = orc.hsd_uniforms(w.seed, b, int(r.accept_len[b]), 0)[1]
        assert lo <= u2 < hi or r.sample_margin[b] < 1e-12


def test_force_accept_len_moves_only_the_stop_row():
    w = _case(B=5, g=4, V=60, seed=4)
    base = orc.verify(w.target, w.draft, w.tokens, w.seed, 1.0, 0.0)
    force = np.array([-1, 0, 4, 2, -1], np.int32)
    r = orc.verify(w.target, w.draft, w.tokens, w.seed, 1.0, 0.0, force_accept_len=force)
    assert r.accept_len[0] == base.accept_len[0] and r.next_token[0] == base.next_token[0]
    assert list(r.accept_len[1:4]) == [0, 4, 2]
    p = _softmax(w.target[2, 4])                                              # forced to the bonus row
    C = np.cumsum(p)
    assert r.next_token[2] == int(np.searchsorted(C, orc.hsd_uniforms(w.seed, 2, 4, 0)[1] * C[-1], side="right"))


# ----------------------------------------------------------------------------- hierarchical driver
def _hier_case(B=20, g=3, V=50, seed=3):
    rng = np.random.default_rng(seed)
    base = (1.5 * rng.standard_normal((B, g + 2, V))).astype(np.float32)
    small = base[:, :g] + rng.standard_normal((B, g, V)).astype(np.float32)
    mid = base[:, :g + 1] + 0.4 * rng.standard_normal((B, g + 1, V)).astype(np.float32)
    q = _softmax(small)
    tok = np.array([[rng.choice(V, p=q[b, j]) for j in range(g)] for b in range(B)], np.int32)
    return [small, mid, base], tok


def test_two_level_is_two_one_level_calls():
    models, tok = _hier_case()
    B, g, V = models[0].shape
    taus = [0.4 * math.log(V), 0.6 * math.log(V)]
    h = orc.hsd_verify(models, tok, 3, 1.0, taus)
    l1 = orc.verify(models[1], models[0], tok, 3, 1.0, taus[0], level=0)
    assert np.array_equal(h.level_accept[0], l1.accept_len) and np.array_equal(h.level_next[0], l1.next_token)
    tok2 = np.full((B, g + 1), -1, np.int32)
    for b in range(B):
        a = l1.accept_len[b]
        tok2[b, :a] = tok[b, :a]
        tok2[b, a] = l1.next_token[b]                                        # accepted prefix + next token
    l2 = orc.verify(models[2], models[1], tok2, 3, 1.0, taus[1], draft_len=l1.accept_len + 1, level=1)
    assert np.array_equal(h.accept_len, l2.accept_len) and np.array_equal(h.next_token, l2.next_token)
    assert np.array_equal(h.tokens[:, :g + 1], tok2) and np.all(h.tokens[:, g + 1] == -1)
    np.testing.assert_array_equal(h.entropy[0][:, :g], l1.entropy)
    np.testing.assert_array_equal(h.entropy[1], l2.entropy)
    # the intermediate's entropy seen by level 2 is what level 1 computed for its target rows
    for b in range(B):
        for j in range(l1.accept_len[b] + 1):
            assert l2.entropy64[b, j] == l1.H_target[b, j]
    # level 2 draws different uniforms than level 1 (level is a counter word)
    assert orc.hsd_uniforms(3, 0, 0, 0) != orc.hsd_uniforms(3, 0, 0, 1)


def test_two_level_survivors_only_reading():
    """The alternative reading: level 2 gets only the tokens level 1 kept (no next token)."""
    models, tok = _hier_case(B=30)
    B, g, V = models[0].shape
    taus = [0.0, 0.5 * math.log(V)]
    h = orc.hsd_verify(models, tok, 3, 1.0, taus, survivors_only=True)
    l1 = orc.verify(models[1], models[0], tok, 3, 1.0, taus[0], level=0)
    tok2 = np.full((B, g + 1), -1, np.int32)
    for b in range(B):
        tok2[b, :l1.accept_len[b]] = tok[b, :l1.accept_len[b]]
    l2 = orc.verify(models[2], models[1], tok2, 3, 1.0, taus[1], draft_len=l1.accept_len, level=1)
    assert np.array_equal(h.accept_len, l2.accept_len) and np.array_equal(h.next_token, l2.next_token)
    assert np.array_equal(h.tokens[:, :g + 1], tok2) and np.all(h.accept_len <= l1.accept_len)
    assert (l1.accept_len == 0).any()                    # an empty survivor list: the level samples its row 0
    dflt = orc.hsd_verify(models, tok, 3, 1.0, taus)
    assert not np.array_equal(dflt.tokens, h.tokens)     # the two readings differ


def test_two_level_first_emitted_token_follows_final_target():
    """Gate off, tiny V: over many sequences with the same logits, the first emitted token of the
    two-level chain is distributed as the final target's p_0 (lossless chain)."""
    rng = np.random.default_rng(17)
    V, g, N = 4, 1, 150_000
    base = (1.3 * rng.standard_normal((g + 2, V))).astype(np.float32)
    small1 = (base[:g] + rng.standard_normal((g, V))).astype(np.float32)
    mid1 = (base[:g + 1] + 0.5 * rng.standard_normal((g + 1, V))).astype(np.float32)
    models = [np.broadcast_to(m, (N,) + m.shape).copy() for m in (small1, mid1, base)]
    q = _softmax(small1)
    tok = rng.choice(V, size=(N, 1), p=q[0]).astype(np.int32)
    h = orc.hsd_verify(models, tok, 77, 1.0, [0.0, 0.0])
    first = np.where(h.accept_len >= 1, h.tokens[:, 0], h.next_token)
    p = _softmax(base)
    assert scipy.stats.chisquare(np.bincount(first, minlength=V), N * p[0]).pvalue > 1e-3
    # whereas the intermediate's p_0 is a different distribution the test can tell apart
    pm = _softmax(mid1)
    assert scipy.stats.chisquare(np.bincount(first, minlength=V), N * pm[0]).pvalue < 1e-6


def test_three_level_runs_and_shapes():
    rng = np.random.default_rng(5)
    B, g, V = 7, 2, 33
    models = [(rng.standard_normal((B, g + k, V))).astype(np.float32) for k in range(4)]
    tok = rng.integers(0, V, (B, g)).astype(np.int32)
    h = orc.hsd_verify(models, tok, 1, 1.0, [1.0, 2.0, 3.0])
    assert h.tokens.shape == (B, g + 3) and h.entropy.shape == (3, B, g + 2)
    assert np.all(h.accept_len <= h.level_accept[1] + 1) and np.all(h.level_accept[1] <= h.level_accept[0] + 1)


def test_three_level_is_three_one_level_calls():
    """The driver's loop at k = 1, 2, 3: each level is the one-level step on the previous level's kept tokens
    followed by its next token, with Philox level word k - 1 and the middle model as the draft."""
    rng = np.random.default_rng(21)
    B, g, V = 24, 3, 61
    base = (1.5 * rng.standard_normal((B, g + 3, V))).astype(np.float32)
    models = [(base[:, :g + k] + (0.9 - 0.3 * k) * rng.standard_normal((B, g + k, V))).astype(np.float32)
              for k in range(3)] + [base]
    q = _softmax(models[0])
    tok = np.array([[rng.choice(V, p=q[b, j]) for j in range(g)] for b in range(B)], np.int32)
    taus = [0.3 * math.log(V), 0.5 * math.log(V), 0.7 * math.log(V)]
    for survivors_only in (False, True):
        h = orc.hsd_verify(models, tok, 9, 1.0, taus, seq_base=1000, survivors_only=survivors_only)
        cur, lens = tok, np.full(B, g, np.int32)
        for k in range(1, 4):
            lv = orc.verify(models[k], models[k - 1], cur, 9, 1.0, taus[k - 1], draft_len=lens, level=k - 1, seq_base=1000)
            np.testing.assert_array_equal(h.level_accept[k - 1], lv.accept_len)
            np.testing.assert_array_equal(h.level_next[k - 1], lv.next_token)
            np.testing.assert_array_equal(h.entropy[k - 1][:, :g + k - 1], lv.entropy)
            assert np.all(h.entropy[k - 1][:, g + k - 1:] == -1.0)
            if k < 3:
                nxt = np.full((B, g + k), -1, np.int32)
                for b in range(B):
                    a = lv.accept_len[b]
                    nxt[b, :a] = cur[b, :a]
                    if not survivors_only:
                        nxt[b, a] = lv.next_token[b]
                cur, lens = nxt, lv.accept_len + (0 if survivors_only else 1)
        np.testing.assert_array_equal(h.accept_len, lv.accept_len)
        np.testing.assert_array_equal(h.next_token, lv.next_token)
        for b in range(B):
            assert np.array_equal(h.tokens[b, :lens[b]], cur[b, :lens[b]]) and np.all(h.tokens[b, lens[b]:] == -1)
        assert len(set(h.level_accept[0].tolist())) > 1 and len(set(h.accept_len.tolist())) > 1
