"""Pins of the oracle's token-tree verify step, CPU only.  The paper drafts one token per position; several
candidates per position follow the published recursive rejection rule (children tried in order against a residual
that loses the draft distribution after every rejection).  Pinned here to the one-token step on chains, to a direct
numpy restatement in the closed form max(0, p - C q), to closed-form accept rates, and to the property the rule
exists for: whatever the tree, the emitted tokens follow the verifier's distributions."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import hola_oracle as orc
from paper_2506_18952_amd import workloads as wl


def _chain_parents(B, g):
    return np.tile(np.arange(-1, g - 1, dtype=np.int32), (B, 1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_is_the_one_token_step(dtype):
    w = wl.small_case(48, 5, 777, dtype=dtype, temperature=0.9, case_id=11)
    par = _chain_parents(w.B, w.gamma)
    dl = np.array([b % (w.gamma + 1) for b in range(w.B)], np.int32)
    for tau in (-1.0, 0.45 * math.log(w.V), 1e9):
        for kw in ({}, {"level": 3, "seq_base": 1 << 33}):
            ref = orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, draft_len=dl, **kw)
            t = orc.verify_tree(w.target, w.draft, w.tokens, par, w.seed, w.temperature, tau, n_nodes=dl, **kw)
            np.testing.assert_array_equal(t.accept_len, ref.accept_len)
            np.testing.assert_array_equal(t.next_token, ref.next_token)
            np.testing.assert_array_equal(t.entropy, ref.entropy)
            np.testing.assert_array_equal(t.sample_margin, ref.sample_margin)
            for b in range(w.B):
                a = t.accept_len[b]
                assert t.path[b, :a].tolist() == list(range(a)) and np.all(t.path[b, a:] == -1)
                tested = ~np.isnan(t.ratio_margin[b])
                np.testing.assert_array_equal(t.ratio_margin[b][tested], ref.ratio_margin[b][tested])
    assert len(set(ref.accept_len.tolist())) > 2


def _walk_numpy(P, D, tok, par, n_nodes, seed, T, tau, b, level=0, seq_base=0):
    """The same walk in the unnormalised closed form: after i rejections at a context the running distribution is
    max(0, p - C q) / Z with Z its sum and C the sum of the earlier Z's (1, then 1 + Z_1, ...)."""
    N = tok.shape[0]
    ctx, path = 0, []
    while True:
        p = scipy.special.softmax(wl.as_f32(P[ctx]).astype(np.float64) / T)
        kids = [n for n in range(n_nodes) if par[n] == ctx - 1]
        u2 = orc.hsd_uniforms(seed, seq_base + b, ctx, level)[1]
        if not kids:
            c = np.cumsum(p)
            return path, int(np.searchsorted(c, u2 * c[-1], side="right")), None
        q = scipy.special.softmax(wl.as_f32(D[ctx]).astype(np.float64) / T)
        gate = scipy.stats.entropy(q) < tau
        C, Z, kept, slack = 0.0, 1.0, None, np.inf
        for i, n in enumerate(kids):
            x = tok[n]
            if i == 0 and gate:
                kept = n
                break
            u = orc.hsd_uniforms(seed, seq_base + b, n, level)[0]
            r = max(0.0, p[x] - C * q[x])
            slack = min(slack, abs(u * q[x] * Z - r) / (q[x] * max(1.0, C)))
            if u * q[x] * Z < r:
                kept = n
                break
            C += Z
            Z = np.maximum(0.0, p - C * q).sum()
        if kept is None:
            wgt = np.maximum(0.0, p - C * q)
            c = np.cumsum(wgt)
            return path, int(np.searchsorted(c, u2 * c[-1], side="right")), slack
        path.append(kept)
        ctx = kept + 1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("widths", [[3], [2, 4, 4], [4, 3, 2, 1, 1], [1, 2, 1, 3]])
def test_walk_matches_a_numpy_restatement_in_closed_form(dtype, widths):
    w = wl.tree_case(24, widths, 211, dtype=dtype, temperature=1.1, draft_sigma=1.2, case_id=701 + len(widths))
    nn = np.array([w.N - (b % 3) for b in range(w.B)], np.int32)
    for tau in (-1.0, w.tau):
        t = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, n_nodes=nn)
        depths = []
        for b in range(w.B):
            path, nxt, _ = _walk_numpy(w.target[b], w.draft[b], w.node_token[b], w.node_parent[b], int(nn[b]), w.seed,
                                       float(np.float32(w.temperature)), tau, b)
            near = np.nanmin(np.r_[t.ratio_margin[b], t.sample_margin[b], t.gate_margin[b], np.inf]) < 1e-9
            if near:
                continue
            assert t.accept_len[b] == len(path) and t.path[b, :len(path)].tolist() == path, (b, path, t.path[b])
            assert t.next_token[b] == nxt, (b, nxt, t.next_token[b])
            depths.append(len(path))
        assert len(depths) >= w.B - 2
    assert max(depths) >= 1 or len(widths) == 1


def test_margin_of_a_later_child_is_in_unnormalised_units():
    V = 7
    rng = np.random.default_rng(3)
    P = rng.standard_normal((1, 4, V)).astype(np.float32)
    D = rng.standard_normal((1, 3, V)).astype(np.float32)
    p, q = scipy.special.softmax(P[0, 0].astype(np.float64)), scipy.special.softmax(D[0, 0].astype(np.float64))
    x = int(np.argmax(q - p))                                  # a token the verifier likes less: likely rejected
    tok = np.array([[x, x, x]], np.int32)
    par = np.array([[-1, -1, -1]], np.int32)
    for seed in range(200):
        t = orc.verify_tree(P, D, tok, par, seed, 1.0, -1.0)
        if t.accept_len[0] == 0 and not np.isnan(t.ratio_margin[0, 2]):
            break
    u0 = orc.hsd_uniforms(seed, 0, 0)[0]
    assert t.ratio_margin[0, 0] == pytest.approx(abs(u0 - p[x] / q[x]), rel=1e-12)
    Z1 = np.maximum(0, p - q).sum()
    r1 = max(0.0, p[x] - q[x])
    u1 = orc.hsd_uniforms(seed, 0, 1)[0]
    assert t.ratio_margin[0, 1] == pytest.approx(abs(u1 * q[x] * Z1 - r1) / q[x], rel=1e-9)
    Z2 = np.maximum(0, p - (1 + Z1) * q).sum()
    r2 = max(0.0, p[x] - (1 + Z1) * q[x])
    u2 = orc.hsd_uniforms(seed, 0, 2)[0]
    assert t.ratio_margin[0, 2] == pytest.approx(abs(u2 * q[x] * Z2 - r2) / (q[x] * (1 + Z1)), rel=1e-9)


def _star_inputs(rng, V, c, N_seq, sigma_q=1.0):
    """One context with c candidates drawn independently from q; the same two rows for every sequence."""
    p_row = (1.2 * rng.standard_normal(V)).astype(np.float32)
    q_row = (p_row + sigma_q * rng.standard_normal(V)).astype(np.float32)
    P = np.broadcast_to(np.r_[[p_row], rng.standard_normal((c, V)).astype(np.float32)], (N_seq, c + 1, V)).copy()
    D = np.broadcast_to(np.r_[[q_row], rng.standard_normal((c - 1, V)).astype(np.float32)], (N_seq, c, V)).copy()
    q = scipy.special.softmax(q_row.astype(np.float64))
    tok = rng.choice(V, size=(N_seq, c), p=q).astype(np.int32)
    par = np.full((N_seq, c), -1, np.int32)
    return P, D, tok, par, scipy.special.softmax(p_row.astype(np.float64)), q


def test_accept_rate_of_several_candidates_has_the_closed_form():
    """P(child i is the first kept) = prod_{j<i} (1 - a_j) * a_i with a_j = sum min(r_j, q), r_0 = p,
    r_{j+1} = max(0, r_j - q) normalised."""
    rng = np.random.default_rng(12)
    V, c, N = 6, 3, 120_000
    P, D, tok, par, p, q = _star_inputs(rng, V, c, N)
    t = orc.verify_tree(P, D, tok, par, 5, 1.0, -1.0)
    r, alive, want = p.copy(), 1.0, []
    for _ in range(c):
        a = np.minimum(r, q).sum()
        want.append(alive * a)
        alive *= 1 - a
        r = np.maximum(0, r - q)
        r /= r.sum()
    want.append(alive)
    which = np.where(t.accept_len == 1, t.path[:, 0], c)
    counts = np.bincount(which, minlength=c + 1)
    assert scipy.stats.chisquare(counts, N * np.asarray(want)).pvalue > 1e-3
    assert want[1] > 0.02 and want[2] > 0.005                   # the later candidates matter in this case
    # one candidate alone: the textbook accept rate sum min(p, q)
    t1 = orc.verify_tree(P[:, :2], D[:, :1], tok[:, :1], par[:, :1], 5, 1.0, -1.0)
    assert abs(t1.accept_len.mean() - np.minimum(p, q).sum()) < 4 * math.sqrt(0.25 / N)


def test_first_token_follows_the_verifier_whatever_the_number_of_candidates():
    rng = np.random.default_rng(21)
    V, N = 5, 150_000
    for c in (2, 4):
        P, D, tok, par, p, q = _star_inputs(rng, V, c, N, sigma_q=1.5)
        t = orc.verify_tree(P, D, tok, par, 9, 1.0, -1.0)
        first = np.where(t.accept_len >= 1, tok[np.arange(N), np.maximum(t.path[:, 0], 0)], t.next_token)
        counts = np.bincount(first, minlength=V)
        assert scipy.stats.chisquare(counts, N * p).pvalue > 1e-3
        assert scipy.stats.chisquare(counts, N * q).pvalue < 1e-6  # the drafter's distribution is told apart


def test_two_emitted_tokens_follow_the_verifier_conditionals():
    """Two candidates at the prefix, two under each of them; the verifier's row after a node depends on that node's
    token.  The first emitted token follows p(.), and given it the second follows p(. | first)."""
    rng = np.random.default_rng(33)
    V, N = 3, 200_000
    p0 = (rng.standard_normal(V)).astype(np.float32)
    q0 = (p0 + rng.standard_normal(V)).astype(np.float32)
    p1 = rng.standard_normal((V, V)).astype(np.float32)         # row x: the verifier after first token x
    q1 = (p1 + rng.standard_normal((V, V))).astype(np.float32)
    par = np.tile(np.array([-1, -1, 0, 0, 1, 1], np.int32), (N, 1))
    sm = lambda z: scipy.special.softmax(z.astype(np.float64), axis=-1)
    tok = np.zeros((N, 6), np.int32)
    tok[:, :2] = rng.choice(V, size=(N, 2), p=sm(q0))
    P = np.zeros((N, 7, V), np.float32)
    D = np.zeros((N, 6, V), np.float32)
    P[:, 0], D[:, 0] = p0, q0
    for k in (0, 1):                                            # contexts 1, 2: after node 0 / node 1
        P[:, 1 + k], D[:, 1 + k] = p1[tok[:, k]], q1[tok[:, k]]
        cdf = np.cumsum(sm(q1)[tok[:, k]], axis=-1)
        for j in (0, 1):
            tok[:, 2 + 2 * k + j] = (rng.random(N)[:, None] > cdf).sum(axis=-1).clip(0, V - 1)
    P[:, 3:] = rng.standard_normal((N, 4, V))                   # after the leaves: any rows
    t = orc.verify_tree(P, D, tok, par, 4, 1.0, -1.0)
    ar = np.arange(N)
    first = np.where(t.accept_len >= 1, tok[ar, np.maximum(t.path[:, 0], 0)], t.next_token)
    assert scipy.stats.chisquare(np.bincount(first, minlength=V), N * sm(p0)).pvalue > 1e-3
    went_on = t.accept_len >= 1
    second = np.where(t.accept_len >= 2, tok[ar, np.maximum(t.path[:, 1], 0)], t.next_token)
    assert (t.accept_len >= 2).mean() > 0.1
    for x in range(V):
        sel = went_on & (first == x)
        assert sel.sum() > 2000
        assert scipy.stats.chisquare(np.bincount(second[sel], minlength=V), sel.sum() * sm(p1[x])).pvalue > 1e-3


def test_gate_keeps_the_first_child_only():
    w = wl.tree_case(16, [3, 3, 2], 97, case_id=720)
    t = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 1e9)     # every context gated
    par = w.node_parent[0]
    spine, ctx = [], 0
    while True:
        kids = [n for n in range(w.N) if par[n] == ctx - 1]
        if not kids:
            break
        spine.append(kids[0])
        ctx = kids[0] + 1
    for b in range(w.B):
        assert t.accept_len[b] == len(spine) and t.path[b, :len(spine)].tolist() == spine
        assert np.all(np.isnan(t.ratio_margin[b]))               # no test was taken
    # the draw after the last kept node is a plain draw from that context's verifier row
    b = 3
    p = scipy.special.softmax(w.target[b, ctx].astype(np.float64))
    c = np.cumsum(p)
    u2 = orc.hsd_uniforms(w.seed, b, ctx)[1]
    assert t.next_token[b] == int(np.searchsorted(c, u2 * c[-1], side="right"))
    # entropies: contexts with children only
    has = np.array([(par == c - 1).any() for c in range(w.N)])
    assert np.all((t.entropy[0] >= 0) == has)
    q = scipy.special.softmax(w.draft[0, 0].astype(np.float64))
    assert t.entropy64[0, 0] == pytest.approx(scipy.stats.entropy(q), abs=1e-12)


def test_edge_cases():
    w = wl.tree_case(6, [2, 2], 53, case_id=730)
    # no node at all: a draw from the verifier's first row = the one-token step without drafts
    t = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, 1, 1.0, 0.0, n_nodes=np.zeros(6, np.int32))
    ref = orc.verify(w.target[:, :2], w.draft[:, :1], w.node_token[:, :1], 1, 1.0, 0.0, draft_len=np.zeros(6, np.int32))
    np.testing.assert_array_equal(t.next_token, ref.next_token)
    assert np.all(t.accept_len == 0) and np.all(t.path == -1) and np.all(t.entropy == -1)
    # a token outside the vocabulary is never kept; its siblings still are
    tok = w.node_token.copy()
    tok[:, 0] = -5
    t = orc.verify_tree(w.target, w.draft, tok, w.node_parent, 1, 1.0, -1.0)
    assert not (t.path[:, 0] == 0).any() and (t.path[:, 0] == 1).any()
    # a parent must be an earlier node
    bad = w.node_parent.copy()
    bad[2, 1] = 1
    with pytest.raises(ValueError):
        orc.verify_tree(w.target, w.draft, w.node_token, bad, 1, 1.0, 0.0)
    with pytest.raises(ValueError):
        orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, 1, 0.0, 0.0)   # greedy trees: not taken
    # q == p: the first child is always kept (u q < p fails only for u >= 1)
    t = orc.verify_tree(w.target, w.target[:, :w.N].copy(), w.node_token, w.node_parent, 1, 1.0, -1.0)
    assert np.all(t.path[:, 0] == 0)


def test_batch_rows_are_independent_and_thread_count_does_not_matter():
    w = wl.tree_case(12, [3, 2, 2], 151, dtype="bf16", temperature=0.9, case_id=740)
    full = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau, seq_base=100,
                           num_threads=4)
    one = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau, seq_base=100,
                          num_threads=1)
    for f in ("accept_len", "path", "next_token", "entropy", "sample_margin"):
        np.testing.assert_array_equal(getattr(full, f), getattr(one, f))
    for b in (0, 5, 11):                                        # a row alone, under its global sequence index
        r = orc.verify_tree(w.target[b:b + 1], w.draft[b:b + 1], w.node_token[b:b + 1], w.node_parent[b:b + 1], w.seed,
                            w.temperature, w.tau, seq_base=100 + b)
        assert r.accept_len[0] == full.accept_len[b] and r.next_token[0] == full.next_token[b]
        np.testing.assert_array_equal(r.path[0], full.path[b])
    other = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau, seq_base=0)
    assert not (np.array_equal(other.next_token, full.next_token) and np.array_equal(other.accept_len, full.accept_len))


def test_forced_node_and_probe_aids():
    """Test aids: forcing a node to the decision it takes anyway changes nothing; forcing the other decision changes
    the walk from that node on exactly as the rule says; the probed interval of the walk's own next token holds the
    sampling uniform and equals a numpy restatement of the final draw's weights."""
    w = wl.tree_case(24, [3, 3, 2], 401, dtype="f32", temperature=0.9, draft_sigma=1.2, case_id=720)
    T = float(np.float32(0.9))
    args = (w.target, w.draft, w.node_token, w.node_parent, w.seed, T, -1.0)
    base = orc.verify_tree(*args, probe_token=None)
    B, N = w.B, w.N
    # (a) a forced decision equal to the walk's own
    fn, fo = np.full(B, -1, np.int32), np.zeros(B, np.int32)
    for b in range(B):
        if base.accept_len[b] > 0:
            fn[b], fo[b] = base.path[b, 0], 1
    same = orc.verify_tree(*args, force_node=fn, force_outcome=fo)
    np.testing.assert_array_equal(same.path, base.path)
    np.testing.assert_array_equal(same.next_token, base.next_token)
    # (b) the first kept node forced to a rejection: the path no longer starts with it, and equals the numpy walk
    # over the tree with that node's token made unacceptable (r(x) = 0 rejects for every u)
    fo[:] = 0
    flipped = orc.verify_tree(*args, force_node=fn, force_outcome=fo)
    for b in range(B):
        if fn[b] >= 0:
            assert flipped.accept_len[b] == 0 or flipped.path[b, 0] != fn[b]
            assert flipped.accept_len[b] == 0 or flipped.path[b, 0] > fn[b]      # a later child of the prefix
        else:
            assert np.array_equal(flipped.path[b], base.path[b]) and flipped.next_token[b] == base.next_token[b]
    # (c) a rejected first child forced to be kept: the walk goes on below it
    fn2, fo2 = np.full(B, -1, np.int32), np.ones(B, np.int32)
    for b in range(B):
        if base.accept_len[b] == 0 or base.path[b, 0] != 0:
            fn2[b] = 0                                       # node 0 is the prefix's first child and was rejected
    kept = orc.verify_tree(*args, force_node=fn2, force_outcome=fo2)
    assert (fn2 >= 0).any()
    for b in range(B):
        if fn2[b] >= 0:
            assert kept.accept_len[b] >= 1 and kept.path[b, 0] == 0
    # (d) probe: the interval of the oracle's own next token
    pr = orc.verify_tree(*args, probe_token=base.next_token)
    for b in range(B):
        a = int(base.accept_len[b])
        ctx = int(base.path[b, a - 1]) + 1 if a else 0
        u2 = orc.hsd_uniforms(w.seed, b, ctx, 0)[1]
        assert pr.probe_lo[b] <= u2 < pr.probe_hi[b] or base.sample_margin[b] < 1e-12
        # numpy restatement of the final weights: max(0, p - C q) after the rejections at ctx
        p = scipy.special.softmax(w.target[b, ctx].astype(np.float64) / T)
        kids = [n for n in range(N) if w.node_parent[b, n] == ctx - 1]
        wgt = p
        if kids:
            q = scipy.special.softmax(w.draft[b, ctx].astype(np.float64) / T)
            C, Z = 0.0, 1.0
            for _ in kids:
                C += Z
                Z = np.maximum(0.0, p - C * q).sum()
            wgt = np.maximum(0.0, p - C * q)
        cs = np.cumsum(wgt)
        k = int(base.next_token[b])
        assert pr.probe_hi[b] - pr.probe_lo[b] == pytest.approx(wgt[k] / cs[-1], rel=1e-9, abs=1e-15)
        assert pr.probe_lo[b] == pytest.approx((cs[k - 1] if k else 0.0) / cs[-1], abs=1e-11)
    none = orc.verify_tree(*args, probe_token=np.full(B, -1, np.int32))
    assert np.all(np.isnan(none.probe_lo))
