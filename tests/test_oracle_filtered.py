"""Pins of the oracle's filtered (top-k / top-p) verify step, CPU only.  The paper does not filter; the
definition is the usual one (stable descending order, top-k prefix, then the shortest prefix reaching top_p of
the top-k mass), pinned here to numpy's stable sort and cumulative sums, to scipy on the kept subset, to closed
forms, to the unfiltered step when the filters are off, and to the property that makes the rule worth having:
with drafts drawn from the filtered q the emitted token follows the filtered p."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import hola_oracle as orc
from paper_2506_18952_amd import workloads as wl


def _np_keep(z, top_k, top_p):
    V = z.shape[0]
    order = np.argsort(-z, kind="stable")
    p = scipy.special.softmax(z)
    m = top_k if 0 < top_k < V else V
    m = min(m, int(np.isfinite(z).sum()))
    if top_p < 1.0:
        ps = p[order[:m]]
        c = np.cumsum(ps)
        m = min(m, int(np.searchsorted(c, top_p * c[-1], side="left")) + 1)
    keep = np.zeros(V, bool)
    keep[order[:m]] = True
    return keep


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("top_k,top_p", [(1, 1.0), (5, 1.0), (50, 1.0), (0, 0.3), (0, 0.9), (0, 0.999), (40, 0.8),
                                         (1000000, 1.0), (3, 0.0001)])
def test_keep_set_is_numpy_stable_sort_prefix(dtype, top_k, top_p):
    w = wl.small_case(3, 2, 2003, dtype=dtype, temperature=0.7, case_id=31)
    T = float(np.float32(0.7))
    for row in w.target.reshape(-1, w.V)[:5]:
        z = wl.as_f32(row).astype(np.float64) / T
        keep, lse, H, mg = orc.filter_row(row, T, top_k, top_p)
        want = _np_keep(z, top_k, top_p)
        if top_p < 1.0 and mg < 1e-12:
            continue                                          # the cut itself is a rounding matter
        assert np.array_equal(keep, want)
        assert lse == pytest.approx(scipy.special.logsumexp(z[keep]), abs=1e-12)
        assert H == pytest.approx(scipy.stats.entropy(scipy.special.softmax(z[keep])), abs=1e-11)
        assert (top_p < 1.0) == (not math.isnan(mg))


def test_ties_are_broken_by_ascending_index_and_closed_forms():
    V = 100
    row = np.zeros(V, np.float32)                              # uniform: every logit ties
    keep, lse, H, _ = orc.filter_row(row, 1.0, 7, 1.0)
    assert np.flatnonzero(keep).tolist() == list(range(7)) and H == pytest.approx(math.log(7), abs=1e-14)
    keep, lse, H, mg = orc.filter_row(row, 1.0, 0, 0.495)
    assert np.flatnonzero(keep).tolist() == list(range(50)) and H == pytest.approx(math.log(50), abs=1e-14)
    assert mg == pytest.approx(0.005, abs=1e-12)               # 50/100 - 0.495
    keep, _, _, _ = orc.filter_row(row, 1.0, 0, 0.505)
    assert keep.sum() == 51
    keep, _, H, mg = orc.filter_row(row, 1.0, 20, 0.26)         # nucleus is taken of the top-k mass: 0.26 * 20 -> 6
    assert np.flatnonzero(keep).tolist() == list(range(6)) and mg == pytest.approx(0.01, abs=1e-12)   # (0.052 - 0.05) / 0.2
    # two-point distribution: p = (0.8, 0.2) in reversed index order
    row = np.log(np.array([0.2, 0.8])).astype(np.float32)
    keep, lse, H, mg = orc.filter_row(row, 1.0, 0, 0.7)
    assert keep.tolist() == [False, True] and H == pytest.approx(0.0, abs=1e-15)
    assert mg == pytest.approx(0.1, abs=1e-7) and lse == pytest.approx(math.log(0.8), abs=1e-7)
    keep, _, H, _ = orc.filter_row(row, 1.0, 0, 0.85)
    assert keep.all() and H == pytest.approx(-(0.8 * math.log(0.8) + 0.2 * math.log(0.2)), abs=1e-7)


def test_masked_logits_are_never_kept():
    row = np.full(10, -np.inf, np.float32)
    row[[2, 7, 8]] = [1.0, 3.0, 1.0]
    keep, lse, H, _ = orc.filter_row(row, 1.0, 5, 1.0)
    assert np.flatnonzero(keep).tolist() == [2, 7, 8]
    keep, _, _, _ = orc.filter_row(row, 1.0, 2, 1.0)
    assert np.flatnonzero(keep).tolist() == [2, 7]              # the tie at 1.0 goes to the lower index
    keep, lse, H, _ = orc.filter_row(np.full(4, -np.inf, np.float32), 1.0, 2, 0.5)
    assert not keep.any() and lse == -math.inf and math.isnan(H)


def test_filters_off_is_the_unfiltered_step():
    for dtype in ("f32", "bf16"):
        w = wl.small_case(8, 4, 301, dtype=dtype, temperature=0.8, case_id=12)
        for tau in (0.0, w.taus[0]):
            a = orc.verify(w.target, w.draft, w.tokens, w.seed, 0.8, tau)
            b = orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, 0.8, tau, top_k=0, top_p=1.0)
            c = orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, 0.8, tau, top_k=w.V, top_p=1.0)
            for r in (b, c):
                assert np.array_equal(a.accept_len, r.accept_len) and np.array_equal(a.next_token, r.next_token)
                assert np.array_equal(a.gate, r.gate) and np.array_equal(a.ratio_ok, r.ratio_ok)
                np.testing.assert_allclose(a.entropy64, r.entropy64, atol=1e-12)
                np.testing.assert_allclose(a.Z, r.Z, rtol=1e-12)
                assert (r.keep_count == w.V).all()


def test_decisions_recomputed_by_brute_force():
    top_k, top_p = 60, 0.85
    w = wl.small_case(10, 5, 401, dtype="bf16", temperature=0.8, case_id=44)
    T = float(np.float32(0.8))
    tau = 0.35 * math.log(w.V)
    tau32 = float(np.float32(tau))
    r = orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, T, tau, top_k=top_k, top_p=top_p)

    def dist(row):
        z = wl.as_f32(row).astype(np.float64) / T
        keep = _np_keep(z, top_k, top_p)
        d = np.where(keep, np.exp(z - scipy.special.logsumexp(z[keep])), 0.0)
        return d

    for b in range(w.B):
        if np.nanmin(r.filter_margin[b]) < 1e-9:
            continue
        a = w.gamma
        for j in range(w.gamma):
            q, p = dist(w.draft[b, j]), dist(w.target[b, j])
            H = scipy.stats.entropy(q[q > 0])
            assert r.entropy64[b, j] == pytest.approx(H, abs=1e-10)
            u = orc.hsd_uniforms(w.seed, b, j, 0)[0]
            x = w.tokens[b, j]
            gate, ok = H < tau32, u * q[x] < p[x]
            if abs(H - tau32) > 1e-9 and (q[x] == 0 or abs(u - p[x] / q[x]) > 1e-9):
                assert bool(r.gate[b, j]) == gate and bool(r.ratio_ok[b, j]) == ok, (b, j)
        acc = np.logical_or(r.gate[b], r.ratio_ok[b])
        rej = np.flatnonzero(~acc)
        a = int(rej[0]) if len(rej) else w.gamma
        assert r.accept_len[b] == a
        u2 = orc.hsd_uniforms(w.seed, b, a, 0)[1]
        p = dist(w.target[b, a])
        wts = p if a == w.gamma else np.maximum(0.0, p - dist(w.draft[b, a]))
        C = np.cumsum(wts)
        if C[-1] > 0 and r.sample_margin[b] > 1e-9:
            assert r.next_token[b] == int(np.searchsorted(C, u2 * C[-1], side="right"))
            assert r.Z[b] == pytest.approx(C[-1], rel=1e-9)
        assert wts[r.next_token[b]] > 0                        # the sample lies in the support


def test_emitted_tokens_follow_the_filtered_target():
    """Monte Carlo through oracle_verify_filtered (gate off): drafts drawn from the filtered q, the token
    emitted at position 0 is distributed as the filtered p_0 and never leaves its support."""
    rng = np.random.default_rng(7)
    V, g, N = 8, 2, 200_000
    top_k, top_p = 6, 0.9
    P1 = (1.3 * rng.standard_normal((g + 1, V))).astype(np.float32)
    D1 = (1.3 * rng.standard_normal((g, V))).astype(np.float32)

    def dist(row):
        z = row.astype(np.float64)
        keep = _np_keep(z, top_k, top_p)
        return np.where(keep, np.exp(z - scipy.special.logsumexp(z[keep])), 0.0)

    q = np.stack([dist(D1[j]) for j in range(g)])
    p = np.stack([dist(P1[j]) for j in range(g + 1)])
    P = np.broadcast_to(P1, (N, g + 1, V)).copy()
    D = np.broadcast_to(D1, (N, g, V)).copy()
    tok = np.stack([rng.choice(V, size=N, p=q[j]) for j in range(g)], axis=1).astype(np.int32)
    r = orc.verify_filtered(P, D, tok, 4242, 1.0, 0.0, top_k=top_k, top_p=top_p)
    first = np.where(r.accept_len >= 1, tok[:, 0], r.next_token)
    cnt = np.bincount(first, minlength=V)
    sup = p[0] > 0
    assert cnt[~sup].sum() == 0 and 2 <= sup.sum() < V
    assert scipy.stats.chisquare(cnt[sup], N * p[0][sup]).pvalue > 1e-3
    rate = np.minimum(p[0], q[0]).sum()
    assert abs((r.accept_len >= 1).mean() - rate) < 5 * math.sqrt(rate * (1 - rate) / N)
    # teeth: the unfiltered target is a different distribution
    pu = scipy.special.softmax(P1[0].astype(np.float64))
    assert scipy.stats.chisquare(cnt[sup], N * pu[sup] / pu[sup].sum() ).pvalue < 1e-6 or abs(pu[sup].sum() - 1) > 0.02


def test_rejects_greedy_rows_and_bad_top_p():
    w = wl.small_case(2, 2, 50, case_id=3)
    with pytest.raises(ValueError):
        orc.verify_filtered(w.target, w.draft, w.tokens, 1, 0.0, 1.0, top_k=5)
    with pytest.raises(ValueError):
        orc.verify_filtered(w.target, w.draft, w.tokens, 1, 1.0, 1.0, top_p=0.0)


def test_forced_keep_count_moves_only_the_cut():
    w = wl.small_case(4, 3, 500, case_id=8)
    base = orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, 1.0, 0.0, top_k=0, top_p=0.8)
    same = orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, 1.0, 0.0, top_k=0, top_p=0.8,
                               force_keep_count=base.keep_count)
    assert np.array_equal(base.accept_len, same.accept_len) and np.array_equal(base.next_token, same.next_token)
    np.testing.assert_array_equal(base.entropy64, same.entropy64)
    fk = np.full_like(base.keep_count, -1)
    fk[2, 0] = base.keep_count[2, 0] + 3                       # three more tokens in one draft row
    moved = orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, 1.0, 0.0, top_k=0, top_p=0.8, force_keep_count=fk)
    assert moved.keep_count[2, 0] == base.keep_count[2, 0] + 3
    assert moved.entropy64[2, 0] > base.entropy64[2, 0]
    mask = np.ones_like(base.keep_count, bool); mask[2, 0] = False
    assert np.array_equal(moved.keep_count[mask], base.keep_count[mask])
    assert np.array_equal(np.delete(moved.entropy64.ravel(), 2 * 3), np.delete(base.entropy64.ravel(), 2 * 3))


# ----------------------------------------------------------------------------- filters in the hierarchy driver
def _hier_case(B=24, g=3, V=60, seed=8):
    rng = np.random.default_rng(seed)
    base = (1.5 * rng.standard_normal((B, g + 2, V))).astype(np.float32)
    small = (base[:, :g] + rng.standard_normal((B, g, V))).astype(np.float32)
    mid = (base[:, :g + 1] + 0.4 * rng.standard_normal((B, g + 1, V))).astype(np.float32)
    tok = np.zeros((B, g), np.int32)
    return [small, mid, base], tok, rng


def test_hierarchy_with_filters_off_is_the_unfiltered_chain():
    models, tok, rng = _hier_case()
    tok[:] = rng.integers(0, models[0].shape[-1], tok.shape)
    taus = [1.0, 2.0]
    plain = orc.hsd_verify(models, tok, 5, 0.9, taus)
    for top_k, top_p in ((0, 1.0), (models[0].shape[-1], 1.0), (10 ** 6, 1.0)):
        h = orc.hsd_verify(models, tok, 5, 0.9, taus, top_k=top_k, top_p=top_p)
        for f in ("tokens", "accept_len", "next_token", "entropy", "level_accept", "level_next"):
            np.testing.assert_array_equal(getattr(h, f), getattr(plain, f))


@pytest.mark.parametrize("top_k,top_p", [(5, 1.0), (0, 0.8), (12, 0.9)])
def test_filtered_hierarchy_is_one_filtered_step_per_level(top_k, top_p):
    models, tok, rng = _hier_case()
    B, g, V = models[0].shape
    for b in range(B):
        for j in range(g):
            keep, _, _, _ = orc.filter_row(models[0][b, j], 1.0, top_k, top_p)
            tok[b, j] = rng.choice(np.flatnonzero(keep))
    taus = [0.3 * math.log(V), 0.5 * math.log(V)]
    h = orc.hsd_verify(models, tok, 3, 1.0, taus, top_k=top_k, top_p=top_p)
    l1 = orc.verify_filtered(models[1], models[0], tok, 3, 1.0, taus[0], top_k=top_k, top_p=top_p, level=0)
    np.testing.assert_array_equal(h.level_accept[0], l1.accept_len)
    np.testing.assert_array_equal(h.level_next[0], l1.next_token)
    tok2 = np.full((B, g + 1), -1, np.int32)
    for b in range(B):
        a = l1.accept_len[b]
        tok2[b, :a] = tok[b, :a]
        tok2[b, a] = l1.next_token[b]
    l2 = orc.verify_filtered(models[2], models[1], tok2, 3, 1.0, taus[1], top_k=top_k, top_p=top_p,
                             draft_len=l1.accept_len + 1, level=1)
    np.testing.assert_array_equal(h.accept_len, l2.accept_len)
    np.testing.assert_array_equal(h.next_token, l2.next_token)
    np.testing.assert_array_equal(h.tokens[:, :g + 1], tok2)
    np.testing.assert_array_equal(h.entropy[0][:, :g], l1.entropy)
    np.testing.assert_array_equal(h.entropy[1], l2.entropy)
    # every token a level hands on lies in that level's verifier's keep set, so the next level's ratio test
    # never divides by a filtered-out draft probability
    for b in range(B):
        a = l1.accept_len[b]
        keep, _, _, _ = orc.filter_row(models[1][b, a], 1.0, top_k, top_p)
        assert keep[l1.next_token[b]]
    plain = orc.hsd_verify(models, tok, 3, 1.0, taus)
    assert not np.array_equal(plain.next_token, h.next_token)    # the filters matter on this case


def test_filtered_two_level_first_token_follows_filtered_final_target():
    """Gate off, tiny V: drafts drawn from the smallest model's filtered distribution; the first token the
    two-level chain emits is distributed as the final target's filtered p_0."""
    rng = np.random.default_rng(23)
    V, g, N, top_k = 6, 1, 150_000, 3
    base = (1.3 * rng.standard_normal((g + 2, V))).astype(np.float32)
    small1 = (base[:g] + rng.standard_normal((g, V))).astype(np.float32)
    mid1 = (base[:g + 1] + 0.6 * rng.standard_normal((g + 1, V))).astype(np.float32)
    models = [np.broadcast_to(m, (N,) + m.shape).copy() for m in (small1, mid1, base)]

    def filtered(row):
        z = row.astype(np.float64)
        keep = _np_keep(z, top_k, 1.0)
        p = np.where(keep, np.exp(z - z.max()), 0.0)
        return p / p.sum()

    tok = rng.choice(V, size=(N, 1), p=filtered(small1[0])).astype(np.int32)
    h = orc.hsd_verify(models, tok, 41, 1.0, [0.0, 0.0], top_k=top_k)
    first = np.where(h.accept_len >= 1, h.tokens[:, 0], h.next_token)
    want = filtered(base[0])
    counts = np.bincount(first, minlength=V)
    assert np.all(counts[want == 0] == 0)
    assert scipy.stats.chisquare(counts[want > 0], N * want[want > 0]).pvalue > 1e-3
    full = scipy.special.softmax(base[0].astype(np.float64))    # the unfiltered target is told apart
    assert scipy.stats.chisquare(counts, N * full).pvalue < 1e-6
    assert set(np.flatnonzero(filtered(mid1[0]))) != set(np.flatnonzero(want))   # the keep sets differ by level


def test_filtered_sample_interval_brackets_the_sampling_uniform():
    """Test aid: the CDF interval of a token in the filtered distribution a stop row is sampled from equals a numpy
    restatement (kept sets by stable sort, renormalised, residual or bonus), follows forced keep counts, and holds
    the sampling uniform for the oracle's own token."""
    w = wl.small_case(12, 3, 257, dtype="f32", temperature=0.8, case_id=601)
    T = float(np.float32(0.8))
    top_k, top_p = 40, 0.9
    call = orc.VerifyCall(w.target, w.draft, w.tokens, w.seed, T, -1.0)
    r = call.run(top_k=top_k, top_p=top_p)

    def kept_probs(row, m):
        z = row.astype(np.float64) / T
        order = np.argsort(-z, kind="stable")[:m]
        p = np.zeros_like(z)
        p[order] = np.exp(z[order] - np.logaddexp.reduce(z[order]))
        return p

    g = w.gamma
    for b in range(w.B):
        a = int(r.accept_len[b])
        p = kept_probs(w.target[b, a], int(r.keep_count[b, g + a]))
        wgt = p if a >= g else np.maximum(0.0, p - kept_probs(w.draft[b, a], int(r.keep_count[b, a])))
        C = np.cumsum(wgt)
        k = int(r.next_token[b])
        lo, hi = call.sample_interval(b, a, k, top_k=top_k, top_p=top_p)
        assert lo == pytest.approx((C[k - 1] if k else 0.0) / C[-1], abs=1e-12) and hi == pytest.approx(C[k] / C[-1], abs=1e-12)
        u2 = orc.hsd_uniforms(w.seed, b, a, 0)[1]
        assert lo <= u2 < hi or r.sample_margin[b] < 1e-12
    # forced keep counts move the interval with the cut
    fk = r.keep_count.copy()
    b = int(np.flatnonzero(r.accept_len < g)[0]) if (r.accept_len < g).any() else 0
    a = int(r.accept_len[b])
    fk[b, g + a] = 3
    p3 = kept_probs(w.target[b, a], 3)
    wgt = p3 if a >= g else np.maximum(0.0, p3 - kept_probs(w.draft[b, a], int(fk[b, a])))
    k = int(np.argmax(wgt))
    C = np.cumsum(wgt)
    lo, hi = call.sample_interval(b, a, k, top_k=top_k, top_p=top_p, force_keep_count=fk)
    assert hi - lo == pytest.approx(wgt[k] / C[-1], abs=1e-12)
    # filters off: the unfiltered interval
    call0 = orc.VerifyCall(w.target, w.draft, w.tokens, w.seed, T, -1.0)
    r0 = call0.run()
    for b in range(4):
        i1 = call0.sample_interval(b, int(r0.accept_len[b]), int(r0.next_token[b]))
        i2 = call0.sample_interval(b, int(r0.accept_len[b]), int(r0.next_token[b]), top_k=0, top_p=1.0)
        assert i1 == pytest.approx(i2, abs=1e-13)
