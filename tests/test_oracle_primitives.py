"""Pins of the oracle's primitives against things other than itself (CPU only).

Philox: published known-answer vectors + an independent pure-Python transcription of the
published round function.  Row statistics: scipy routines and closed forms.  Acceptance test:
closed form min(1, p/q) over the full uniform lattice.  Inverse CDF: numpy cumsum+searchsorted.
"""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from conftest import golden_path
from oracle import hola_oracle as orc
from paper_2506_18952_amd import workloads as wl


# ----------------------------------------------------------------------------- Philox
def _kat_rows():
    rows = []
    with open(golden_path("philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v = [int(x, 16) for x in line.split()]
            rows.append((v[0:4], v[4:6], tuple(v[6:10])))
    return rows


def _philox_py(ctr, key):
    """Independent statement of Philox4x32-10 with Python integers."""
    c, k = list(ctr), list(key)
    for rnd in range(10):
        if rnd:
            k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return tuple(c)


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert orc.philox4x32_10(ctr, key) == want
        assert _philox_py(ctr, key) == want


def test_philox_matches_python_on_random_inputs():
    rng = np.random.default_rng(0)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert orc.philox4x32_10(ctr, key) == _philox_py(ctr, key)


def test_u24_lattice():
    assert orc.u24(0) == 0.0
    assert orc.u24(0xFF) == 0.0                    # low 8 bits dropped
    assert orc.u24(0x100) == 2.0 ** -24
    assert orc.u24(0xFFFFFFFF) == 1.0 - 2.0 ** -24  # never reaches 1
    # exactly representable in float32
    for r in (0x12345678, 0xFFFFFFFF, 0x80000000):
        assert float(np.float32(orc.u24(r))) == orc.u24(r)


def test_hsd_uniform_keying():
    """Counter = (position, seq lo, seq hi, level), key = (seed lo, seed hi); word0/word1."""
    seed, seq, pos, level = 0x1122334455667788, 0x1_0000_0005, 3, 2
    r = _philox_py([pos, seq & 0xFFFFFFFF, seq >> 32, level], [seed & 0xFFFFFFFF, seed >> 32])
    u, u2 = orc.hsd_uniforms(seed, seq, pos, level)
    assert u == (r[0] >> 8) / 2 ** 24 and u2 == (r[1] >> 8) / 2 ** 24
    # every coordinate matters
    base = orc.hsd_uniforms(5, 7, 1, 0)
    assert len({base, orc.hsd_uniforms(6, 7, 1, 0), orc.hsd_uniforms(5, 8, 1, 0),
                orc.hsd_uniforms(5, 7, 2, 0), orc.hsd_uniforms(5, 7, 1, 1),
                orc.hsd_uniforms(5 + (1 << 32), 7, 1, 0), orc.hsd_uniforms(5, 7 + (1 << 32), 1, 0)}) == 7


# ----------------------------------------------------------------------------- row statistics
@pytest.mark.parametrize("V", [1, 2, 7, 1000, 32000])
def test_entropy_of_uniform_logits_is_lnV(V):
    for c in (0.0, -3.5, 11.0):
        lse, H, am = orc.row_stats(np.full(V, c, np.float32), 1.0)
        assert H == pytest.approx(math.log(V), abs=1e-12 * max(1, V))
        assert lse == pytest.approx(c + math.log(V), abs=1e-12)
        assert am == 0                                   # lowest index on ties


def test_one_hot_with_minus_inf_has_zero_entropy():
    row = np.full(50, -np.inf, np.float32)
    row[17] = 2.5
    lse, H, am = orc.row_stats(row, 0.7)
    assert H == 0.0 and am == 17
    assert lse == pytest.approx(2.5 / 0.7, rel=1e-15)


def test_all_minus_inf_row():
    lse, H, am = orc.row_stats(np.full(9, -np.inf, np.float32), 1.0)
    assert lse == -np.inf and math.isnan(H) and am == -1


@pytest.mark.parametrize("a,b", [(0.0, 0.0), (1.0, -1.0), (3.0, -4.0), (-20.0, 20.0)])
def test_two_point_entropy_is_binary_entropy(a, b):
    _, H, _ = orc.row_stats(np.array([a, b], np.float32), 1.0)
    p = 1.0 / (1.0 + math.exp(b - a))
    hb = 0.0
    for x in (p, 1 - p):
        if x > 0:
            hb -= x * math.log(x)
    assert H == pytest.approx(hb, abs=1e-14)


@pytest.mark.parametrize("V,a", [(10, 0.5), (1000, 2.0 ** -7), (128256, 2.0 ** -13), (128256, 2.0 ** -5)])
def test_geometric_logits_closed_form(V, a):
    """z_i = -a*i: lse = ln((1-r^V)/(1-r)), H = lse + a*(r/(1-r) - V r^V/(1-r^V)), r = e^-a.

    a is a power of two, so every z_i is exact in float32 and the closed form applies at full V."""
    z32 = (-a * np.arange(V, dtype=np.float64)).astype(np.float32)
    assert np.array_equal(z32.astype(np.float64), -a * np.arange(V, dtype=np.float64))
    lse, H, am = orc.row_stats(z32, 1.0)
    r = math.exp(-a)
    lse_cf = math.log(-math.expm1(-a * V) / -math.expm1(-a))
    H_cf = lse_cf + a * (r / -math.expm1(-a) - V * r ** V / -math.expm1(-a * V))
    assert lse == pytest.approx(lse_cf, abs=1e-11)
    assert H == pytest.approx(H_cf, abs=1e-10)
    assert am == 0


@pytest.mark.parametrize("T", [1.0, 0.8, 0.7, 2.5])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_stats_match_scipy(T, dtype):
    rng = np.random.default_rng(3)
    for V in (5, 257, 4099):
        x = (3.0 * rng.standard_normal(V)).astype(np.float32)
        x[rng.integers(0, V)] += 9.0
        if V > 5:
            x[rng.integers(0, V, 3)] = -np.inf          # masked vocabulary entries
        row = wl.f32_to_bf16_bits(x) if dtype == "bf16" else x
        xs = wl.as_f32(row).astype(np.float64)
        T32 = float(np.float32(T))
        lse, H, am = orc.row_stats(row, T32)
        z = xs / T32
        assert lse == pytest.approx(scipy.special.logsumexp(z), rel=1e-14)
        p = scipy.special.softmax(z)
        assert H == pytest.approx(scipy.stats.entropy(p), rel=1e-12)
        assert am == int(np.argmax(xs))


def test_shift_invariance_and_temperature_monotonicity():
    rng = np.random.default_rng(4)
    x = (2.0 * rng.standard_normal(3000)).astype(np.float32)
    lse0, H0, _ = orc.row_stats(x, 1.0)
    lse1, H1, _ = orc.row_stats((x.astype(np.float64) + 8.0).astype(np.float32), 1.0)
    # the shift is applied in float32, so compare with its stored value
    assert H1 == pytest.approx(H0, abs=2e-5)
    assert lse1 - 8.0 == pytest.approx(lse0, abs=2e-5)
    Hs = [orc.row_stats(x, float(np.float32(T)))[1] for T in (0.25, 0.5, 0.8, 1.0, 1.5, 3.0, 10.0)]
    assert all(b > a for a, b in zip(Hs, Hs[1:]))        # entropy grows with temperature
    assert Hs[-1] < math.log(3000)


def test_greedy_temperature_zero_uses_unscaled_logits_and_argmax_ties():
    x = np.array([1.0, 5.0, 5.0, -2.0], np.float32)
    lse0, H0, am0 = orc.row_stats(x, 0.0)
    lse1, H1, am1 = orc.row_stats(x, 1.0)
    assert (lse0, H0) == (lse1, H1) and am0 == am1 == 1   # lowest index among ties


# ----------------------------------------------------------------------------- acceptance test
def test_ratio_accept_special_cases():
    # p = q accepts for every u in [0,1); p_x = 0 rejects for every u, also u = 0
    for u in (0.0, 2.0 ** -24, 0.5, 1.0 - 2.0 ** -24):
        assert orc.ratio_accept(u, 0.3, 0.3)
        assert not orc.ratio_accept(u, 0.0, 0.3)
        assert not orc.ratio_accept(u, 0.0, 0.0)
        assert orc.ratio_accept(u, 1e-30, 0.0)            # q_x = 0 < p_x accepts
        assert orc.ratio_accept(u, 0.9, 0.3)              # p_x > q_x accepts
    assert orc.ratio_accept(0.49, 0.5, 1.0) and not orc.ratio_accept(0.5, 0.5, 1.0)  # strict


@pytest.mark.parametrize("p,q", [(0.2, 0.7), (0.7, 0.2), (0.123456789, 0.987654321),
                                 (1e-9, 1e-3), (0.5, 0.5), (0.0, 0.4), (3e-5, 4e-5)])
def test_ratio_accept_frequency_over_full_lattice(p, q):
    """Accepted fraction of all 2^24 lattice uniforms equals min(1, p/q) within one lattice step."""
    n = orc.ratio_accept_lattice_count(p, q, 1)
    want = min(1.0, p / q) if q > 0 else 1.0
    assert abs(n / 2 ** 24 - want) <= 2.0 ** -24


# ----------------------------------------------------------------------------- inverse CDF
def _np_inverse_cdf(w, u):
    C = np.cumsum(w)
    return int(np.searchsorted(C, u * C[-1], side="right"))


def test_inverse_cdf_matches_cumsum_searchsorted():
    rng = np.random.default_rng(5)
    for V in (1, 2, 3, 17, 1000, 50000):
        w = rng.random(V) ** 4
        w[rng.random(V) < 0.3] = 0.0
        if w.sum() == 0:
            w[0] = 1.0
        for u in list(rng.random(25)) + [0.0, 1.0 - 2.0 ** -24]:
            tok, Z, margin = orc.inverse_cdf(w, u)
            ref = _np_inverse_cdf(w, u)
            assert tok == min(ref, V - 1) or (ref >= V and w[tok] > 0)
            assert Z == pytest.approx(w.sum(), rel=1e-12)
            assert w[tok] > 0.0                           # zero-weight tokens are never selected
            C = np.cumsum(w)
            lo = (C[tok - 1] if tok else 0.0)
            assert margin == pytest.approx(min(u * Z - lo, C[tok] - u * Z) / Z, abs=1e-12)


def test_inverse_cdf_edge_cases():
    assert orc.inverse_cdf(np.zeros(5), 0.3)[0] == -1      # no positive weight
    w = np.array([0.0, 0.0, 2.0, 0.0, 1.0, 0.0])
    assert orc.inverse_cdf(w, 0.0)[0] == 2                 # u = 0 picks the first positive weight
    assert orc.inverse_cdf(w, 0.6666)[0] == 2
    assert orc.inverse_cdf(w, 0.6667)[0] == 4
    assert orc.inverse_cdf(w, 1.0 - 2.0 ** -24)[0] == 4    # never an index past the last positive weight
    assert orc.inverse_cdf(w, 2.0 / 3.0)[0] in (2, 4)      # exactly on a boundary: C_i > t is strict


def test_inverse_cdf_lattice_frequencies():
    w = np.array([0.1, 0.0, 0.25, 0.4, 0.0, 0.25])
    hist = orc.inverse_cdf_lattice_hist(w, 1)
    assert hist.sum() == 2 ** 24
    assert np.all(np.abs(hist / 2 ** 24 - w / w.sum()) <= 2.0 ** -23)
    assert hist[1] == 0 and hist[4] == 0


# ----------------------------------------------------------------------------- residual weights
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_residual_weights_definition_and_invariants(dtype):
    rng = np.random.default_rng(6)
    V, T = 777, float(np.float32(0.8))
    P = (2 * rng.standard_normal(V)).astype(np.float32)
    D = (P + 0.7 * rng.standard_normal(V)).astype(np.float32)
    if dtype == "bf16":
        P, D = wl.f32_to_bf16_bits(P), wl.f32_to_bf16_bits(D)
    p = scipy.special.softmax(wl.as_f32(P).astype(np.float64) / T)
    q = scipy.special.softmax(wl.as_f32(D).astype(np.float64) / T)
    w = orc.residual_weights(P, D, T)
    np.testing.assert_allclose(w, np.maximum(0.0, p - q), rtol=0, atol=1e-15)
    assert w.sum() == pytest.approx(1.0 - np.minimum(p, q).sum(), abs=1e-13)   # Z = 1 - sum min(p,q)
    assert w.sum() == pytest.approx(0.5 * np.abs(p - q).sum(), abs=1e-13)      #   = total variation
    wb = orc.residual_weights(P, None, T, bonus=True)
    np.testing.assert_allclose(wb, p, rtol=1e-13, atol=0)
    # identical rows leave no residual at all
    assert orc.residual_weights(P, P, T).sum() == 0.0


def _entropy_unclamped(row, T):
    """lse - sum z p in IEEE double, ascending index order, exactly as Section 3.1's definition is evaluated."""
    z = [float(x) / T for x in np.asarray(row, np.float32).astype(np.float64)]
    m = max(z)
    S = 0.0
    for x in z:
        S += math.exp(x - m)
    lse = m + math.log(S)
    acc = 0.0
    for x in z:
        pr = math.exp(x - lse)
        if pr > 0.0:
            acc += x * pr
    return lse - acc


def test_entropy_is_never_negative_and_tau_zero_never_gates():
    """Shannon entropy (Section 3.1) is >= 0.  On nearly one-hot rows lse - sum z p cancels to rounding; whatever
    is left below zero is not entropy, so the oracle returns 0 there and a threshold of 0 (strict <) gates nothing."""
    rows = [np.array([35.14083480834961, -0.257364958524704, -1.2592607736587524, 1.5822691917419434], np.float32),
            np.array([1.6672909259796143, 35.24894332885742, -0.6074924468994141], np.float32),
            np.array([0.8733947277069092, 0.8153969049453735, 36.382686614990234, -0.076581209897995, 2.817026376724243],
                     np.float32)]
    for row in rows:
        assert _entropy_unclamped(row, 1.0) < 0.0              # rounding alone goes below zero on these rows
        lse, H, _ = orc.row_stats(row, 1.0)
        assert H == 0.0
    rng = np.random.default_rng(5)
    n_neg = 0
    for trial in range(3000):
        V = int(rng.integers(2, 6))
        row = rng.normal(0, 1, V).astype(np.float32)
        row[rng.integers(0, V)] += np.float32(rng.uniform(20, 40))
        T = float(rng.choice([0.7, 1.0, 1.3]))
        naive = _entropy_unclamped(row, T)
        n_neg += naive < 0.0
        lse, H, _ = orc.row_stats(row, T)
        assert H >= 0.0 and H == max(naive, 0.0)               # the clamp and nothing else
    # through the entry point: such rows are never gated at tau = 0
    P = np.zeros((3, 2, 5), np.float32)
    D = np.zeros((3, 1, 5), np.float32)
    for b, row in enumerate(rows):
        D[b, 0, :row.shape[0]] = row
        D[b, 0, row.shape[0]:] = -np.inf
    r = orc.verify(P, D, np.zeros((3, 1), np.int32), 0, 1.0, 0.0)
    assert not r.gate.any() and np.all(r.entropy64 == 0.0)


def test_plus_inf_or_nan_logit_gives_nan_statistics():
    """A row holding +inf or NaN has no softmax: both statistics are NaN (and a NaN entropy never gates)."""
    for bad in (np.inf, np.nan):
        row = np.array([0.5, bad, -1.0, 2.0], np.float32)
        lse, H, _ = orc.row_stats(row, 1.0)
        assert math.isnan(lse) and math.isnan(H)
        bits = wl.f32_to_bf16_bits(row)
        lse, H, _ = orc.row_stats(bits, 0.8)
        assert math.isnan(lse) and math.isnan(H)
    P = np.zeros((1, 2, 4), np.float32); D = np.zeros((1, 1, 4), np.float32)
    D[0, 0, 1] = np.inf
    r = orc.verify(P, D, np.zeros((1, 1), np.int32), 0, 1.0, 1e30)
    assert not r.gate.any()
